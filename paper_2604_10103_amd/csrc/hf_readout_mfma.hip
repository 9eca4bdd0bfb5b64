// History readout on bf16 MFMA (placeholder until the tiled kernel lands).
#include "hf_common.h"

namespace hf {

bool readout_mfma_supported(const hf_config&) { return false; }

int launch_readout_mfma(const hf_config&, const void*, int, const void*, const float*, const float*,
                        const float*, void*, hipStream_t) {
  set_error("MFMA readout kernel not available for this shape");
  return HF_ERR_SHAPE;
}

}  // namespace hf
