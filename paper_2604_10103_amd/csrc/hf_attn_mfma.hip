// Block-sparse flash forward on bf16 MFMA (placeholder until the tiled kernel lands).
#include "hf_common.h"

namespace hf {

bool attn_mfma_supported(const hf_config&) { return false; }

int launch_attn_mfma(const hf_config&, const void*, int, const void*, const void*, int, const int32_t*, int,
                     void*, hipStream_t) {
  set_error("MFMA attention kernel not available for this shape");
  return HF_ERR_SHAPE;
}

}  // namespace hf
