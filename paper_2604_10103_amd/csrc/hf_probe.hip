// Measurement helper: the rate at which this chip issues the MFMA of the attention kernels, as a practical
// ceiling next to the nominal peak.  No part of the method.
#include "hf_common.h"

namespace hf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kProbeWgs = 512;      // two workgroups per compute unit,
constexpr int kProbeThreads = 256;  // one wavefront per SIMD each: two wavefronts per SIMD
constexpr int kProbeUnroll = 16;

// every wavefront issues iters x 16 independent v_mfma_f32_32x32x16_bf16 (eight accumulators in turn) on
// operands that are neither zero nor constant across lanes (the clock a chip holds depends on what toggles)
__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(int iters, float* __restrict__ sink) {
  bf16x8 a[4], b[4];
  const unsigned seed = threadIdx.x * 2654435761u + blockIdx.x * 40503u;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const unsigned r = (seed >> ((3 * i + e) & 15)) & 127u;
      a[i][e] = static_cast<__bf16>(0.5f - (float)r * (1.0f / 128.0f));
      b[i][e] = static_cast<__bf16>((float)(r ^ 85u) * (1.0f / 256.0f) - 0.25f);
    }
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u)
      acc[u & 7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u & 3], b[(u >> 2) & 3], acc[u & 7], 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (s == 123456.789f) sink[0] = s;   // (keeps the products alive; practically never true)
}

}  // namespace

}  // namespace hf

using namespace hf;

extern "C" {

int hf_probe_mfma_bf16(int32_t iters, void* scratch4, double* flops_out, void* stream) {
  if (iters < 1 || iters > (1 << 20)) { set_error("iters must be in [1, 2^20]"); return HF_ERR_SHAPE; }
  if (!scratch4) { set_error("scratch4 is NULL"); return HF_ERR_NULL; }
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(kProbeWgs), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream), iters,
                     static_cast<float*>(scratch4));
  if (flops_out)
    *flops_out = (double)kProbeWgs * (kProbeThreads / 64) * (double)iters * kProbeUnroll * (2.0 * 32 * 32 * 16);
  return check_launch("hf_probe_mfma_bf16");
}

}  // extern "C"
