// History readout and hybrid sum (Eq. 3 without the Linear map, Eq. 6):
//   O[r][j] = O_local[r][j] + ( sum_i R_r(phi(q_r))[i] L[i][j] ) / ( z_scale * sum_i phi(q_r)[i] z[i] + eps )
//
// fp32-arithmetic kernel: a workgroup keeps the head's L (d x d fp32) in LDS and streams query
// rows through it, R rows per wavefront at a time; lanes own output features.
#include "hf_common.h"

namespace hf {

namespace {

template <typename T, int D, int R>
__global__ __launch_bounds__(256) void readout_fma_kernel(const T* __restrict__ Q, const T* __restrict__ Oloc,
                                                          const float* __restrict__ state,
                                                          const float* __restrict__ cosq,
                                                          const float* __restrict__ sinq, int n_q,
                                                          int rows_per_wg, int phi_kind, float eps, float z_scale,
                                                          int BH, T* __restrict__ O) {
  constexpr int C = D / kWave;
  extern __shared__ float smem[];
  float* sL = smem;                 // [D][D]
  float* sz = sL + D * D;           // [D]
  float* sf = sz + D;               // [4][R][2][D]: rotated phi(q) and plain phi(q)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int bh = blockIdx.y;
  const int row_begin = blockIdx.x * rows_per_wg;
  const int row_end = min(n_q, row_begin + rows_per_wg);
  const float* L = state + (size_t)bh * D * D;
  const float* z = state + (size_t)BH * D * D + (size_t)bh * D;
  for (int w = threadIdx.x * 4; w < D * D; w += 256 * 4)
    *reinterpret_cast<float4*>(sL + w) = *reinterpret_cast<const float4*>(L + w);
  if (threadIdx.x < D) sz[threadIdx.x] = z[threadIdx.x];
  __syncthreads();

  const T* Qh = Q + (size_t)bh * n_q * D;
  const T* Lh = Oloc + (size_t)bh * n_q * D;
  T* Oh = O + (size_t)bh * n_q * D;
  float* frot = sf + (size_t)wave * R * 2 * D;
  for (int r0 = row_begin + wave * R; r0 < row_end; r0 += 4 * R) {
    for (int w = lane; w < R * (D / 2); w += kWave) {
      const int rr = w / (D / 2), p = w % (D / 2);
      const int row = min(r0 + rr, n_q - 1);
      const float f0 = phi_apply(Elem<T>::load(Qh + (size_t)row * D + 2 * p), phi_kind);
      const float f1 = phi_apply(Elem<T>::load(Qh + (size_t)row * D + 2 * p + 1), phi_kind);
      float g0 = f0, g1 = f1;
      if (cosq) {
        const float c = cosq[(size_t)row * (D / 2) + p], s = sinq[(size_t)row * (D / 2) + p];
        g0 = f0 * c - f1 * s;
        g1 = f0 * s + f1 * c;
      }
      frot[(rr * 2 + 0) * D + 2 * p] = g0;
      frot[(rr * 2 + 0) * D + 2 * p + 1] = g1;
      frot[(rr * 2 + 1) * D + 2 * p] = f0;
      frot[(rr * 2 + 1) * D + 2 * p + 1] = f1;
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);
    float num[R][C], den[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      den[rr] = 0.0f;
#pragma unroll
      for (int e = 0; e < C; ++e) num[rr][e] = 0.0f;
    }
    for (int i = 0; i < D; ++i) {
      float lv[C];
#pragma unroll
      for (int e = 0; e < C; ++e) lv[e] = sL[i * D + e * kWave + lane];
      const float zi = sz[i];
#pragma unroll
      for (int rr = 0; rr < R; ++rr) {
        const float g = frot[(rr * 2 + 0) * D + i];
        den[rr] = fmaf(frot[(rr * 2 + 1) * D + i], zi, den[rr]);
#pragma unroll
        for (int e = 0; e < C; ++e) num[rr][e] = fmaf(g, lv[e], num[rr][e]);
      }
    }
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      const int row = r0 + rr;
      if (row < row_end) {
        const float inv = 1.0f / (z_scale * den[rr] + eps);
#pragma unroll
        for (int e = 0; e < C; ++e) {
          const size_t off = (size_t)row * D + e * kWave + lane;
          Elem<T>::store(Oh + off, Elem<T>::load(Lh + off) + num[rr][e] * inv);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

}  // namespace

int launch_readout_mfma(const hf_config& c, const void* Q, int n_q, const void* O_local, const float* state,
                        const float* cosq, const float* sinq, void* planes, void* O,
                        hipStream_t s);  // hf_readout_mfma.hip
bool readout_mfma_supported(const hf_config& c);

template <typename T, int D>
static int launch_readout_fma(const hf_config& c, const void* Q, int n_q, const void* O_local,
                              const float* state, const float* cosq, const float* sinq, void* O,
                              hipStream_t s) {
  constexpr int R = 4;
  const int BH = c.batch * c.heads;
  const int rows_per_wg = 256;
  const dim3 grid((n_q + rows_per_wg - 1) / rows_per_wg, BH), block(256);
  const size_t smem = (size_t)(D * D + D + 4 * R * 2 * D) * sizeof(float);
  auto kern = readout_fma_kernel<T, D, R>;
  if (smem > 64 * 1024) {
    static LdsGrant grant;   // (one per instantiation of this function template, i.e. per kernel)
    const int rc = grant_lds(grant, reinterpret_cast<const void*>(kern), (int)smem, "the readout kernel");
    if (rc != HF_OK) return rc;
  }
  hipLaunchKernelGGL(kern, grid, block, smem, s, static_cast<const T*>(Q), static_cast<const T*>(O_local), state,
                     cosq, sinq, n_q, rows_per_wg, c.phi, c.eps, c.z_scale, BH, static_cast<T*>(O));
  return check_launch("hf_hybrid_attn_fwd(readout)");
}

int launch_readout(const hf_config& c, const void* Q, int n_q, const void* O_local, const float* state,
                   const float* cosq, const float* sinq, void* planes, void* O, hipStream_t s) {
  if (readout_mfma_supported(c)) return launch_readout_mfma(c, Q, n_q, O_local, state, cosq, sinq, planes, O, s);
  if (c.dtype == HF_F32) {
    return c.head_dim == 128 ? launch_readout_fma<float, 128>(c, Q, n_q, O_local, state, cosq, sinq, O, s)
                             : launch_readout_fma<float, 64>(c, Q, n_q, O_local, state, cosq, sinq, O, s);
  }
  return c.head_dim == 128 ? launch_readout_fma<bf16_t, 128>(c, Q, n_q, O_local, state, cosq, sinq, O, s)
                           : launch_readout_fma<bf16_t, 64>(c, Q, n_q, O_local, state, cosq, sinq, O, s);
}

}  // namespace hf
