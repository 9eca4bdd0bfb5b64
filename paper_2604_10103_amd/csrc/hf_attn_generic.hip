// Block-sparse window attention (Eq. 5), shape-generic fp32-arithmetic kernel.
//
// Used for fp32 inputs (all arithmetic fp32, so the fp32-mode error bound holds) and for
// bf16 shapes the MFMA kernel does not cover.  One workgroup per (batch*head, query block);
// each wavefront carries R query rows at a time through the selected KV blocks:
//   scores : lane = key (64 keys per step), q broadcast from LDS, K row read by its lane
//   softmax: online (running max m, running sum l) in the exp2 domain, wave reductions
//   P V    : lanes = value features, p broadcast with a lane read, V row read coalesced
#include <stdlib.h>

#include "hf_common.h"

namespace hf {

namespace {

template <typename T, int D, int R>
__global__ __launch_bounds__(256) void attn_generic_kernel(const T* __restrict__ Q, const T* __restrict__ K,
                                                           const T* __restrict__ V,
                                                           const int32_t* __restrict__ idx, int k, int n_q,
                                                           int n_kv, int kv_stride, int bq, int bkv, int t_m,
                                                           int t_n, float scale_log2e, T* __restrict__ O,
                                                           float* __restrict__ lse2, const T* __restrict__ dO,
                                                           float* __restrict__ Dv) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int C = D / kWave;  // value features per lane
  __shared__ float sq[4][R][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int qb = blockIdx.x, bh = blockIdx.y;
  const T* Qh = Q + (size_t)bh * n_q * D;
  const T* Kh = K + (size_t)bh * kv_stride * D;  // heads of a cache buffer are kv_stride tokens apart
  const T* Vh = V + (size_t)bh * kv_stride * D;
  T* Oh = O + (size_t)bh * n_q * D;
  const int32_t* row_idx = idx ? idx + ((size_t)bh * t_m + qb) * k : nullptr;
  const int nsel = idx ? k : t_n;
  const int q_end = min(n_q, (qb + 1) * bq);

  // every wavefront runs the same number of passes; rows past the block end are computed on
  // clamped addresses and never written
  for (int pass0 = qb * bq; pass0 < q_end; pass0 += 4 * R) {
    const int r0 = pass0 + wave * R;
    for (int w = lane; w < R * D; w += kWave) {
      const int rr = w / D, c = w % D;
      const int row = min(r0 + rr, n_q - 1);
      sq[wave][rr][c] = Elem<T>::load(Qh + (size_t)row * D + c) * scale_log2e;
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);

    float m[R], l[R], o[R][C];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      m[rr] = -INFINITY;
      l[rr] = 0.0f;
#pragma unroll
      for (int e = 0; e < C; ++e) o[rr][e] = 0.0f;
    }

    for (int s = 0; s < nsel; ++s) {
      const int jb = row_idx ? row_idx[s] : s;
      if ((unsigned)jb >= (unsigned)t_n) continue;  // ignore an out-of-range block index
      const int k_end = min(n_kv, (jb + 1) * bkv);
      for (int kc = jb * bkv; kc < k_end; kc += kWave) {
        const int key = kc + lane;
        const bool valid = key < k_end;
        const T* krow = Kh + (size_t)(valid ? key : kc) * D;
        float sc[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) sc[rr] = 0.0f;
#pragma unroll 4
        for (int c = 0; c < D; c += E) {
          float kv[E];
          load16B<T>(krow + c, kv);
#pragma unroll
          for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int e = 0; e < E; ++e) sc[rr] = fmaf(sq[wave][rr][c + e], kv[e], sc[rr]);
        }
        float p[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
          const float sv = valid ? sc[rr] : -INFINITY;
          const float m_new = fmaxf(m[rr], wave_max(sv));  // finite: lane 0 of the step is a real key
          const float alpha = exp2f(m[rr] - m_new);
          p[rr] = valid ? exp2f(sv - m_new) : 0.0f;
          l[rr] = l[rr] * alpha + wave_sum(p[rr]);
          m[rr] = m_new;
#pragma unroll
          for (int e = 0; e < C; ++e) o[rr][e] *= alpha;
        }
        const int cnt = min(kWave, k_end - kc);
        for (int kk = 0; kk < cnt; ++kk) {
          const T* vrow = Vh + (size_t)(kc + kk) * D + lane * C;
          float vv[C];
#pragma unroll
          for (int e = 0; e < C; ++e) vv[e] = Elem<T>::load(vrow + e);
#pragma unroll
          for (int rr = 0; rr < R; ++rr) {
            const float pk = __shfl(p[rr], kk, kWave);
#pragma unroll
            for (int e = 0; e < C; ++e) o[rr][e] = fmaf(pk, vv[e], o[rr][e]);
          }
        }
      }
    }
    if (lse2) {
      // statistics for the backward pass instead of the output: log2 of the sum of 2^(scaled logit), and
      // D = dO . O_local from the unrounded output (uniform branch: every lane of the wavefront takes it)
#pragma unroll
      for (int rr = 0; rr < R; ++rr) {
        const int row = min(r0 + rr, n_q - 1);
        const float inv = l[rr] > 0.0f ? 1.0f / l[rr] : 0.0f;   // a row without a single real key: O_local = 0
        float acc = 0.0f;
#pragma unroll
        for (int e = 0; e < C; ++e)
          acc = fmaf(o[rr][e] * inv, Elem<T>::load(dO + ((size_t)bh * n_q + row) * D + lane * C + e), acc);
        acc = wave_sum(acc);
        if (lane == 0 && r0 + rr < q_end) {
          lse2[(size_t)bh * n_q + row] = l[rr] > 0.0f ? m[rr] + log2f(l[rr]) : INFINITY;  // no real key: P = 0
          Dv[(size_t)bh * n_q + row] = acc;
        }
      }
      __builtin_amdgcn_wave_barrier();
      continue;
    }
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      const int row = r0 + rr;
      if (row < q_end) {
        const float inv = l[rr] > 0.0f ? 1.0f / l[rr] : 0.0f;   // a row without a single real key: O_local = 0
#pragma unroll
        for (int e = 0; e < C; ++e) Elem<T>::store(Oh + (size_t)row * D + lane * C + e, o[rr][e] * inv);
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

}  // namespace

int launch_attn_generic(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                        const int32_t* idx, int k, void* O_local, hipStream_t s, float* lse2, const void* dO,
                        float* Dv) {
  const int BH = c.batch * c.heads;
  const int t_m = (n_q + c.block_q - 1) / c.block_q, t_n = (n_kv + c.block_kv - 1) / c.block_kv;
  const float scale = c.softmax_scale > 0.0f ? c.softmax_scale : 1.0f / sqrtf((float)c.head_dim);
  const float sl2 = scale * 1.4426950408889634f;
  const dim3 grid(t_m, BH), block(256);
#define HF_LAUNCH_GENERIC(T, DD)                                                                           \
  hipLaunchKernelGGL((attn_generic_kernel<T, DD, 4>), grid, block, 0, s, static_cast<const T*>(Q),         \
                     static_cast<const T*>(K), static_cast<const T*>(V), idx, k, n_q, n_kv, kv_stride_of(c, n_kv), c.block_q, \
                     c.block_kv, t_m, t_n, sl2, static_cast<T*>(O_local), lse2, static_cast<const T*>(dO), Dv)
  if (c.dtype == HF_F32) {
    if (c.head_dim == 128) HF_LAUNCH_GENERIC(float, 128); else HF_LAUNCH_GENERIC(float, 64);
  } else {
    if (c.head_dim == 128) HF_LAUNCH_GENERIC(bf16_t, 128); else HF_LAUNCH_GENERIC(bf16_t, 64);
  }
#undef HF_LAUNCH_GENERIC
  return check_launch("hf_hybrid_attn_fwd(attention)");
}

int launch_attn_mfma(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                     const int32_t* idx, int k, void* O_local, hipStream_t s);  // hf_attn_mfma.hip
bool attn_mfma_supported(const hf_config& c);
int launch_attn_w64(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                    const int32_t* idx, int k, void* O_local, hipStream_t s);  // hf_attn_w64.hip
bool attn_w64_supported(const hf_config& c);

int launch_attn(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                const int32_t* idx, int k, void* O_local, hipStream_t s) {
  if (c.batch * c.heads > 65535 || (n_q + c.block_q - 1) / c.block_q > (1 << 30)) {
    set_error("grid too large");
    return HF_ERR_SHAPE;
  }
  // bf16, head_dim 128: block_q 64 / 128 take the workgroup-per-query-block MFMA kernel, other
  // multiples of 64 the wavefront-per-64-rows MFMA kernel; everything else the fp32-arithmetic one
  if (attn_mfma_supported(c)) return launch_attn_mfma(c, Q, n_q, K, V, n_kv, idx, k, O_local, s);
  if (attn_w64_supported(c)) return launch_attn_w64(c, Q, n_q, K, V, n_kv, idx, k, O_local, s);
  return launch_attn_generic(c, Q, n_q, K, V, n_kv, idx, k, O_local, s, nullptr, nullptr, nullptr);
}

}  // namespace hf
