// Gradients of the hybrid attention for the training algorithm of the supplement (the one step per
// chunk that runs with gradients enabled): dQ, dK, dV of the block-sparse softmax attention (Eq. 5)
// for a fixed Top-K mask, and the gradient of the history readout (Eq. 3) with respect to its
// queries for a constant state.  This file: the kernels every shape and type can take (fp32
// arithmetic, one wavefront per few rows) and the small helpers shared with the matrix-core path.
//
// With P recomputed from the saved row statistic lse2 = log2 sum_j 2^(c s_ij) (c = scale log2 e):
//     D_i  = dO_i . O_local_i      (from the recomputed forward pass, before O_local is rounded)
//     dV_j = sum_i P_ij dO_i               dP_ij = dO_i . v_j
//     dS_ij = P_ij (dP_ij - D_i)
//     dQ_i = scale sum_j dS_ij k_j         dK_j = scale sum_i dS_ij q_i
// dQ walks the index list of its query block; dK, dV walk the inverse list (the query blocks that
// selected a KV block), so both accumulate in registers and nothing is added atomically.
#include <math.h>

#include "hf_common.h"

namespace hf {
namespace {

// ---- inverse of the index lists: for every KV block the query blocks whose row holds it, ascending ----
// One wavefront per (head, KV block): lane = query block, 64 at a time; a ballot and a prefix count compact
// the hits in order.
__global__ __launch_bounds__(256) void invert_index_kernel(const int32_t* __restrict__ idx, int k, int t_m, int t_n,
                                                           int32_t* __restrict__ inv_cnt,
                                                           int32_t* __restrict__ inv_list) {
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6), bh = blockIdx.y;
  if (j >= t_n) return;
  const int32_t* rows = idx + (size_t)bh * t_m * k;
  int32_t* out = inv_list + ((size_t)bh * t_n + j) * t_m;
  int cnt = 0;
  for (int i0 = 0; i0 < t_m; i0 += kWave) {
    const int i = i0 + lane;
    bool hit = false;
    if (i < t_m)
      for (int s = 0; s < k; ++s) hit |= rows[(size_t)i * k + s] == j;   // by contract a row lists a block at most once
    const unsigned long long mask = __ballot(hit);
    if (hit) out[cnt + __popcll(mask & ((1ull << lane) - 1ull))] = i;
    cnt += __popcll(mask);
  }
  if (lane == 0) inv_cnt[(size_t)bh * t_n + j] = cnt;
}

// The same lists by counting, one workgroup per head (used when a head's index rows and eight histograms fit in
// LDS): the rows are copied to LDS once; wavefront w owns a contiguous run of query blocks and walks it in order,
// first counting the hits per KV block, then, from the exclusive sums over the wavefronts, placing its query blocks
// behind those of the wavefronts before it.  Lanes of a wavefront work on one row at a time, whose entries are
// distinct by contract, so their counters are distinct: no atomics.  Ascending lists, as above.
constexpr int kInvWaves = 8;
__global__ __launch_bounds__(64 * kInvWaves) void invert_index_lds_kernel(const int32_t* __restrict__ idx, int k,
                                                                          int t_m, int t_n,
                                                                          int32_t* __restrict__ inv_cnt,
                                                                          int32_t* __restrict__ inv_list) {
  extern __shared__ int32_t inv_smem[];
  int32_t* rows = inv_smem;              // [t_m][k]
  int32_t* hist = inv_smem + t_m * k;    // [kInvWaves][t_n]
  const int bh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int32_t* src = idx + (size_t)bh * t_m * k;
  for (int e = tid; e < t_m * k; e += 64 * kInvWaves) rows[e] = src[e];
  for (int e = tid; e < kInvWaves * t_n; e += 64 * kInvWaves) hist[e] = 0;
  __syncthreads();
  const int seg = (t_m + kInvWaves - 1) / kInvWaves;
  const int i_begin = min(w * seg, t_m), i_end = min(i_begin + seg, t_m);
  int32_t* mine = hist + w * t_n;
  for (int i = i_begin; i < i_end; ++i)
    for (int s = lane; s < k; s += 64) {
      const int j = rows[i * k + s];
      if ((unsigned)j < (unsigned)t_n) mine[j] += 1;
    }
  __syncthreads();
  for (int j = tid; j < t_n; j += 64 * kInvWaves) {
    int base = 0;
    for (int v = 0; v < kInvWaves; ++v) {
      const int c = hist[v * t_n + j];
      hist[v * t_n + j] = base;
      base += c;
    }
    inv_cnt[(size_t)bh * t_n + j] = min(base, t_m);
  }
  __syncthreads();
  int32_t* out = inv_list + (size_t)bh * t_n * t_m;
  for (int i = i_begin; i < i_end; ++i)
    for (int s = lane; s < k; s += 64) {
      const int j = rows[i * k + s];
      if ((unsigned)j < (unsigned)t_n) {
        const int pos = mine[j];
        mine[j] = pos + 1;
        if (pos < t_m) out[(size_t)j * t_m + pos] = i;   // (a row that breaks the contract cannot write past a list)
      }
    }
}

// ---- dQ: R query rows per wavefront, lanes = keys for the dot products, lanes = features for dQ ------
template <typename T, int D, int R>
__global__ __launch_bounds__(256) void bwd_dq_generic_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, const T* __restrict__ dO,
    const int32_t* __restrict__ idx, int k, int n_q, int n_kv, int kv_stride, int bq, int bkv, int t_m, int t_n,
    float scale_log2e, float scale, const float* __restrict__ lse2, const float* __restrict__ Dv,
    const float* __restrict__ dqh32, T* __restrict__ dQ) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int C = D / kWave;
  __shared__ float sq[4][R][D];
  __shared__ float sdo[4][R][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int qb = blockIdx.x, bh = blockIdx.y;
  const T* Qh = Q + (size_t)bh * n_q * D;
  const T* dOh = dO + (size_t)bh * n_q * D;
  const T* Kh = K + (size_t)bh * kv_stride * D;
  const T* Vh = V + (size_t)bh * kv_stride * D;
  const int32_t* row_idx = idx ? idx + ((size_t)bh * t_m + qb) * k : nullptr;
  const int nsel = idx ? k : t_n;
  const int q_end = min(n_q, (qb + 1) * bq);

  for (int pass0 = qb * bq; pass0 < q_end; pass0 += 4 * R) {
    const int r0 = pass0 + wave * R;
    for (int w = lane; w < R * D; w += kWave) {
      const int rr = w / D, c = w % D;
      const int row = min(r0 + rr, n_q - 1);
      sq[wave][rr][c] = Elem<T>::load(Qh + (size_t)row * D + c) * scale_log2e;
      sdo[wave][rr][c] = Elem<T>::load(dOh + (size_t)row * D + c);
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);
    float lse[R], dv[R], dq[R][C];
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      const size_t row = (size_t)bh * n_q + min(r0 + rr, n_q - 1);
      lse[rr] = lse2[row];
      dv[rr] = Dv[row];
#pragma unroll
      for (int e = 0; e < C; ++e) dq[rr][e] = 0.0f;
    }
    for (int s = 0; s < nsel; ++s) {
      const int jb = row_idx ? row_idx[s] : s;
      if ((unsigned)jb >= (unsigned)t_n) continue;
      const int k_end = min(n_kv, (jb + 1) * bkv);
      for (int kc = jb * bkv; kc < k_end; kc += kWave) {
        const int key = kc + lane;
        const bool valid = key < k_end;
        const T* krow = Kh + (size_t)(valid ? key : kc) * D;
        const T* vrow = Vh + (size_t)(valid ? key : kc) * D;
        float sc[R], dp[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) { sc[rr] = 0.0f; dp[rr] = 0.0f; }
#pragma unroll 2
        for (int c = 0; c < D; c += E) {
          float kv[E], vv[E];
          load16B<T>(krow + c, kv);
          load16B<T>(vrow + c, vv);
#pragma unroll
          for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int e = 0; e < E; ++e) {
              sc[rr] = fmaf(sq[wave][rr][c + e], kv[e], sc[rr]);
              dp[rr] = fmaf(sdo[wave][rr][c + e], vv[e], dp[rr]);
            }
        }
        float ds[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
          const float p = valid ? exp2f(sc[rr] - lse[rr]) : 0.0f;
          ds[rr] = p * (dp[rr] - dv[rr]);
        }
        const int cnt = min(kWave, k_end - kc);
        for (int kk = 0; kk < cnt; ++kk) {
          const T* kr = Kh + (size_t)(kc + kk) * D + lane * C;
          float kv[C];
#pragma unroll
          for (int e = 0; e < C; ++e) kv[e] = Elem<T>::load(kr + e);
#pragma unroll
          for (int rr = 0; rr < R; ++rr) {
            const float d1 = __shfl(ds[rr], kk, kWave);
#pragma unroll
            for (int e = 0; e < C; ++e) dq[rr][e] = fmaf(d1, kv[e], dq[rr][e]);
          }
        }
      }
    }
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      const int row = r0 + rr;
      if (row < q_end) {
        const size_t off = ((size_t)bh * n_q + row) * D + lane * C;
#pragma unroll
        for (int e = 0; e < C; ++e)
          Elem<T>::store(dQ + off + e, dq[rr][e] * scale + (dqh32 ? dqh32[off + e] : 0.0f));
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// ---- dK, dV: R keys per wavefront, lanes = query rows for the dot products, lanes = features after ---
template <typename T, int D, int R>
__global__ __launch_bounds__(256) void bwd_dkv_generic_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, const T* __restrict__ dO,
    const int32_t* __restrict__ inv_cnt, const int32_t* __restrict__ inv_list, int n_q, int n_kv, int kv_stride,
    int bq, int bkv, int t_m, int t_n, float scale_log2e, float scale, const float* __restrict__ lse2,
    const float* __restrict__ Dv, T* __restrict__ dK, T* __restrict__ dV) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int C = D / kWave;
  __shared__ float sk[4][R][D];
  __shared__ float sv[4][R][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int jb = blockIdx.x, bh = blockIdx.y;
  const T* Qh = Q + (size_t)bh * n_q * D;
  const T* dOh = dO + (size_t)bh * n_q * D;
  const T* Kh = K + (size_t)bh * kv_stride * D;
  const T* Vh = V + (size_t)bh * kv_stride * D;
  const float* lseh = lse2 + (size_t)bh * n_q;
  const float* Dvh = Dv + (size_t)bh * n_q;
  const int n_lists = inv_cnt ? inv_cnt[(size_t)bh * t_n + jb] : t_m;   // no lists: every query block (dense)
  const int32_t* list = inv_list ? inv_list + ((size_t)bh * t_n + jb) * t_m : nullptr;
  const int k_end = min(n_kv, (jb + 1) * bkv);

  for (int pass0 = jb * bkv; pass0 < k_end; pass0 += 4 * R) {
    const int r0 = pass0 + wave * R;
    for (int w = lane; w < R * D; w += kWave) {
      const int rr = w / D, c = w % D;
      const int key = min(r0 + rr, n_kv - 1);
      sk[wave][rr][c] = Elem<T>::load(Kh + (size_t)key * D + c) * scale_log2e;
      sv[wave][rr][c] = Elem<T>::load(Vh + (size_t)key * D + c);
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);
    float dk[R][C], dv[R][C];
#pragma unroll
    for (int rr = 0; rr < R; ++rr)
#pragma unroll
      for (int e = 0; e < C; ++e) { dk[rr][e] = 0.0f; dv[rr][e] = 0.0f; }
    for (int t = 0; t < n_lists; ++t) {
      const int qb = list ? list[t] : t;
      const int q_end = min(n_q, (qb + 1) * bq);
      for (int qc = qb * bq; qc < q_end; qc += kWave) {
        const int row = qc + lane;
        const bool valid = row < q_end;
        const int rrow = valid ? row : qc;
        const T* qrow = Qh + (size_t)rrow * D;
        const T* drow = dOh + (size_t)rrow * D;
        const float lse = lseh[rrow], dvec = Dvh[rrow];
        float sc[R], dp[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) { sc[rr] = 0.0f; dp[rr] = 0.0f; }
#pragma unroll 2
        for (int c = 0; c < D; c += E) {
          float qv[E], dv_[E];
          load16B<T>(qrow + c, qv);
          load16B<T>(drow + c, dv_);
#pragma unroll
          for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int e = 0; e < E; ++e) {
              sc[rr] = fmaf(sk[wave][rr][c + e], qv[e], sc[rr]);
              dp[rr] = fmaf(sv[wave][rr][c + e], dv_[e], dp[rr]);
            }
        }
        float p[R], ds[R];
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
          p[rr] = valid ? exp2f(sc[rr] - lse) : 0.0f;
          ds[rr] = p[rr] * (dp[rr] - dvec);
        }
        const int cnt = min(kWave, q_end - qc);
        for (int kk = 0; kk < cnt; ++kk) {
          const T* qr = Qh + (size_t)(qc + kk) * D + lane * C;
          const T* dr = dOh + (size_t)(qc + kk) * D + lane * C;
          float qv[C], dov[C];
#pragma unroll
          for (int e = 0; e < C; ++e) { qv[e] = Elem<T>::load(qr + e); dov[e] = Elem<T>::load(dr + e); }
#pragma unroll
          for (int rr = 0; rr < R; ++rr) {
            const float p1 = __shfl(p[rr], kk, kWave), d1 = __shfl(ds[rr], kk, kWave);
#pragma unroll
            for (int e = 0; e < C; ++e) {
              dv[rr][e] = fmaf(p1, dov[e], dv[rr][e]);
              dk[rr][e] = fmaf(d1, qv[e], dk[rr][e]);
            }
          }
        }
      }
    }
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
      const int key = r0 + rr;
      if (key < k_end) {
        const size_t off = ((size_t)bh * kv_stride + key) * D + lane * C;
#pragma unroll
        for (int e = 0; e < C; ++e) {
          Elem<T>::store(dK + off + e, dk[rr][e] * scale);
          Elem<T>::store(dV + off + e, dv[rr][e]);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// ---- gradient of the history readout with respect to its queries, one wavefront per row -------------
//   f = phi(q), r = R f, num = r L, den = z_scale f.z + eps, out = num / den
//   dnum = g / den, dden = -(g . num) / den^2, df = R^T (dnum L^T) + z_scale dden z, dq = df phi'(q)
// TO = float writes the result for the dQ kernel to add before its one rounding; TO = T writes the
// gradient of a query tensor of its own.
template <typename T, typename TO, int D>
__global__ __launch_bounds__(256) void bwd_hist_generic_kernel(const T* __restrict__ Qh, const T* __restrict__ dO,
                                                               const float* __restrict__ state, int BH, int n_q,
                                                               const float* __restrict__ cosq,
                                                               const float* __restrict__ sinq, int phi_kind,
                                                               float eps, float z_scale, TO* __restrict__ out) {
  constexpr int C = D / kWave;   // 2 (one rotation pair per lane) or 1 (pair = lanes l, l^1)
  __shared__ float sr[4][D];
  __shared__ float sd[4][D];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int bh = blockIdx.y;
  const int row = blockIdx.x * 4 + wave;
  if (row >= n_q) return;
  const float* L = state + (size_t)bh * D * D;
  const float* z = state + (size_t)BH * D * D + (size_t)bh * D;
  const size_t off = ((size_t)bh * n_q + row) * D + lane * C;
  float q[C], f[C], r[C], g[C];
  float den = 0.0f;
#pragma unroll
  for (int e = 0; e < C; ++e) {
    q[e] = Elem<T>::load(Qh + off + e);
    g[e] = Elem<T>::load(dO + off + e);
    f[e] = phi_apply(q[e], phi_kind);
    den = fmaf(f[e], z[lane * C + e], den);
  }
  den = z_scale * wave_sum(den) + eps;
  // rotation of adjacent pairs (2p, 2p+1)
  float cs = 1.0f, sn = 0.0f;
  if (cosq) {
    const int pair = C == 2 ? lane : lane >> 1;
    cs = cosq[(size_t)row * (D / 2) + pair];
    sn = sinq[(size_t)row * (D / 2) + pair];
  }
  if (C == 2) {
    r[0] = f[0] * cs - f[C - 1] * sn;
    r[C - 1] = f[0] * sn + f[C - 1] * cs;
  } else {
    const float other = __shfl_xor(f[0], 1, kWave);
    r[0] = (lane & 1) ? other * sn + f[0] * cs : f[0] * cs - other * sn;
  }
#pragma unroll
  for (int e = 0; e < C; ++e) sr[wave][lane * C + e] = r[e];
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);
  // num_j = sum_i r_i L[i][j], lanes = j
  float num[C];
#pragma unroll
  for (int e = 0; e < C; ++e) num[e] = 0.0f;
  for (int i = 0; i < D; ++i) {
    const float ri = sr[wave][i];
#pragma unroll
    for (int e = 0; e < C; ++e) num[e] = fmaf(ri, L[(size_t)i * D + lane * C + e], num[e]);
  }
  float gn = 0.0f;
#pragma unroll
  for (int e = 0; e < C; ++e) gn = fmaf(g[e], num[e], gn);
  const float inv = 1.0f / den;
  const float dden = -wave_sum(gn) * inv * inv;
#pragma unroll
  for (int e = 0; e < C; ++e) sd[wave][lane * C + e] = g[e] * inv;   // dnum
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);
  // t_i = sum_j dnum_j L[i][j], lanes = i
  float t[C];
#pragma unroll
  for (int e = 0; e < C; ++e) {
    const float* Lrow = L + (size_t)(lane * C + e) * D;
    float acc = 0.0f;
    for (int j = 0; j < D; j += 4) {
      const float4 l4 = *reinterpret_cast<const float4*>(Lrow + j);
      acc = fmaf(sd[wave][j], l4.x, acc);
      acc = fmaf(sd[wave][j + 1], l4.y, acc);
      acc = fmaf(sd[wave][j + 2], l4.z, acc);
      acc = fmaf(sd[wave][j + 3], l4.w, acc);
    }
    t[e] = acc;
  }
  // back through the rotation (opposite angle), add the denominator's share, times phi'
  float df[C];
  if (C == 2) {
    df[0] = t[0] * cs + t[C - 1] * sn;
    df[C - 1] = -t[0] * sn + t[C - 1] * cs;
  } else {
    const float other = __shfl_xor(t[0], 1, kWave);
    df[0] = (lane & 1) ? -other * sn + t[0] * cs : t[0] * cs + other * sn;
  }
#pragma unroll
  for (int e = 0; e < C; ++e) {
    const float d1 = df[e] + z_scale * dden * z[lane * C + e];
    const float dphi = phi_kind == HF_PHI_RELU ? (q[e] > 0.0f ? 1.0f : 0.0f) : (q[e] > 0.0f ? 1.0f : __expf(q[e]));
    const float v = d1 * dphi;
    if (sizeof(TO) == 4) reinterpret_cast<float*>(out)[off + e] = v;
    else reinterpret_cast<bf16_t*>(out)[off + e] = f32_to_bf16(v);
  }
}

}  // namespace

int launch_invert_index(const hf_config& c, const int32_t* idx, int k, int t_m, int t_n, int32_t* inv_cnt,
                        int32_t* inv_list, hipStream_t s) {
  const size_t lds = ((size_t)t_m * k + (size_t)kInvWaves * t_n) * sizeof(int32_t);
  if (lds <= 48 * 1024) {
    hipLaunchKernelGGL(invert_index_lds_kernel, dim3(c.batch * c.heads), dim3(64 * kInvWaves), lds, s, idx, k, t_m, t_n,
                       inv_cnt, inv_list);
    return check_launch("hf_hybrid_attn_bwd(inverse lists)");
  }
  hipLaunchKernelGGL(invert_index_kernel, dim3((t_n + 3) / 4, c.batch * c.heads), dim3(256), 0, s, idx, k, t_m, t_n,
                     inv_cnt, inv_list);
  return check_launch("hf_hybrid_attn_bwd(inverse lists)");
}

int launch_bwd_generic(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                       const int32_t* idx, int k, const void* dO, const float* lse2, const float* Dv,
                       const int32_t* inv_cnt, const int32_t* inv_list, const float* dqh32, void* dQ, void* dK,
                       void* dV, hipStream_t s) {
  const int BH = c.batch * c.heads;
  const int t_m = (n_q + c.block_q - 1) / c.block_q, t_n = (n_kv + c.block_kv - 1) / c.block_kv;
  const float scale = c.softmax_scale > 0.0f ? c.softmax_scale : 1.0f / sqrtf((float)c.head_dim);
  const float sl2 = scale * 1.4426950408889634f;
  const int kvs = kv_stride_of(c, n_kv);
#define HF_LAUNCH_BWD(T, DD)                                                                                        \
  do {                                                                                                              \
    hipLaunchKernelGGL((bwd_dq_generic_kernel<T, DD, 4>), dim3(t_m, BH), dim3(256), 0, s, static_cast<const T*>(Q), \
                       static_cast<const T*>(K), static_cast<const T*>(V), static_cast<const T*>(dO), idx, k, n_q,  \
                       n_kv, kvs, c.block_q, c.block_kv, t_m, t_n, sl2, scale, lse2, Dv, dqh32,                     \
                       static_cast<T*>(dQ));                                                                        \
    hipLaunchKernelGGL((bwd_dkv_generic_kernel<T, DD, 4>), dim3(t_n, BH), dim3(256), 0, s,                          \
                       static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V),                \
                       static_cast<const T*>(dO), inv_cnt, inv_list, n_q, n_kv, kvs, c.block_q, c.block_kv, t_m,    \
                       t_n, sl2, scale, lse2, Dv, static_cast<T*>(dK), static_cast<T*>(dV));                        \
  } while (0)
  if (c.dtype == HF_F32) { if (c.head_dim == 128) HF_LAUNCH_BWD(float, 128); else HF_LAUNCH_BWD(float, 64); }
  else { if (c.head_dim == 128) HF_LAUNCH_BWD(bf16_t, 128); else HF_LAUNCH_BWD(bf16_t, 64); }
#undef HF_LAUNCH_BWD
  return check_launch("hf_hybrid_attn_bwd(dQ, dK, dV)");
}

int launch_bwd_hist_generic(const hf_config& c, const void* Q_hist, const void* dO, const float* state, int n_q,
                            const float* cosq, const float* sinq, void* out, bool out_f32, hipStream_t s) {
  const int BH = c.batch * c.heads;
  const dim3 grid((n_q + 3) / 4, BH), block(256);
#define HF_LAUNCH_HIST(T, TO, DD)                                                                                  \
  hipLaunchKernelGGL((bwd_hist_generic_kernel<T, TO, DD>), grid, block, 0, s, static_cast<const T*>(Q_hist),        \
                     static_cast<const T*>(dO), state, BH, n_q, cosq, sinq, c.phi, c.eps, c.z_scale,               \
                     static_cast<TO*>(out))
  if (c.dtype == HF_F32) {
    if (c.head_dim == 128) HF_LAUNCH_HIST(float, float, 128); else HF_LAUNCH_HIST(float, float, 64);
  } else if (out_f32) {
    if (c.head_dim == 128) HF_LAUNCH_HIST(bf16_t, float, 128); else HF_LAUNCH_HIST(bf16_t, float, 64);
  } else {
    if (c.head_dim == 128) HF_LAUNCH_HIST(bf16_t, bf16_t, 128); else HF_LAUNCH_HIST(bf16_t, bf16_t, 64);
  }
#undef HF_LAUNCH_HIST
  return check_launch("hf_hybrid_attn_bwd(history)");
}

// out[row] = A[row] . B[row] over head_dim features (bf16 storage, fp32 arithmetic): D = dO . O_local from a
// saved O_local.  16 lanes per row, 16 bytes per lane and tensor.
__global__ __launch_bounds__(256) void row_dot_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                                      long long rows, float* __restrict__ out) {
  const long long row = (long long)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int part = threadIdx.x & 15;
  float acc = 0.0f;
  if (row < rows) {
    const uint4 a = *reinterpret_cast<const uint4*>(A + row * 128 + part * 8);
    const uint4 b = *reinterpret_cast<const uint4*>(B + row * 128 + part * 8);
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc = fmaf(__uint_as_float(aw[i] << 16), __uint_as_float(bw[i] << 16), acc);
      acc = fmaf(__uint_as_float(aw[i] & 0xffff0000u), __uint_as_float(bw[i] & 0xffff0000u), acc);
    }
  }
#pragma unroll
  for (int off = 8; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 16);
  if (row < rows && part == 0) out[row] = acc;
}

int launch_row_dot(const hf_config& c, const void* A, const void* B, long long rows, float* out, hipStream_t s) {
  if (c.dtype != HF_BF16 || c.head_dim != 128) { set_error("row dot: bf16, head_dim 128 only"); return HF_ERR_SHAPE; }
  if (rows > (1ll << 34)) { set_error("too many rows"); return HF_ERR_SHAPE; }
  hipLaunchKernelGGL(row_dot_kernel, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, s,
                     static_cast<const bf16_t*>(A), static_cast<const bf16_t*>(B), rows, out);
  return check_launch("hf_hybrid_attn_bwd_saved(D)");
}

}  // namespace hf
