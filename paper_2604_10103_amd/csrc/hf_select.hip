// Block importance scores and Top-K block selection (Eq. 4 and the mask M of the sparse branch).
//
//  pool kernel    : one wavefront per block of b tokens; 16-byte loads, fp32 sums, mean over the
//                   block's real length (the last block may be short).  HBM-bound streaming read.
//  select kernel  : one wavefront per query-block row.  Lane j computes A[i][j] = qbar_i . kbar_j
//                   for its blocks, the row of scores is kept in LDS, every block gets its rank
//                   (number of blocks that beat it; ties go to the lower index), the k blocks of
//                   rank < k are written in ascending order with a ballot prefix sum.
#include "hf_common.h"

namespace hf {

namespace {

template <typename T, int D>
__global__ __launch_bounds__(256) void pool_kernel(const T* __restrict__ X, int n, int b, int t,
                                                   float* __restrict__ pooled) {
  constexpr int E = Elem<T>::kPer16B;  // elements per 16-byte load
  constexpr int LPR = D / E;           // lanes covering one row
  constexpr int RPP = kWave / LPR;     // rows per pass of the wavefront
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int blk = blockIdx.x * 4 + wave;
  const int bh = blockIdx.y;
  if (blk >= t) return;
  const int r0 = blk * b, r1 = min(n, r0 + b);
  const int sub = lane / LPR, col = (lane % LPR) * E;
  const T* base = X + (size_t)bh * n * D + col;
  float acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.0f;
  int r = r0 + sub;
  // four independent loads in flight per lane
  for (; r + 3 * RPP < r1; r += 4 * RPP) {
    float v[4][E];
#pragma unroll
    for (int u = 0; u < 4; ++u) load16B<T>(base + (size_t)(r + u * RPP) * D, v[u]);
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < E; ++e) acc[e] += v[u][e];
  }
  for (; r < r1; r += RPP) {
    float v[E];
    load16B<T>(base + (size_t)r * D, v);
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] += v[e];
  }
#pragma unroll
  for (int o = LPR; o < kWave; o <<= 1)
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] += __shfl_xor(acc[e], o, kWave);
  if (sub == 0) {
    const float inv = 1.0f / (float)(r1 - r0);
    float* out = pooled + ((size_t)bh * t + blk) * D + col;
#pragma unroll
    for (int e = 0; e < E; e += 4)
      *reinterpret_cast<float4*>(out + e) =
          make_float4(acc[e] * inv, acc[e + 1] * inv, acc[e + 2] * inv, acc[e + 3] * inv);
  }
}

template <int D>
__global__ __launch_bounds__(256) void score_select_kernel(const float* __restrict__ qbar,
                                                           const float* __restrict__ kbar, int t_m, int t_n,
                                                           int k, int32_t* __restrict__ idx,
                                                           float* __restrict__ scores) {
  extern __shared__ float smem[];  // [4][D] pooled query rows, then [4][t_n] scores
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row = blockIdx.x * 4 + wave;
  const int bh = blockIdx.y;
  if (row >= t_m) return;  // whole wavefront leaves; no workgroup barrier is used below
  float* sq = smem + wave * D;
  float* sc = smem + 4 * D + (size_t)wave * t_n;
  const float* q = qbar + ((size_t)bh * t_m + row) * D;
  for (int c = lane; c < D; c += kWave) sq[c] = q[c];
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): LDS writes of this wavefront are visible

  for (int j = lane; j < t_n; j += kWave) {
    const float* kr = kbar + ((size_t)bh * t_n + j) * D;
    float a = 0.0f;
#pragma unroll 8
    for (int c = 0; c < D; c += 4) {
      const float4 kv = *reinterpret_cast<const float4*>(kr + c);
      a = fmaf(sq[c], kv.x, a);
      a = fmaf(sq[c + 1], kv.y, a);
      a = fmaf(sq[c + 2], kv.z, a);
      a = fmaf(sq[c + 3], kv.w, a);
    }
    sc[j] = a;
    if (scores) scores[((size_t)bh * t_m + row) * t_n + j] = a;
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);

  int32_t* out = idx + ((size_t)bh * t_m + row) * k;
  int base = 0;
  for (int j0 = 0; j0 < t_n; j0 += kWave) {
    const int j = j0 + lane;
    bool keep = false;
    if (j < t_n) {
      const float mine = sc[j];
      int rank = 0;
      for (int o = 0; o < t_n; ++o) {
        const float other = sc[o];
        rank += (other > mine || (other == mine && o < j)) ? 1 : 0;
      }
      keep = rank < k;
    }
    const unsigned long long m = __ballot(keep);
    const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
    if (keep && pos < k) out[pos] = j;
    base += __popcll(m);
  }
}

}  // namespace

int launch_pool(const hf_config& c, const void* X, int n, int b, int t, float* pooled, hipStream_t s) {
  const int BH = c.batch * c.heads;
  const dim3 grid((t + 3) / 4, BH), block(256);
  if (c.dtype == HF_BF16) {
    const bf16_t* x = static_cast<const bf16_t*>(X);
    if (c.head_dim == 128) hipLaunchKernelGGL((pool_kernel<bf16_t, 128>), grid, block, 0, s, x, n, b, t, pooled);
    else hipLaunchKernelGGL((pool_kernel<bf16_t, 64>), grid, block, 0, s, x, n, b, t, pooled);
  } else {
    const float* x = static_cast<const float*>(X);
    if (c.head_dim == 128) hipLaunchKernelGGL((pool_kernel<float, 128>), grid, block, 0, s, x, n, b, t, pooled);
    else hipLaunchKernelGGL((pool_kernel<float, 64>), grid, block, 0, s, x, n, b, t, pooled);
  }
  return check_launch("hf_block_select(pool)");
}

int launch_score_select(const hf_config& c, const float* qbar, const float* kbar, int t_m, int t_n, int k,
                        int32_t* idx, float* scores, hipStream_t s) {
  const int BH = c.batch * c.heads;
  const dim3 grid((t_m + 3) / 4, BH), block(256);
  const size_t smem = (size_t)(4 * c.head_dim + 4 * (size_t)t_n) * sizeof(float);
  if (c.head_dim == 128)
    hipLaunchKernelGGL((score_select_kernel<128>), grid, block, smem, s, qbar, kbar, t_m, t_n, k, idx, scores);
  else
    hipLaunchKernelGGL((score_select_kernel<64>), grid, block, smem, s, qbar, kbar, t_m, t_n, k, idx, scores);
  return check_launch("hf_block_select(select)");
}

}  // namespace hf
