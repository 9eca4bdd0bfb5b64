// Block importance scores and Top-K block selection (Eq. 4 and the mask M of the sparse branch).
//
//  pool kernel    : one launch for Q and K_win, one wavefront per block of b tokens; 16-byte
//                   loads, fp32 sums, mean over the block's real length (the last block may be
//                   short).  HBM-bound streaming read.
//  select kernel  : one workgroup per query-block row.  The dot products A[i][j] = qbar_i . kbar_j are
//                   split over the four wavefronts by feature quarter, the row of scores is kept in
//                   LDS, every block gets its rank (number of blocks that beat it; ties go to the
//                   lower index), the k blocks of rank < k are written in ascending order with a
//                   ballot prefix sum.
#include "hf_common.h"

namespace hf {

namespace {

// Pooled keys are stored feature-group-major, kbar_t[bh][D/4][t_n][4], so that in the scoring
// kernel consecutive lanes (= consecutive KV blocks) read consecutive 16-byte groups.
// Pooled queries stay row-major, qbar[bh][t_m][D].
template <typename T, int D>
__global__ __launch_bounds__(256) void pool_kernel(const T* __restrict__ Q, int n_q, int bq, int t_m,
                                                   const T* __restrict__ K, int n_kv, int kv_stride, int bkv,
                                                   int t_n, int kv_first, int kv_end, float* __restrict__ qbar,
                                                   float* __restrict__ kbar_t) {
  constexpr int E = Elem<T>::kPer16B;  // elements per 16-byte load
  constexpr int LPR = D / E;           // lanes covering one row
  constexpr int RPP = kWave / LPR;     // rows per pass of the wavefront
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int blk = blockIdx.x * 4 + wave;
  const int bh = blockIdx.y;
  if (blk >= t_m + kv_end - kv_first) return;
  const bool is_q = blk < t_m;
  if (!is_q) blk += kv_first - t_m;  // KV blocks outside [kv_first, kv_end) keep the pooled means already stored
  const T* X = is_q ? Q : K;
  const int n = is_q ? n_q : n_kv, b = is_q ? bq : bkv;
  const int r0 = blk * b, r1 = min(n, r0 + b);
  const int sub = lane / LPR, col = (lane % LPR) * E;
  const T* base = X + (size_t)bh * (is_q ? n_q : kv_stride) * D + col;
  float acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.0f;
  int r = r0 + sub;
  // sixteen, then eight independent 16-byte loads in flight per lane
  for (; r + 15 * RPP < r1; r += 16 * RPP) {
    float v[16][E];
#pragma unroll
    for (int u = 0; u < 16; ++u) load16B<T>(base + (size_t)(r + u * RPP) * D, v[u]);
#pragma unroll
    for (int u = 0; u < 16; ++u)
#pragma unroll
      for (int e = 0; e < E; ++e) acc[e] += v[u][e];
  }
  for (; r + 7 * RPP < r1; r += 8 * RPP) {
    float v[8][E];
#pragma unroll
    for (int u = 0; u < 8; ++u) load16B<T>(base + (size_t)(r + u * RPP) * D, v[u]);
#pragma unroll
    for (int u = 0; u < 8; ++u)
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
#pragma unroll
    for (int e = 0; e < E; e += 4) {
      const float4 v = make_float4(acc[e] * inv, acc[e + 1] * inv, acc[e + 2] * inv, acc[e + 3] * inv);
      if (is_q)
        *reinterpret_cast<float4*>(qbar + ((size_t)bh * t_m + blk) * D + col + e) = v;
      else
        *reinterpret_cast<float4*>(kbar_t + (((size_t)bh * (D / 4) + (col + e) / 4) * t_n + blk) * 4) = v;
    }
  }
}

// One workgroup (four wavefronts) per query-block row.
// Scoring: wavefront w takes a quarter of the head dimension and lane l the KV blocks l, l + 64, ...;
// all of a thread's pooled-key loads are independent and issued together (the kernel is a chain of
// latencies, not of bytes), the four partial dot products of a block meet in LDS.
// Selection: thread j ranks block j against the row in LDS (rank = number of blocks that beat it;
// ties go to the lower index); the blocks of rank < k are written in ascending order with a ballot
// and a cross-wave prefix sum.
template <int D>
__global__ __launch_bounds__(256) void score_select_kernel(const float* __restrict__ qbar,
                                                           const float* __restrict__ kbar_t, int t_m, int t_n,
                                                           int k, int32_t* __restrict__ idx,
                                                           float* __restrict__ scores) {
  extern __shared__ __attribute__((aligned(16))) float smem[];  // [D] query, [4][t_pad] partials, [t_pad] scores
  __shared__ int wave_count[4];
  constexpr int CW = D / 16;  // 16-byte feature groups per wavefront
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x, bh = blockIdx.y;
  const int t_pad = (t_n + 3) & ~3;
  float* sq = smem;
  float* part = smem + D;
  float* sc = part + 4 * t_pad;
  if (tid < D) sq[tid] = qbar[((size_t)bh * t_m + row) * D + tid];
  if (tid < t_pad - t_n) sc[t_n + tid] = -INFINITY;  // padding never outranks a block
  __syncthreads();

  const float4* kt = reinterpret_cast<const float4*>(kbar_t) + ((size_t)bh * (D / 4) + wave * CW) * t_n;
  float4 q[CW];
#pragma unroll
  for (int c = 0; c < CW; ++c) q[c] = *reinterpret_cast<const float4*>(sq + 4 * (wave * CW + c));
  for (int j0 = lane; j0 < t_n; j0 += 256) {
    float4 kv[4][CW];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = min(j0 + 64 * u, t_n - 1);  // clamped: a valid address, the result is dropped
#pragma unroll
      for (int c = 0; c < CW; ++c) kv[u][c] = kt[(size_t)c * t_n + j];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
      for (int c = 0; c < CW; c += 2) {
        a0 = fmaf(q[c].x, kv[u][c].x, a0); a0 = fmaf(q[c].y, kv[u][c].y, a0);
        a0 = fmaf(q[c].z, kv[u][c].z, a0); a0 = fmaf(q[c].w, kv[u][c].w, a0);
        a1 = fmaf(q[c + 1].x, kv[u][c + 1].x, a1); a1 = fmaf(q[c + 1].y, kv[u][c + 1].y, a1);
        a1 = fmaf(q[c + 1].z, kv[u][c + 1].z, a1); a1 = fmaf(q[c + 1].w, kv[u][c + 1].w, a1);
      }
      if (j0 + 64 * u < t_n) part[wave * t_pad + j0 + 64 * u] = a0 + a1;
    }
  }
  __syncthreads();
  for (int j = tid; j < t_n; j += 256) {
    const float a = (part[j] + part[t_pad + j]) + (part[2 * t_pad + j] + part[3 * t_pad + j]);
    sc[j] = a;
    if (scores) scores[((size_t)bh * t_m + row) * t_n + j] = a;
  }
  __syncthreads();

  int32_t* out = idx + ((size_t)bh * t_m + row) * k;
  // First pass: rank by strict comparison only (two instructions per element).  Blocks with equal
  // scores share a rank, so the pass is exact unless a tie straddles the k-th place, which shows
  // as more than k blocks of rank < k; only then the row is redone with the tie rule.
  for (int pass = 0; pass < 2; ++pass) {
    int base = 0;
    for (int j0 = 0; j0 < t_n; j0 += 256) {  // uniform trip count: barriers inside
      const int j = j0 + tid;
      bool keep = false;
      if (j < t_n) {
        const float mine = sc[j];
        int rank = 0;
        if (pass == 0) {
          for (int o = 0; o < t_pad; o += 4) {
            const float4 v = *reinterpret_cast<const float4*>(sc + o);
            rank += (v.x > mine) ? 1 : 0;
            rank += (v.y > mine) ? 1 : 0;
            rank += (v.z > mine) ? 1 : 0;
            rank += (v.w > mine) ? 1 : 0;
          }
        } else {
          for (int o = 0; o < t_pad; o += 4) {
            const float4 v = *reinterpret_cast<const float4*>(sc + o);
            rank += (v.x > mine || (v.x == mine && o < j)) ? 1 : 0;
            rank += (v.y > mine || (v.y == mine && o + 1 < j)) ? 1 : 0;
            rank += (v.z > mine || (v.z == mine && o + 2 < j)) ? 1 : 0;
            rank += (v.w > mine || (v.w == mine && o + 3 < j)) ? 1 : 0;
          }
        }
        keep = rank < k;
      }
      const unsigned long long m = __ballot(keep);
      if (lane == 0) wave_count[wave] = __popcll(m);
      __syncthreads();
      int pos = base + __popcll(m & ((1ull << lane) - 1ull));
      int total = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int cw = wave_count[w];
        if (w < wave) pos += cw;
        total += cw;
      }
      if (keep && pos < k) out[pos] = j;
      base += total;
      __syncthreads();
    }
    if (base == k) break;  // uniform over the workgroup
  }
}

// Three query-block rows per workgroup of eight wavefronts: every row of a head reads that head's
// pooled keys from L2 (the launch is bound by that traffic: T_m x 75 KB per head at the 832x480
// shape), so sharing one read between three rows cuts it threefold.
// Scoring: wavefront w takes an eighth of the head dimension, lane l the KV blocks l, l + 64, ...,
// each loaded pooled key meets the three pooled queries (held in registers); the eight partial dot
// products of a (row, block) meet in LDS and are added in a fixed order.
// Selection: the 3 x T_n (row, block) pairs are ranked one per thread (441 or 507 of the 512
// threads at the two workloads' shapes) by strict comparison; wavefront r then turns row r's keep
// flags into the ascending list with a ballot prefix sum and, if a tie straddles the k-th place
// (more than k kept), redoes that row with the tie rule.
constexpr int kRows = 3;

template <int D>
__global__ __launch_bounds__(512) void score_select3_kernel(const float* __restrict__ qbar,
                                                            const float* __restrict__ kbar_t, int t_m, int t_n,
                                                            int k, int32_t* __restrict__ idx,
                                                            float* __restrict__ scores) {
  // LDS: [kRows][D] queries | [8][kRows][t_pad] partials (later: keep flags) | [kRows][t_pad] scores
  extern __shared__ __attribute__((aligned(16))) float smem[];
  constexpr int CW = D / 32;  // 16-byte feature groups per wavefront
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row0 = blockIdx.x * kRows, bh = blockIdx.y;
  const int t_pad = (t_n + 3) & ~3;
  float* sq = smem;
  float* part = smem + kRows * D;
  float* sc = part + 8 * kRows * t_pad;
  if (tid < kRows * D) {
    const int r = min(row0 + tid / D, t_m - 1);  // rows past the end repeat the last one; never written
    sq[tid] = qbar[((size_t)bh * t_m + r) * D + (tid % D)];
  }
  const int pad = t_pad - t_n;  // at most 3
  if (pad > 0 && tid < kRows * pad) sc[(tid / pad) * t_pad + t_n + tid % pad] = -INFINITY;  // never outranks a block
  __syncthreads();

  const float4* kt = reinterpret_cast<const float4*>(kbar_t) + ((size_t)bh * (D / 4) + wave * CW) * t_n;
  float4 q[kRows][CW];
#pragma unroll
  for (int r = 0; r < kRows; ++r)
#pragma unroll
    for (int c = 0; c < CW; ++c) q[r][c] = *reinterpret_cast<const float4*>(sq + r * D + 4 * (wave * CW + c));
  for (int j0 = lane; j0 < t_n; j0 += 256) {
    float4 kv[4][CW];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = min(j0 + 64 * u, t_n - 1);  // clamped: a valid address, the result is dropped
#pragma unroll
      for (int c = 0; c < CW; ++c) kv[u][c] = kt[(size_t)c * t_n + j];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int r = 0; r < kRows; ++r) {
        float a = 0.0f;
#pragma unroll
        for (int c = 0; c < CW; ++c) {
          a = fmaf(q[r][c].x, kv[u][c].x, a); a = fmaf(q[r][c].y, kv[u][c].y, a);
          a = fmaf(q[r][c].z, kv[u][c].z, a); a = fmaf(q[r][c].w, kv[u][c].w, a);
        }
        if (j0 + 64 * u < t_n) part[(wave * kRows + r) * t_pad + j0 + 64 * u] = a;
      }
  }
  __syncthreads();
  for (int it = tid; it < kRows * t_n; it += 512) {
    const int r = it / t_n, j = it - r * t_n;
    const float* p = part + r * t_pad + j;
    const int ws = kRows * t_pad;  // stride between wavefronts' partials
    const float a = ((p[0] + p[ws]) + (p[2 * ws] + p[3 * ws])) + ((p[4 * ws] + p[5 * ws]) + (p[6 * ws] + p[7 * ws]));
    sc[r * t_pad + j] = a;
    if (scores && row0 + r < t_m) scores[((size_t)bh * t_m + row0 + r) * t_n + j] = a;
  }
  __syncthreads();

  // rank every (row, block) pair by strict comparison: blocks with equal scores share a rank
  int* flags = reinterpret_cast<int*>(part);  // the partials are dead
  for (int it = tid; it < kRows * t_n; it += 512) {
    const int r = it / t_n, j = it - r * t_n;
    const float* my = sc + r * t_pad;
    const float mine = my[j];
    int rank = 0;
    for (int o = 0; o < t_pad; o += 4) {
      const float4 v = *reinterpret_cast<const float4*>(my + o);
      rank += (v.x > mine) ? 1 : 0;
      rank += (v.y > mine) ? 1 : 0;
      rank += (v.z > mine) ? 1 : 0;
      rank += (v.w > mine) ? 1 : 0;
    }
    flags[r * t_pad + j] = rank < k ? 1 : 0;
  }
  __syncthreads();

  if (wave >= kRows || row0 + wave >= t_m) return;
  const float* my = sc + wave * t_pad;
  const int* fl = flags + wave * t_pad;
  int32_t* out = idx + ((size_t)bh * t_m + row0 + wave) * k;
  int base = 0;
  for (int j0 = 0; j0 < t_n; j0 += 64) {  // wave-uniform
    const int j = j0 + lane;
    const bool keep = j < t_n && fl[j] != 0;
    const unsigned long long m = __ballot(keep);
    const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
    if (keep && pos < k) out[pos] = j;
    base += __popcll(m);
  }
  if (base == k) return;
  // a tie straddles the k-th place: exact ranks with the tie rule (lower index wins), this row only
  base = 0;
  for (int j0 = 0; j0 < t_n && base < k; j0 += 64) {
    const int j = j0 + lane;
    bool keep = false;
    if (j < t_n) {
      const float mine = my[j];
      int rank = 0;
      for (int o = 0; o < t_pad; o += 4) {
        const float4 v = *reinterpret_cast<const float4*>(my + o);
        rank += (v.x > mine || (v.x == mine && o < j)) ? 1 : 0;
        rank += (v.y > mine || (v.y == mine && o + 1 < j)) ? 1 : 0;
        rank += (v.z > mine || (v.z == mine && o + 2 < j)) ? 1 : 0;
        rank += (v.w > mine || (v.w == mine && o + 3 < j)) ? 1 : 0;
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

int launch_pool_both(const hf_config& c, const void* Q, int n_q, int t_m, const void* K, int n_kv, int t_n,
                     int kv_first, int kv_end, float* qbar, float* kbar_t, hipStream_t s) {
  const int BH = c.batch * c.heads;
  const dim3 grid((t_m + kv_end - kv_first + 3) / 4, BH), block(256);
#define HF_LAUNCH_POOL(T, DD)                                                                                  \
  hipLaunchKernelGGL((pool_kernel<T, DD>), grid, block, 0, s, static_cast<const T*>(Q), n_q, c.block_q, t_m,   \
                     static_cast<const T*>(K), n_kv, kv_stride_of(c, n_kv), c.block_kv, t_n, kv_first, kv_end, qbar, kbar_t)
  if (c.dtype == HF_BF16) {
    if (c.head_dim == 128) HF_LAUNCH_POOL(bf16_t, 128); else HF_LAUNCH_POOL(bf16_t, 64);
  } else {
    if (c.head_dim == 128) HF_LAUNCH_POOL(float, 128); else HF_LAUNCH_POOL(float, 64);
  }
#undef HF_LAUNCH_POOL
  return check_launch("hf_block_select(pool)");
}

int launch_score_select(const hf_config& c, const float* qbar, const float* kbar_t, int t_m, int t_n, int k,
                        int32_t* idx, float* scores, hipStream_t s) {
  const int BH = c.batch * c.heads;
  const int t_pad = (t_n + 3) & ~3;
  // three rows per workgroup while its LDS need stays within the default 64 KB
  const size_t smem3 = (size_t)(kRows * c.head_dim + 9 * kRows * t_pad) * sizeof(float);
  if (smem3 <= 64 * 1024) {
    const dim3 grid((t_m + kRows - 1) / kRows, BH), block(512);
    if (c.head_dim == 128)
      hipLaunchKernelGGL((score_select3_kernel<128>), grid, block, smem3, s, qbar, kbar_t, t_m, t_n, k, idx, scores);
    else
      hipLaunchKernelGGL((score_select3_kernel<64>), grid, block, smem3, s, qbar, kbar_t, t_m, t_n, k, idx, scores);
    return check_launch("hf_block_select(select)");
  }
  const dim3 grid(t_m, BH), block(256);
  const size_t smem = (size_t)(c.head_dim + 5 * t_pad) * sizeof(float);
  if (c.head_dim == 128)
    hipLaunchKernelGGL((score_select_kernel<128>), grid, block, smem, s, qbar, kbar_t, t_m, t_n, k, idx, scores);
  else
    hipLaunchKernelGGL((score_select_kernel<64>), grid, block, smem, s, qbar, kbar_t, t_m, t_n, k, idx, scores);
  return check_launch("hf_block_select(select)");
}

}  // namespace hf
