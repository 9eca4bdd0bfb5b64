// Block-sparse flash forward (Eq. 5) on bf16 MFMA for gfx950: head_dim 128, block_q 64 or 128.
//
// One workgroup owns one query block; each of its wavefronts owns 32 query rows and walks the
// block's selected KV blocks in tiles of 32 keys.  The products are formed TRANSPOSED so that
// every softmax statistic is private to a lane:
//
//   S^T (keys x queries) = K_tile (A operand, from LDS)   x  Q^T (B operand, registers)
//   O^T (d x queries)   += V_tile^T (A operand, from LDS) x  P^T (B operand, registers)
//
// With the 32x32x16 MFMA a lane then holds, for ONE query, 16 of the tile's 32 scores: row max
// and row sum are in-lane reductions plus one exchange with lane^32, the rescale factor is a
// per-lane scalar, and the exp'd accumulators of S^T are, after rounding to bf16, already the
// B operand of the second product.  The k index of that MFMA is thereby bound to the order in
// which a lane holds keys: 16 t2 + 8 x + 4 (lane / 32) + 0..3.
//
// Staging.  K and V tiles go global -> LDS directly (buffer loads with the LDS bit: 16 bytes per lane,
// 1 KB = 4 key rows per instruction, no staging registers, no LDS stores), row-major with the 16-byte
// units of a row permuted (K: u ^ (row & 15), V: u ^ (4 (row & 3) | (row >> 2 & 3))) by choosing which global unit a lane
// fetches.  A K fragment is one 16-byte read; a V^T fragment is two transposing 8-byte reads
// (ds_read_b64_tr_b16: a 16-lane group fetches 4 key rows x 16 features and every lane receives the
// four keys of its own feature), which is exactly the key order above.  Both patterns are conflict free.
// Key rows past the head's end are written as zeros (a load past the descriptor's end stores zero).
// LDS holds three K tiles (requested two tiles ahead) and two V tiles (one ahead); one workgroup barrier per
// tile, placed behind the S^T products,
// whose K fragments were read into registers during the previous tile's softmax: see tile_step.
//
// Two things ride in the same launch where the caller asks for them (the kSel instances): every workgroup selects its
// own KV blocks first (Eq. 4 and the Top-K, select_in_workgroup), and workgroups of their own absorb another chunk's
// tokens into a second state buffer (Eq. 2, absorb_role) in the slots that the attending workgroups leave free.
//
// What bounds this kernel at block_q 64: the matrix work and the vector work of the softmax do not
// overlap on a SIMD of this chip; with no loads, no exponentials and no barrier the loop still takes
// twice the time of its MFMAs.
#include <stdlib.h>

#include "hf_common.h"

namespace hf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int D = 128;
constexpr int TK = 32;      // keys per tile
constexpr int KSTR = 256;   // bytes per key row of a K tile in LDS; 16-byte units XOR-swizzled by (row & 15)
constexpr int OSTR = 272;   // bytes per query row of the staged output
constexpr int KTILE = TK * KSTR;
constexpr float kRescaleThreshold = 8.0f;  // log2 units: rescale only when a row max grew by more than 2^8

// History branch fused into the epilogue (kFused): planes = the fp32 state split into two bf16
// planes (hi, lo), transposed (Lt[plane][j][i], see hf_readout_mfma.hip), of which the first
// n_planes are used; zvec = the state's normaliser.
// max without the NaN-quieting canonicalisation the compiler adds around fmaxf (scores are finite
// or -inf here): one instruction per three inputs
__device__ __forceinline__ float max3f(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float max2f(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

struct HistArgs {
  const bf16_t* planes;  // [BH][2][d][d]
  const float* zvec;     // [BH][d]
  float eps, z_scale;
  int n_planes;          // 2 = hi + lo, 1 = hi only
  int phi_kind;          // feature map of the history branch
  const float* cosq;     // [n_q][d/2] rotation of phi(q) in the numerator, or NULL
  const float* sinq;
  const bf16_t* q_hist;  // [BH][n_q][d] queries of the history branch when they are not Q, or NULL
  // kFused == 3 (row statistics for the backward pass instead of the output):
  const bf16_t* d_out;   // [BH][n_q][d] gradient of the output
  float* lse2;           // [BH][n_q] log2 of the softmax denominator in the scaled-logit domain
  float* dvec;           // [BH][n_q] d_out . O_local
  // by-products of an ordinary forward pass for the backward pass, each optional (kFused != 3):
  float* lse2_out;       // [BH][n_q] the same row statistic
  bf16_t* olocal_out;    // [BH][n_q][d] the sparse branch's output alone, rounded once
  // kSel (the workgroup selects its own KV blocks, Eq. 4, before it attends to them):
  const float* kbar_t;   // [BH][d/4][T_n][4] pooled keys, feature-group-major (pool kernel)
  int32_t* idx_out;      // [BH][T_m][k] the ascending block list of every query block (also read back by the kernel)
  float* scores_out;     // [BH][T_m][T_n] the scores A of Eq. 4, or NULL
};

// ---- Eq. 4 and the Top-K of a query block inside the attention workgroup (kSel).
// q-bar from the block's rows (they are read for the fragments anyway), A_j = q-bar . k-bar_j against the head's pooled
// keys (wavefront w a slice of the head dimension, lane l the KV blocks l, l + 64, ...; partial sums meet in LDS in a
// fixed order), rank by counting (strict comparison; the exact tie rule, lower index wins, only when a tie straddles
// the k-th place), ascending list by ballot prefix sums.  The list is left in LDS at `sel` (k entries) and written to
// idx_row.  All scratch lies in the tile space, which is not in use yet.  t_n <= kSelMaxBlocks.
constexpr int kSelMaxBlocks = kMaxFusedSelectBlocks;

template <int NW>
__device__ __forceinline__ int* select_in_workgroup(char* smem, const bf16_t* Qh, int q0, int n_q, const float* kbar_head,
                                                    int t_n, int k, int32_t* idx_row, float* scores_row) {
  constexpr int NT = 64 * NW, BQ = 32 * NW, G = NT / 16, CW = D / 4 / NW;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int t_pad = (t_n + 3) & ~3;
  float* qpart = reinterpret_cast<float*>(smem);      // [G][D] partial column sums
  float* qbar = qpart + G * D;                          // [D]
  float* part = qbar + D;                               // [NW][t_pad]
  float* sc = part + NW * t_pad;                        // [t_pad]
  int* sel = reinterpret_cast<int*>(sc + t_pad);        // [k]
  int* wave_count = sel + t_n;                          // [2][NW]
  const int rows = min(BQ, n_q - q0);
  // the block's rows and, right behind them, the first pass of pooled keys: both are on their way while the
  // pooled query is formed (the chain of this prologue is memory round trips, not arithmetic)
  const int u16 = tid & 15, g = tid >> 4;
  bf16x8 v[BQ / G];
#pragma unroll
  for (int i = 0; i < BQ / G; ++i)
    v[i] = *reinterpret_cast<const bf16x8*>(Qh + (size_t)min(q0 + g + G * i, n_q - 1) * D + 8 * u16);
  // pooled keys through a buffer descriptor: one offset register per block, the feature group's offset is scalar
  // (forty-eight 64-bit addresses would not fit next to the loads they feed)
  const __amdgpu_buffer_rsrc_t krsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(kbar_head), 0, (D / 4) * t_n * 16, 0x00020000);
  auto kload = [&](int j, int c) {
    typedef unsigned int u32v4 __attribute__((vector_size(16)));
    const u32v4 r = __builtin_amdgcn_raw_buffer_load_b128(krsrc, j * 16, (wave * CW + c) * t_n * 16, 0);
    return make_float4(__uint_as_float(r[0]), __uint_as_float(r[1]), __uint_as_float(r[2]), __uint_as_float(r[3]));
  };
  constexpr int U = 48 / CW;   // KV blocks per lane and pass (3 or 6): 48 loads of 16 bytes in flight
  float4 kv[U][CW];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int j = min(lane + 64 * u, t_n - 1);   // clamped: a valid address, the result is dropped
#pragma unroll
    for (int c = 0; c < CW; ++c) kv[u][c] = kload(j, c);
  }
  {
    // column sums of the thread's rows, two rows per instruction: (x_r, x_r') . (1, 1) + acc in fp32
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 one2 = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
    const bf16x8 zero = {};
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
#pragma unroll
    for (int i = 0; i < BQ / G; i += 2) {
      const bf16x8 r0 = (g + G * i < rows) ? v[i] : zero, r1 = (g + G * (i + 1) < rows) ? v[i + 1] : zero;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const bf16x2 pr = {r0[e], r1[e]};
        acc[e] = __builtin_amdgcn_fdot2_f32_bf16(pr, one2, acc[e], false);
      }
    }
    *reinterpret_cast<float4*>(qpart + g * D + 8 * u16) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    *reinterpret_cast<float4*>(qpart + g * D + 8 * u16 + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
  }
  __syncthreads();
  if (tid < D) {
    float a = 0.0f;
#pragma unroll
    for (int gg = 0; gg < G; ++gg) a += qpart[gg * D + tid];
    qbar[tid] = a * (1.0f / (float)rows);
  }
  if (tid < t_pad - t_n) sc[t_n + tid] = -INFINITY;   // padding never outranks a block
  __syncthreads();

  // ---- scores: wavefront w a slice of the head dimension, lane l the KV blocks l, l + 64, ...
  const float4* q4 = reinterpret_cast<const float4*>(qbar) + wave * CW;
  for (int j0 = lane; j0 < t_n; j0 += 64 * U) {
    if (j0 != lane) {   // (uniform) windows of more than 64 U blocks: further passes
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = min(j0 + 64 * u, t_n - 1);
#pragma unroll
        for (int c = 0; c < CW; ++c) kv[u][c] = kload(j, c);
      }
    }
    // (feature groups outermost: the pooled query passes through a few registers instead of staying in sixty-four)
    float a0[U], a1[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a0[u] = a1[u] = 0.0f;
#pragma unroll
    for (int c = 0; c < CW; c += 2) {
      const float4 qa = q4[c], qb4 = q4[c + 1];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        a0[u] = fmaf(qa.x, kv[u][c].x, a0[u]); a0[u] = fmaf(qa.y, kv[u][c].y, a0[u]);
        a0[u] = fmaf(qa.z, kv[u][c].z, a0[u]); a0[u] = fmaf(qa.w, kv[u][c].w, a0[u]);
        a1[u] = fmaf(qb4.x, kv[u][c + 1].x, a1[u]); a1[u] = fmaf(qb4.y, kv[u][c + 1].y, a1[u]);
        a1[u] = fmaf(qb4.z, kv[u][c + 1].z, a1[u]); a1[u] = fmaf(qb4.w, kv[u][c + 1].w, a1[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (j0 + 64 * u < t_n) part[wave * t_pad + j0 + 64 * u] = a0[u] + a1[u];
  }
  __syncthreads();

  if (t_n <= 256) {
    // ---- Top-K by the k-th largest key, found bit by bit (a few comparisons and population counts per step, every
    // wavefront for itself on the whole row: lane l holds the blocks l, l + 64, ..., their scores summed from the
    // wavefronts' parts in wavefront order).  Keys order like the scores; kept: every block above the k-th key, and
    // of the blocks equal to it the lowest indices (the tie rule).
    uint32_t key[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j = lane + 64 * e, jc = min(j, t_n - 1);
      float a = part[jc];
#pragma unroll
      for (int w = 1; w < NW; ++w) a += part[w * t_pad + jc];
      if (scores_row && wave == 0 && j < t_n) scores_row[j] = a;
      const uint32_t b = __float_as_uint(a + 0.0f);   // (-0 counts as +0)
      key[e] = j < t_n ? (b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u)) : 0u;   // padding lies below every score
    }
    // Two bits per step (the three candidates are counted side by side: the steps are a chain of latencies), and the
    // search ends as soon as exactly k keys reach a candidate: they are the list, whatever the lower bits say.
    uint32_t kth = 0;
    bool cut = false;
    for (int bit = 30; bit >= 0; bit -= 2) {
      const uint32_t c1 = kth | (1u << bit), c2 = kth | (2u << bit), c3 = kth | (3u << bit);
      int n1 = 0, n2 = 0, n3 = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        n1 += __popcll(__ballot(key[e] >= c1));
        n2 += __popcll(__ballot(key[e] >= c2));
        n3 += __popcll(__ballot(key[e] >= c3));
      }
      int n;   // (all uniform)
      if (n3 >= k) { kth = c3; n = n3; }
      else if (n2 >= k) { kth = c2; n = n2; }
      else if (n1 >= k) { kth = c1; n = n1; }
      else continue;
      if (n == k) { cut = true; break; }
    }
    if (cut) --kth;   // kept: the keys above kth, i.e. the k that reach the candidate; none of them ties with the rest
    int above = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) above += __popcll(__ballot(key[e] > kth));
    const int ties_kept = k - above;
    const unsigned long long below = (1ull << lane) - 1ull;
    int base = 0, ties_seen = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int j = lane + 64 * e;
      const bool eq = key[e] == kth;
      const unsigned long long bal_eq = __ballot(eq);
      const bool keep = key[e] > kth || (eq && ties_seen + __popcll(bal_eq & below) < ties_kept);
      const unsigned long long bal = __ballot(keep);
      const int pos = base + __popcll(bal & below);
      if (keep && wave == 0) { sel[pos] = j; idx_row[pos] = j; }
      base += __popcll(bal);
      ties_seen += __popcll(bal_eq);
    }
    __syncthreads();
    return sel;
  }
  for (int j = tid; j < t_n; j += NT) {
    float a = part[j];
#pragma unroll
    for (int w = 1; w < NW; ++w) a += part[w * t_pad + j];
    sc[j] = a;
    if (scores_row) scores_row[j] = a;
  }
  __syncthreads();
  // ---- rank and list (windows of more than 256 blocks), two blocks per thread and scan of the row (j and j + NT share every score they are
  // compared with).  First pass: strict comparison only (blocks with equal scores share a rank), exact unless
  // a tie straddles the k-th place, which shows as more than k blocks of rank < k; then the row is redone with the rule.
  for (int pass = 0; pass < 2; ++pass) {
    int base = 0;
    for (int j0 = 0; j0 < t_n; j0 += 2 * NT) {   // uniform trip count: barriers inside
      const int ja = j0 + tid, jb = ja + NT;
      const float ma = ja < t_n ? sc[ja] : INFINITY, mb = jb < t_n ? sc[jb] : INFINITY;
      int ra = 0, rb = 0;
      if (pass == 0) {
#pragma unroll 4
        for (int o = 0; o < t_pad; o += 4) {
          const float4 x = *reinterpret_cast<const float4*>(sc + o);
          ra += (x.x > ma) ? 1 : 0; ra += (x.y > ma) ? 1 : 0; ra += (x.z > ma) ? 1 : 0; ra += (x.w > ma) ? 1 : 0;
          rb += (x.x > mb) ? 1 : 0; rb += (x.y > mb) ? 1 : 0; rb += (x.z > mb) ? 1 : 0; rb += (x.w > mb) ? 1 : 0;
        }
      } else {
        for (int o = 0; o < t_pad; o += 4) {
          const float4 x = *reinterpret_cast<const float4*>(sc + o);
          ra += (x.x > ma || (x.x == ma && o < ja)) ? 1 : 0;
          ra += (x.y > ma || (x.y == ma && o + 1 < ja)) ? 1 : 0;
          ra += (x.z > ma || (x.z == ma && o + 2 < ja)) ? 1 : 0;
          ra += (x.w > ma || (x.w == ma && o + 3 < ja)) ? 1 : 0;
          rb += (x.x > mb || (x.x == mb && o < jb)) ? 1 : 0;
          rb += (x.y > mb || (x.y == mb && o + 1 < jb)) ? 1 : 0;
          rb += (x.z > mb || (x.z == mb && o + 2 < jb)) ? 1 : 0;
          rb += (x.w > mb || (x.w == mb && o + 3 < jb)) ? 1 : 0;
        }
      }
      const bool keep_a = ja < t_n && ra < k, keep_b = jb < t_n && rb < k;
      const unsigned long long bal_a = __ballot(keep_a), bal_b = __ballot(keep_b);
      if (lane == 0) {
        wave_count[wave] = __popcll(bal_a);
        wave_count[NW + wave] = __popcll(bal_b);
      }
      __syncthreads();
      const unsigned long long below = (1ull << lane) - 1ull;
      int pos_a = base + __popcll(bal_a & below), pos_b = __popcll(bal_b & below), tot_a = 0, tot_b = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const int ca = wave_count[w], cb = wave_count[NW + w];
        if (w < wave) { pos_a += ca; pos_b += cb; }
        tot_a += ca;
        tot_b += cb;
      }
      pos_b += base + tot_a;
      if (keep_a && pos_a < k) { sel[pos_a] = ja; idx_row[pos_a] = ja; }
      if (keep_b && pos_b < k) { sel[pos_b] = jb; idx_row[pos_b] = jb; }
      base += tot_a + tot_b;
      __syncthreads();
    }
    if (base == k) break;  // uniform over the workgroup
  }
  return sel;
}

// ---- Eq. 2 in workgroups of their own inside the attention launch (kSel instances; AbsorbArgs::role_blocks > 0).
// A query block's workgroup occupies its compute-unit slot for the whole launch, and the launch seldom fills every
// slot (888 workgroups on 1024 slots at the 832x480 shape): the first role_blocks workgroup ids therefore do not
// attend.  Each takes one token slice of one head of the evicted chunk and accumulates that slice's 128 x 128
// contribution  sum_t phi(k_t)^T v_t  (A operand phi(K)^T, B operand V, both by transposing reads of row-major
// 16-token stages that travel global -> LDS directly, five stages in the tile space, four in flight) and  sum_t
// phi(k_t)  (a B operand of ones), stores it as a partial, and the last workgroup of a head to arrive adds the
// partials in slice order to state_in and writes state_out and its two bf16 planes.  state_out / planes_out are
// other buffers than the ones the attending workgroups read: the chunk absorbed here is the one the NEXT chunk's
// eviction removes, and nothing of this launch depends on it.  ReLU, no rotation.
struct AbsorbArgs {
  const bf16_t* K;         // [BH][stride][d] tokens to absorb (first n of every head)
  const bf16_t* V;
  int n, stride, slices, role_blocks, BH;
  const float* state_in;   // L [BH][d][d] then z [BH][d]
  float* state_out;
  bf16_t* planes_out;      // [BH][2][d][d] or NULL
  float* partials;         // [BH][slices][d*d + d]
  unsigned long long* counters;   // [BH] arrival counters, (tag << 16) | count
  unsigned long long tag;
};

template <int NW>
__device__ __forceinline__ void absorb_role(char* smem, const AbsorbArgs& ab) {
  constexpr int NT = 64 * NW;
  constexpr int IB = 4 / NW;                 // 32-row blocks of key features per wavefront
  constexpr int PARTB = 16 * KSTR;           // bytes of 16 tokens of K (or V)
  constexpr int STAGE = 2 * PARTB;           // a stage: 16 tokens of K, then of V (8 KB)
  constexpr int NSTG = 5;
  constexpr int HP = (PARTB / 1024) / NW;    // 1 KB pieces (4 token rows) of a part per wavefront (2 or 1)
  constexpr int PART = D * D + D;
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  int* const s_last = reinterpret_cast<int*>(smem);   // (the stages are dead when it is written)
  const int wg = blockIdx.x;
  if (wg >= ab.BH * ab.slices) return;      // (padding up to a multiple of eight workgroup ids)
  const int bh = wg / ab.slices, slice = wg - bh * ab.slices;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, h = lane >> 5;
  const int nst_total = (ab.n + 15) / 16;
  const int st0 = (int)((long long)slice * nst_total / ab.slices);
  const int nst = (int)((long long)(slice + 1) * nst_total / ab.slices) - st0;

  const uint64_t kbase = reinterpret_cast<uint64_t>(ab.K + (size_t)bh * ab.stride * D);
  const uint64_t vbase = reinterpret_cast<uint64_t>(ab.V + (size_t)bh * ab.stride * D);
  const int head_bytes = ab.n * (D * 2);
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
  int lane_off[HP];
#pragma unroll
  for (int j = 0; j < HP; ++j) {
    const int r = 4 * (wave + NW * j) + (lane >> 4), u = lane & 15;
    lane_off[j] = r * (D * 2) + ((u ^ (((r & 3) << 2) | ((r >> 2) & 3))) * 16);
  }
  // stage c of this slice (16 tokens from token 16 (st0 + c)) into slot c mod NSTG; stages past the slice's end
  // get an empty descriptor (zeros, nothing read), so that every wavefront issues the same number of requests
  auto fetch = [&](int c) {
    const int start = __builtin_amdgcn_readfirstlane((st0 + c) * 16);
    const int skip = start * (D * 2);
    const int left = c < nst ? min(head_bytes - skip, 16 * D * 2) : 0;   // the slice's own tokens only
    const uint32_t slot = lds0 + (uint32_t)(c % NSTG) * STAGE;
#pragma unroll
    for (int part = 0; part < 2; ++part) {
      const uint64_t base = (part ? vbase : kbase) + (uint64_t)(uint32_t)(left > 0 ? skip : 0);
      const i32x4 d2 = {(int)(uint32_t)base, (int)(uint32_t)(base >> 32), left > 0 ? left : 0, 0x00020000};
#pragma unroll
      for (int j = 0; j < HP; ++j) {
        const uint32_t dst = slot + part * PARTB + 4 * (wave + NW * j) * KSTR;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                     :: "s"(dst), "v"(lane_off[j]), "s"(d2) : "memory", "m0");
      }
    }
  };
  // transposing reads of a 16-token part: feature 32 dt + l32 as the row, the lane's eight tokens as the k index
  const int j16 = lane & 15, grp16 = lane >> 4;
  const int key_l = 4 * h + (j16 >> 2);
  const int w_l = (4 * (key_l & 3)) | ((2 * (grp16 & 1) + ((j16 & 3) >> 1)) ^ h);
  const uint32_t rd = key_l * KSTR + w_l * 16 + 8 * (j16 & 1);
  auto frag = [&](const char* part, int dt) {
    const char* p = part + (rd ^ (64u * dt));
    const char* q = part + ((rd ^ (64u * dt)) ^ 32u) + 2048;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(q));
    const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return both;
  };

  // the head's arrival counter has to carry this call's tag before anybody's ticket is drawn: one lane looks at it
  // now (its oldest request) and claims it if the tag is another call's
  unsigned long long* const ctr = ab.counters + bh;
  const bool claimer = tid == NT - 64;
  unsigned long long seen = 0;
  if (claimer) asm volatile("global_load_dwordx2 %0, %1, off sc1" : "=&v"(seen) : "v"(ctr) : "memory");
#pragma unroll
  for (int c = 0; c < NSTG - 1; ++c) fetch(c);
  if (claimer) {
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(seen) : "n"(2 * HP * (NSTG - 1)) : "memory");
    if ((seen >> 16) != ab.tag)
      (void)__hip_atomic_compare_exchange_strong(ctr, &seen, ab.tag << 16, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
  }

  f32x16 acc[IB][4], zacc[IB];
#pragma unroll
  for (int ib = 0; ib < IB; ++ib) {
#pragma unroll
    for (int r = 0; r < 16; ++r) zacc[ib][r] = 0.0f;
#pragma unroll
    for (int jb = 0; jb < 4; ++jb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[ib][jb][r] = 0.0f;
  }
  const s16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  const s16x8 ones8 = {0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80, 0x3f80};   // bf16 1.0
  for (int c = 0; c < nst; ++c) {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * HP * (NSTG - 2)) : "memory");   // this wavefront's rows of stage c
    __syncthreads();             // ... and everybody's; everybody has read stage c - 1
    fetch(c + NSTG - 1);         // into the slot of stage c - 1
    const char* st = smem + (c % NSTG) * STAGE;
    bf16x8 a[IB], b[4];
#pragma unroll
    for (int ib = 0; ib < IB; ++ib)   // phi = ReLU on bf16 values as a packed signed-integer max with zero
      a[ib] = __builtin_bit_cast(bf16x8, __builtin_elementwise_max(frag(st, IB * wave + ib), zero8));
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) b[jb] = __builtin_bit_cast(bf16x8, frag(st + PARTB, jb));
#pragma unroll
    for (int ib = 0; ib < IB; ++ib) {
#pragma unroll
      for (int jb = 0; jb < 4; ++jb) acc[ib][jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ib], b[jb], acc[ib][jb], 0, 0, 0);
      zacc[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ib], __builtin_bit_cast(bf16x8, ones8), zacc[ib], 0, 0, 0);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // (requests past the slice's end were empty; the claim is done)

  // ---- the slice's partial, in the state's layout.  Partials meet workgroups on other XCDs, whose L2 caches do not
  // see each other's lines: device-scope stores and loads (through to memory), no fence.
  float* part = ab.partials + ((size_t)bh * ab.slices + slice) * PART;
#pragma unroll
  for (int ib = 0; ib < IB; ++ib)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = 32 * (IB * wave + ib) + 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
      for (int jb = 0; jb < 4; ++jb)
        __hip_atomic_store(part + i * D + 32 * jb + l32, acc[ib][jb][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (l32 == 0) __hip_atomic_store(part + D * D + i, zacc[ib][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  // ---- arrival: every store above has been acknowledged before the workgroup draws its ticket
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0) {
    const unsigned long long before = __hip_atomic_fetch_add(ctr, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *s_last = (int)(before & 0xffffull) + 1 == ab.slices;
    // the last one leaves the count at zero under this call's tag: a captured launch replays with the same tag
    if (*s_last) __hip_atomic_store(ctr, ab.tag << 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (!*s_last) return;

  // ---- the head's last workgroup: state_out = state_in + (partials in slice order), one addition at the state's
  // magnitude; a thread owns value feature j and a run of key features i, eight at a time, so that the planes
  // [plane][j][i] leave as 16-byte pieces
  constexpr int G = NT / D, RUN = D / G;
  const int j = tid & (D - 1), i_begin = (tid / D) * RUN;
  const float* p0 = ab.partials + (size_t)bh * ab.slices * PART;
  const float* Lin = ab.state_in + (size_t)bh * D * D;
  float* Lout = ab.state_out + (size_t)bh * D * D;
  constexpr int KB = 8;    // slices whose loads are in flight together
  constexpr int RB = 16;   // key features per trip: 16 x 8 loads of the partials in flight per thread (the trips are
                           // round trips to memory, a handful of them is the whole tail of this role)
  for (int i0 = i_begin; i0 < i_begin + RUN; i0 += RB) {
    float sum[RB], old[RB];
#pragma unroll
    for (int q = 0; q < RB; ++q) { old[q] = Lin[(size_t)(i0 + q) * D + j]; sum[q] = 0.0f; }
    for (int s0 = 0; s0 < ab.slices; s0 += KB) {
      float v[KB][RB];
#pragma unroll
      for (int u = 0; u < KB; ++u) {
        const float* ps = p0 + (size_t)min(s0 + u, ab.slices - 1) * PART;   // (past the last slice: re-read, not added)
#pragma unroll
        for (int q = 0; q < RB; ++q)
          v[u][q] = __hip_atomic_load(const_cast<float*>(ps) + (size_t)(i0 + q) * D + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
#pragma unroll
      for (int u = 0; u < KB; ++u)
        if (s0 + u < ab.slices) {   // uniform; slice order
#pragma unroll
          for (int q = 0; q < RB; ++q) sum[q] += v[u][q];
        }
    }
#pragma unroll
    for (int q = 0; q < RB; ++q) {
      sum[q] += old[q];
      Lout[(size_t)(i0 + q) * D + j] = sum[q];
    }
    if (ab.planes_out) {
#pragma unroll
      for (int half = 0; half < RB / 8; ++half) {
        uint32_t hw[4], lw[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float v0 = sum[8 * half + 2 * q], v1 = sum[8 * half + 2 * q + 1];
          const bf16_t h0 = f32_to_bf16(v0), h1 = f32_to_bf16(v1);
          hw[q] = (uint32_t)h0 | ((uint32_t)h1 << 16);
          lw[q] = (uint32_t)f32_to_bf16(v0 - bf16_to_f32(h0)) | ((uint32_t)f32_to_bf16(v1 - bf16_to_f32(h1)) << 16);
        }
        bf16_t* hi = ab.planes_out + (size_t)bh * 2 * D * D + (size_t)j * D + i0 + 8 * half;
        *reinterpret_cast<uint4*>(hi) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
        *reinterpret_cast<uint4*>(hi + D * D) = make_uint4(lw[0], lw[1], lw[2], lw[3]);
      }
    }
  }
  if (tid < D) {
    float zsum = 0.0f;
    for (int sl = 0; sl < ab.slices; ++sl)
      zsum += __hip_atomic_load(const_cast<float*>(p0) + (size_t)sl * PART + D * D + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const size_t zat = (size_t)ab.BH * D * D + (size_t)bh * D + tid;
    ab.state_out[zat] = zsum + ab.state_in[zat];
  }
}

// kSel: 1 = the workgroup first selects its KV blocks itself (Eq. 4 from hist.kbar_t, list to hist.idx_out); the
// first ab.role_blocks workgroup ids (a multiple of eight) absorb evicted tokens instead (absorb_role)
template <int NW, int kFused, int kSel = 0>
__global__ __launch_bounds__(64 * NW, 2) void attn_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const int32_t* __restrict__ idx, int k, int n_q, int n_kv, int kv_stride, int bkv, int t_m, int t_n,
    int items_per_xcd, int total_items, float c_scale, HistArgs hist, AbsorbArgs ab, bf16_t* __restrict__ O) {
  constexpr int NT = 64 * NW;
  constexpr int BQ = 32 * NW;
  constexpr int CPT = (TK * D * 2 / 16) / NT;  // 1 KB pieces (4 key rows) of a tile per wavefront (4 or 2)
  __shared__ __attribute__((aligned(16))) char smem[5 * KTILE];
  char* const sK = smem;                // three K tiles (requested two tiles ahead)
  char* const sV = smem + 3 * KTILE;    // two V tiles (requested one tile ahead)
  static_assert(BQ * OSTR <= 5 * KTILE, "staged output must fit in the tiles");

  // consecutive workgroup ids go to consecutive XCDs: give every XCD one contiguous run of
  // (head, query block) items so that its L2 sees few heads
  if (kSel && (int)blockIdx.x < ab.role_blocks) {
    absorb_role<NW>(smem, ab);
    return;
  }
  const int wgid = kSel ? (int)blockIdx.x - ab.role_blocks : (int)blockIdx.x;
  const int xcd = wgid & 7, slot = wgid >> 3;
  const int item = xcd * items_per_xcd + slot;
  if (slot >= items_per_xcd || item >= total_items) return;
  const int bh = item / t_m, qb = item % t_m;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps LDS slot arithmetic on the scalar unit
  const int l32 = lane & 31, h = lane >> 5;
  const bf16_t* Qh = Q + (size_t)bh * n_q * D;
  const bf16_t* Kh = K + (size_t)bh * kv_stride * D;  // heads of a cache buffer are kv_stride tokens apart
  const bf16_t* Vh = V + (size_t)bh * kv_stride * D;
  bf16_t* Oh = O + (size_t)bh * n_q * D;
  const int32_t* row_idx = kSel ? hist.idx_out + ((size_t)bh * t_m + qb) * k : (idx ? idx + ((size_t)bh * t_m + qb) * k : nullptr);
  const int nsel = (kSel || idx) ? k : t_n;
  const int* sel_lds = nullptr;   // kSel: the list in LDS, valid until the first tile is requested
  if (kSel)
    sel_lds = select_in_workgroup<NW>(smem, Qh, qb * BQ, n_q, hist.kbar_t + (size_t)bh * (D / 4) * t_n * 4, t_n, k,
                                      hist.idx_out + ((size_t)bh * t_m + qb) * k,
                                      hist.scores_out ? hist.scores_out + ((size_t)bh * t_m + qb) * t_n : nullptr);
  const int subs = (bkv + TK - 1) / TK;
  const int ntiles = nsel * subs;

  // ---- this lane's query row as B-operand fragments (d = 16 s + 8 h .. +8)
  const int q_row = qb * BQ + 32 * wave + l32;
  bf16x8 qf[8];
  {
    const bf16_t* qp = Qh + (size_t)min(q_row, n_q - 1) * D + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
  }

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;
  float m_ref = -INFINITY, l_run = 0.0f;

  // ---- tile list: (selected block, 32-key part) -> (first key, number of real keys).  Tiles past
  // the end of the list and out-of-range block indices give (0, 0): such a tile reads real rows and
  // is masked entirely.  The descriptors are formed 64 tiles at a time, lane l holding tile 64 c + l,
  // and handed out with one v_readlane per tile: the bookkeeping and the load of the block index stay
  // out of the tile loop.
  int d_tile = 0, tq = 0;  // first key (24 bits: the window has fewer than 2^23 keys) | real keys << 24
  auto refill = [&](int t0) {
    const int t = t0 + lane;
    const int sel = t / subs, sub = t - sel * subs;
    const int sc = min(sel, nsel - 1);
    int jb;
    if (kSel)   // the first 64 tiles from the list in LDS; later ones from the copy in memory, past this CU's L1
      jb = t0 == 0 ? sel_lds[sc] : __hip_atomic_load(const_cast<int32_t*>(row_idx) + sc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
      jb = row_idx ? row_idx[sc] : sc;
    const bool ok = (sel < nsel) && ((unsigned)jb < (unsigned)t_n);
    const int st = jb * bkv + TK * sub;
    d_tile = ok ? (st | (max(0, min(TK, min(n_kv, (jb + 1) * bkv) - st)) << 24)) : 0;
  };
  refill(0);
  if (kSel) __syncthreads();   // every wavefront has its descriptors before a tile lands on the list
  auto next_tile = [&](int& start, int& valid) {
    if ((tq & 63) == 0 && tq > 0) refill(tq);  // uniform
    const int d = __builtin_amdgcn_readlane(d_tile, tq & 63);
    start = d & 0xffffff;
    valid = d >> 24;
    ++tq;
  };

  // ---- staging: K and V tiles go global -> LDS directly (16 bytes per lane, 1 KB = 4 key rows per
  // instruction), row-major with swizzled 16-byte units: K unit u of row r sits at u ^ (r & 15), V unit u
  // at u ^ (4 (r & 3) | (r >> 2 & 3)).  Rows past n_kv arrive as zeros (range check of the descriptor).
  // K has three slots, V two: in iteration t, V of tile t+1 and then K of tile t+3 are requested.
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  const uint64_t kbase = reinterpret_cast<uint64_t>(Kh), vbase = reinterpret_cast<uint64_t>(Vh);
  const i32x4 k_desc = {(int)(uint32_t)kbase, (int)(uint32_t)(kbase >> 32), n_kv * (D * 2), 0x00020000};
  const i32x4 v_desc = {(int)(uint32_t)vbase, (int)(uint32_t)(vbase >> 32), n_kv * (D * 2), 0x00020000};
  const uint32_t sK_lds = (uint32_t)(uintptr_t)sK, sV_lds = (uint32_t)(uintptr_t)sV;
  int k_lane_off[CPT], v_lane_off[CPT];
#pragma unroll
  for (int j = 0; j < CPT; ++j) {
    const int r = 4 * (wave + NW * j) + (lane >> 4), u = lane & 15;
    k_lane_off[j] = r * (D * 2) + ((u ^ (r & 15)) * 16);
    v_lane_off[j] = r * (D * 2) + ((u ^ (((r & 3) << 2) | ((r >> 2) & 3))) * 16);
  }
  // the tile's first key moves into the descriptor (base and size, scalar arithmetic): the per-lane offsets
  // stay constant and the range check still ends at the head's last key
  auto dma_tile = [&](const i32x4& desc, uint32_t lds_slot, int start_v, const int (&lane_off)[CPT]) {
    const int start = __builtin_amdgcn_readfirstlane(start_v);   // uniform already; this pins it to a scalar register
    // a tile that starts at or past the head's end (an empty part of a short block) gets a descriptor of
    // size zero: every load of it returns zero and nothing outside the head is touched
    const int skip = start * (D * 2), left = desc.z - skip;
    const uint64_t base = (((uint64_t)(uint32_t)desc.y << 32) | (uint32_t)desc.x) + (uint64_t)(uint32_t)(left > 0 ? skip : 0);
    const i32x4 d2 = {(int)(uint32_t)base, (int)(uint32_t)(base >> 32), left > 0 ? left : 0, desc.w};
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      const uint32_t dst = lds_slot + 4 * (wave + NW * j) * KSTR;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                   :: "s"(dst), "v"(lane_off[j]), "s"(d2) : "memory", "m0");
    }
  };

  // per-lane LDS read offsets
  // K operand of step s: unit (2 s + h) ^ (row & 15) of row l32, i.e. byte k_rd ^ (32 s)
  const uint32_t k_rd = l32 * KSTR + 16 * (h ^ (l32 & 1)) + 32 * ((l32 & 15) >> 1);
  // V operand (feature 32 dt + l32, keys 16 t2 + 8 x + 4 h .. + 4) by transposing reads: a 16-lane group
  // fetches 4 key rows x 16 features as 16 chunks of 8 bytes, lane j the chunk (key j / 4, features 4 (j % 4));
  // each lane receives the four keys of its own feature column
  const int j16 = lane & 15, grp16 = lane >> 4;
  const int key_l = 4 * h + (j16 >> 2);                                  // key within the group of 8, = key & 7
  // unit u of key row r sits at u ^ (4 (r & 3) | (r >> 2 & 3)): the 32 lanes of two groups then touch 4 rows x 4
  // units = 16 different units.  For the row 16 t2 + 8 x + key_l that is 4 (key_l & 3) | 2 x | h.
  const int w_l = (4 * (key_l & 3)) | ((2 * (grp16 & 1) + ((j16 & 3) >> 1)) ^ h);   // swizzled unit for dt = 0, x = 0
  const uint32_t v_rd = key_l * KSTR + w_l * 16 + 8 * (j16 & 1);   // ^ (64 dt) ^ (32 x), + 4096 t2 + 2048 x

  // ---- prologue: K and V of tile 0 land (K of tiles 1 and 2 are on their way), the K fragments of tile 0 are
  // read into registers
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  uint32_t k_addr[8], v_addr[4][2];
#pragma unroll
  for (int s = 0; s < 8; ++s) k_addr[s] = k_rd ^ (32u * s);
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    v_addr[dt][0] = v_rd ^ (64u * dt);
    v_addr[dt][1] = v_rd ^ (64u * dt) ^ 32u;
  }
  int start_a, start_b, start_c, valid0, valid1, valid2, valid3;   // starts of tiles t+1, t+2, t+3
  {
    int st0;
    next_tile(st0, valid0);
    dma_tile(k_desc, sK_lds, st0, k_lane_off);
    dma_tile(v_desc, sV_lds, st0, v_lane_off);
    next_tile(start_a, valid1);
    dma_tile(k_desc, sK_lds + KTILE, start_a, k_lane_off);
    next_tile(start_b, valid2);
    dma_tile(k_desc, sK_lds + 2 * KTILE, start_b, k_lane_off);
    next_tile(start_c, valid3);
  }
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * CPT) : "memory");   // K and V of tile 0 (K of tiles 1, 2 may fly)
  __syncthreads();
  bf16x8 kf[8];   // K operand fragments of the tile whose scores come next
#pragma unroll
  for (int s = 0; s < 8; ++s) kf[s] = *reinterpret_cast<const bf16x8*>(sK + k_addr[s]);

  int va = valid0, vb = valid1, vc = valid2, vd = valid3;  // real keys of tiles t .. t+3
  // One tile (kslot = t mod 3, par = t mod 2, literals at every call site).  The scores of tile t are formed from
  // fragments already in registers; the one barrier of the iteration follows them.  Behind it every wavefront is
  // done with K slot kslot (fragments of tile t were read during tile t-1) and with V half par^1 (tile t-1), so V
  // of tile t+1 (at once) and K of tile t+3 (between the P.V products) are requested into them; K of tile t+1 and
  // V of tile t have landed (awaited before the barrier) and their fragments are read while the softmax runs.
  auto tile_step = [&](const int kslot, const int par) {
    const int valid_cur = va;
    // ---- S^T = K Q^T : 32 keys, 8 steps over d
    f32x16 sacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = 0.0f;
#pragma unroll
    for (int s = 0; s < 8; ++s) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[s], sacc, 0, 0, 0);

    // this wavefront's parts of K of tile t+1 and V of tile t have landed; K of tile t+2, requested last, may fly
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(CPT) : "memory");
    __syncthreads();

    dma_tile(v_desc, sV_lds + (par ^ 1) * KTILE, start_a, v_lane_off);     // V of tile t+1
    const int start_k = start_c;   // K of tile t+3 is requested further down
    start_a = start_b;
    start_b = start_c;
    int vnew;
    next_tile(start_c, vnew);

    // V fragments of tile t and K fragments of tile t+1: the reads complete under the softmax
    auto v_frag = [&](int dt, int t2) {
      const char* p = sV + v_addr[dt][0] + par * KTILE + 4096 * t2;
      const char* q = sV + v_addr[dt][1] + par * KTILE + 4096 * t2 + 2048;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(q));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, both);
    };
    bf16x8 vf[4], vg[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) vf[dt] = v_frag(dt, 0);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) vg[dt] = v_frag(dt, 1);
#pragma unroll
    for (int s = 0; s < 8; ++s) kf[s] = *reinterpret_cast<const bf16x8*>(sK + k_addr[s] + ((kslot + 1) % 3) * KTILE);
    __builtin_amdgcn_sched_barrier(0);

    if (valid_cur < TK) {  // keys that do not exist never contribute
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = 8 * (r >> 2) + 4 * h + (r & 3);
        if (key >= valid_cur) sacc[r] = -INFINITY;
      }
    }

    // ---- online softmax in the exp2 domain; statistics are per lane (= per query)
    float mx;
    {
      const float m0 = max3f(sacc[0], sacc[1], sacc[2]), m1 = max3f(sacc[3], sacc[4], sacc[5]);
      const float m2 = max3f(sacc[6], sacc[7], sacc[8]), m3 = max3f(sacc[9], sacc[10], sacc[11]);
      const float m4 = max3f(sacc[12], sacc[13], sacc[14]);
      mx = max2f(max3f(m0, m1, m2), max3f(m3, m4, sacc[15]));
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
      mx = max2f(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * c_scale;  // both lanes of a query agree
    }
    // lazy rescale: keep the reference max unless some row's max grew by more than the threshold
    if (__any(mx > m_ref + kRescaleThreshold)) {
      const float m_new = fmaxf(m_ref, mx);
      const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;  // nothing seen yet: keep exp2 finite
      const float alpha = __builtin_amdgcn_exp2f(m_ref - m_use);
      m_ref = m_new;
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
    }
    const float m_use = (m_ref == -INFINITY) ? 0.0f : m_ref;
    float psum = 0.0f;
    bf16x8 pf[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = __builtin_amdgcn_exp2f(fmaf(sacc[r], c_scale, -m_use));
      psum += p;
      pf[r >> 3][r & 7] = static_cast<__bf16>(p);
    }
    l_run += psum;

    // ---- O^T += V^T P^T : 2 steps of 16 keys, 4 tiles of 32 features
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[dt], pf[0], o[dt], 0, 0, 0);
    // K of tile t+3 into the slot of tile t, here rather than with V behind the barrier: eight transfers in a row
    // from every wavefront of the CU at once queue up at the memory pipeline, and a wavefront that cannot issue
    // its transfer cannot issue anything else (1.2 % of the kernel's time)
    dma_tile(k_desc, sK_lds + kslot * KTILE, start_k, k_lane_off);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vg[dt], pf[1], o[dt], 0, 0, 0);
    va = vb;
    vb = vc;
    vc = vd;
    vd = vnew;
  };
  // six tiles per trip: every (t mod 3, t mod 2) pair once, so that all slot offsets are immediates
  for (int t = 0; t < ntiles; t += 6) {
    tile_step(0, 0);
    if (t + 1 >= ntiles) break;
    tile_step(1, 1);
    if (t + 2 >= ntiles) break;
    tile_step(2, 0);
    if (t + 3 >= ntiles) break;
    tile_step(0, 1);
    if (t + 4 >= ntiles) break;
    tile_step(1, 0);
    if (t + 5 >= ntiles) break;
    tile_step(2, 1);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may land in LDS after the tiles' space is reused
  __syncthreads();
  // ---- normalise, transpose through LDS (the tiles are dead now) and store coalesced rows
  float l_tot;
  {
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
    l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
  }
  const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] *= inv;

  // the accumulators as bf16 rows of a [n_q][d] head: transposed through LDS (whose tiles or planes are dead at
  // every call), stored as coalesced rows; LDS may be reused after the barrier that follows the last call
  auto store_rows = [&](bf16_t* dst_head) {
    char* stage = smem;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        uint2 w;
        w.x = (uint32_t)f32_to_bf16(o[dt][4 * rq]) | ((uint32_t)f32_to_bf16(o[dt][4 * rq + 1]) << 16);
        w.y = (uint32_t)f32_to_bf16(o[dt][4 * rq + 2]) | ((uint32_t)f32_to_bf16(o[dt][4 * rq + 3]) << 16);
        *reinterpret_cast<uint2*>(stage + (32 * wave + l32) * OSTR + (32 * dt + 8 * rq + 4 * h) * 2) = w;
      }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < (BQ * 16) / NT; ++i) {
      const int c = tid + NT * i, row = c >> 4, col = c & 15;
      if (qb * BQ + row < n_q)
        *reinterpret_cast<uint4*>(dst_head + (size_t)(qb * BQ + row) * D + col * 8) =
            *reinterpret_cast<const uint4*>(stage + row * OSTR + col * 16);
    }
  };
  if (kFused != 3) {
    // ---- by-products for a later backward pass (training forward): the row statistic and O_local itself
    if (hist.lse2_out && h == 0 && q_row < n_q)
      hist.lse2_out[(size_t)bh * n_q + q_row] = l_tot > 0.0f ? m_ref + __log2f(l_tot) : INFINITY;
    if (kFused != 0 && hist.olocal_out) {   // (without a history term O is O_local)
      store_rows(hist.olocal_out + (size_t)bh * n_q * D);
      __syncthreads();
    }
  }

  if (kFused == 3) {
    // ---- backward-pass statistics: lse2 = m + log2(l) and D = dO . O_local, O_local still unrounded
    const bf16_t* gp = hist.d_out + ((size_t)bh * n_q + min(q_row, n_q - 1)) * D + 4 * h;
    float acc = 0.0f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const uint2 w = *reinterpret_cast<const uint2*>(gp + 32 * dt + 8 * rq);
        acc = fmaf(o[dt][4 * rq], __uint_as_float(w.x << 16), acc);
        acc = fmaf(o[dt][4 * rq + 1], __uint_as_float(w.x & 0xffff0000u), acc);
        acc = fmaf(o[dt][4 * rq + 2], __uint_as_float(w.y << 16), acc);
        acc = fmaf(o[dt][4 * rq + 3], __uint_as_float(w.y & 0xffff0000u), acc);
      }
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc), __float_as_uint(acc), false, false);
    acc = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    if (h == 0 && q_row < n_q) {
      // a row without a single real key keeps probability zero everywhere
      hist.lse2[(size_t)bh * n_q + q_row] = l_tot > 0.0f ? m_ref + __log2f(l_tot) : INFINITY;
      hist.dvec[(size_t)bh * n_q + q_row] = acc;
    }
    return;
  }

  if (kFused) {
    // ---- O += R(phi(q)) L / (z_scale phi(q).z + eps) (Eq. 3, 6): the query fragments already in
    // registers become the B operand of O_hist^T = Lt x R(phi(Q))^T; the A operand comes from the
    // L2-resident plane(s) through LDS.
    // The plane of the state is on its way before anything else: it travels global -> LDS like the tiles (four
    // "tiles" of 32 value features x 128 key features in the K layout, so that an A fragment is the K fragment's
    // read), under the arithmetic of the denominator.
    const uint64_t plane_base = reinterpret_cast<uint64_t>(hist.planes + (size_t)bh * 2 * D * D);
    auto dma_plane = [&](int plane) {
      const uint64_t b = plane_base + (uint64_t)plane * (D * D * 2);
      const i32x4 p_desc = {(int)(uint32_t)b, (int)(uint32_t)(b >> 32), D * D * 2, 0x00020000};
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) dma_tile(p_desc, sK_lds + dt * KTILE, 32 * dt, k_lane_off);
    };
    dma_plane(0);
    const float* zv = hist.zvec + (size_t)bh * D + 8 * h;
    float den = 0.0f;
    if (kFused == 1) {
      // ReLU of a bf16 value as a packed integer max: the fragments stay exact
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      const s16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        qf[s] = __builtin_bit_cast(bf16x8, __builtin_elementwise_max(__builtin_bit_cast(s16x8, qf[s]), zero8));
        const float4 z0 = *reinterpret_cast<const float4*>(zv + 16 * s);
        const float4 z1 = *reinterpret_cast<const float4*>(zv + 16 * s + 4);
        den += static_cast<float>(qf[s][0]) * z0.x + static_cast<float>(qf[s][1]) * z0.y +
               static_cast<float>(qf[s][2]) * z0.z + static_cast<float>(qf[s][3]) * z0.w +
               static_cast<float>(qf[s][4]) * z1.x + static_cast<float>(qf[s][5]) * z1.y +
               static_cast<float>(qf[s][6]) * z1.z + static_cast<float>(qf[s][7]) * z1.w;
      }
    } else {
      // any feature map, optional rotation of adjacent feature pairs: phi in fp32, the denominator from
      // the unrotated phi(q), the rotated numerator operand rounded to bf16 (2^-9, like P)
      const size_t trow = (size_t)min(q_row, n_q - 1) * (D / 2) + 4 * h;
      if (hist.q_hist) {
        const bf16_t* qp = hist.q_hist + ((size_t)bh * n_q + min(q_row, n_q - 1)) * D + 8 * h;
#pragma unroll
        for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
      }
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        float f[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = phi_apply(static_cast<float>(qf[s][e]), hist.phi_kind);
        const float4 z0 = *reinterpret_cast<const float4*>(zv + 16 * s);
        const float4 z1 = *reinterpret_cast<const float4*>(zv + 16 * s + 4);
        den += f[0] * z0.x + f[1] * z0.y + f[2] * z0.z + f[3] * z0.w + f[4] * z1.x + f[5] * z1.y + f[6] * z1.z +
               f[7] * z1.w;
        if (hist.cosq) {
          const float4 c4 = *reinterpret_cast<const float4*>(hist.cosq + trow + 8 * s);
          const float4 s4 = *reinterpret_cast<const float4*>(hist.sinq + trow + 8 * s);
          const float cc[4] = {c4.x, c4.y, c4.z, c4.w}, ss[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
          for (int p2 = 0; p2 < 4; ++p2) {
            const float a = f[2 * p2], b = f[2 * p2 + 1];
            f[2 * p2] = a * cc[p2] - b * ss[p2];
            f[2 * p2 + 1] = a * ss[p2] + b * cc[p2];
          }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[s][e] = static_cast<__bf16>(f[e]);
      }
    }
    {
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(den), __float_as_uint(den), false, false);
      den = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    // O_local is scaled by the denominator, the matrix cores add the numerator straight into the
    // same accumulators, and one multiplication by 1/denominator finishes O_local + O_hist
    const float den_eps = hist.z_scale * den + hist.eps;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] *= den_eps;
    static_assert(D * D * 2 <= 4 * KTILE, "a state plane must fit in the tiles' space");
    for (int plane = 0; plane < hist.n_planes; ++plane) {  // each plane goes through LDS once per workgroup
      if (plane) {
        __syncthreads();  // everybody is done with the previous plane
        dma_plane(plane);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(sK + k_addr[s] + dt * KTILE);
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s], o[dt], 0, 0, 0);
        }
    }
    const float inv_den = 1.0f / den_eps;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] *= inv_den;
    __syncthreads();  // the plane's space becomes the output staging area
  }

  store_rows(Oh);
}

}  // namespace

bool attn_mfma_supported(const hf_config& c) {
  return c.dtype == HF_BF16 && c.head_dim == 128 && (c.block_q == 64 || c.block_q == 128);
}

// byte offsets inside one head are 32-bit in the buffer loads
constexpr int kMfmaMaxKeys = 1 << 23;

static int launch_attn_mfma_impl(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                                 const int32_t* idx, int k, const HistArgs* hist, void* O, hipStream_t s,
                                 const AbsorbArgs* absorb = nullptr) {
  if (n_kv >= kMfmaMaxKeys) { set_error("window longer than %d keys", kMfmaMaxKeys); return HF_ERR_SHAPE; }
  const int BH = c.batch * c.heads;
  const int t_m = (n_q + c.block_q - 1) / c.block_q, t_n = (n_kv + c.block_kv - 1) / c.block_kv;
  const long long total = (long long)BH * t_m;
  if (total > (1ll << 30)) { set_error("too many query blocks"); return HF_ERR_SHAPE; }
  const int per_xcd = (int)((total + 7) / 8);
  const float scale = c.softmax_scale > 0.0f ? c.softmax_scale : 1.0f / sqrtf((float)c.head_dim);
  const float c_scale = scale * 1.4426950408889634f;
  const AbsorbArgs ab = absorb ? *absorb : AbsorbArgs{};
  const dim3 grid(8 * per_xcd + ab.role_blocks);
  const bf16_t* q = static_cast<const bf16_t*>(Q);
  const bf16_t* kk = static_cast<const bf16_t*>(K);
  const bf16_t* v = static_cast<const bf16_t*>(V);
  bf16_t* o = static_cast<bf16_t*>(O);
  const HistArgs h = hist ? *hist : HistArgs{};
#define HF_LAUNCH_ATTN_SEL(NWV, FUSED, SEL)                                                                      \
  hipLaunchKernelGGL((attn_mfma_kernel<NWV, FUSED, SEL>), grid, dim3(64 * NWV), 0, s, q, kk, v, idx, k, n_q, n_kv, \
                     kv_stride_of(c, n_kv), c.block_kv, t_m, t_n, per_xcd, (int)total, c_scale, h, ab, o)
#define HF_LAUNCH_ATTN(NWV, FUSED) HF_LAUNCH_ATTN_SEL(NWV, FUSED, 0)
  const int fused = !h.planes && !h.lse2 ? 0 : (h.lse2 ? 3 : ((h.phi_kind == HF_PHI_RELU && h.cosq == nullptr && h.q_hist == nullptr) ? 1 : 2));
  if (ab.role_blocks && !h.kbar_t) { set_error("absorbing workgroups ride only in the selecting launch"); return HF_ERR_SHAPE; }
  if (h.kbar_t) {
    // the workgroups select their KV blocks themselves
    if (fused == 3 || idx || !h.idx_out) { set_error("in-kernel selection: bad operands"); return HF_ERR_SHAPE; }
    if (t_n > kSelMaxBlocks) {
      set_error("window has %d KV blocks; the attention kernel selects among at most %d (select with hf_block_select)", t_n,
                kSelMaxBlocks);
      return HF_ERR_SHAPE;
    }
    if (c.block_q == 64) {
      if (fused == 0) HF_LAUNCH_ATTN_SEL(2, 0, 1); else if (fused == 1) HF_LAUNCH_ATTN_SEL(2, 1, 1); else HF_LAUNCH_ATTN_SEL(2, 2, 1);
    } else {
      if (fused == 0) HF_LAUNCH_ATTN_SEL(4, 0, 1); else if (fused == 1) HF_LAUNCH_ATTN_SEL(4, 1, 1); else HF_LAUNCH_ATTN_SEL(4, 2, 1);
    }
    return check_launch("hf_select_attn_fwd(attention)");
  }
  if (c.block_q == 64) {
    if (fused == 0) HF_LAUNCH_ATTN(2, 0); else if (fused == 1) HF_LAUNCH_ATTN(2, 1); else if (fused == 2) HF_LAUNCH_ATTN(2, 2); else HF_LAUNCH_ATTN(2, 3);
  } else {
    if (fused == 0) HF_LAUNCH_ATTN(4, 0); else if (fused == 1) HF_LAUNCH_ATTN(4, 1); else if (fused == 2) HF_LAUNCH_ATTN(4, 2); else HF_LAUNCH_ATTN(4, 3);
  }
#undef HF_LAUNCH_ATTN
#undef HF_LAUNCH_ATTN_SEL
  return check_launch("hf_hybrid_attn_fwd(attention)");
}

int launch_attn_mfma(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                     const int32_t* idx, int k, void* O_local, hipStream_t s) {
  return launch_attn_mfma_impl(c, Q, n_q, K, V, n_kv, idx, k, nullptr, O_local, s);
}

// the same with the row statistic of the softmax as a by-product (training forward without a history term)
int launch_attn_mfma_lse(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                         const int32_t* idx, int k, void* O_local, float* lse2_out, hipStream_t s) {
  HistArgs h = {};
  h.lse2_out = lse2_out;
  return launch_attn_mfma_impl(c, Q, n_q, K, V, n_kv, idx, k, &h, O_local, s);
}

// the history term rides in the attention epilogue (any feature map, with or without rotation)
bool attn_mfma_fused_supported(const hf_config& c) { return attn_mfma_supported(c); }

int launch_attn_mfma_fused(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                           const int32_t* idx, int k, const void* planes, const float* zvec, const float* cosq,
                           const float* sinq, const void* Q_hist, void* O, hipStream_t s, float* lse2_out,
                           void* olocal_out, const float* kbar_t, int32_t* idx_out, float* scores_out) {
  // One bf16 plane of L (2^-9 per element, errors of the d terms of a readout average out) costs the
  // output nothing measurable next to the bf16 rounding of P and O; HF_FLAG_HISTORY_TWO_PLANES adds the low plane.
  const HistArgs h = {static_cast<const bf16_t*>(planes), zvec, c.eps, c.z_scale, (c.flags & HF_FLAG_HISTORY_TWO_PLANES) ? 2 : 1,
                      c.phi, cosq, sinq, Q_hist == Q ? nullptr : static_cast<const bf16_t*>(Q_hist), nullptr, nullptr, nullptr,
                      lse2_out, static_cast<bf16_t*>(olocal_out), kbar_t, idx_out, scores_out};
  return launch_attn_mfma_impl(c, Q, n_q, K, V, n_kv, idx, k, &h, O, s);
}

// Workgroups that absorb next to the ones that attend: how many token slices per head, given what the attending
// workgroups leave free of the chip's slots (256 compute units; 4 workgroups of two wavefronts or 2 of four each)
int step_absorb_slices(const hf_config& c, int n_q, int n_ev) {
  const int BH = c.batch * c.heads;
  const long long attending = (long long)BH * ((n_q + c.block_q - 1) / c.block_q);
  const long long slots = 256ll * (c.block_q == 64 ? 4 : 2);
  long long room = slots - attending;          // a launch of several rounds has no room to speak of: few, long slices
  int s = room >= BH ? (int)(room / BH) : 2;
  if (s > 8) s = 8;
  const int by_len = (n_ev + 255) / 256;       // a slice should hold some hundred tokens
  if (s > by_len) s = by_len;
  return s < 1 ? 1 : s;
}

size_t step_absorb_workspace_bytes(const hf_config& c, int n_q, int n_ev) {
  const size_t BH = (size_t)c.batch * c.heads, d = c.head_dim;
  const size_t counters = (BH * 8 + 255) & ~(size_t)255;
  return counters + BH * step_absorb_slices(c, n_q, n_ev) * (d * d + d) * sizeof(float);
}

// selection, attention with the history term, and Eq. 2 for another chunk, in one launch
int launch_attn_mfma_step(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv, int k,
                          const float* kbar_t, int32_t* idx_out, float* scores_out, const void* planes,
                          const float* zvec, const float* cosq, const float* sinq, const void* Q_hist, void* O,
                          const void* K_ev, const void* V_ev, int n_ev, int ev_stride, const float* state_in,
                          float* state_out, void* planes_out, void* workspace, hipStream_t s) {
  const int BH = c.batch * c.heads;
  AbsorbArgs ab = {};
  ab.K = static_cast<const bf16_t*>(K_ev);
  ab.V = static_cast<const bf16_t*>(V_ev);
  ab.n = n_ev;
  ab.stride = ev_stride;
  ab.slices = step_absorb_slices(c, n_q, n_ev);
  ab.role_blocks = (BH * ab.slices + 7) & ~7;
  ab.BH = BH;
  ab.state_in = state_in;
  ab.state_out = state_out;
  ab.planes_out = static_cast<bf16_t*>(planes_out);
  ab.counters = static_cast<unsigned long long*>(workspace);
  ab.partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + (((size_t)BH * 8 + 255) & ~(size_t)255));
  ab.tag = next_call_tag();
  HistArgs h = {};
  if (planes) {
    h = HistArgs{static_cast<const bf16_t*>(planes), zvec, c.eps, c.z_scale, (c.flags & HF_FLAG_HISTORY_TWO_PLANES) ? 2 : 1,
                 c.phi, cosq, sinq, Q_hist == Q ? nullptr : static_cast<const bf16_t*>(Q_hist), nullptr, nullptr, nullptr,
                 nullptr, nullptr, kbar_t, idx_out, scores_out};
  } else {
    h.kbar_t = kbar_t;
    h.idx_out = idx_out;
    h.scores_out = scores_out;
  }
  return launch_attn_mfma_impl(c, Q, n_q, K, V, n_kv, nullptr, k, &h, O, s, &ab);
}

// selection (Eq. 4) and attention (Eq. 5) in one launch, no history term
int launch_attn_mfma_select(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv, int k,
                            const float* kbar_t, int32_t* idx_out, float* scores_out, void* O_local, hipStream_t s) {
  HistArgs h = {};
  h.kbar_t = kbar_t;
  h.idx_out = idx_out;
  h.scores_out = scores_out;
  return launch_attn_mfma_impl(c, Q, n_q, K, V, n_kv, nullptr, k, &h, O_local, s);
}

// the forward pass recomputed for the backward pass: row statistics out, no attention output
int launch_attn_mfma_stats(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                           const int32_t* idx, int k, const void* dO, float* lse2, float* dvec, hipStream_t s) {
  const HistArgs h = {nullptr, nullptr, 0.0f, 0.0f, 0, 0, nullptr, nullptr, nullptr, static_cast<const bf16_t*>(dO),
                      lse2, dvec, nullptr, nullptr, nullptr, nullptr, nullptr};
  return launch_attn_mfma_impl(c, Q, n_q, K, V, n_kv, idx, k, &h, nullptr, s);
}

}  // namespace hf
