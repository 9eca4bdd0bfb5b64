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
constexpr int PSTR = 272;   // bytes per row of a staged state plane (256 + 16)
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
};

// kFused: 0 = attention only, 1 = + history term for ReLU without rotation, 2 = + history term, general,
// 3 = no output: the row statistics the backward pass needs
template <int NW, int kFused>
__global__ __launch_bounds__(64 * NW, 2) void attn_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const int32_t* __restrict__ idx, int k, int n_q, int n_kv, int kv_stride, int bkv, int t_m, int t_n,
    int items_per_xcd, int total_items, float c_scale, HistArgs hist, bf16_t* __restrict__ O) {
  constexpr int NT = 64 * NW;
  constexpr int BQ = 32 * NW;
  constexpr int CPT = (TK * D * 2 / 16) / NT;  // 1 KB pieces (4 key rows) of a tile per wavefront (4 or 2)
  __shared__ __attribute__((aligned(16))) char smem[5 * KTILE];
  char* const sK = smem;                // three K tiles (requested two tiles ahead)
  char* const sV = smem + 3 * KTILE;    // two V tiles (requested one tile ahead)
  static_assert(BQ * OSTR <= 5 * KTILE, "staged output must fit in the tiles");

  // consecutive workgroup ids go to consecutive XCDs: give every XCD one contiguous run of
  // (head, query block) items so that its L2 sees few heads
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
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
  const int32_t* row_idx = idx ? idx + ((size_t)bh * t_m + qb) * k : nullptr;
  const int nsel = idx ? k : t_n;
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
    const int jb = row_idx ? row_idx[sc] : sc;
    const bool ok = (sel < nsel) && ((unsigned)jb < (unsigned)t_n);
    const int st = jb * bkv + TK * sub;
    d_tile = ok ? (st | (max(0, min(TK, min(n_kv, (jb + 1) * bkv) - st)) << 24)) : 0;
  };
  refill(0);
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
    constexpr int PCH = (D * D * 2 / 16) / NT;  // 16-byte chunks of one plane per thread
    static_assert(D * PSTR <= 5 * KTILE, "a state plane must fit in the tiles' space");
    const u32x4* gp = reinterpret_cast<const u32x4*>(hist.planes + (size_t)bh * 2 * D * D);
    for (int plane = 0; plane < hist.n_planes; ++plane) {  // each plane goes through LDS once per workgroup
      u32x4 preg[PCH];
#pragma unroll
      for (int i = 0; i < PCH; ++i) preg[i] = gp[plane * (D * D * 2 / 16) + tid + NT * i];
      if (plane) __syncthreads();  // everybody is done with the previous plane
#pragma unroll
      for (int i = 0; i < PCH; ++i) {
        const int c = tid + NT * i;
        *reinterpret_cast<u32x4*>(smem + (c >> 4) * PSTR + (c & 15) * 16) = preg[i];
      }
      __syncthreads();
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(smem + (32 * dt + l32) * PSTR + 16 * h + 32 * s);
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
                                 const int32_t* idx, int k, const HistArgs* hist, void* O, hipStream_t s) {
  if (n_kv >= kMfmaMaxKeys) { set_error("window longer than %d keys", kMfmaMaxKeys); return HF_ERR_SHAPE; }
  const int BH = c.batch * c.heads;
  const int t_m = (n_q + c.block_q - 1) / c.block_q, t_n = (n_kv + c.block_kv - 1) / c.block_kv;
  const long long total = (long long)BH * t_m;
  if (total > (1ll << 30)) { set_error("too many query blocks"); return HF_ERR_SHAPE; }
  const int per_xcd = (int)((total + 7) / 8);
  const float scale = c.softmax_scale > 0.0f ? c.softmax_scale : 1.0f / sqrtf((float)c.head_dim);
  const float c_scale = scale * 1.4426950408889634f;
  const dim3 grid(8 * per_xcd);
  const bf16_t* q = static_cast<const bf16_t*>(Q);
  const bf16_t* kk = static_cast<const bf16_t*>(K);
  const bf16_t* v = static_cast<const bf16_t*>(V);
  bf16_t* o = static_cast<bf16_t*>(O);
  const HistArgs h = hist ? *hist : HistArgs{};
#define HF_LAUNCH_ATTN(NWV, FUSED)                                                                              \
  hipLaunchKernelGGL((attn_mfma_kernel<NWV, FUSED>), grid, dim3(64 * NWV), 0, s, q, kk, v, idx, k, n_q, n_kv,   \
                     kv_stride_of(c, n_kv), c.block_kv, t_m, t_n, per_xcd, (int)total, c_scale, h, o)
  const int fused = !h.planes && !h.lse2 ? 0 : (h.lse2 ? 3 : ((h.phi_kind == HF_PHI_RELU && h.cosq == nullptr && h.q_hist == nullptr) ? 1 : 2));
  if (c.block_q == 64) {
    if (fused == 0) HF_LAUNCH_ATTN(2, 0); else if (fused == 1) HF_LAUNCH_ATTN(2, 1); else if (fused == 2) HF_LAUNCH_ATTN(2, 2); else HF_LAUNCH_ATTN(2, 3);
  } else {
    if (fused == 0) HF_LAUNCH_ATTN(4, 0); else if (fused == 1) HF_LAUNCH_ATTN(4, 1); else if (fused == 2) HF_LAUNCH_ATTN(4, 2); else HF_LAUNCH_ATTN(4, 3);
  }
#undef HF_LAUNCH_ATTN
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
                           void* olocal_out) {
  // One bf16 plane of L (2^-9 per element, errors of the d terms of a readout average out) costs the
  // output nothing measurable next to the bf16 rounding of P and O; HF_FLAG_HISTORY_TWO_PLANES adds the low plane.
  const HistArgs h = {static_cast<const bf16_t*>(planes), zvec, c.eps, c.z_scale, (c.flags & HF_FLAG_HISTORY_TWO_PLANES) ? 2 : 1,
                      c.phi, cosq, sinq, Q_hist == Q ? nullptr : static_cast<const bf16_t*>(Q_hist), nullptr, nullptr, nullptr,
                      lse2_out, static_cast<bf16_t*>(olocal_out)};
  return launch_attn_mfma_impl(c, Q, n_q, K, V, n_kv, idx, k, &h, O, s);
}

// the forward pass recomputed for the backward pass: row statistics out, no attention output
int launch_attn_mfma_stats(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                           const int32_t* idx, int k, const void* dO, float* lse2, float* dvec, hipStream_t s) {
  const HistArgs h = {nullptr, nullptr, 0.0f, 0.0f, 0, 0, nullptr, nullptr, nullptr, static_cast<const bf16_t*>(dO),
                      lse2, dvec, nullptr, nullptr};
  return launch_attn_mfma_impl(c, Q, n_q, K, V, n_kv, idx, k, &h, nullptr, s);
}

}  // namespace hf
