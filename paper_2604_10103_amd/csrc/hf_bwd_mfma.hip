// Backward pass of the block-sparse attention on the matrix cores (bf16, head_dim 128, block_q 64 or
// 128; training algorithm of the supplement).  Two kernels, both built from 32x32x16 bf16 MFMAs on
// transposed products, so that every statistic of a softmax row is private to a lane or comes from a
// 32-entry table, and every accumulated gradient stays in registers until it is stored once:
//
//  dQ  (one workgroup per query block, one wavefront per 32 query rows, tiles of 32 keys)
//      S^T  = K Q^T          D - dP^T = D + V (-dO)^T  lane = query row, registers = keys
//      dS^T = (-2^(c S^T - lse2)) (D - dP^T)           -> bf16, B operand
//      dQ^T += K^T dS^T                                A operand = K transposed in LDS
//  dK, dV  (one workgroup per 64 keys of a KV block, a wavefront per 32 keys x 128 features, one wavefront per
//      SIMD with the 128 accumulators in the accumulation half of the register file, tiles of 32 query rows
//      taken from the inverse index lists)
//      S  = Q K^T            D - dP = D + dO (-V)^T   lane = key, registers = query rows
//      P  = 2^(c S - lse2),  dS = (-P) (D - dP)       -> bf16, B operands
//      dV^T += dO^T P        dK^T += Q^T dS           A operands = dO, Q transposed in LDS
//
// A tile of 32 tokens x 128 features goes global -> LDS directly (buffer loads with the LDS bit; rows past the
// end of the head arrive as zeros), row-major with swizzled 16-byte units, and serves both kinds of A operand:
// tokens as rows by 16-byte reads, features as rows by gfx950's transposing reads (ds_read_b64_tr_b16).
// No staging registers, no LDS stores, no transposing permutes; one barrier per tile.  Both kernels run one
// wavefront per SIMD with their accumulators and loop-invariant operands in the accumulation half of the register
// file, all MFMAs of their loops as inline assembly, four tile slots and a loop pipelined over three tiles; the
// dK/dV workgroups are launched longest list first (dkv_order_kernel).
#include <math.h>
#include <stdlib.h>

#include "hf_common.h"

namespace hf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int D = 128;
constexpr int TT = 32;       // tokens per tile
constexpr int RSTR = 256;    // bytes per token row of a row-major tile
constexpr int RTILE = TT * RSTR;
constexpr int OSTR = 272;    // bytes per token row of a staged output

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// A 32-token tile sits in LDS row-major, 256 B per token, the 16-byte units of a row permuted:
// unit u of row r is stored at u ^ swz(r), swz(r) = 4 (r & 3) | (r >> 2 & 3).  With it both access patterns
// below are free of bank conflicts: 16-byte reads of one unit from 16 consecutive rows (16 different units)
// and the transposing reads, whose 32 lanes of two groups touch 4 consecutive rows x 4 units (16 different units).
__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// buffer descriptor of [rows x 128] bf16 at p (range check ends at the last row)
__device__ __forceinline__ i32x4 desc_of(const bf16_t* p, int rows) {
  const uint64_t a = reinterpret_cast<uint64_t>(p);
  return i32x4{(int)(uint32_t)a, (int)(uint32_t)(a >> 32), rows * (D * 2), 0x00020000};
}

// Per-wavefront constants of the tile transfer global -> LDS (buffer loads with the LDS bit, 16 bytes per
// lane, 1 KB = 4 token rows per instruction): a lane's place in LDS is fixed, the swizzle is done by
// choosing which global unit it fetches.
template <int NWAVES>
struct TileDma {
  static constexpr int CPT = 8 / NWAVES;   // 1 KB pieces per wavefront
  int lane_off[CPT];
  int wave;
  __device__ TileDma(int wave_, int lane) : wave(wave_) {
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      const int r = 4 * (wave + NWAVES * j) + (lane >> 4), u = lane & 15;
      lane_off[j] = r * (D * 2) + ((u ^ swz(r)) * 16);
    }
  }
  // rows [first, first + 32) of the tensor behind desc -> LDS at byte address lds; rows past the end (or a
  // tile that starts past it) arrive as zeros (a load past the descriptor's end stores zero in LDS).  Completion
  // is counted by vmcnt.
  __device__ __forceinline__ void fetch(const i32x4& desc, uint32_t lds, int first_v) const {
    const i32x4 d2 = moved(desc, first_v);
#pragma unroll
    for (int j = 0; j < CPT; ++j) piece(d2, lds, j);
  }
  // the same in two steps, for a caller that spreads the pieces between other instructions: the descriptor moved
  // to the tile's first row, then piece j of this wavefront
  __device__ __forceinline__ i32x4 moved(const i32x4& desc, int first_v) const {
    const int first = __builtin_amdgcn_readfirstlane(first_v);
    const int skip = first * (D * 2), left = desc.z - skip;
    const uint64_t base = (((uint64_t)(uint32_t)desc.y << 32) | (uint32_t)desc.x) + (uint64_t)(uint32_t)(left > 0 ? skip : 0);
    return i32x4{(int)(uint32_t)base, (int)(uint32_t)(base >> 32), left > 0 ? left : 0, desc.w};
  }
  // the same without moving the descriptor: voff = lane_off[j] + 256 first (rows past the end lie past the
  // descriptor's range either way)
  __device__ __forceinline__ int offset_of(int j, int first_bytes) const { return lane_off[j] + first_bytes; }
  __device__ __forceinline__ uint32_t place_of(uint32_t lds, int j) const { return lds + 4 * (wave + NWAVES * j) * RSTR; }
  __device__ __forceinline__ void piece_at(const i32x4& desc, uint32_t lds, int j, int voff) const {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(place_of(lds, j)), "v"(voff), "s"(desc) : "memory", "m0");
  }
  __device__ __forceinline__ void piece(const i32x4& d2, uint32_t lds, int j) const {
    const uint32_t dst = lds + 4 * (wave + NWAVES * j) * RSTR;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(dst), "v"(lane_off[j]), "s"(d2) : "memory", "m0");
  }
};

// A operand, tokens as rows: row l32, features 16 s + 8 h .. + 8: byte rows_base(l32, h) ^ (32 s)
__device__ __forceinline__ uint32_t rows_base(int l32, int h) {
  const int w = swz(l32);
  return l32 * RSTR + 16 * (h ^ (w & 1)) + 32 * (w >> 1);
}
__device__ __forceinline__ bf16x8 rows_frag(const char* sX, uint32_t base, int s) {
  return *reinterpret_cast<const bf16x8*>(sX + (base ^ (32u * s)));
}
// A operand, features as rows: feature 32 ft + l32, tokens 16 t2 + 8 x + 4 h .. + 4 for x = 0, 1, by two
// transposing reads (a 16-lane group fetches 4 token rows x 16 features as 16 chunks of 8 bytes, lane j the
// chunk (row j / 4, features 4 (j % 4)); every lane receives the four tokens of its own feature):
// byte (tr_base(lane) ^ (64 ft) ^ (32 x)) + 4096 t2 + 2048 x   (row 16 t2 + 8 x + key_l: swz = 4 (key_l & 3) | 2 x | h)
__device__ __forceinline__ uint32_t tr_base(int lane) {
  const int j = lane & 15, g = lane >> 4, h = lane >> 5;
  const int key_l = 4 * h + (j >> 2);
  const int c = (4 * (key_l & 3)) | ((2 * (g & 1) + ((j & 3) >> 1)) ^ h);
  return key_l * RSTR + 16 * c + 8 * (j & 1);
}
__device__ __forceinline__ bf16x8 transposed_frag(const char* sX, uint32_t base, int ft, int t2) {
  const char* p0 = sX + (base ^ (64u * ft)) + 4096 * t2;
  const char* p1 = sX + (base ^ (64u * ft) ^ 32u) + 4096 * t2 + 2048;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p1));
  const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, both);
}

// this lane's token row as B-operand fragments (features 16 s + 8 h .. + 8), zero past the end
__device__ __forceinline__ void row_frags(__amdgpu_buffer_rsrc_t rsrc, int row, int h, bf16x8 (&f)[8]) {
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, row * (D * 2) + 16 * h + 32 * s, 0, 0);
    f[s] = __builtin_bit_cast(bf16x8, v);
  }
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc_of(const bf16_t* p, int rows) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(p), 0, rows * (D * 2), 0x00020000);
}

// C-layout accumulators (feature 32 dt + 8 (r >> 2) + 4 h + (r & 3), token l32) -> bf16 rows in LDS
__device__ __forceinline__ void stage_rows(char* stage, int row, int h, const f32x16 (&acc)[4], float mul) {
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      uint2 w;
      w.x = (uint32_t)f32_to_bf16(acc[dt][4 * rq] * mul) | ((uint32_t)f32_to_bf16(acc[dt][4 * rq + 1] * mul) << 16);
      w.y = (uint32_t)f32_to_bf16(acc[dt][4 * rq + 2] * mul) | ((uint32_t)f32_to_bf16(acc[dt][4 * rq + 3] * mul) << 16);
      *reinterpret_cast<uint2*>(stage + row * OSTR + (32 * dt + 8 * rq + 4 * h) * 2) = w;
    }
}

// History branch (Eq. 3) in the dQ kernel's epilogue: with f = phi(q), r = R f, den = z_scale f.z + eps
//     num^T = Lt r^T            (first plane:  Lt[j][i] = bf16(L[i][j]), rows = value features)
//     dden  = -(dO . num) / den^2
//     t^T   = L (dO / den)^T    (second plane: bf16(L[i][j]), rows = key features)
//     dq    = (R^T t + z_scale dden z) * phi'(q)
// Both products have the query fragments' layout on the B side (lane = query row), so the result lands
// in the accumulator layout of dQ and joins it before the one rounding (kHist 1) or is stored as the
// gradient of a query tensor of its own (kHist 2).
struct BwdHist {
  const bf16_t* planes;   // [BH][2][d][d]
  const float* zvec;      // [BH][d]
  const float* cosq;      // [n_q][d/2] or NULL
  const float* sinq;
  const bf16_t* q_hist;   // [BH][n_q][d] queries of the history branch (kHist 2)
  bf16_t* dq_hist;        // [BH][n_q][d] their gradient (kHist 2)
  float eps, z_scale;
  int phi_kind;
};

// fp32 state -> the two bf16 planes of the backward pass: Lt (transposed) and L
__global__ __launch_bounds__(256) void state_planes_bwd_kernel(const float* __restrict__ state,
                                                               bf16_t* __restrict__ planes) {
  __shared__ float tile[32][33];
  const int bh = blockIdx.z, i0 = blockIdx.y * 32, j0 = blockIdx.x * 32;
  const float* L = state + (size_t)bh * D * D;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  bf16_t* lt = planes + (size_t)bh * 2 * D * D;
  bf16_t* ln = lt + D * D;
  for (int r = ty; r < 32; r += 8) {
    const float v = L[(size_t)(i0 + r) * D + j0 + tx];
    tile[r][tx] = v;
    ln[(size_t)(i0 + r) * D + j0 + tx] = f32_to_bf16(v);
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) lt[(size_t)(j0 + r) * D + i0 + tx] = f32_to_bf16(tile[tx][r]);
}

// acc += A B with the accumulator pinned to the accumulation half of the register file (the compiler, left to
// itself, keeps such accumulators in ordinary registers and shuttles others through that half).  The compiler
// counts no wait states for inline assembly, so they are provided here: A comes from LDS reads, which it awaits as
// for any use; C is the same accumulator's previous value, eight MFMAs back; B is a vector ALU result, and an MFMA
// may not read one in the two issue slots after it was written: kWait = true puts two idle slots first, for the
// first reader of a B operand.  volatile keeps the MFMAs in program order, so that the first reader stays the first.
template <bool kWait>
__device__ __forceinline__ void mfma_acc(f32x16& acc, const bf16x8 a, const bf16x8 b) {
  if (kWait) asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}

// Scores-type products of the two pipelined kernels: the loop-invariant B operand sits in the accumulation half of
// the register file, the result in ordinary registers (its first reader is vector work a phase of MFMAs later).
__device__ __forceinline__ void mfma_zero(f32x16& acc, const bf16x8 a, const bf16x8& b) {   // acc = A B
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_from(f32x16& acc, const bf16x8 a, const bf16x8& b, const f32x16& c) {   // = A B + C
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(acc) : "v"(a), "a"(b), "v"(c));
}
__device__ __forceinline__ void mfma_more(f32x16& acc, const bf16x8 a, const bf16x8& b) {   // acc += A B
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b));
}
// acc += A B, accumulator in the accumulation half, with a 1 KB transfer global -> LDS behind it (LDS address through
// m0, written in front of the MFMA, which is the wait state that the transfer needs behind that write)
__device__ __forceinline__ void mfma_acc_piece(f32x16& acc, const bf16x8 a, const bf16x8 b, const bool wait,
                                               const uint32_t lds, const int voff, const i32x4& desc) {
  if (wait)
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\t"
                 "buffer_load_dwordx4 %4, %5, 0 offen lds"
                 : "+a"(acc) : "v"(a), "v"(b), "s"(lds), "v"(voff), "s"(desc) : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %3\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\t"
                 "buffer_load_dwordx4 %4, %5, 0 offen lds"
                 : "+a"(acc) : "v"(a), "v"(b), "s"(lds), "v"(voff), "s"(desc) : "memory", "m0");
}

// ---------------------------------------------------------------------------------------------- dQ
// One workgroup per query block, a wavefront per 32 query rows, one wavefront per SIMD: the 64 accumulators of
// dQ^T and the loop-invariant Q and -dO fragments sit in the accumulation half of the register file; only MFMAs
// touch the accumulators inside the loop, whose body has no vector branch (see the dK/dV kernel below for why).
// kRagged: block_kv is no multiple of 32, so that the last part of a block is cut short and its missing keys have
// to be masked (they are keys of the next block).
constexpr int kDqSlots = 4;   // tiles in LDS: K and V each
constexpr int kDqLds = kDqSlots * 2 * RTILE;
template <int NW, int kHist, bool kRagged>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(1, 1))) void bwd_dq_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const int32_t* __restrict__ idx, int k, int n_q, int n_kv, int kv_stride, int bkv,
    int t_m, int t_n, int items_per_xcd, int total_items, float c_scale, float scale,
    const float* __restrict__ lse2, const float* __restrict__ Dv, BwdHist hist, bf16_t* __restrict__ dQ) {
  constexpr int NT = 64 * NW;
  constexpr int BQ = 32 * NW;
  constexpr int NSLOT = kDqSlots;
  extern __shared__ __attribute__((aligned(16))) char smem[];   // kDqLds bytes: K and V per slot; a state plane later
  static_assert(4 * RTILE <= kDqLds, "a state plane (four pieces of 32 rows) must fit in the tiles' space");
  char* const sK = smem;
  char* const sV = smem + NSLOT * RTILE;
  static_assert(BQ * OSTR <= kDqLds, "staged output must fit");

  // consecutive workgroup ids go to consecutive XCDs: every XCD gets one contiguous run of (head, query
  // block) items, so that its L2 holds the keys and values of few heads
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int item = xcd * items_per_xcd + slot;
  if (slot >= items_per_xcd || item >= total_items) return;
  const int bh = item / t_m, qb = item - bh * t_m;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, h = lane >> 5;
  const TileDma<NW> dma(wave, lane);
  const __amdgpu_buffer_rsrc_t q_rsrc = rsrc_of(Q + (size_t)bh * n_q * D, n_q);
  const __amdgpu_buffer_rsrc_t do_rsrc = rsrc_of(dO + (size_t)bh * n_q * D, n_q);
  const i32x4 k_desc = desc_of(K + (size_t)bh * kv_stride * D, n_kv);
  const i32x4 v_desc = desc_of(V + (size_t)bh * kv_stride * D, n_kv);
  const uint32_t sK_lds = (uint32_t)(uintptr_t)sK, sV_lds = (uint32_t)(uintptr_t)sV;
  const uint32_t rb = rows_base(l32, h), tb = tr_base(lane);
  const int32_t* row_idx = idx ? idx + ((size_t)bh * t_m + qb) * k : nullptr;
  const int nsel = idx ? k : t_n;
  const int subs = (bkv + TT - 1) / TT;

  const int q_row = qb * BQ + 32 * wave + l32;   // rows past n_q read zeros and are not stored
  bf16x8 qf[8], dof[8];
  row_frags(q_rsrc, q_row, h, qf);
  row_frags(do_rsrc, q_row, h, dof);
  const size_t stat = (size_t)bh * n_q + min(q_row, n_q - 1);
  const float lse = lse2[stat], dvec = Dv[stat];
  // (requested now, used after the first tiles have been requested: the latencies overlap)
  f32x16 dq[4], dinit;

  // Tile list: (selected block, 32-key part) -> first key.  A tile past the end of the list, an out-of-range block
  // index or an empty part of a short block starts at n_kv: past the head's end, where the transfers deliver
  // zeros, and zeros for K contribute nothing to dQ whatever P is.  Block indices come by scalar loads one tile
  // ahead of their use, awaited behind the next barrier (a vector load in the loop would share the transfers'
  // counter and drain them); the counters (sel, sub) of the next tile to look up advance without a branch.
  const int ntiles = nsel * subs;
  const int32_t* list_base = row_idx ? row_idx : reinterpret_cast<const int32_t*>(Q);   // dense: any readable word
  int sel_n = 0, sub_n = 0;
  auto entry_issue_at = [&](const int sel) {
    int jb;
    const int off = __builtin_amdgcn_readfirstlane(row_idx ? 4 * min(sel, nsel - 1) : 0);
    asm volatile("s_load_dword %0, %1, %2" : "=s"(jb) : "s"(list_base), "s"(off) : "memory");
    return jb;
  };
  auto entry_issue = [&]() { return entry_issue_at(sel_n); };
  auto entry_wait = [&](int& e) { asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(e) :: "memory"); };
  // first key and number of real keys of the tile (sel_n, sub_n) whose block index was loaded; then step on
  auto tile_of = [&](int jb_loaded, int& start, int& valid) {
    const int jb = row_idx ? jb_loaded : sel_n;
    const int first = jb * bkv + TT * sub_n;
    const int n = min(TT, min(n_kv, (jb + 1) * bkv) - first);
    const bool ok = sel_n < nsel && (unsigned)jb < (unsigned)t_n && n > 0;
    start = ok ? first : n_kv;
    valid = ok ? n : 0;
    const bool wrap = sub_n + 1 == subs;
    sub_n = wrap ? 0 : sub_n + 1;
    sel_n += wrap ? 1 : 0;
  };
  constexpr int CPT = TileDma<NW>::CPT;
  constexpr int kPerTile = 2 * CPT;   // transfers a wavefront issues per tile
  auto fetch_tile = [&](const int slot_, const int start_v) {
    const int first = __builtin_amdgcn_readfirstlane(start_v) * (D * 2);
#pragma unroll
    for (int j = 0; j < CPT; ++j) dma.piece_at(k_desc, sK_lds + slot_ * RTILE, j, dma.offset_of(j, first));
#pragma unroll
    for (int j = 0; j < CPT; ++j) dma.piece_at(v_desc, sV_lds + slot_ * RTILE, j, dma.offset_of(j, first));
  };
  int v1, v2, v3, e_next;   // real keys of tiles n + 1 .. n + 3
  {
    // the block indices of tiles 0 .. 3 in one round trip (tile t belongs to selection t / subs)
    int st, v0;
    int e0 = entry_issue_at(0), e1 = entry_issue_at(1 / subs), e2 = entry_issue_at(2 / subs), e3 = entry_issue_at(3 / subs);
    entry_wait(e0);
    entry_wait(e1);
    entry_wait(e2);
    entry_wait(e3);
    tile_of(e0, st, v0); fetch_tile(0, st);
    tile_of(e1, st, v1); fetch_tile(1, st);
    tile_of(e2, st, v2); fetch_tile(2, st);
    tile_of(e3, st, v3); fetch_tile(3, st);
    e_next = entry_issue();
    v1 = kRagged ? v1 : TT;   // (only the ragged instance looks at them)
    (void)v0;
    // Q, dO and the row statistics were requested before the tiles: complete once at most the tiles are in flight
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(4 * kPerTile) : "memory");
    // dO enters negated: the dP accumulator starts at D and ends at D - dP, so that dS = (-P) (D - dP) costs one
    // multiplication per element (the history branch below turns the sign back)
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      u32x4 w = __builtin_bit_cast(u32x4, dof[s]);
      w ^= 0x80008000u;
      dof[s] = __builtin_bit_cast(bf16x8, w);
    }
    // inside the loop Q and -dO of this wavefront's rows live in the accumulation half of the register file
#pragma unroll
    for (int s = 0; s < 8; ++s) asm volatile("" : "+a"(qf[s]), "+a"(dof[s]));
    // (dinit: the dP accumulator's start)
#pragma unroll
    for (int r = 0; r < 16; ++r) dinit[r] = dvec;

#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) dq[dt][r] = 0.0f;

    // The loop is pipelined over three tiles like the dK/dV kernel's (see there): a trip forms S^T and D - dP^T of
    // tile n + 1 next to dS^T of tile n and the transposing reads of its keys, passes the barrier (tile n + 2 has
    // landed, tile n's slot is free) and accumulates tile n into dQ^T next to the row reads of tile n + 2 and the
    // requests for tile n + 4.  Source order is issue order.
    f32x16 s0, p0, s1, p1;   // S^T and D - dP^T, two generations
    bf16x8 ka[8], va_[8];    // rows of the tile whose scores come next
    auto rows_read = [&](const int par, const int s) {
      ka[s] = rows_frag(sK + par * RTILE, rb, s);
      va_[s] = rows_frag(sV + par * RTILE, rb, s);
    };
    // a key that the part of a short block does not have starts at -inf: its probability is zero
    auto scores = [&](const int s, const int valid, f32x16& sacc) {
      if (s == 0 && kRagged) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = (8 * (r >> 2) + 4 * h + (r & 3) >= valid) ? -INFINITY : 0.0f;
        asm volatile("s_nop 1" : "+v"(sacc));   // (vector results, read by an MFMA the compiler does not know)
      }
      if (s == 0 && !kRagged) mfma_zero(sacc, ka[0], qf[0]);
      else mfma_more(sacc, ka[s], qf[s]);
    };
    auto grads = [&](const int s, f32x16& dpacc) {
      if (s == 0) mfma_from(dpacc, va_[0], dof[0], dinit);
      else mfma_more(dpacc, va_[s], dof[s]);
    };
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(3 * kPerTile) : "memory");   // tile 0
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 8; ++s) rows_read(0, s);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < 8; ++s) { scores(s, kRagged ? v0 : TT, s0); grads(s, p0); }
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * kPerTile) : "memory");   // tile 1
    __syncthreads();
#pragma unroll
    for (int s = 0; s < 8; ++s) rows_read(1, s);
    __builtin_amdgcn_sched_barrier(0);

    auto tile_step = [&](const int par, f32x16& sc, f32x16& dp, f32x16& sn, f32x16& dn) {
      // par = n mod 4 (a literal at the call sites): the slot of tile n.  sc, dp belong to tile n, sn, dn to n + 1.
      const char* tK = sK + par * RTILE;
      bf16x8 kt[8];          // K^T of tile n: 4 t2 + dt
      u32x4 dsw[2];          // dS^T, two bf16 per word
      float dse;
      // dS^T = (-P) (D - dP) with P = 2^(c S^T - lse2), clamped to [0, 1] (an output modifier of the exponential: a
      // real key's probability is there anyway, and a row of zeros standing in for a key past the head's end must
      // not reach infinity, 0 * inf would follow).  The empty statements that name the results keep the vector work
      // between the MFMAs where it is written.
      auto ds_even = [&](const int s) {
        dse = -__builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(fmaf(sc[2 * s], c_scale, -lse)), 0.0f, 1.0f) * dp[2 * s];
        asm volatile("" : "+v"(dse));
      };
      auto ds_odd = [&](const int s) {
        const float dso =
            -__builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(fmaf(sc[2 * s + 1], c_scale, -lse)), 0.0f, 1.0f) * dp[2 * s + 1];
        const bf16x2 dw = {static_cast<__bf16>(dse), static_cast<__bf16>(dso)};
        uint32_t dwi = __builtin_bit_cast(uint32_t, dw);
        asm volatile("" : "+v"(dwi));
        dsw[s >> 2][s & 3] = dwi;
      };
      // ---- phase one
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        scores(s, v1, sn);
        kt[s] = transposed_frag(tK, tb, s & 3, s >> 2);
        ds_even(s);
        __builtin_amdgcn_sched_barrier(0);
        grads(s, dn);
        ds_odd(s);
        __builtin_amdgcn_sched_barrier(0);
      }
      // ---- tile n + 2 visible, tile n's slot free (every transposing read of it has returned)
      asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kPerTile) : "memory");   // this wavefront's parts of tile n + 2
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __syncthreads();
      entry_wait(e_next);
      int st4, v4;
      tile_of(e_next, st4, v4);
      e_next = entry_issue();
      const int first = __builtin_amdgcn_readfirstlane(st4) * (D * 2);
      v1 = v2; v2 = v3; v3 = v4;
      // ---- phase two: tile n into the accumulators
      const int p2 = (par + 2) % NSLOT;
#pragma unroll
      for (int u = 0; u < 8; ++u) {   // u = 4 t2 + dt
        const int dt = u & 3;
        const bf16x8 dsf = __builtin_bit_cast(bf16x8, dsw[u >> 2]);
        if (u < 2 * CPT) {   // a piece of tile n + 4 rides along: K first, then V
          const int j = u % CPT;
          const int voff = dma.offset_of(j, first);
          if (u < CPT) mfma_acc_piece(dq[dt], kt[u], dsf, dt == 0, dma.place_of(sK_lds + par * RTILE, j), voff, k_desc);
          else mfma_acc_piece(dq[dt], kt[u], dsf, dt == 0, dma.place_of(sV_lds + par * RTILE, j), voff, v_desc);
        } else {
          if (dt == 0) mfma_acc<true>(dq[dt], kt[u], dsf);
          else mfma_acc<false>(dq[dt], kt[u], dsf);
        }
        rows_read(p2, u);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // slot numbers are literals, hence four trips per turn of the loop; the last one to three tiles take two or
    // four more trips (a tile past the list is zeros)
    const int whole = ntiles & ~3;
    for (int n = 0; n < whole; n += 4) {
      tile_step(0, s0, p0, s1, p1);
      tile_step(1, s1, p1, s0, p0);
      tile_step(2, s0, p0, s1, p1);
      tile_step(3, s1, p1, s0, p0);
    }
    if (ntiles > whole) {
      tile_step(0, s0, p0, s1, p1);
      tile_step(1, s1, p1, s0, p0);
    }
    if (ntiles > whole + 2) {
      tile_step(2, s0, p0, s1, p1);
      tile_step(3, s1, p1, s0, p0);
    }
  }
  // nothing may land in LDS once the tiles' space is reused; and the last accumulating MFMAs (inline assembly: the
  // compiler does not count wait states for them) must have written their results before these are read: the idle
  // slots name the accumulators as operands, or the compiler moves the reads above them
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  asm volatile("s_nop 15\n\ts_nop 15" : "+a"(dq[0]), "+a"(dq[1]), "+a"(dq[2]), "+a"(dq[3]));

  f32x16 acc[4];   // history branch: num^T, then t^T, then the gradient itself
  if (kHist) {
    // both planes of the state go global -> LDS like the tiles (four pieces of 32 rows each, no registers in
    // between) into the tiles' space, requested here so that they travel under the arithmetic below
    static_assert(8 * RTILE <= kDqLds, "two state planes must fit in the tiles' space");
    const uint32_t smem_lds = (uint32_t)(uintptr_t)smem;
    __syncthreads();   // the tiles are consumed
#pragma unroll
    for (int plane = 0; plane < 2; ++plane) {
      const i32x4 p_desc = desc_of(hist.planes + ((size_t)bh * 2 + plane) * D * D, D);
#pragma unroll
      for (int part = 0; part < 4; ++part) dma.fetch(p_desc, smem_lds + (4 * plane + part) * RTILE, 32 * part);
    }
    bf16x8 hq[8];
    if (kHist == 2) {
      row_frags(rsrc_of(hist.q_hist + (size_t)bh * n_q * D, n_q), q_row, h, hq);
    } else {
#pragma unroll
      for (int s = 0; s < 8; ++s) hq[s] = qf[s];
    }
    const int crow = min(q_row, n_q - 1);
    const float* zv = hist.zvec + (size_t)bh * D;
    // f = phi(q), den = z_scale f.z + eps, r = R f as bf16 fragments
    float den = 0.0f;   // (R f is written back into hq, dO / den into dof: the epilogue must not need more registers)
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      float f[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = phi_apply(static_cast<float>(hq[s][e]), hist.phi_kind);
      const float4 z0 = *reinterpret_cast<const float4*>(zv + 16 * s + 8 * h);
      const float4 z1 = *reinterpret_cast<const float4*>(zv + 16 * s + 8 * h + 4);
      den += f[0] * z0.x + f[1] * z0.y + f[2] * z0.z + f[3] * z0.w + f[4] * z1.x + f[5] * z1.y + f[6] * z1.z +
             f[7] * z1.w;
      if (hist.cosq) {
        const size_t tp = (size_t)crow * (D / 2) + 8 * s + 4 * h;
        const float4 c4 = *reinterpret_cast<const float4*>(hist.cosq + tp);
        const float4 s4 = *reinterpret_cast<const float4*>(hist.sinq + tp);
        const float cc[4] = {c4.x, c4.y, c4.z, c4.w}, ss[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
        for (int p2 = 0; p2 < 4; ++p2) {
          const float a = f[2 * p2], b = f[2 * p2 + 1];
          f[2 * p2] = a * cc[p2] - b * ss[p2];
          f[2 * p2 + 1] = a * ss[p2] + b * cc[p2];
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) hq[s][e] = static_cast<__bf16>(f[e]);
    }
    {
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(den), __float_as_uint(den), false, false);
      den = hist.z_scale * (__uint_as_float(sw[0]) + __uint_as_float(sw[1])) + hist.eps;
    }
    const float inv_den = 1.0f / den;

    float dden = 0.0f;
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) dof[s][e] = static_cast<__bf16>(-static_cast<float>(dof[s][e]) * inv_den);   // dnum
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's pieces of both planes
    __syncthreads();
    for (int plane = 0; plane < 2; ++plane) {
      const char* sP = smem + 4 * plane * RTILE;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] = 0.0f;
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows_frag(sP + dt * RTILE, rb, s), plane ? dof[s] : hq[s],
                                                            acc[dt], 0, 0, 0);
        }
      if (plane == 0) {
        // dden = -(dO . num) / den^2
        const bf16_t* gq = dO + ((size_t)bh * n_q + crow) * D + 4 * h;
        float gn = 0.0f;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const uint2 w = *reinterpret_cast<const uint2*>(gq + 32 * dt + 8 * rq);
            gn = fmaf(acc[dt][4 * rq], __uint_as_float(w.x << 16), gn);
            gn = fmaf(acc[dt][4 * rq + 1], __uint_as_float(w.x & 0xffff0000u), gn);
            gn = fmaf(acc[dt][4 * rq + 2], __uint_as_float(w.y << 16), gn);
            gn = fmaf(acc[dt][4 * rq + 3], __uint_as_float(w.y & 0xffff0000u), gn);
          }
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(gn), __float_as_uint(gn), false, false);
        dden = -(__uint_as_float(sw[0]) + __uint_as_float(sw[1])) * inv_den * inv_den;
      }
    }
    // back through the rotation, the denominator's share, phi'
    const bf16_t* qsrc = (kHist == 2 ? hist.q_hist : Q) + ((size_t)bh * n_q + crow) * D + 4 * h;
    const float zd = hist.z_scale * dden;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int f0 = 32 * dt + 8 * rq + 4 * h;
        float t[4] = {acc[dt][4 * rq], acc[dt][4 * rq + 1], acc[dt][4 * rq + 2], acc[dt][4 * rq + 3]};
        if (hist.cosq) {
          const float2 c2 = *reinterpret_cast<const float2*>(hist.cosq + (size_t)crow * (D / 2) + f0 / 2);
          const float2 s2 = *reinterpret_cast<const float2*>(hist.sinq + (size_t)crow * (D / 2) + f0 / 2);
          const float a0 = t[0], b0 = t[1], a1 = t[2], b1 = t[3];
          t[0] = a0 * c2.x + b0 * s2.x;
          t[1] = -a0 * s2.x + b0 * c2.x;
          t[2] = a1 * c2.y + b1 * s2.y;
          t[3] = -a1 * s2.y + b1 * c2.y;
        }
        const float4 z4 = *reinterpret_cast<const float4*>(zv + f0);
        const float zz[4] = {z4.x, z4.y, z4.z, z4.w};
        const uint2 w = *reinterpret_cast<const uint2*>(qsrc + 32 * dt + 8 * rq);
        const float qv[4] = {__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u),
                             __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xffff0000u)};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float dphi = hist.phi_kind == HF_PHI_RELU ? (qv[i] > 0.0f ? 1.0f : 0.0f)
                                                          : (qv[i] > 0.0f ? 1.0f : __expf(qv[i]));
          const float g = (t[i] + zd * zz[i]) * dphi;
          if (kHist == 1) dq[dt][4 * rq + i] = fmaf(dq[dt][4 * rq + i], scale, g);
          else acc[dt][4 * rq + i] = g;
        }
      }
  }
  bf16_t* dQh = dQ + (size_t)bh * n_q * D;
  for (int which = 0; which < (kHist == 2 ? 2 : 1); ++which) {
    __syncthreads();
    if (which == 0) stage_rows(smem, 32 * wave + l32, h, dq, kHist == 1 ? 1.0f : scale);
    else stage_rows(smem, 32 * wave + l32, h, acc, 1.0f);
    __syncthreads();
    bf16_t* out = which ? hist.dq_hist + (size_t)bh * n_q * D : dQh;
#pragma unroll
    for (int i = 0; i < (BQ * 16) / NT; ++i) {
      const int c = tid + NT * i, row = c >> 4, col = c & 15;
      if (qb * BQ + row < n_q)
        *reinterpret_cast<uint4*>(out + (size_t)(qb * BQ + row) * D + col * 8) =
            *reinterpret_cast<const uint4*>(smem + row * OSTR + col * 16);
    }
  }
}

// ------------------------------------------------------------------------------------------ dK, dV
// Launch order of the dK/dV workgroups.  A workgroup's time is proportional to the length of its KV block's list
// of query blocks, and the lists differ (top-k selection: a binomial spread around t_m k / t_n), while a GPU takes
// workgroups in index order as slots free up.  Longest first within every XCD's share of the items leaves the short
// ones to fill the end.  The kernel writes one record of 8 words per place: the item that runs there (rank by list
// length descending, item ascending, found by counting), the length of its list and the list's first three entries,
// so that a workgroup has all it needs for its first tiles after ONE dependent load (a workgroup is alone on its
// two SIMDs: every round trip to memory before its first MFMA is idle time).
// One workgroup per share; the share's keys sit in LDS.
constexpr int kOrderMax = 4096;   // items per share this kernel takes (4 per thread, 2 x 16 KB of LDS)
constexpr int kOrderRec = 8;      // words per record
__global__ __launch_bounds__(1024) void dkv_order_kernel(const int32_t* __restrict__ inv_cnt,
                                                          const int32_t* __restrict__ inv_list, int t_m, int slabs,
                                                          int items_per_xcd, int total_items,
                                                          int32_t* __restrict__ order) {
  __shared__ int32_t key[kOrderMax], rank[kOrderMax];
  const int first = blockIdx.x * items_per_xcd;
  const int n = max(0, min(items_per_xcd, total_items - first));
  // a thread per item: list length and first entries, all loads in flight together
  int4 head[kOrderMax / 1024];
#pragma unroll
  for (int q = 0; q < kOrderMax / 1024; ++q) {
    const int j = threadIdx.x + 1024 * q;
    if (j < n) {
      const int kvb = (first + j) / slabs;
      const int32_t* list = inv_list + (size_t)kvb * t_m;
      head[q] = int4{inv_cnt[kvb], list[0], list[min(1, t_m - 1)], list[min(2, t_m - 1)]};
      key[j] = head[q].x;
      rank[j] = 0;
    }
  }
  __syncthreads();
  // the n x n comparisons spread over all threads: `per` threads share an item, each takes every per-th key and
  // adds its count to the item's rank
  int per = 1;
  while (per < 64 && 2 * per * n <= 1024) per *= 2;
  const int sub = threadIdx.x & (per - 1);
  for (int j = threadIdx.x / per; j < n; j += 1024 / per) {
    const int mine = key[j];
    int before = 0;
    for (int i = sub; i < n; i += per) {
      const int other = key[i];
      before += (other > mine || (other == mine && i < j)) ? 1 : 0;
    }
    atomicAdd(&rank[j], before);
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < kOrderMax / 1024; ++q) {
    const int j = threadIdx.x + 1024 * q;
    if (j < n) {
      int4* rec = reinterpret_cast<int4*>(order + (size_t)(first + rank[j]) * kOrderRec);
      rec[0] = int4{first + j, head[q].x, head[q].y, head[q].z};
      rec[1] = int4{head[q].w, 0, 0, 0};
    }
  }
}

// One workgroup per slab of 64 keys of a KV block, two wavefronts of 32 keys each; a wavefront owns all 128
// features of dK and dV of its keys: 128 accumulator registers that only MFMAs touch until the end, which is what
// the second half of the register file (one wavefront per SIMD: 512 registers) is for.  Per tile of 32 query rows
// a wavefront issues 16 MFMAs for S and dP and 16 for dV and dK, nothing is computed twice.
constexpr int kDkvSlots = 4;   // tiles in LDS: one in use, three on their way
constexpr int kDkvLds = kDkvSlots * (2 * RTILE + 512);
__global__ __launch_bounds__(128) __attribute__((amdgpu_waves_per_eu(1, 1))) void bwd_dkv_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const int32_t* __restrict__ inv_cnt, const int32_t* __restrict__ inv_list,
    int n_q, int n_kv, int kv_stride, int bq, int bkv, int t_m, int t_n, int slabs, int items_per_xcd,
    int total_items, const int32_t* __restrict__ order, float c_scale, float scale,
    const float* __restrict__ lse2, const float* __restrict__ Dv, bf16_t* __restrict__ dK, bf16_t* __restrict__ dV) {
  constexpr int NT = 128;
  constexpr int NSLOT = kDkvSlots;
  extern __shared__ __attribute__((aligned(16))) char smem[];   // kDkvLds bytes: Q, dO, row statistics per slot
  char* const sQ = smem;
  char* const sdO = smem + NSLOT * RTILE;
  float* const sStat = reinterpret_cast<float*>(smem + 2 * NSLOT * RTILE);   // per slot: lse2[32] twice, D[32] twice
  static_assert(64 * OSTR <= 2 * NSLOT * RTILE, "staged output must fit");

  // XCD-aware placement as in the dQ kernel: an XCD's L2 then holds the queries and output gradients of few heads
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int place = xcd * items_per_xcd + slot;   // the slot-th workgroup of this XCD's share, longest lists first
  if (slot >= items_per_xcd || place >= total_items) return;
  // the record of this place: item, list length, first three list entries (no record: index order, entries loaded)
  const int32_t* rec = order ? order + (size_t)place * kOrderRec : nullptr;
  const int item = rec ? rec[0] : place;
  const int bh = item / (t_n * slabs);
  const int rest = item - bh * (t_n * slabs);
  const int jb = rest / slabs, slab = rest - jb * slabs;
  const int tid = threadIdx.x, lane = tid & 63;
  const int kw = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, h = lane >> 5;
  const TileDma<2> dma(kw, lane);
  const i32x4 q_desc = desc_of(Q + (size_t)bh * n_q * D, n_q);
  const i32x4 do_desc = desc_of(dO + (size_t)bh * n_q * D, n_q);
  const uint32_t sQ_lds = (uint32_t)(uintptr_t)sQ, sdO_lds = (uint32_t)(uintptr_t)sdO;
  const uint32_t rb = rows_base(l32, h), tb = tr_base(lane);
  const __amdgpu_buffer_rsrc_t k_rsrc = rsrc_of(K + (size_t)bh * kv_stride * D, n_kv);
  const __amdgpu_buffer_rsrc_t v_rsrc = rsrc_of(V + (size_t)bh * kv_stride * D, n_kv);
  const float* lseh = lse2 + (size_t)bh * n_q;
  const float* Dvh = Dv + (size_t)bh * n_q;
  const int n_lists = rec ? rec[1] : inv_cnt ? inv_cnt[(size_t)bh * t_n + jb] : t_m;   // no lists: every query block (dense)
  const int32_t* list = inv_list ? inv_list + ((size_t)bh * t_n + jb) * t_m : nullptr;

  // this wavefront's 32 keys (keys past the block's end are computed along and never stored)
  const int blk_end = min(n_kv, (jb + 1) * bkv);
  const int first_key = jb * bkv + 64 * slab;
  const int key0 = first_key + 32 * kw;
  // (requested now, used after the first tiles have been requested: the latencies overlap)
  bf16x8 kf[8], vf[8];
  row_frags(k_rsrc, key0 + l32, h, kf);
  row_frags(v_rsrc, key0 + l32, h, vf);

  f32x16 dk[4], dv[4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[a][r] = 0.0f; dv[a][r] = 0.0f; }

  // tiles of 32 query rows of the listed query blocks.  The rows come from all over the head (whatever query
  // blocks selected this KV block), so a tile is requested two trips of the loop before its first use, into one of
  // four slots (Q, dO and the row statistics).  Rows past n_q, and whole tiles past the end of the list, read zeros.
  const int qtiles = bq / TT;
  const int ntiles = n_lists * qtiles;
  // List entries are fetched with scalar loads issued one tile ahead of their use and awaited behind the next
  // barrier (where no LDS read is in flight): a vector load inside the tile loop would have to be awaited together
  // with every transfer in flight, they share one counter.
  const int qshift = bq == 64 ? 1 : 2;   // tiles per query block = 2 or 4
  auto entry_issue = [&](int n) {   // query block of tile n; valid after entry_wait
    const int t = n >> qshift;
    int e = t;
    if (list) {
      // (an entry past the list's end is never used, so the load need not wait for the list's length)
      const int off = __builtin_amdgcn_readfirstlane(4 * min(t, t_m - 1));
      asm volatile("s_load_dword %0, %1, %2" : "=s"(e) : "s"(list), "s"(off) : "memory");
    }
    return e;
  };
  auto entry_wait = [&](int& e) { asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(e) :: "memory"); };
  auto tile_row0 = [&](int n, int e) {   // first row of tile n, a tile of query block e; uniform over the workgroup
    return n < ntiles ? e * bq + TT * (n & (qtiles - 1)) : n_q;   // a tile past the list lies past the head: zeros
  };
  // row statistics global -> LDS like the tiles (4 bytes per lane; both halves of the wavefront fetch the same 32
  // rows).  Both wavefronts issue them, so that they count the same number of transfers per tile.
  const __amdgpu_buffer_rsrc_t lse_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(lseh), 0, n_q * 4, 0x00020000);
  const __amdgpu_buffer_rsrc_t dv_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(Dvh), 0, n_q * 4, 0x00020000);
  const uint32_t sStat_lds = (uint32_t)(uintptr_t)sStat;
  auto stat_fetch = [&](const int slot_, const int r0, const int which) {   // which: 0 = lse2, 1 = D
    const int off = 4 * (r0 + l32);   // a row past n_q is past the descriptor's end: zero
    if (which == 0)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                   :: "s"(sStat_lds + slot_ * 512), "v"(off), "s"(lse_rsrc) : "memory", "m0");
    else
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                   :: "s"(sStat_lds + slot_ * 512 + 256), "v"(off), "s"(dv_rsrc) : "memory", "m0");
  };
  auto fetch_tile = [&](const int slot_, const int r0_v) {
    const int r0 = __builtin_amdgcn_readfirstlane(r0_v);
#pragma unroll
    for (int j = 0; j < TileDma<2>::CPT; ++j) dma.piece_at(q_desc, sQ_lds + slot_ * RTILE, j, dma.offset_of(j, r0 * (D * 2)));
#pragma unroll
    for (int j = 0; j < TileDma<2>::CPT; ++j) dma.piece_at(do_desc, sdO_lds + slot_ * RTILE, j, dma.offset_of(j, r0 * (D * 2)));
    stat_fetch(slot_, r0, 0);
    stat_fetch(slot_, r0, 1);
  };
  constexpr int kPerTile = 2 * TileDma<2>::CPT + 2;   // transfers a wavefront issues per tile
  int e0, e1, e2, e3, e_next;   // entries of tiles 0 .. 4
  if (rec) {
    const int r0 = rec[2], r1 = rec[3], r2 = rec[4];
    e0 = r0;
    e1 = r0;
    e2 = qshift == 1 ? r1 : r0;
    e3 = e2;
    e_next = qshift == 1 ? r2 : r1;
  } else {
    e0 = entry_issue(0), e1 = entry_issue(1), e2 = entry_issue(2), e3 = entry_issue(3), e_next = entry_issue(4);
    entry_wait(e0);
    entry_wait(e1);
    entry_wait(e2);
    entry_wait(e3);
    entry_wait(e_next);
  }
  fetch_tile(0, tile_row0(0, e0));
  fetch_tile(1, tile_row0(1, e1));
  fetch_tile(2, tile_row0(2, e2));
  fetch_tile(3, tile_row0(3, e3));
  // K and V of this wavefront's keys (requested before the tiles: complete once at most the tiles are in flight).
  // V enters negated: the dP accumulator starts at D and ends at D - dP, so that dS = (-P) (D - dP) costs one
  // multiplication per element.
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(4 * kPerTile) : "memory");
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    u32x4 w = __builtin_bit_cast(u32x4, vf[s]);
    w ^= 0x80008000u;
    vf[s] = __builtin_bit_cast(bf16x8, w);
  }
  // from here on they live in the accumulation half of the register file (every use below asks for them there;
  // defined there, they are not copied before each use)
#pragma unroll
  for (int s = 0; s < 8; ++s) asm volatile("" : "+a"(kf[s]), "+a"(vf[s]));
  // All MFMAs of the loop are inline assembly.  The loop-invariant B operands (K and -V of this wavefront's keys) and
  // the accumulators sit in the accumulation half of the register file; S and D - dP come out in ordinary registers,
  // and their first reader is vector work a whole phase (16 MFMAs) later.
  // A wavefront alone on its SIMD issues in order, one instruction per four cycles, and an MFMA keeps the matrix
  // pipeline busy for 32: everything that is not an MFMA (56 LDS reads, 10 transfers, ~70 vector instructions per
  // tile, about as many issue cycles as the 32 MFMAs take to execute) has to sit BETWEEN MFMAs or the pipeline
  // idles.  Hence a loop pipelined over three tiles, the source order below being the issue order (a fence after
  // every group).  Trip n:
  //   phase one   S and D - dP of tile n + 1 (16 MFMAs; its rows were read in the trip before) next to P and dS of
  //               tile n (vector work on the previous trip's S and D - dP) and the transposing reads of tile n;
  //   barrier     tile n + 2 has landed, tile n's slot is free: tile n + 4 requested into it;
  //   phase two   tile n into dV and dK (16 MFMAs) next to the reads of tile n + 2's rows and D, tile n + 1's
  //               row statistic, and the requests.
  f32x16 s0, p0, s1, p1;   // S and D - dP, two generations
  bf16x8 qa[8], ga[8];     // rows of the tile whose scores come next
  float lsr[16];           // row statistic of the tile whose probabilities come next
  auto d_read = [&](const int par, const int g, f32x16& dpacc) {   // rows 8 g + 4 h .. + 4 of D
    const float4 d4 = *reinterpret_cast<const float4*>(sStat + 128 * par + 64 + 8 * g + 4 * h);
    dpacc[4 * g] = d4.x; dpacc[4 * g + 1] = d4.y; dpacc[4 * g + 2] = d4.z; dpacc[4 * g + 3] = d4.w;
  };
  auto lse_read = [&](const int par, const int g) {
    const float4 l4 = *reinterpret_cast<const float4*>(sStat + 128 * par + 8 * g + 4 * h);
    lsr[4 * g] = l4.x; lsr[4 * g + 1] = l4.y; lsr[4 * g + 2] = l4.z; lsr[4 * g + 3] = l4.w;
  };
  auto rows_read = [&](const int par, const int s) {
    qa[s] = rows_frag(sQ + par * RTILE, rb, s);
    ga[s] = rows_frag(sdO + par * RTILE, rb, s);
  };
  // prologue: S and D - dP of tile 0; rows and D of tile 1, row statistic of tile 0
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(3 * kPerTile) : "memory");   // tile 0
  __syncthreads();
#pragma unroll
  for (int g = 0; g < 4; ++g) d_read(0, g, p0);
#pragma unroll
  for (int s = 0; s < 8; ++s) rows_read(0, s);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    if (s == 0) mfma_zero(s0, qa[0], kf[0]);
    else mfma_more(s0, qa[s], kf[s]);
    mfma_more(p0, ga[s], vf[s]);
  }
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * kPerTile) : "memory");   // tile 1
  __syncthreads();
#pragma unroll
  for (int g = 0; g < 4; ++g) { d_read(1, g, p1); lse_read(0, g); }
#pragma unroll
  for (int s = 0; s < 8; ++s) rows_read(1, s);
  __builtin_amdgcn_sched_barrier(0);

  auto tile_step = [&](const int n, const int par, f32x16& sc, f32x16& dp, f32x16& sn, f32x16& dn) {
    // par = n mod 4 (a literal at the call sites): the slot of tile n.  sc, dp: S and D - dP of tile n;
    // sn, dn: those of tile n + 1, dn holding D so far.
    const char* tQ = sQ + par * RTILE;
    const char* tdO = sdO + par * RTILE;
    // ---- phase one.  P = 2^(c S - lse2) and dS = (-P) (D - dP).  Nothing is masked: a query row that does not
    // exist has zeros for Q, dO, lse2 and D in LDS (P = 1, dS = 0, and its columns of Q^T and dO^T are zero), and a
    // key that does not exist owns a column of dK^T and dV^T that is never stored.
    bf16x8 trf[16];         // transposed fragments of tile n in the order of their use: 8 t2 + 2 ft + (0: dO^T, 1: Q^T)
    u32x4 pfw[2], dsw[2];   // P and dS, two bf16 per word
    auto tr_read = [&](const int f) {
      trf[f] = transposed_frag((f & 1) ? tQ : tdO, tb, (f >> 1) & 3, f >> 3);
    };
    // rows 2 s and 2 s + 1 of this lane's P and dS, in two halves.  (The empty statements that name the results keep
    // the vector work where it is written: without them the compiler collects all of it behind the phase's MFMAs.)
    float pe, dse;
    auto rows_even = [&](const int s) {
      pe = __builtin_amdgcn_exp2f(fmaf(sc[2 * s], c_scale, -lsr[2 * s]));
      dse = -pe * dp[2 * s];
      asm volatile("" : "+v"(pe), "+v"(dse));
    };
    auto rows_odd = [&](const int s) {
      const float po = __builtin_amdgcn_exp2f(fmaf(sc[2 * s + 1], c_scale, -lsr[2 * s + 1]));
      const bf16x2 pw = {static_cast<__bf16>(pe), static_cast<__bf16>(po)};
      const bf16x2 dw = {static_cast<__bf16>(dse), static_cast<__bf16>(-po * dp[2 * s + 1])};
      uint32_t pwi = __builtin_bit_cast(uint32_t, pw), dwi = __builtin_bit_cast(uint32_t, dw);
      asm volatile("" : "+v"(pwi), "+v"(dwi));
      pfw[s >> 2][s & 3] = pwi;
      dsw[s >> 2][s & 3] = dwi;
    };
    // The vector work of the first 16 tokens sits in the first half of phase one, that of the other 16 in the first
    // half of phase two; the halves without it carry more of the reads and the requests.
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      if (s == 0) mfma_zero(sn, qa[0], kf[0]);
      else mfma_more(sn, qa[s], kf[s]);
      if (s < 4) { tr_read(s); rows_even(s); }
      else { tr_read(3 * s - 8); tr_read(3 * s - 7); }
      __builtin_amdgcn_sched_barrier(0);
      mfma_more(dn, ga[s], vf[s]);
      if (s < 4) rows_odd(s);
      else tr_read(3 * s - 6);
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---- tile n + 2 visible, tile n's slot free (every transposing read of it has returned)
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kPerTile) : "memory");   // this wavefront's parts of tile n + 2
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();
    entry_wait(e_next);
    const int r0 = __builtin_amdgcn_readfirstlane(tile_row0(n + 4, e_next));
    e_next = entry_issue(n + 5);
    static_assert(TileDma<2>::CPT == 4, "four pieces per tensor");
    // ---- phase two: tile n into the accumulators; dp (spent) takes D of tile n + 2
    const int p2 = (par + 2) % NSLOT, p1n = (par + 1) % NSLOT;
#pragma unroll
    for (int u = 0; u < 8; ++u) {   // u = 4 t2 + ft
      const int t2 = u >> 2, ft = u & 3;
      const bf16x8 pf = __builtin_bit_cast(bf16x8, pfw[t2]), dsf = __builtin_bit_cast(bf16x8, dsw[t2]);
      // (in the second half an MFMA and a piece of tile n + 4 share a statement: the MFMA is the wait state that the
      // transfer needs behind the write of m0)
      const int voff = u >= 4 ? dma.offset_of(u - 4, r0 * (D * 2)) : 0;
      if (u == 0) mfma_acc<true>(dv[ft], trf[2 * u], pf);   // first reader of pf
      else if (u < 4) mfma_acc<false>(dv[ft], trf[2 * u], pf);
      else mfma_acc_piece(dv[ft], trf[2 * u], pf, u == 4, dma.place_of(sQ_lds + par * RTILE, u - 4), voff, q_desc);
      qa[u] = rows_frag(sQ + p2 * RTILE, rb, u);
      if (u < 4) rows_even(4 + u);
      __builtin_amdgcn_sched_barrier(0);
      if (u == 0) mfma_acc<true>(dk[ft], trf[2 * u + 1], dsf);
      else if (u < 4) mfma_acc<false>(dk[ft], trf[2 * u + 1], dsf);
      else mfma_acc_piece(dk[ft], trf[2 * u + 1], dsf, u == 4, dma.place_of(sdO_lds + par * RTILE, u - 4), voff, do_desc);
      ga[u] = rows_frag(sdO + p2 * RTILE, rb, u);
      if (u < 4) {
        rows_odd(4 + u);
      } else {
        d_read(p2, u - 4, dp);
        lse_read(p1n, u - 4);
        if (u == 5) stat_fetch(par, r0, 0);
        if (u == 6) stat_fetch(par, r0, 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // slot numbers are literals, hence four trips per turn of the loop; the last one to three tiles take two or four
  // more trips (a tile past the list is zeros)
  const int whole = ntiles & ~3;
  for (int n = 0; n < whole; n += 4) {
    tile_step(n, 0, s0, p0, s1, p1);
    tile_step(n + 1, 1, s1, p1, s0, p0);
    tile_step(n + 2, 2, s0, p0, s1, p1);
    tile_step(n + 3, 3, s1, p1, s0, p0);
  }
  if (ntiles > whole) {
    tile_step(whole, 0, s0, p0, s1, p1);
    tile_step(whole + 1, 1, s1, p1, s0, p0);
  }
  if (ntiles > whole + 2) {
    tile_step(whole + 2, 2, s0, p0, s1, p1);
    tile_step(whole + 3, 3, s1, p1, s0, p0);
  }
  // (the idle slots name the accumulators as operands, or the compiler moves the reads above them)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  asm volatile("s_nop 15\n\ts_nop 15" : "+a"(dk[0]), "+a"(dk[1]), "+a"(dk[2]), "+a"(dk[3]), "+a"(dv[0]), "+a"(dv[1]),
               "+a"(dv[2]), "+a"(dv[3]));

  // transpose through LDS and store the rows of real keys, dK first, then dV
  for (int which = 0; which < 2; ++which) {
    __syncthreads();
    if (which == 0) stage_rows(smem, 32 * kw + l32, h, dk, scale);
    else stage_rows(smem, 32 * kw + l32, h, dv, 1.0f);
    __syncthreads();
    bf16_t* out = (which ? dV : dK) + (size_t)bh * kv_stride * D;
#pragma unroll
    for (int i = 0; i < (64 * 16) / NT; ++i) {
      const int c = tid + NT * i, row = c >> 4, col = c & 15;
      if (first_key + row < blk_end)
        *reinterpret_cast<uint4*>(out + (size_t)(first_key + row) * D + col * 8) =
            *reinterpret_cast<const uint4*>(smem + row * OSTR + col * 16);
    }
  }
}

}  // namespace

bool bwd_mfma_supported(const hf_config& c) {
  return c.dtype == HF_BF16 && c.head_dim == 128 && (c.block_q == 64 || c.block_q == 128);
}

size_t bwd_planes_bytes(const hf_config& c) {
  return bwd_mfma_supported(c) ? (size_t)c.batch * c.heads * 2 * D * D * sizeof(bf16_t) : 0;
}

// state == NULL: no history branch.  Q_hist != Q: its gradient goes to dQ_hist, else it joins dQ.
int launch_bwd_mfma(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                    const int32_t* idx, int k, const void* dO, const float* lse2, const float* Dv,
                    const int32_t* inv_cnt, const int32_t* inv_list, int32_t* dkv_order, const float* state,
                    const float* cosq, const float* sinq, const void* Q_hist, void* planes, void* dQ, void* dQ_hist,
                    void* dK, void* dV, hipStream_t s) {
  if (n_kv >= (1 << 23) || n_q >= (1 << 23)) { set_error("more than 2^23 tokens"); return HF_ERR_SHAPE; }
  const int BH = c.batch * c.heads;
  const int t_m = (n_q + c.block_q - 1) / c.block_q, t_n = (n_kv + c.block_kv - 1) / c.block_kv;
  const float scale = c.softmax_scale > 0.0f ? c.softmax_scale : 1.0f / sqrtf((float)c.head_dim);
  const float c_scale = scale * 1.4426950408889634f;
  const int kvs = kv_stride_of(c, n_kv);
  const bf16_t* q = static_cast<const bf16_t*>(Q);
  const bf16_t* kk = static_cast<const bf16_t*>(K);
  const bf16_t* v = static_cast<const bf16_t*>(V);
  const bf16_t* g = static_cast<const bf16_t*>(dO);
  const int hist_mode = !state ? 0 : (Q_hist != Q ? 2 : 1);
  BwdHist hist = {};
  if (hist_mode) {
    hipLaunchKernelGGL(state_planes_bwd_kernel, dim3(D / 32, D / 32, BH), dim3(256), 0, s, state,
                       static_cast<bf16_t*>(planes));
    hist.planes = static_cast<const bf16_t*>(planes);
    hist.zvec = state + (size_t)BH * D * D;
    hist.cosq = cosq;
    hist.sinq = sinq;
    hist.q_hist = static_cast<const bf16_t*>(Q_hist);
    hist.dq_hist = static_cast<bf16_t*>(dQ_hist);
    hist.eps = c.eps;
    hist.z_scale = c.z_scale;
    hist.phi_kind = c.phi;
  }
  const long long q_items = (long long)BH * t_m;
  if (q_items > (1ll << 30)) { set_error("too many query blocks"); return HF_ERR_SHAPE; }
  const int q_per_xcd = (int)((q_items + 7) / 8);
  // more than 64 KB of LDS has to be granted per kernel instance, once
#define HF_LAUNCH_DQ3(NWV, HM, RG)                                                                                  \
  do {                                                                                                             \
    static LdsGrant grant;                                                                                         \
    const int rc_grant = grant_lds(grant, reinterpret_cast<const void*>(bwd_dq_mfma_kernel<NWV, HM, RG>), kDqLds,  \
                                   "the dQ kernel");                                                               \
    if (rc_grant != HF_OK) return rc_grant;                                                                        \
    hipLaunchKernelGGL((bwd_dq_mfma_kernel<NWV, HM, RG>), dim3(8 * q_per_xcd), dim3(64 * NWV), kDqLds, s, q, kk, v, \
                       g, idx, k, n_q, n_kv, kvs, c.block_kv, t_m, t_n, q_per_xcd, (int)q_items, c_scale, scale,    \
                       lse2, Dv, hist, static_cast<bf16_t*>(dQ));                                                  \
  } while (0)
#define HF_LAUNCH_DQ(NWV, HM) do { if (c.block_kv % 32) HF_LAUNCH_DQ3(NWV, HM, true); else HF_LAUNCH_DQ3(NWV, HM, false); } while (0)
  if (c.block_q == 64) {
    if (hist_mode == 0) HF_LAUNCH_DQ(2, 0); else if (hist_mode == 1) HF_LAUNCH_DQ(2, 1); else HF_LAUNCH_DQ(2, 2);
  } else {
    if (hist_mode == 0) HF_LAUNCH_DQ(4, 0); else if (hist_mode == 1) HF_LAUNCH_DQ(4, 1); else HF_LAUNCH_DQ(4, 2);
  }
#undef HF_LAUNCH_DQ
#undef HF_LAUNCH_DQ3
  int rc = check_launch("hf_hybrid_attn_bwd(dQ)");
  if (rc != HF_OK) return rc;
  const int slabs = (c.block_kv + 63) / 64;   // 64 keys per workgroup
  const long long kv_items = (long long)BH * t_n * slabs;
  if (kv_items > (1ll << 30)) { set_error("too many KV slabs"); return HF_ERR_SHAPE; }
  const int kv_per_xcd = (int)((kv_items + 7) / 8);
  static LdsGrant dkv_grant;
  const int rc_dkv = grant_lds(dkv_grant, reinterpret_cast<const void*>(bwd_dkv_mfma_kernel), kDkvLds, "the dK/dV kernel");
  if (rc_dkv != HF_OK) return rc_dkv;
  const int32_t* order = nullptr;   // equal lists (dense), or a share too long for the ordering kernel: index order
  if (inv_cnt && dkv_order && kv_per_xcd <= kOrderMax && !(c.flags & HF_FLAG_DKV_INDEX_ORDER)) {
    hipLaunchKernelGGL(dkv_order_kernel, dim3(8), dim3(1024), 0, s, inv_cnt, inv_list, t_m, slabs, kv_per_xcd,
                       (int)kv_items, dkv_order);
    order = dkv_order;
  }
  hipLaunchKernelGGL(bwd_dkv_mfma_kernel, dim3(8 * kv_per_xcd), dim3(128), kDkvLds, s, q, kk, v, g, inv_cnt, inv_list, n_q,
                     n_kv, kvs, c.block_q, c.block_kv, t_m, t_n, slabs, kv_per_xcd, (int)kv_items, order, c_scale, scale,
                     lse2, Dv, static_cast<bf16_t*>(dK), static_cast<bf16_t*>(dV));
  return check_launch("hf_hybrid_attn_bwd(dK, dV)");
}

}  // namespace hf
