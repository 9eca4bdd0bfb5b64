// Eq. 2 on the matrix cores (bf16 inputs, head_dim 128, fp32 state).
//
// Per (batch, head) the update is the contraction  L += A^T B  with A = R(phi(K_ev)) and B = V_ev,
// both stored token-major, while an MFMA operand wants the contraction index (the token)
// contiguous in each lane.  The workgroup therefore transposes on the way into LDS: two
// consecutive tokens of one feature are packed into one dword and stored at
// [feature][token pair], so that an operand fragment (8 tokens of one feature) is one 16-byte
// LDS read.
//
// The kernel is bound by the HBM read of K_ev and V_ev, which at this size (tens of MB) is a
// latency problem.  Two kernels:
//   - absorb_quad_kernel (ReLU, no rotation, caller workspace: the fast path, see there): tiles travel
//     global -> LDS directly, operands by transposing LDS reads, ONE launch that also reduces;
//   - absorb_mfma_kernel (any feature map, rotated keys, or no workspace): register-staged, described above; a
//     workgroup requests ALL the tokens of its run (up to 320) before it touches the first one.  The evicted
//     tokens of one head are cut into slices, one workgroup each; slice partials are combined through the
//     workspace by a small reduction kernel, or, without workspace, with device-scope float atomics straight
//     into the state (the L2 atomic units retire one dword per channel and clock, which costs more than the
//     read itself).
#include <stdlib.h>

#include "hf_common.h"

namespace hf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int D = 128;
constexpr int CH = 64;              // tokens per chunk (one LDS image)
constexpr int NP = CH / 2;          // token pairs per chunk
constexpr int SP = NP + 16;         // LDS row stride in dwords (see pair_col)
constexpr int RUN_CHUNKS = 5;       // chunks requested up front
constexpr int RUN = RUN_CHUNKS * CH;
constexpr int PART = D * D + D;     // floats of one partial: L then z
constexpr int NT = 512;             // threads per workgroup: 8 wavefronts, two per SIMD
constexpr int ITEMS = 16 * NP / NT; // (token pair, feature group) items per thread and chunk
constexpr int TPI = NT / 16;        // token pairs between two items of a thread

// column of token pair `tp` in the row of `feature`: rows are rotated by one 16-byte group per 8
// features.  LDS serves dword stores 32 lanes at a time from 32 banks: a half-wavefront holds 8
// feature groups x 4 adjacent token pairs, which the rotation spreads over all 32; with 48-dword
// rows the 16-byte operand reads are conflict free as well (both measured on the exact patterns
// with SQ_LDS_BANK_CONFLICT), and the 4-pair groups of an operand read stay intact.
__device__ __forceinline__ int pair_col(int feature, int tp) {
  return (tp + (((feature >> 3) & 7) << 2)) & (NP - 1);
}

struct Regs {
  uint4 k[ITEMS][2];  // [item][token of the pair]
  uint4 v[ITEMS][2];
};

typedef short s16x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t relu_pk(uint32_t x) {
  // bf16 ReLU on two packed values: as signed 16-bit integers negative numbers (also -0) are < 0,
  // so a packed integer max with zero clears them (one v_pk_max_i16)
  const s16x2 v = __builtin_bit_cast(s16x2, x);
  const s16x2 zero = {0, 0};
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(v, zero));
}

template <bool kPlain>
__global__ __launch_bounds__(NT, 1) void absorb_mfma_kernel(float* __restrict__ state, float* __restrict__ partials,
                                                             const bf16_t* __restrict__ K,
                                                             const bf16_t* __restrict__ V, int n, int head_stride,
                                                             int tokens_per_slice, const float* __restrict__ cosv,
                                                             const float* __restrict__ sinv, int phi_kind, int BH,
                                                             int slices) {
  __shared__ __attribute__((aligned(16))) uint32_t Kt[D * SP];
  __shared__ __attribute__((aligned(16))) uint32_t Vt[D * SP];
  __shared__ float zs[D];

  int bh, slice;
  if (partials) {  // plain (head, slice) order: every XCD streams the same number of bytes
    bh = blockIdx.x / slices;
    slice = blockIdx.x - bh * slices;
  } else {
    // Consecutive workgroup ids land on consecutive XCDs; all slices of one (batch, head) go to
    // one XCD (head index mod 8), which keeps that head's atomics in a single L2.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    bh = xcd + 8 * (slot / slices);
    slice = slot % slices;
  }
  if (bh >= BH) return;
  const int t0 = slice * tokens_per_slice;
  const int t1 = min(n, t0 + tokens_per_slice);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bf16_t* Kh = K + (size_t)bh * head_stride * D;  // head_stride tokens between heads (= n when packed)
  const bf16_t* Vh = V + (size_t)bh * head_stride * D;
  const int g = (lane & 7) + 8 * (lane >> 5);      // feature group: features 8g .. 8g+7
  const int tp0 = 4 * wave + ((lane >> 3) & 3);    // token pair of item 0; further items are TPI pairs apart

  if (tid < D) zs[tid] = 0.0f;

  auto load = [&](int tb, Regs& r) {
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int tok = tb + 2 * (tp0 + TPI * it);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        if (tok + u < t1) {
          r.k[it][u] = *reinterpret_cast<const uint4*>(Kh + (size_t)(tok + u) * D + 8 * g);
          r.v[it][u] = *reinterpret_cast<const uint4*>(Vh + (size_t)(tok + u) * D + 8 * g);
        } else {
          r.k[it][u] = make_uint4(0, 0, 0, 0);
          r.v[it][u] = make_uint4(0, 0, 0, 0);
        }
      }
    }
  };

  float zacc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) zacc[e] = 0.0f;

  constexpr int TA = 8 / (NT / 64);   // 32x32 tiles per wave along the key features (4x4 tiles in all)
  f32x16 acc[TA][2];
#pragma unroll
  for (int a = 0; a < TA; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

  const int mi0 = TA * (wave >> 1), nj0 = 2 * (wave & 1);  // this wave's TA x 2 grid of 32x32 tiles
  const int h = lane >> 5, l32 = lane & 31;

  // transform one chunk held in registers, pack token pairs, transposing store to LDS
  auto stage = [&](int tb, Regs& cur) {
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
      const int tp = tp0 + TPI * it;
      uint32_t kw[2][4] = {{cur.k[it][0].x, cur.k[it][0].y, cur.k[it][0].z, cur.k[it][0].w},
                           {cur.k[it][1].x, cur.k[it][1].y, cur.k[it][1].z, cur.k[it][1].w}};
      const uint32_t vw[2][4] = {{cur.v[it][0].x, cur.v[it][0].y, cur.v[it][0].z, cur.v[it][0].w},
                                 {cur.v[it][1].x, cur.v[it][1].y, cur.v[it][1].z, cur.v[it][1].w}};
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int tok = tb + 2 * tp + u;
        if (kPlain) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            kw[u][q] = relu_pk(kw[u][q]);
            zacc[2 * q] += __uint_as_float(kw[u][q] << 16);
            zacc[2 * q + 1] += __uint_as_float(kw[u][q] & 0xffff0000u);
          }
        } else if (tok < t1) {
          float4 c4 = make_float4(1.f, 1.f, 1.f, 1.f), s4 = make_float4(0.f, 0.f, 0.f, 0.f);
          if (cosv) {
            c4 = *reinterpret_cast<const float4*>(cosv + (size_t)tok * (D / 2) + 4 * g);
            s4 = *reinterpret_cast<const float4*>(sinv + (size_t)tok * (D / 2) + 4 * g);
          }
          const float cc[4] = {c4.x, c4.y, c4.z, c4.w}, ss[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const float f0 = phi_apply(__uint_as_float(kw[u][q] << 16), phi_kind);
            const float f1 = phi_apply(__uint_as_float(kw[u][q] & 0xffff0000u), phi_kind);
            zacc[2 * q] += f0;
            zacc[2 * q + 1] += f1;
            const float r0 = f0 * cc[q] - f1 * ss[q], r1 = f0 * ss[q] + f1 * cc[q];
            kw[u][q] = (uint32_t)f32_to_bf16(r0) | ((uint32_t)f32_to_bf16(r1) << 16);
          }
        }
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int f = 8 * g + 2 * q;
        const int col = pair_col(f, tp);
        // one byte permute per dword: (token, token + 1) of feature f, then of feature f + 1
        Kt[f * SP + col] = __builtin_amdgcn_perm(kw[1][q], kw[0][q], 0x05040100u);
        Kt[(f + 1) * SP + col] = __builtin_amdgcn_perm(kw[1][q], kw[0][q], 0x07060302u);
        Vt[f * SP + col] = __builtin_amdgcn_perm(vw[1][q], vw[0][q], 0x05040100u);
        Vt[(f + 1) * SP + col] = __builtin_amdgcn_perm(vw[1][q], vw[0][q], 0x07060302u);
      }
    }
  };

  // 4 contraction steps of 16 tokens over the chunk in LDS
  auto contract = [&]() {
#pragma unroll
    for (int ks = 0; ks < CH / 16; ++ks) {
      bf16x8 af[TA], bf[2];
#pragma unroll
      for (int a = 0; a < TA; ++a) {
        const int f = 32 * (mi0 + a) + l32;
        af[a] = *reinterpret_cast<const bf16x8*>(&Kt[f * SP + pair_col(f, 8 * ks + 4 * h)]);
      }
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int f = 32 * (nj0 + b) + l32;
        bf[b] = *reinterpret_cast<const bf16x8*>(&Vt[f * SP + pair_col(f, 8 * ks + 4 * h)]);
      }
#pragma unroll
      for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[b], af[a], acc[a][b], 0, 0, 0);  // L^T tile
    }
  };

  for (int run0 = t0; run0 < t1; run0 += RUN) {
    Regs r[RUN_CHUNKS];
#pragma unroll
    for (int c = 0; c < RUN_CHUNKS; ++c) load(run0 + c * CH, r[c]);  // the whole run is requested before use
#pragma unroll
    for (int c = 0; c < RUN_CHUNKS; ++c) {
      if (run0 + c * CH < t1) {  // uniform
        stage(run0 + c * CH, r[c]);
        __syncthreads();
        contract();
        __syncthreads();
      }
    }
  }

  // ---- hand the partial over
  float* L;
  float* z;
  if (partials) {
    L = partials + ((size_t)bh * slices + slice) * PART;
    z = L + D * D;
  } else {
    L = state + (size_t)bh * D * D;
    z = state + (size_t)BH * D * D + (size_t)bh * D;
  }
  // lanes l, l + 8, l + 16, l + 24 of a half-wavefront hold the same feature group: sum them first
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    zacc[e] += __shfl_xor(zacc[e], 8, kWave);
    zacc[e] += __shfl_xor(zacc[e], 16, kWave);
  }
  if ((lane & 24) == 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) atomicAdd(&zs[8 * g + e], zacc[e]);
  }
  // The tiles were accumulated transposed (V fragment as the A operand): a lane holds, for ONE key
  // feature i, four consecutive value features j per register group, i.e. 16 contiguous bytes of
  // row i of L.  Two straight-line epilogues (a choice per element costs a branch each).
  if (partials) {
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int i = 32 * (mi0 + a) + l32;
          const int j = 32 * (nj0 + b) + 8 * rq + 4 * h;
          *reinterpret_cast<float4*>(L + i * D + j) =
              make_float4(acc[a][b][4 * rq], acc[a][b][4 * rq + 1], acc[a][b][4 * rq + 2], acc[a][b][4 * rq + 3]);
        }
  } else {
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = 32 * (mi0 + a) + l32;
          const int j = 32 * (nj0 + b) + 8 * (r >> 2) + 4 * h + (r & 3);
          atomicAdd(L + i * D + j, acc[a][b][r]);
        }
  }
  __syncthreads();
  if (tid < D) {
    if (partials) z[tid] = zs[tid];
    else atomicAdd(z + tid, zs[tid]);
  }
}

// ---- the plain case (ReLU, no rotation, workspace given): ONE launch, partials of a few fat slices ---------------
// Work item = (head, token slice, quadrant of L).  The evicted tokens of a head are cut into a FEW slices (about
// 256 / (4 heads) of them), and the four workgroups of a (head, slice) share its tokens: each accumulates one
// 64 x 64 quadrant L[64a .. , 64b ..] over the slice, reading the matching halves of the K and V rows.  The four
// run on the same XCD, so the slice crosses HBM once and is served to the other three from that XCD's L2.  Few
// slices keep the partials small (slices x state size, 3-4 MB at the 832x480 shape, where one workgroup per 288
// tokens wrote 13 MB); many quadrant workgroups keep every compute unit streaming.
//
// Tiles of 32 tokens x 64 features (128-byte rows) travel global -> LDS directly (buffer loads with the LDS bit,
// 16 bytes per lane, 1 KB = 8 token rows per instruction) through a ring of kRing tiles per tensor that is kept
// full: tile c + kRing - 1 is requested as soon as tile c - 1 is consumed.  Both MFMA operands want tokens as
// the contraction index, i.e. features as rows, and come from transposing LDS reads (ds_read_b64_tr_b16) of the
// row-major tiles; 16-byte unit u of row r sits at u ^ (4 (r >> 1 & 1)), which spreads the 4 rows x 64 bytes a
// half-wavefront reads over all 64 banks.  Tokens past the slice's end arrive as zeros (descriptor range).
//
// The slices of a quadrant meet in the workspace: every workgroup stores its 64 x 64 partial (coalesced, through
// LDS), then takes a ticket from the quadrant's arrival counter; the workgroup that draws the last ticket adds
// the partials IN SLICE ORDER to the state (so the sum does not depend on who came last), and writes the
// quadrant of the readout's two transposed bf16 planes when asked.  No second launch, nothing waits for anyone.
// The counter needs no initialisation: its upper 48 bits carry a tag that the host draws per call, and a counter
// whose tag is not this call's counts from zero (the last workgroup also leaves the count at zero, so that a
// launch replayed from a captured graph, tag and all, finds it ready).
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
constexpr int QT = 32;                  // tokens per tile
constexpr int QROW = 128;               // bytes per token row of a tile (64 features)
constexpr int QTILE = QT * QROW;        // bytes of one tile of one tensor
constexpr int QSLOT = 4 * QTILE;        // a ring slot: a pair of tiles (even, odd) of both tensors, 64 tokens
constexpr int QNT = 512;                // threads per workgroup: two groups of four wavefronts (even / odd tiles),
                                        // one 32 x 32 tile of the quadrant per wavefront
constexpr int LSTR = 68;                // floats per row of the staged 64 x 64 block (16-byte aligned rows)
constexpr int QUADS = 4;

__device__ __forceinline__ bf16x8 tr_frag64(const char* tile, uint32_t base, int ft, int t2) {
  const char* p0 = tile + (base ^ (64u * ft)) + 2048 * t2;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0 + 1024));
  const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, both);
}

template <int kRing>
__global__ __launch_bounds__(QNT) void absorb_quad_kernel(float* __restrict__ state, bf16_t* __restrict__ planes,
                                                          unsigned long long* __restrict__ counters,
                                                          float* __restrict__ partials, const bf16_t* __restrict__ K,
                                                          const bf16_t* __restrict__ V, int n, int head_stride,
                                                          int tokens_per_slice, int slices, int BH,
                                                          unsigned long long tag) {
  extern __shared__ __attribute__((aligned(16))) char smem[];   // kRing x 2 x (K tile, V tile); later the staged block
  static_assert(kRing * QSLOT >= (64 * LSTR + 64) * 4, "the staged block must fit in the ring");
  static_assert(2 * (kRing - 2) <= 63, "vmcnt holds six bits");
  __shared__ int s_last;
  // consecutive workgroup ids go to consecutive XCDs: the four quadrants of a (head, slice) share one
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int item = xcd + 8 * (slot >> 2), quad = slot & 3;
  if (item >= BH * slices) return;
  const int bh = item / slices, slice = item - bh * slices;
  const int qa = quad >> 1, qb = quad & 1;   // key-feature half, value-feature half
  const int t0 = slice * tokens_per_slice;
  const int t1 = min(n, t0 + tokens_per_slice);
  const int npairs = (t1 - t0 + 2 * QT - 1) / (2 * QT);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // wavefronts 0-3 take the even tiles, 4-7 the odd ones; within a group one 32 x 32 tile of the quadrant each
  const int grp = wave >> 2, wa = (wave >> 1) & 1, wb = wave & 1;
  const int l32 = lane & 31, h = lane >> 5;

  // transfer: a wavefront moves token rows 8 (w & 3) .. + 7 of its own group's tile, lane l the physical unit
  // l & 7 of row l >> 3
  const int row = 8 * (wave & 3) + (lane >> 3);
  const int unit = (lane & 7) ^ (4 * ((row >> 1) & 1));
  const int k_off = row * (D * 2) + 128 * qa + 16 * unit;
  const int v_off = row * (D * 2) + 128 * qb + 16 * unit;
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem + grp * (2 * QTILE) + 1024 * (wave & 3);
  const uint64_t kbase = reinterpret_cast<uint64_t>(K + (size_t)bh * head_stride * D);
  const uint64_t vbase = reinterpret_cast<uint64_t>(V + (size_t)bh * head_stride * D);
  auto fetch = [&](int c) {   // pair c of the slice into slot c mod kRing; rows past t1 (and whole tiles) as zeros
    const int first = t0 + (2 * c + grp) * QT;
    const int left = (t1 - first) * (D * 2);
    const uint64_t ka = kbase + (uint64_t)(left > 0 ? first : 0) * (D * 2);
    const uint64_t va = vbase + (uint64_t)(left > 0 ? first : 0) * (D * 2);
    const i32x4 kd = {(int)(uint32_t)ka, (int)(uint32_t)(ka >> 32), left > 0 ? left : 0, 0x00020000};
    const i32x4 vd = {(int)(uint32_t)va, (int)(uint32_t)(va >> 32), left > 0 ? left : 0, 0x00020000};
    const uint32_t dst = lds0 + (uint32_t)(c % kRing) * QSLOT;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(dst), "v"(k_off), "s"(kd) : "memory", "m0");
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(dst + QTILE), "v"(v_off), "s"(vd) : "memory", "m0");
  };
  // operand address of a lane inside a tile: the 16-lane group g reads 4 token rows x 16 features, lane j of it
  // supplies the 8-byte chunk (row 4 h + j / 4, features 4 (j % 4) .. + 4) and receives feature 16 (g & 1) + j
  uint32_t tb;
  {
    const int j = lane & 15, g = lane >> 4;
    const int key_l = 4 * h + (j >> 2);
    const int low2 = 2 * (g & 1) + ((j & 3) >> 1);
    tb = key_l * QROW + 64 * ((key_l >> 1) & 1) + 16 * low2 + 8 * (j & 1);   // ^ 64 ft, + 1024 x + 2048 t2
  }

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
  float zacc = 0.0f;   // sum over this lane's tokens of phi(k) for key feature 64 qa + 32 wa + l32
  const s16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  bf16x8 kf[2], vf[2];   // fragments of the tile read in the previous trip (zeros before the first)
#pragma unroll
  for (int t2 = 0; t2 < 2; ++t2) kf[t2] = vf[t2] = __builtin_bit_cast(bf16x8, zero8);
  auto contract = [&]() {
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      // ReLU of bf16 values as a packed signed-integer max with zero
      const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_elementwise_max(__builtin_bit_cast(s16x8, kf[t2]), zero8));
#pragma unroll
      for (int e = 0; e < 8; ++e) zacc += static_cast<float>(a[e]);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t2], a, acc, 0, 0, 0);   // L^T tile
    }
  };

  // The quadrant's arrival counter has to carry this call's tag before anybody's ticket is drawn.  One lane looks
  // at it now (the load is this wavefront's oldest request, so it has returned once at most the transfers issued
  // behind it are in flight) and claims it if the tag is another call's; whether this exchange or another
  // workgroup's wins does not matter.  Two round trips to memory, hidden behind the first tiles' latency.
  unsigned long long* const ctr = counters + (size_t)bh * QUADS + quad;
  const bool claimer = tid == QNT - 64;
  unsigned long long seen = 0;
  if (claimer) asm volatile("global_load_dwordx2 %0, %1, off sc1" : "=&v"(seen) : "v"(ctr) : "memory");
  // every wavefront issues the same two requests per pair (tiles past the end have an empty descriptor), so the
  // number in flight when a tile is needed is a constant
#pragma unroll
  for (int c = 0; c < kRing - 1; ++c) fetch(c);
  if (claimer) {
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(seen) : "n"(2 * (kRing - 1)) : "memory");
    if ((seen >> 16) != tag)
      (void)__hip_atomic_compare_exchange_strong(ctr, &seen, tag << 16, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
  }
  for (int c = 0; c < npairs; ++c) {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * (kRing - 2)) : "memory");   // this wavefront's rows of pair c
    __syncthreads();              // ... and everybody's; everybody has read pair c - 1
    fetch(c + kRing - 1);         // into the slot of pair c - 1
    const char* tK = smem + (c % kRing) * QSLOT + grp * (2 * QTILE);
    bf16x8 nk[2], nv[2];
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      nk[t2] = tr_frag64(tK, tb, wa, t2);
      nv[t2] = tr_frag64(tK + QTILE, tb, wb, t2);
    }
    contract();   // the previous trip's tile, while this trip's reads are on their way
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) { kf[t2] = nk[t2]; vf[t2] = nv[t2]; }
  }
  contract();
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // nothing may land in LDS once the ring's space is reused
  __syncthreads();

  // ---- the quadrant's partial: both groups' tiles summed in LDS (a lane holds 4 x 4 consecutive value features
  // of ONE key feature), then row pieces of 256 bytes into this slice's partial, which has the state's layout
  float* tile = reinterpret_cast<float*>(smem);   // [64 key features][LSTR]
  float* zs = tile + 64 * LSTR;                   // [64]
  zacc += __shfl_xor(zacc, 32, kWave);   // the two halves of a tile's tokens
  float* trow = tile + (32 * wa + l32) * LSTR + 32 * wb + 4 * h;
  if (grp == 0) {
#pragma unroll
    for (int rq = 0; rq < 4; ++rq)
      *reinterpret_cast<float4*>(trow + 8 * rq) = make_float4(acc[4 * rq], acc[4 * rq + 1], acc[4 * rq + 2], acc[4 * rq + 3]);
    if (wb == 0 && h == 0) zs[32 * wa + l32] = zacc;
  }
  __syncthreads();
  if (grp == 1) {
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      float4 t = *reinterpret_cast<const float4*>(trow + 8 * rq);
      t.x += acc[4 * rq]; t.y += acc[4 * rq + 1]; t.z += acc[4 * rq + 2]; t.w += acc[4 * rq + 3];
      *reinterpret_cast<float4*>(trow + 8 * rq) = t;
    }
    if (wb == 0 && h == 0) zs[32 * wa + l32] += zacc;
  }
  __syncthreads();
  // Partials are exchanged between workgroups on different XCDs, whose L2 caches do not see each other's lines:
  // they are written and read with device-scope accesses (they go through to memory; a device-scope FENCE would
  // instead write back and invalidate the whole L2 of the XCD, per workgroup: measured 45-120 us per launch).
  float* part = partials + ((size_t)bh * slices + slice) * PART;
  const int er = tid >> 6, ec = tid & 63;   // a wavefront moves one 256-byte row piece; rows er + 8 p
#pragma unroll
  for (int p = 0; p < 8; ++p)
    __hip_atomic_store(part + (64 * qa + er + 8 * p) * D + 64 * qb + ec, tile[(er + 8 * p) * LSTR + ec],
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (qb == 0 && tid < 64)
    __hip_atomic_store(part + D * D + 64 * qa + tid, zs[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  // ---- arrival: every store above has been acknowledged before the workgroup draws its ticket
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0) {   // (the claim above has long been carried out: the wait behind the loop covers it)
    const unsigned long long before = __hip_atomic_fetch_add(ctr, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (int)(before & 0xffffull) + 1 == slices;
    // the last one leaves the count at zero under this call's tag: a captured launch replays with the same tag
    if (s_last) __hip_atomic_store(ctr, tag << 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (!s_last) return;

  // ---- the last workgroup of the quadrant: state += partials in slice order; planes of the updated quadrant
  // (these loads come from memory, not from L2: all eight of a thread for up to four slices are in flight at once)
  const float* p0 = partials + (size_t)bh * slices * PART;
  float* Lq = state + (size_t)bh * D * D;
  // the slices are summed first and meet the state in ONE addition per call: over a long stream the state is much
  // larger than a chunk's contribution, and every addition at its magnitude costs a rounding of its size
  float sum[8], old[8];
  const size_t at0 = (size_t)(64 * qa + er) * D + 64 * qb + ec;   // + 8 p rows
#pragma unroll
  for (int p = 0; p < 8; ++p) { old[p] = Lq[at0 + (size_t)8 * p * D]; sum[p] = 0.0f; }
  const bool zrow = qb == 0 && tid < 64;
  float* zq = state + (size_t)BH * D * D + (size_t)bh * D + 64 * qa + ec;
  const float zold = zrow ? *zq : 0.0f;
  float zsum = 0.0f;
  constexpr int kBatch = 6;   // slices whose loads are in flight together (one round trip for the usual 4-6 slices)
  for (int s0 = 0; s0 < slices; s0 += kBatch) {
    float v[kBatch][8], zv[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const float* ps = p0 + (size_t)min(s0 + u, slices - 1) * PART;   // (past the last slice: re-read, not added)
#pragma unroll
      for (int p = 0; p < 8; ++p)
        v[u][p] = __hip_atomic_load(ps + at0 + (size_t)8 * p * D, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      zv[u] = zrow ? __hip_atomic_load(ps + D * D + 64 * qa + ec, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u)
      if (s0 + u < slices) {   // uniform; slice order
#pragma unroll
        for (int p = 0; p < 8; ++p) sum[p] += v[u][p];
        zsum += zv[u];
      }
  }
#pragma unroll
  for (int p = 0; p < 8; ++p) sum[p] += old[p];
  zsum += zold;
#pragma unroll
  for (int p = 0; p < 8; ++p) tile[(er + 8 * p) * LSTR + ec] = sum[p];
  __syncthreads();   // (the planes' transposed reads; in front of the state's stores so that all stores leave together)
#pragma unroll
  for (int p = 0; p < 8; ++p) Lq[at0 + (size_t)8 * p * D] = sum[p];
  if (zrow) *zq = zsum;
  if (planes != nullptr) {
    // planes[bh][plane][j][i]: thread (j, eighth) writes 8 consecutive key features i of value feature j
    const int j = tid >> 3, i0 = 8 * (tid & 7);
    uint32_t hw[4], lw[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float v0 = tile[(i0 + 2 * q) * LSTR + j], v1 = tile[(i0 + 2 * q + 1) * LSTR + j];
      const bf16_t h0 = f32_to_bf16(v0), h1 = f32_to_bf16(v1);
      hw[q] = (uint32_t)h0 | ((uint32_t)h1 << 16);
      lw[q] = (uint32_t)f32_to_bf16(v0 - bf16_to_f32(h0)) | ((uint32_t)f32_to_bf16(v1 - bf16_to_f32(h1)) << 16);
    }
    bf16_t* hi = planes + (size_t)bh * 2 * D * D + (size_t)(64 * qb + j) * D + 64 * qa + i0;
    *reinterpret_cast<uint4*>(hi) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
    *reinterpret_cast<uint4*>(hi + D * D) = make_uint4(lw[0], lw[1], lw[2], lw[3]);
  }
}

// state += sum over slices of the partials; one thread per 4 consecutive floats of a partial.
// planes != NULL: the updated L also leaves as the two transposed bf16 planes (high part and remainder,
// planes[bh][plane][j][i]) that the attention kernel's history epilogue multiplies with: the conversion rides
// in the kernel that produces the state instead of running as a launch of its own before every attention call.
__global__ __launch_bounds__(256) void absorb_reduce_kernel(float* __restrict__ state,
                                                            const float* __restrict__ partials, int slices,
                                                            int BH, bf16_t* __restrict__ planes) {
  __shared__ float tile[8][D + 1];   // the block's 8 rows of L, for the transposed write
  const int e4 = blockIdx.x * 256 + threadIdx.x;  // float4 index inside a partial
  const int bh = blockIdx.y;
  if (e4 >= PART / 4) return;   // (only in the block of z, which takes no part in the planes)
  const float4* p = reinterpret_cast<const float4*>(partials + (size_t)bh * slices * PART) + e4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  int sl = 0;
  for (; sl + 3 < slices; sl += 4) {  // four independent loads in flight
    const float4 a = p[(size_t)sl * (PART / 4)], b = p[(size_t)(sl + 1) * (PART / 4)];
    const float4 c = p[(size_t)(sl + 2) * (PART / 4)], d = p[(size_t)(sl + 3) * (PART / 4)];
    s.x += (a.x + b.x) + (c.x + d.x);
    s.y += (a.y + b.y) + (c.y + d.y);
    s.z += (a.z + b.z) + (c.z + d.z);
    s.w += (a.w + b.w) + (c.w + d.w);
  }
  for (; sl < slices; ++sl) {
    const float4 a = p[(size_t)sl * (PART / 4)];
    s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
  }
  const int e = 4 * e4;
  float* dst = e < D * D ? state + (size_t)bh * D * D + e : state + (size_t)BH * D * D + (size_t)bh * D + (e - D * D);
  float4 cur = *reinterpret_cast<float4*>(dst);
  cur.x += s.x; cur.y += s.y; cur.z += s.z; cur.w += s.w;
  *reinterpret_cast<float4*>(dst) = cur;
  if (planes == nullptr || e >= D * D) return;   // uniform over a block: a block holds 8 whole rows of L, or z
  {
    const int r = threadIdx.x >> 5, c0 = 4 * (threadIdx.x & 31);
    tile[r][c0] = cur.x; tile[r][c0 + 1] = cur.y; tile[r][c0 + 2] = cur.z; tile[r][c0 + 3] = cur.w;
  }
  __syncthreads();
  const int j = threadIdx.x & (D - 1), half = threadIdx.x >> 7;   // column j, rows 4 half .. + 4 of the block
  const int i0 = 8 * blockIdx.x + 4 * half;
  uint32_t hw[2], lw[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const float v0 = tile[4 * half + 2 * q][j], v1 = tile[4 * half + 2 * q + 1][j];
    const bf16_t h0 = f32_to_bf16(v0), h1 = f32_to_bf16(v1);
    hw[q] = (uint32_t)h0 | ((uint32_t)h1 << 16);
    lw[q] = (uint32_t)f32_to_bf16(v0 - bf16_to_f32(h0)) | ((uint32_t)f32_to_bf16(v1 - bf16_to_f32(h1)) << 16);
  }
  bf16_t* hi = planes + (size_t)bh * 2 * D * D + (size_t)j * D + i0;
  *reinterpret_cast<uint2*>(hi) = make_uint2(hw[0], hw[1]);
  *reinterpret_cast<uint2*>(hi + D * D) = make_uint2(lw[0], lw[1]);
}

// slice length (a multiple of the 64-token chunk) and slice count for n tokens: the register-staged kernel
void slice_plan(int BH, int n, bool with_workspace, int& per, int& slices) {
  if (with_workspace) {
    // one run (320 tokens) per workgroup until there are ~4 workgroups per compute unit, then longer slices
    const int max_slices = (1024 + BH - 1) / BH;
    per = RUN;
    if ((n + per - 1) / per > max_slices) per = ((n + max_slices - 1) / max_slices + RUN - 1) / RUN * RUN;
  } else {
    // atomics: fewer, longer slices (the atomic traffic is slices x state size)
    const int max_slices = (160 + BH - 1) / BH;
    per = (((n + max_slices - 1) / max_slices) + CH - 1) / CH * CH;
    if (per < 2 * CH) per = 2 * CH;
  }
  slices = (n + per - 1) / per;
}

// the quadrant kernel: about one workgroup per compute unit (4 quadrants x BH heads x slices ~ 256), slices of whole tiles
struct QuadPlan {
  int per, slices;
  size_t counters_bytes, total_bytes;
};
QuadPlan quad_plan(int BH, int n, int want_slices) {
  const int tiles = (n + 2 * QT - 1) / (2 * QT);   // pairs of tiles
  int sl = want_slices > 0 ? want_slices : (256 + 2 * BH) / (QUADS * BH);
  if (sl < 1) sl = 1;
  if (sl > tiles) sl = tiles;
  if (sl > 4096) sl = 4096;   // the arrival counter holds 16 bits
  QuadPlan p;
  p.per = (tiles + sl - 1) / sl * (2 * QT);
  p.slices = (n + p.per - 1) / p.per;
  p.counters_bytes = ((size_t)BH * QUADS * sizeof(unsigned long long) + 255) & ~(size_t)255;
  p.total_bytes = p.counters_bytes + (size_t)BH * p.slices * PART * sizeof(float);
  return p;
}

}  // namespace

size_t absorb_mfma_workspace_bytes(const hf_config& c, int n) {
  int per, slices;   // whichever kernel runs: the larger of the two plans
  slice_plan(c.batch * c.heads, n, true, per, slices);
  const size_t staged = (size_t)c.batch * c.heads * slices * PART * sizeof(float);
  const size_t quad = quad_plan(c.batch * c.heads, n, 0).total_bytes;
  return staged > quad ? staged : quad;
}

// ReLU without rotation, workspace given: one launch.  want_slices / ring: 0 = the plan's choice (other values:
// tuning runs of a development harness)
int launch_absorb_quad(const hf_config& c, float* state, const void* K, const void* V, int n, int head_stride,
                       void* workspace, hipStream_t s, void* planes_out, int want_slices, int ring) {
  const int BH = c.batch * c.heads;
  const QuadPlan p = quad_plan(BH, n, want_slices);
  const int items = BH * p.slices;
  const dim3 grid(8 * QUADS * ((items + 7) / 8));
  // four slots of 64 tokens (64 KB of LDS, three in flight per workgroup) measured as fast as eight and leave
  // room for a second workgroup per compute unit
  const bool deep = ring >= 8;
  unsigned long long* counters = static_cast<unsigned long long*>(workspace);
  float* partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + p.counters_bytes);
  const unsigned long long tag = next_call_tag();
#define HF_LAUNCH_QUAD(RING)                                                                                       \
  do {                                                                                                             \
    static LdsGrant grant;                                                                                         \
    constexpr int lds = RING * QSLOT;                                                                              \
    const int rc = grant_lds(grant, reinterpret_cast<const void*>(absorb_quad_kernel<RING>), lds, "the absorb kernel"); \
    if (rc != HF_OK) return rc;                                                                                    \
    hipLaunchKernelGGL((absorb_quad_kernel<RING>), grid, dim3(QNT), lds, s, state, static_cast<bf16_t*>(planes_out), \
                       counters, partials, static_cast<const bf16_t*>(K), static_cast<const bf16_t*>(V), n,        \
                       head_stride, p.per, p.slices, BH, tag);                                                              \
  } while (0)
  if (deep) HF_LAUNCH_QUAD(8); else HF_LAUNCH_QUAD(4);
#undef HF_LAUNCH_QUAD
  return check_launch("hf_absorb_evicted");
}

int launch_absorb_mfma(const hf_config& c, float* state, const void* K, const void* V, int n, int head_stride,
                       const float* cosv, const float* sinv, void* workspace, size_t workspace_bytes,
                       hipStream_t s, void* planes_out) {
  const int BH = c.batch * c.heads;
  bf16_t* planes = static_cast<bf16_t*>(planes_out);   // NULL: the state alone
  const bool use_ws = workspace != nullptr && workspace_bytes >= absorb_mfma_workspace_bytes(c, n);
  const bool plain = (c.phi == HF_PHI_RELU) && cosv == nullptr;
  if (plain && use_ws) return launch_absorb_quad(c, state, K, V, n, head_stride, workspace, s, planes_out, 0, 0);
  int per, slices;
  slice_plan(BH, n, use_ws, per, slices);
  float* partials = use_ws ? static_cast<float*>(workspace) : nullptr;
  const bf16_t* Kp = static_cast<const bf16_t*>(K);
  const bf16_t* Vp = static_cast<const bf16_t*>(V);
  const int heads_per_xcd = (BH + 7) / 8;
  const dim3 grid(use_ws ? BH * slices : 8 * heads_per_xcd * slices);
  if (plain) {
    hipLaunchKernelGGL((absorb_mfma_kernel<true>), grid, dim3(NT), 0, s, state, partials, Kp, Vp, n, head_stride, per, cosv,
                       sinv, c.phi, BH, slices);
  } else {
    hipLaunchKernelGGL((absorb_mfma_kernel<false>), grid, dim3(NT), 0, s, state, partials, Kp, Vp, n, head_stride, per, cosv,
                       sinv, c.phi, BH, slices);
  }
  const int rc = check_launch("hf_absorb_evicted");
  if (rc != HF_OK) return rc;
  if (!use_ws) return planes ? launch_state_planes(c, state, planes, s) : HF_OK;   // (atomics: no reduce kernel)
  hipLaunchKernelGGL(absorb_reduce_kernel, dim3((PART / 4 + 255) / 256, BH), dim3(256), 0, s, state, partials,
                     slices, BH, planes);
  return check_launch("hf_absorb_evicted(reduce)");
}

}  // namespace hf
