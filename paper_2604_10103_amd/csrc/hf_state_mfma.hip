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
// latency problem: a workgroup requests ALL the tokens of its run (up to 320) before it touches
// the first one, so that a whole run is in flight per compute unit.  The evicted tokens of one
// head are cut into slices, one workgroup each.  Slice partials are combined either
//   - through a caller workspace: plain coalesced stores of the d x d + d partial, then a small
//     reduction kernel adds the slices to the state (the fast path), or
//   - with device-scope float atomics straight into the state (no workspace; the L2 atomic units
//     retire one dword per channel and clock, which costs more than the read itself).
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

// ---- the same update with tiles streamed global -> LDS directly (plain case: ReLU, no rotation, partials) ----
// A workgroup requests a whole run of 9 tiles of 32 tokens (K and V, 144 KB: one workgroup per CU) before it
// touches the first: buffer loads with the LDS bit, 16 bytes per lane, no staging registers, no LDS stores;
// tokens past the slice's end arrive as zeros (descriptor range), which ReLU and the products leave at zero.
// Tiles are row-major with swizzled 16-byte units; both MFMA operands want tokens as the contraction index,
// i.e. features as rows, and come from gfx950's transposing LDS reads (ds_read_b64_tr_b16: a 16-lane group
// fetches 4 token rows x 16 features, every lane receives the four tokens of its own feature).
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
constexpr int TT = 32;               // tokens per tile
constexpr int RTILE = TT * D * 2;    // bytes of one tile of one tensor
constexpr int RUN_TILES = 9;         // tiles requested up front
constexpr int DMA_LDS = RUN_TILES * 2 * RTILE;

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }   // see hf_bwd_mfma.hip

__device__ __forceinline__ bf16x8 tr_frag(const char* tile, uint32_t base, int ft, int t2) {
  const char* p0 = tile + (base ^ (64u * ft)) + 4096 * t2;
  const char* p1 = tile + (base ^ (64u * ft) ^ 32u) + 4096 * t2 + 2048;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p1));
  const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, both);
}

__global__ __launch_bounds__(NT, 1) void absorb_dma_kernel(float* __restrict__ partials, const bf16_t* __restrict__ K,
                                                           const bf16_t* __restrict__ V, int n, int head_stride,
                                                           int tokens_per_slice, int slices) {
  extern __shared__ __attribute__((aligned(16))) char smem[];   // RUN_TILES x (K tile, V tile)
  const int bh = blockIdx.x / slices, slice = blockIdx.x - bh * slices;
  const int t0 = slice * tokens_per_slice;
  const int t1 = min(n, t0 + tokens_per_slice);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, h = lane >> 5;

  // transfer: wavefront w moves token rows 4 w .. 4 w + 3 of every tile (1 KB per instruction)
  const int row = 4 * wave + (lane >> 4);
  const int lane_off = row * (D * 2) + (((lane & 15) ^ swz(row)) * 16);
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem + 4 * wave * (D * 2);
  auto fetch = [&](const bf16_t* base_ptr, uint32_t dst, int first) {   // rows [first, first + 32), zeros from t1 on
    const uint64_t a = reinterpret_cast<uint64_t>(base_ptr + (size_t)bh * head_stride * D) + (uint64_t)first * (D * 2);
    const int left = (t1 - first) * (D * 2);
    const i32x4 desc = {(int)(uint32_t)a, (int)(uint32_t)(a >> 32), left > 0 ? left : 0, 0x00020000};
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(dst), "v"(lane_off), "s"(desc) : "memory", "m0");
  };
  // operand addresses of a lane inside a tile (see tr_frag)
  uint32_t tb;
  {
    const int j = lane & 15, g = lane >> 4;
    const int key_l = 4 * h + (j >> 2);
    const int c = (4 * (key_l & 3)) | ((2 * (g & 1) + ((j & 3) >> 1)) ^ h);
    tb = key_l * (D * 2) + 16 * c + 8 * (j & 1);
  }

  const int mi0 = wave >> 1, nj0 = 2 * (wave & 1);   // this wavefront's key-feature tile and its two value-feature tiles
  f32x16 acc[2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[b][r] = 0.0f;
  float zacc = 0.0f;   // sum over tokens of phi(k) for key feature 32 mi0 + l32 (this lane's half of the tokens)

  typedef short s16x8v __attribute__((ext_vector_type(8)));
  const s16x8v zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  auto consume = [&](const int c) {
    const char* tK = smem + c * 2 * RTILE;
    const char* tV = tK + RTILE;
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2) {
      // ReLU of bf16 values as a packed signed-integer max with zero
      const bf16x8 af = __builtin_bit_cast(
          bf16x8, __builtin_elementwise_max(__builtin_bit_cast(s16x8v, tr_frag(tK, tb, mi0, t2)), zero8));
#pragma unroll
      for (int e = 0; e < 8; ++e) zacc += static_cast<float>(af[e]);
#pragma unroll
      for (int b = 0; b < 2; ++b)
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(tV, tb, nj0 + b, t2), af, acc[b], 0, 0, 0);  // L^T tile
    }
  };

  for (int run0 = t0; run0 < t1; run0 += RUN_TILES * TT) {
    if (run0 > t0) __syncthreads();   // the previous run is consumed
    // every wavefront issues the same 2 x RUN_TILES requests (tiles past the end have an empty descriptor), so
    // that the number still in flight when tile c is needed is a constant
#pragma unroll
    for (int c = 0; c < RUN_TILES; ++c) {
      fetch(K, lds0 + c * 2 * RTILE, run0 + c * TT);
      fetch(V, lds0 + c * 2 * RTILE + RTILE, run0 + c * TT);
    }
#pragma unroll
    for (int c = 0; c < RUN_TILES; ++c) {
      asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * (RUN_TILES - 1 - c)) : "memory");
      __syncthreads();   // every wavefront's rows of tile c have landed
      if (run0 + c * TT < t1) consume(c);   // uniform
    }
  }

  // ---- hand the partial over: plain coalesced stores (16 contiguous bytes of a row of L per register group)
  float* L = partials + ((size_t)bh * slices + slice) * PART;
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int i = 32 * mi0 + l32;
      const int j = 32 * (nj0 + b) + 8 * rq + 4 * h;
      *reinterpret_cast<float4*>(L + i * D + j) =
          make_float4(acc[b][4 * rq], acc[b][4 * rq + 1], acc[b][4 * rq + 2], acc[b][4 * rq + 3]);
    }
  zacc += __shfl_xor(zacc, 32, kWave);   // the two halves of the tokens
  if ((wave & 1) == 0 && h == 0) L[D * D + 32 * mi0 + l32] = zacc;   // one of the two wavefronts of a key tile
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

// slice length (a multiple of the 64-token chunk) and slice count for n tokens
// dma: the plan of absorb_dma_kernel, whose run is RUN_TILES tiles of 32 tokens
void slice_plan(int BH, int n, bool with_workspace, bool dma, int& per, int& slices) {
  if (with_workspace && dma) {
    // one run (288 tokens) per workgroup, one workgroup per CU; longer slices only for very long inputs
    const int run = RUN_TILES * TT;
    const int max_slices = (1024 + BH - 1) / BH;
    per = run;
    if ((n + per - 1) / per > max_slices) per = ((n + max_slices - 1) / max_slices + run - 1) / run * run;
  } else if (with_workspace) {
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

}  // namespace

size_t absorb_mfma_workspace_bytes(const hf_config& c, int n) {
  int per, slices, per2, slices2;   // whichever kernel runs: the larger of the two plans
  slice_plan(c.batch * c.heads, n, true, false, per, slices);
  slice_plan(c.batch * c.heads, n, true, true, per2, slices2);
  return (size_t)c.batch * c.heads * (slices > slices2 ? slices : slices2) * PART * sizeof(float);
}

int launch_absorb_mfma(const hf_config& c, float* state, const void* K, const void* V, int n, int head_stride,
                       const float* cosv, const float* sinv, void* workspace, size_t workspace_bytes,
                       hipStream_t s, void* planes_out) {
  const int BH = c.batch * c.heads;
  bf16_t* planes = static_cast<bf16_t*>(planes_out);   // NULL: the state alone
  const bool use_ws = workspace != nullptr && workspace_bytes >= absorb_mfma_workspace_bytes(c, n);
  const bool plain = (c.phi == HF_PHI_RELU) && cosv == nullptr;
  const bool dma = plain && use_ws;
  int per, slices;
  slice_plan(BH, n, use_ws, dma, per, slices);
  float* partials = use_ws ? static_cast<float*>(workspace) : nullptr;
  const bf16_t* Kp = static_cast<const bf16_t*>(K);
  const bf16_t* Vp = static_cast<const bf16_t*>(V);
  if (dma) {
    static LdsGrant grant;
    const int rc_grant = grant_lds(grant, reinterpret_cast<const void*>(absorb_dma_kernel), DMA_LDS, "the absorb kernel");
    if (rc_grant != HF_OK) return rc_grant;
    hipLaunchKernelGGL(absorb_dma_kernel, dim3(BH * slices), dim3(NT), DMA_LDS, s, partials, Kp, Vp, n, head_stride, per,
                       slices);
    const int rc2 = check_launch("hf_absorb_evicted");
    if (rc2 != HF_OK) return rc2;
    hipLaunchKernelGGL(absorb_reduce_kernel, dim3((PART / 4 + 255) / 256, BH), dim3(256), 0, s, state, partials,
                       slices, BH, planes);
    return check_launch("hf_absorb_evicted(reduce)");
  }
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
