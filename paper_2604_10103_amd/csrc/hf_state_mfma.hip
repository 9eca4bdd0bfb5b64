// Eq. 2 on the matrix cores (bf16 inputs, head_dim 128, fp32 state).
//
// Per (batch, head) the update is the contraction  L += A^T B  with A = R(phi(K_ev)) and B = V_ev,
// both stored token-major, while an MFMA operand wants the contraction index (the token)
// contiguous in each lane.  The workgroup therefore transposes on the way into LDS: two
// consecutive tokens of one feature are packed into one dword and stored at
// [feature][token pair], so that an operand fragment (8 tokens of one feature) is one 16-byte
// LDS read.  The kernel is bound by the HBM read of K_ev and V_ev; the next 64-token chunk is
// fetched into registers while the matrix cores work on the current one.
#include <stdlib.h>

#include "hf_common.h"

namespace hf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int D = 128;
constexpr int CH = 64;        // tokens per chunk
constexpr int NP = CH / 2;    // token pairs per chunk
constexpr int SP = NP + 4;    // LDS row stride in dwords: keeps 16-byte operand reads conflict free

// column of token pair `tp` in the row of `feature`: rows are rotated by one 16-byte group per
// 16 features, which spreads the transposing dword stores of a wave (16 feature groups x 4
// token pairs) over all 64 banks and keeps the 4-pair groups of an operand read intact
__device__ __forceinline__ int pair_col(int feature, int tp) {
  return (tp + (((feature >> 4) & 7) << 2)) & (NP - 1);
}

struct Regs {
  uint4 k[2][2];  // [item][token of the pair]
  uint4 v[2][2];
};

__device__ __forceinline__ uint32_t relu_pk(uint32_t x) {
  // bf16 ReLU on two packed values: a set sign bit (also -0) gives +0
  const uint32_t lo = (x & 0x8000u) ? 0u : (x & 0xffffu);
  const uint32_t hi = (x & 0x80000000u) ? 0u : (x & 0xffff0000u);
  return lo | hi;
}

template <bool kPlain>
__global__ __launch_bounds__(256) void absorb_mfma_kernel(float* __restrict__ state, const bf16_t* __restrict__ K,
                                                          const bf16_t* __restrict__ V, int n, int tokens_per_slice,
                                                          const float* __restrict__ cosv,
                                                          const float* __restrict__ sinv, int phi_kind, int BH,
                                                          int slices) {
  __shared__ __attribute__((aligned(16))) uint32_t Kt[D * SP];
  __shared__ __attribute__((aligned(16))) uint32_t Vt[D * SP];
  __shared__ float zs[D];

  // Consecutive workgroup ids land on consecutive XCDs.  All slices of one (batch, head) are
  // given to ONE XCD (head index mod 8), so the float atomics that add the partials to that
  // head's state meet in a single L2 instead of bouncing between the XCDs' caches.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int bh = xcd + 8 * (slot / slices);
  if (bh >= BH) return;
  const int t0 = (slot % slices) * tokens_per_slice;
  const int t1 = min(n, t0 + tokens_per_slice);
  if (t0 >= t1) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bf16_t* Kh = K + (size_t)bh * n * D;
  const bf16_t* Vh = V + (size_t)bh * n * D;
  const int g = tid & 15;   // feature group: features 8g .. 8g+7
  const int tp0 = tid >> 4; // token pair of item 0; item 1 is 16 pairs further

  if (tid < D) zs[tid] = 0.0f;

  auto load = [&](int tb, Regs& r) {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int tok = tb + 2 * (tp0 + 16 * it);
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

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;

  const int mi0 = 2 * (wave >> 1), nj0 = 2 * (wave & 1);  // this wave's 2x2 grid of 32x32 tiles
  const int h = lane >> 5, l32 = lane & 31;

  Regs cur;
  load(t0, cur);
  for (int tb = t0; tb < t1; tb += CH) {
    // ---- transform, pack token pairs, transposing store to LDS
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int tp = tp0 + 16 * it;
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
        Kt[f * SP + col] = (kw[0][q] & 0xffffu) | (kw[1][q] << 16);
        Kt[(f + 1) * SP + col] = (kw[0][q] >> 16) | (kw[1][q] & 0xffff0000u);
        Vt[f * SP + col] = (vw[0][q] & 0xffffu) | (vw[1][q] << 16);
        Vt[(f + 1) * SP + col] = (vw[0][q] >> 16) | (vw[1][q] & 0xffff0000u);
      }
    }
    __syncthreads();
    if (tb + CH < t1) load(tb + CH, cur);  // in flight while the matrix cores run

    // ---- 4 contraction steps of 16 tokens
#pragma unroll
    for (int ks = 0; ks < CH / 16; ++ks) {
      bf16x8 af[2], bf[2];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const int f = 32 * (mi0 + a) + l32;
        af[a] = *reinterpret_cast<const bf16x8*>(&Kt[f * SP + pair_col(f, 8 * ks + 4 * h)]);
      }
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const int f = 32 * (nj0 + b) + l32;
        bf[b] = *reinterpret_cast<const bf16x8*>(&Vt[f * SP + pair_col(f, 8 * ks + 4 * h)]);
      }
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
    }
    __syncthreads();
  }

  // ---- add the partial to the state
  float* L = state + (size_t)bh * D * D;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = 32 * (mi0 + a) + 8 * (r >> 2) + 4 * h + (r & 3);
        const int j = 32 * (nj0 + b) + l32;
        atomicAdd(L + i * D + j, acc[a][b][r]);
      }
#pragma unroll
  for (int e = 0; e < 8; ++e) atomicAdd(&zs[8 * g + e], zacc[e]);
  __syncthreads();
  if (tid < D) atomicAdd(state + (size_t)BH * D * D + (size_t)bh * D + tid, zs[tid]);
}

int env_int(const char* name, int dflt) {
  const char* v = getenv(name);
  if (!v || !*v) return dflt;
  const int x = atoi(v);
  return x > 0 ? x : dflt;
}

}  // namespace

int launch_absorb_mfma(const hf_config& c, float* state, const void* K, const void* V, int n,
                       const float* cosv, const float* sinv, hipStream_t s) {
  const int BH = c.batch * c.heads;
  // slice length: a multiple of the 64-token chunk; default aims at ~2 workgroups per compute unit
  const int forced = env_int("HF_ABSORB_SLICE_TOKENS", 0);
  int per;
  if (forced > 0) {
    per = (forced + CH - 1) / CH * CH;
  } else {
    int slices = (512 + BH - 1) / BH;
    per = (n + slices - 1) / slices;
    per = (per + CH - 1) / CH * CH;
    if (per < 2 * CH) per = 2 * CH;
  }
  const int slices = (n + per - 1) / per;
  const bool plain = (c.phi == HF_PHI_RELU) && cosv == nullptr;
  const bf16_t* Kp = static_cast<const bf16_t*>(K);
  const bf16_t* Vp = static_cast<const bf16_t*>(V);
  const int heads_per_xcd = (BH + 7) / 8;
  const dim3 grid(8 * heads_per_xcd * slices);
  if (plain) {
    hipLaunchKernelGGL((absorb_mfma_kernel<true>), grid, dim3(256), 0, s, state, Kp, Vp, n, per, cosv, sinv,
                       c.phi, BH, slices);
  } else {
    hipLaunchKernelGGL((absorb_mfma_kernel<false>), grid, dim3(256), 0, s, state, Kp, Vp, n, per, cosv, sinv,
                       c.phi, BH, slices);
  }
  return check_launch("hf_absorb_evicted");
}

}  // namespace hf
