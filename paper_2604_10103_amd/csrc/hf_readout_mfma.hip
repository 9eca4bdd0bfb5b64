// History readout and hybrid sum (Eq. 3 without the Linear map, Eq. 6) on bf16 MFMA:
//   O[r][j] = O_local[r][j] + ( sum_i R_r(phi(q_r))[i] L[i][j] ) / ( z_scale * phi(q_r).z + eps )
// for bf16 inputs and head_dim 128.  The kernel streams Q and O_local in and O out (HBM bound).
//
// The fp32 state is first split into two bf16 planes L ~ hi + lo (error ~2^-17 relative) and
// transposed so that the contraction index i is contiguous: Lt[j][i].  A workgroup of four
// wavefronts keeps both planes in LDS, each wavefront owns 32 query rows and forms
//   O_hist^T (j x queries) = Lt (A operand, LDS)  x  phi(Q)^T (B operand, registers)
// so the denominator and the scaling are per-lane scalars.  The result is transposed back
// through LDS (reusing the planes' space) and combined with O_local in coalesced 16-byte rows.
#include "hf_common.h"

namespace hf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int D = 128;
constexpr int LSTR = 272;  // bytes per row of a bf16 plane in LDS (256 + 16)
constexpr int OSTR = 528;  // bytes per staged fp32 output row in LDS (512 + 16)
constexpr int PLANE = D * LSTR;

// state L[i][j] fp32 -> planes hi/lo, transposed: Lt[plane][j][i] bf16
__global__ __launch_bounds__(256) void state_planes_kernel(const float* __restrict__ state,
                                                           bf16_t* __restrict__ planes) {
  __shared__ float tile[32][33];
  const int bh = blockIdx.z, i0 = blockIdx.y * 32, j0 = blockIdx.x * 32;
  const float* L = state + (size_t)bh * D * D;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int r = ty; r < 32; r += 8) tile[r][tx] = L[(size_t)(i0 + r) * D + j0 + tx];
  __syncthreads();
  bf16_t* hi = planes + (size_t)bh * 2 * D * D;
  bf16_t* lo = hi + D * D;
  for (int r = ty; r < 32; r += 8) {
    const float v = tile[tx][r];  // i = i0 + tx, j = j0 + r
    const bf16_t h = f32_to_bf16(v);
    hi[(size_t)(j0 + r) * D + i0 + tx] = h;
    lo[(size_t)(j0 + r) * D + i0 + tx] = f32_to_bf16(v - bf16_to_f32(h));
  }
}

template <bool kPlain>
__global__ __launch_bounds__(256) void readout_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Oloc, const bf16_t* __restrict__ planes,
    const float* __restrict__ state, const float* __restrict__ cosq, const float* __restrict__ sinq, int n_q,
    int phi_kind, float eps, float z_scale, int BH, bf16_t* __restrict__ O) {
  extern __shared__ __attribute__((aligned(16))) char smem[];  // planes hi|lo, later the staged output
  __shared__ float sz[D];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  const int bh = blockIdx.y;
  const int row0 = blockIdx.x * 128 + 32 * wave;
  const bf16_t* Qh = Q + (size_t)bh * n_q * D;
  const bf16_t* Lh = Oloc + (size_t)bh * n_q * D;
  bf16_t* Oh = O + (size_t)bh * n_q * D;

  // ---- everything this workgroup reads is requested up front
  uint4 lreg[16];
  {
    const uint4* src = reinterpret_cast<const uint4*>(planes + (size_t)bh * 2 * D * D);
#pragma unroll
    for (int i = 0; i < 16; ++i) lreg[i] = src[tid + 256 * i];
  }
  const int q_row = min(row0 + l32, n_q - 1);
  uint4 qraw[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) qraw[s] = *reinterpret_cast<const uint4*>(Qh + (size_t)q_row * D + 16 * s + 8 * h);
  uint4 oraw[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int c = lane + 64 * i, r = min(row0 + (c >> 4), n_q - 1);
    oraw[i] = *reinterpret_cast<const uint4*>(Lh + (size_t)r * D + (c & 15) * 8);
  }
  if (tid < D) sz[tid] = state[(size_t)BH * D * D + (size_t)bh * D + tid];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = tid + 256 * i;             // 16-byte chunk of the two planes: 16 per row
    const int row = c >> 4, col = c & 15;    // row counts over hi rows then lo rows
    *reinterpret_cast<uint4*>(smem + row * LSTR + col * 16) = lreg[i];
  }
  __syncthreads();

  // ---- phi(q): B-operand fragments (features 16 s + 8 h + e) and the denominator
  bf16x8 qhi[8], qlo[8];
  float den = 0.0f;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const uint32_t w[4] = {qraw[s].x, qraw[s].y, qraw[s].z, qraw[s].w};
    float f[8];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      f[2 * p] = phi_apply(__uint_as_float(w[p] << 16), phi_kind);
      f[2 * p + 1] = phi_apply(__uint_as_float(w[p] & 0xffff0000u), phi_kind);
    }
    const float4 z0 = *reinterpret_cast<const float4*>(&sz[16 * s + 8 * h]);
    const float4 z1 = *reinterpret_cast<const float4*>(&sz[16 * s + 8 * h + 4]);
    den += f[0] * z0.x + f[1] * z0.y + f[2] * z0.z + f[3] * z0.w + f[4] * z1.x + f[5] * z1.y + f[6] * z1.z +
           f[7] * z1.w;
    if (!kPlain && cosq) {
      const size_t toff = (size_t)q_row * (D / 2) + 8 * s + 4 * h;
      const float4 c4 = *reinterpret_cast<const float4*>(cosq + toff);
      const float4 s4 = *reinterpret_cast<const float4*>(sinq + toff);
      const float cc[4] = {c4.x, c4.y, c4.z, c4.w}, ss[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const float a = f[2 * p], b = f[2 * p + 1];
        f[2 * p] = a * cc[p] - b * ss[p];
        f[2 * p + 1] = a * ss[p] + b * cc[p];
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const __bf16 hi = static_cast<__bf16>(f[e]);
      qhi[s][e] = hi;
      if (!kPlain) qlo[s][e] = static_cast<__bf16>(f[e] - static_cast<float>(hi));
    }
  }
  den += __shfl_xor(den, 32, kWave);
  const float inv = 1.0f / (z_scale * den + eps);

  // ---- O_hist^T = Lt x phi(Q)^T, hi and lo planes (and the low part of phi(q) when it is inexact)
  f32x16 acc[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[dt][r] = 0.0f;
  const char* a_base = smem + l32 * LSTR + 16 * h;
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
      const bf16x8 ahi = *reinterpret_cast<const bf16x8*>(a_base + 32 * dt * LSTR + 32 * s);
      const bf16x8 alo = *reinterpret_cast<const bf16x8*>(a_base + PLANE + 32 * dt * LSTR + 32 * s);
      acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(alo, qhi[s], acc[dt], 0, 0, 0);
      if (!kPlain) acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ahi, qlo[s], acc[dt], 0, 0, 0);
      acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ahi, qhi[s], acc[dt], 0, 0, 0);
    }
  __syncthreads();  // all wavefronts are done with the planes: their space becomes the staging area

  // ---- transpose back through LDS: lane (query l32) holds features 32 dt + 8 (r/4) + 4 h + (r%4)
  char* stage = smem + wave * 32 * OSTR;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq)
      *reinterpret_cast<float4*>(stage + l32 * OSTR + (32 * dt + 8 * rq + 4 * h) * 4) =
          make_float4(acc[dt][4 * rq] * inv, acc[dt][4 * rq + 1] * inv, acc[dt][4 * rq + 2] * inv,
                      acc[dt][4 * rq + 3] * inv);
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_s_waitcnt(0xc07f);

  // ---- O = O_local + O_hist, coalesced 16-byte pieces
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int c = lane + 64 * i, r = c >> 4, col = c & 15;
    if (row0 + r < n_q) {
      const float4 h0 = *reinterpret_cast<const float4*>(stage + r * OSTR + col * 32);
      const float4 h1 = *reinterpret_cast<const float4*>(stage + r * OSTR + col * 32 + 16);
      const uint32_t w[4] = {oraw[i].x, oraw[i].y, oraw[i].z, oraw[i].w};
      const float hh[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
      uint32_t out[4];
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const float a = __uint_as_float(w[p] << 16) + hh[2 * p];
        const float b = __uint_as_float(w[p] & 0xffff0000u) + hh[2 * p + 1];
        out[p] = (uint32_t)f32_to_bf16(a) | ((uint32_t)f32_to_bf16(b) << 16);
      }
      *reinterpret_cast<uint4*>(Oh + (size_t)(row0 + r) * D + col * 8) = make_uint4(out[0], out[1], out[2], out[3]);
    }
  }
}

}  // namespace

bool readout_mfma_supported(const hf_config& c) { return c.dtype == HF_BF16 && c.head_dim == 128; }

size_t readout_planes_bytes(const hf_config& c) {
  return readout_mfma_supported(c) ? (size_t)c.batch * c.heads * 2 * D * D * sizeof(bf16_t) : 0;
}

int launch_state_planes(const hf_config& c, const float* state, void* planes, hipStream_t s) {
  hipLaunchKernelGGL(state_planes_kernel, dim3(D / 32, D / 32, c.batch * c.heads), dim3(256), 0, s, state,
                     static_cast<bf16_t*>(planes));
  return check_launch("hf_hybrid_attn_fwd(state planes)");
}

int launch_readout_mfma(const hf_config& c, const void* Q, int n_q, const void* O_local, const float* state,
                        const float* cosq, const float* sinq, void* planes, void* O, hipStream_t s) {
  const int BH = c.batch * c.heads;
  bf16_t* pl = static_cast<bf16_t*>(planes);
  hipLaunchKernelGGL(state_planes_kernel, dim3(D / 32, D / 32, BH), dim3(256), 0, s, state, pl);
  const size_t smem = 2 * PLANE;  // 69632 B >= 4 * 32 * OSTR = 67584 B of staging
  static_assert(2 * PLANE >= 4 * 32 * OSTR, "staging must fit in the planes' space");
  const bool plain = (c.phi == HF_PHI_RELU) && cosq == nullptr;
  const dim3 grid((n_q + 127) / 128, BH), block(256);
  const bf16_t* q = static_cast<const bf16_t*>(Q);
  const bf16_t* ol = static_cast<const bf16_t*>(O_local);
  bf16_t* o = static_cast<bf16_t*>(O);
  static LdsGrant grants[2];
  const void* fn = plain ? reinterpret_cast<const void*>(readout_mfma_kernel<true>)
                         : reinterpret_cast<const void*>(readout_mfma_kernel<false>);
  {
    const int rc = grant_lds(grants[plain], fn, (int)smem, "the readout kernel");
    if (rc != HF_OK) return rc;
  }
  if (plain)
    hipLaunchKernelGGL((readout_mfma_kernel<true>), grid, block, smem, s, q, ol, pl, state, cosq, sinq, n_q, c.phi,
                       c.eps, c.z_scale, BH, o);
  else
    hipLaunchKernelGGL((readout_mfma_kernel<false>), grid, block, smem, s, q, ol, pl, state, cosq, sinq, n_q, c.phi,
                       c.eps, c.z_scale, BH, o);
  return check_launch("hf_hybrid_attn_fwd(readout)");
}

}  // namespace hf
