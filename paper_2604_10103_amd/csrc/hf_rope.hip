// Relative, capped temporal RoPE (Sec. 3.3, Eq. 7): construction of the per-token cos/sin tables
// from frame indices and the token grid, and rotation of a Q or K tensor by such tables.
//
// Both kernels are small and HBM-bound.  The rotation is a pass of its own, not folded into the
// attention kernel's tile loads: that kernel is bound by its vector ALU work next to the matrix
// cores, a rotated copy of the window's K costs one read and one write of it per chunk, and the
// copy is then read by every denoising step of the chunk.
#include <math.h>

#include "hf_common.h"

namespace hf {

struct RopeSpec {
  int frame_idx[HF_ROPE_MAX_FRAMES];
  double omega[HF_ROPE_MAX_PAIRS];  // radians per position step of every feature pair
};

// one thread per (token, pair); angles and their sine / cosine in fp64, rounded once to fp32
__global__ __launch_bounds__(256) void rope_tables_kernel(const RopeSpec spec, int n_tokens, int height, int width,
                                                          int pairs_t, int pairs_h, int pairs_w, int temporal_only,
                                                          float* __restrict__ cosv, float* __restrict__ sinv) {
  const int P = pairs_t + pairs_h + pairs_w;
  const long long e = (long long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long long)n_tokens * P) return;
  const int tok = (int)(e / P), p = (int)(e - (long long)tok * P);
  const int frame = tok / (height * width);
  const int rem = tok - frame * height * width;
  const int row = rem / width, col = rem - row * width;
  int pos;
  if (p < pairs_t) pos = spec.frame_idx[frame];
  else if (temporal_only) pos = 0;
  else pos = p < pairs_t + pairs_h ? row : col;
  double sn, cs;
  sincos((double)pos * spec.omega[p], &sn, &cs);
  cosv[e] = (float)cs;
  sinv[e] = (float)sn;
}

// 8 consecutive features (4 adjacent pairs) of one token per thread, for every head in turn: the thread's
// slice of the tables is read once and stays in registers (a table row is shared by all heads; read per head
// it would cross HBM once per head, the table being larger than an XCD's L2).  fp32 arithmetic, one rounding
// to the storage type.  X and Y may be the same buffer: a thread writes only what it has read.
template <typename T, int D>
__global__ __launch_bounds__(256) void rope_apply_kernel(const T* X, int n_tokens, int BH,
                                                         const float* __restrict__ cosv,
                                                         const float* __restrict__ sinv, T* Y) {
  constexpr int TPT = D / 8;         // threads per token
  constexpr int TOK = 256 / TPT;     // tokens per workgroup
  const int tok = blockIdx.x * TOK + threadIdx.x / TPT;
  if (tok >= n_tokens) return;
  const int g = threadIdx.x % TPT;
  const float4 c4 = *reinterpret_cast<const float4*>(cosv + (size_t)tok * (D / 2) + 4 * g);
  const float4 s4 = *reinterpret_cast<const float4*>(sinv + (size_t)tok * (D / 2) + 4 * g);
  const float cc[4] = {c4.x, c4.y, c4.z, c4.w}, ss[4] = {s4.x, s4.y, s4.z, s4.w};
  const int bh0 = blockIdx.y, bh_step = gridDim.y;
#pragma unroll 4
  for (int bh = bh0; bh < BH; bh += bh_step) {
    const size_t off = ((size_t)bh * n_tokens + tok) * D + 8 * g;
    float x[8];
    load16B<T>(X + off, x);
    if (Elem<T>::kPer16B == 4) load16B<T>(X + off + 4, x + 4);
    float y[8];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      y[2 * p] = x[2 * p] * cc[p] - x[2 * p + 1] * ss[p];
      y[2 * p + 1] = x[2 * p] * ss[p] + x[2 * p + 1] * cc[p];
    }
    if (Elem<T>::kPer16B == 8) {
      uint4 o;
      uint32_t w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) w[i] = (uint32_t)f32_to_bf16(y[2 * i]) | ((uint32_t)f32_to_bf16(y[2 * i + 1]) << 16);
      o.x = w[0]; o.y = w[1]; o.z = w[2]; o.w = w[3];
      *reinterpret_cast<uint4*>(Y + off) = o;
    } else {
      *reinterpret_cast<float4*>(Y + off) = make_float4(y[0], y[1], y[2], y[3]);
      *reinterpret_cast<float4*>(Y + off + 4) = make_float4(y[4], y[5], y[6], y[7]);
    }
  }
}

// The chunk's new keys take their place in the window buffer and the KV blocks they touch are pooled (Eq. 4's
// k-bar) in the same pass: one workgroup per (KV block, head) walks the block's tokens, 8 features of a token per
// thread; a token of the new range is read from X, rotated by its table row (fp32, one rounding to the storage type;
// no tables: copied) and stored, any other token of the block is read from the window as it stands; the column sums
// of the STORED values meet by lane exchanges and through LDS, and the mean over the block's real length goes to
// kbar_t[bh][D/4][t_n][4].
template <typename T, int D>
__global__ __launch_bounds__(256) void rope_append_pool_kernel(const T* __restrict__ X, int n_new,
                                                               const float* __restrict__ cosv,
                                                               const float* __restrict__ sinv, T* Kwin, int kv_stride,
                                                               int first, int n_kv, int bkv, int t_n, int blk0,
                                                               float* __restrict__ kbar_t) {
  constexpr int TPT = D / 8;         // threads per token
  constexpr int TOK = 256 / TPT;     // tokens per pass of the workgroup
  __shared__ float red[4][D];
  const int blk = blk0 + blockIdx.x, bh = blockIdx.y;
  const int t0 = blk * bkv, t1 = min(n_kv, t0 + bkv);
  const int g = threadIdx.x % TPT, tl = threadIdx.x / TPT;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
#pragma unroll 4
  for (int t = t0 + tl; t < t1; t += TOK) {
    T* dst = Kwin + ((size_t)bh * kv_stride + t) * D + 8 * g;
    float x[8];
    if (t >= first && t < first + n_new) {
      const size_t src = ((size_t)bh * n_new + (t - first)) * D + 8 * g;
      load16B<T>(X + src, x);
      if (Elem<T>::kPer16B == 4) load16B<T>(X + src + 4, x + 4);
      if (cosv != nullptr) {
        const float4 c4 = *reinterpret_cast<const float4*>(cosv + (size_t)(t - first) * (D / 2) + 4 * g);
        const float4 s4 = *reinterpret_cast<const float4*>(sinv + (size_t)(t - first) * (D / 2) + 4 * g);
        const float cc[4] = {c4.x, c4.y, c4.z, c4.w}, ss[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const float a = x[2 * p], b = x[2 * p + 1];
          x[2 * p] = a * cc[p] - b * ss[p];
          x[2 * p + 1] = a * ss[p] + b * cc[p];
        }
      }
      if (Elem<T>::kPer16B == 8) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bf16_t lo = f32_to_bf16(x[2 * i]), hi = f32_to_bf16(x[2 * i + 1]);
          w[i] = (uint32_t)lo | ((uint32_t)hi << 16);
          x[2 * i] = bf16_to_f32(lo);          // what is pooled is what is stored
          x[2 * i + 1] = bf16_to_f32(hi);
        }
        *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
      } else {
        *reinterpret_cast<float4*>(dst) = make_float4(x[0], x[1], x[2], x[3]);
        *reinterpret_cast<float4*>(dst + 4) = make_float4(x[4], x[5], x[6], x[7]);
      }
    } else {
      load16B<T>(dst, x);
      if (Elem<T>::kPer16B == 4) load16B<T>(dst + 4, x + 4);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += x[e];
  }
  // lanes g, g + TPT, ... of a wavefront hold the same features of different tokens
#pragma unroll
  for (int o = TPT; o < kWave; o <<= 1)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], o, kWave);
  if (lane < TPT) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wave][8 * lane + e] = acc[e];
  }
  __syncthreads();
  if (threadIdx.x < D) {
    const int f = threadIdx.x;
    const float sum = (red[0][f] + red[1][f]) + (red[2][f] + red[3][f]);
    kbar_t[(((size_t)bh * (D / 4) + f / 4) * t_n + blk) * 4 + (f & 3)] = sum * (1.0f / (float)(t1 - t0));
  }
}

int launch_rope_append_pool(const hf_config& c, const void* X, int n_new, const float* cosv, const float* sinv, void* Kwin,
                            int first, int n_kv, float* kbar_t, hipStream_t s) {
  const int BH = c.batch * c.heads;
  const int t_n = (n_kv + c.block_kv - 1) / c.block_kv;
  const int blk0 = first / c.block_kv, blk1 = (first + n_new + c.block_kv - 1) / c.block_kv;   // blocks the new tokens touch
  const dim3 grid(blk1 - blk0, BH);
  const int stride = kv_stride_of(c, n_kv);
#define HF_LAUNCH_RAP(T, DD)                                                                                         \
  hipLaunchKernelGGL((rope_append_pool_kernel<T, DD>), grid, dim3(256), 0, s, static_cast<const T*>(X), n_new, cosv, \
                     sinv, static_cast<T*>(Kwin), stride, first, n_kv, c.block_kv, t_n, blk0, kbar_t)
  if (c.dtype == HF_BF16) {
    if (c.head_dim == 128) HF_LAUNCH_RAP(bf16_t, 128); else HF_LAUNCH_RAP(bf16_t, 64);
  } else {
    if (c.head_dim == 128) HF_LAUNCH_RAP(float, 128); else HF_LAUNCH_RAP(float, 64);
  }
#undef HF_LAUNCH_RAP
  return check_launch("hf_rope_append_keys");
}

int launch_rope_tables(const int32_t* frame_idx, int n_frames, int height, int width, int pairs_t, int pairs_h,
                       int pairs_w, double theta, int temporal_only, float* cosv, float* sinv, hipStream_t s) {
  RopeSpec spec;
  for (int f = 0; f < HF_ROPE_MAX_FRAMES; ++f) spec.frame_idx[f] = f < n_frames ? frame_idx[f] : 0;
  const int np[3] = {pairs_t, pairs_h, pairs_w};
  int at = 0;
  for (int a = 0; a < 3; ++a)
    for (int p = 0; p < np[a]; ++p) spec.omega[at++] = pow(theta, -(double)p / (double)np[a]);
  for (; at < HF_ROPE_MAX_PAIRS; ++at) spec.omega[at] = 0.0;
  const long long n_tokens = (long long)n_frames * height * width;
  const long long total = n_tokens * (pairs_t + pairs_h + pairs_w);
  hipLaunchKernelGGL(rope_tables_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, spec,
                     (int)n_tokens, height, width, pairs_t, pairs_h, pairs_w, temporal_only, cosv, sinv);
  return check_launch("hf_rope_tables");
}

template <typename T>
static int launch_rope_apply_t(const hf_config& c, const void* X, int n, const float* cosv, const float* sinv,
                               void* Y, hipStream_t s) {
  const int D = c.head_dim;
  const int tok_per_wg = 256 / (D / 8);
  const int BH = c.batch * c.heads;
  const int chunks = (n + tok_per_wg - 1) / tok_per_wg;
  // heads are split over grid.y only as far as it takes to fill the chip (about 2000 workgroups)
  int ysplit = (2048 + chunks - 1) / chunks;
  if (ysplit > BH) ysplit = BH;
  if (ysplit < 1) ysplit = 1;
  const dim3 grid(chunks, ysplit);
  if (D == 128)
    hipLaunchKernelGGL((rope_apply_kernel<T, 128>), grid, dim3(256), 0, s, static_cast<const T*>(X), n, BH, cosv, sinv,
                       static_cast<T*>(Y));
  else
    hipLaunchKernelGGL((rope_apply_kernel<T, 64>), grid, dim3(256), 0, s, static_cast<const T*>(X), n, BH, cosv, sinv,
                       static_cast<T*>(Y));
  return check_launch("hf_rope_apply");
}

int launch_rope_apply(const hf_config& c, const void* X, int n, const float* cosv, const float* sinv, void* Y,
                      hipStream_t s) {
  return c.dtype == HF_BF16 ? launch_rope_apply_t<bf16_t>(c, X, n, cosv, sinv, Y, s)
                            : launch_rope_apply_t<float>(c, X, n, cosv, sinv, Y, s);
}

}  // namespace hf
