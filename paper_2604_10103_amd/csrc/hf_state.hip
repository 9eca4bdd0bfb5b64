// Linear state of the history branch: zero fill and absorption of evicted tokens (Eq. 2).
//
//   L[i][j] += sum_t R_t(phi(k_t))[i] * v_t[j]        z[i] += sum_t phi(k_t)[i]
//
// This file: the fill kernel and the fp32-arithmetic absorb kernel (fp32 inputs, or head_dim 64).
// The evicted tokens of one (batch, head) are cut into slices; a workgroup reduces one slice to
// a d x d partial in registers and adds it to the fp32 state with device-scope float atomics.
// bf16 inputs with head_dim 128 take the MFMA kernel of hf_state_mfma.hip.
#include "hf_common.h"

namespace hf {

__global__ void fill_zero_kernel(float* __restrict__ p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0.0f;
}

int launch_fill_zero(float* p, size_t n, hipStream_t s) {
  const int threads = 256;
  size_t blocks = (n + threads - 1) / threads;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(threads), 0, s, p, n);
  return check_launch("hf_state_init");
}

// ---------------------------------------------------------------------------------------------
// Linear map of Eq. 3 folded into the state: L'[bh] = L[bh] W[h], z' = z.  Runs once per chunk on
// 0.8 MB, fp32 FMA: one workgroup per 16 rows of one head's L; thread (row, column group) forms 8
// (or 4) output columns; the 16 rows of L sit in LDS (broadcast reads), W streams from L2 with
// the 16 column groups of a row reading 512 (256) contiguous bytes.
template <int D>
__global__ __launch_bounds__(256) void fold_linear_kernel(const float* __restrict__ state_in,
                                                          const float* __restrict__ W,
                                                          float* __restrict__ state_out, int H, int BH) {
  constexpr int C = D / 16;  // output columns per thread
  __shared__ float sL[16][D];
  const int tid = threadIdx.x, row = tid >> 4, cg = tid & 15;
  const int bh = blockIdx.y, h = bh % H, i0 = blockIdx.x * 16;
  const float* Lin = state_in + (size_t)bh * D * D + (size_t)i0 * D;
  for (int e = tid; e < 16 * D; e += 256) sL[e / D][e % D] = Lin[e];
  if (blockIdx.x == 0 && tid < D)  // the normaliser is copied unchanged
    state_out[(size_t)BH * D * D + (size_t)bh * D + tid] = state_in[(size_t)BH * D * D + (size_t)bh * D + tid];
  __syncthreads();
  const float* Wh = W + (size_t)h * D * D + cg * C;
  float acc[C];
#pragma unroll
  for (int c = 0; c < C; ++c) acc[c] = 0.0f;
#pragma unroll 4
  for (int j = 0; j < D; ++j) {
    const float l = sL[row][j];
    float w[C];
#pragma unroll
    for (int c = 0; c < C; c += 4) {
      const float4 v = *reinterpret_cast<const float4*>(Wh + (size_t)j * D + c);
      w[c] = v.x; w[c + 1] = v.y; w[c + 2] = v.z; w[c + 3] = v.w;
    }
#pragma unroll
    for (int c = 0; c < C; ++c) acc[c] = fmaf(l, w[c], acc[c]);
  }
  float* out = state_out + (size_t)bh * D * D + (size_t)(i0 + row) * D + cg * C;
#pragma unroll
  for (int c = 0; c < C; c += 4) *reinterpret_cast<float4*>(out + c) = make_float4(acc[c], acc[c + 1], acc[c + 2], acc[c + 3]);
}

int launch_fold_linear(const hf_config& c, const float* state_in, const float* W, float* state_out, hipStream_t s) {
  const int BH = c.batch * c.heads;
  const dim3 grid(c.head_dim / 16, BH), block(256);
  if (c.head_dim == 128)
    hipLaunchKernelGGL((fold_linear_kernel<128>), grid, block, 0, s, state_in, W, state_out, c.heads, BH);
  else
    hipLaunchKernelGGL((fold_linear_kernel<64>), grid, block, 0, s, state_in, W, state_out, c.heads, BH);
  return check_launch("hf_state_fold_linear");
}

// ---------------------------------------------------------------------------------------------
// fp32 FMA path (any storage dtype, fp32 arithmetic): used for fp32 inputs.
// 256 threads own a D x D register tile grid: thread (ti, tj) holds an E x E tile, E = D / 16.
// Tokens are staged TT at a time in LDS as fp32 (rotated phi(k) and v).
template <typename T, int D>
__global__ __launch_bounds__(256) void absorb_fma_kernel(float* __restrict__ state, const T* __restrict__ K,
                                                         const T* __restrict__ V, int n, int head_stride,
                                                         int tokens_per_slice, const float* __restrict__ cosv,
                                                         const float* __restrict__ sinv, int phi_kind, int BH) {
  constexpr int E = D / 16;
  constexpr int TT = 32;
  __shared__ float sk[TT][D + 4];
  __shared__ float sv[TT][D + 4];
  const int bh = blockIdx.y;
  const int t0 = blockIdx.x * tokens_per_slice;
  const int t1 = min(n, t0 + tokens_per_slice);
  if (t0 >= t1) return;
  const int tid = threadIdx.x;
  const int ti = tid / 16, tj = tid % 16;
  const T* Kh = K + (size_t)bh * head_stride * D;  // head_stride tokens between heads (= n when packed)
  const T* Vh = V + (size_t)bh * head_stride * D;
  float acc[E][E];
#pragma unroll
  for (int a = 0; a < E; ++a)
#pragma unroll
    for (int b = 0; b < E; ++b) acc[a][b] = 0.0f;
  float zsum = 0.0f;  // thread tid < D sums feature tid

  for (int tb = t0; tb < t1; tb += TT) {
    const int cnt = min(TT, t1 - tb);
    // stage: one feature pair per work item so the rotation has both partners
    for (int w = tid; w < TT * (D / 2); w += 256) {
      const int r = w / (D / 2), p = w % (D / 2);
      float k0 = 0.f, k1 = 0.f, v0 = 0.f, v1 = 0.f;
      if (r < cnt) {
        const size_t off = (size_t)(tb + r) * D + 2 * p;
        k0 = phi_apply(Elem<T>::load(Kh + off), phi_kind);
        k1 = phi_apply(Elem<T>::load(Kh + off + 1), phi_kind);
        v0 = Elem<T>::load(Vh + off);
        v1 = Elem<T>::load(Vh + off + 1);
        if (cosv) {
          const float c = cosv[(size_t)(tb + r) * (D / 2) + p], s = sinv[(size_t)(tb + r) * (D / 2) + p];
          const float r0 = k0 * c - k1 * s, r1 = k0 * s + k1 * c;
          k0 = r0; k1 = r1;
        }
      }
      sk[r][2 * p] = k0; sk[r][2 * p + 1] = k1;
      sv[r][2 * p] = v0; sv[r][2 * p + 1] = v1;
    }
    if (tid < D) {  // normaliser: un-rotated phi(k), straight from memory
      for (int r = 0; r < cnt; ++r) zsum += phi_apply(Elem<T>::load(Kh + (size_t)(tb + r) * D + tid), phi_kind);
    }
    __syncthreads();
    for (int r = 0; r < TT; ++r) {
      float kk[E], vv[E];
#pragma unroll
      for (int a = 0; a < E; ++a) kk[a] = sk[r][ti * E + a];
#pragma unroll
      for (int b = 0; b < E; ++b) vv[b] = sv[r][tj * E + b];
#pragma unroll
      for (int a = 0; a < E; ++a)
#pragma unroll
        for (int b = 0; b < E; ++b) acc[a][b] = fmaf(kk[a], vv[b], acc[a][b]);
    }
    __syncthreads();
  }
  float* L = state + (size_t)bh * D * D;
  float* z = state + (size_t)BH * D * D + (size_t)bh * D;
#pragma unroll
  for (int a = 0; a < E; ++a)
#pragma unroll
    for (int b = 0; b < E; ++b) atomicAdd(L + (size_t)(ti * E + a) * D + tj * E + b, acc[a][b]);
  if (tid < D) atomicAdd(z + tid, zsum);
}

template <typename T, int D>
static int launch_absorb_fma(const hf_config& c, float* state, const void* K, const void* V, int n,
                             int head_stride, const float* cosv, const float* sinv, hipStream_t s) {
  const int BH = c.batch * c.heads;
  // aim at ~4 workgroups per compute unit, at least 64 tokens per slice
  int slices = (1024 + BH - 1) / BH;
  int per = (n + slices - 1) / slices;
  if (per < 64) per = 64;
  per = (per + 31) / 32 * 32;
  slices = (n + per - 1) / per;
  hipLaunchKernelGGL((absorb_fma_kernel<T, D>), dim3(slices, BH), dim3(256), 0, s, state,
                     static_cast<const T*>(K), static_cast<const T*>(V), n, head_stride, per, cosv, sinv, c.phi, BH);
  return check_launch("hf_absorb_evicted");
}

int launch_absorb_mfma(const hf_config& c, float* state, const void* K, const void* V, int n, int head_stride,
                       const float* cosv, const float* sinv, void* workspace, size_t workspace_bytes,
                       hipStream_t s, void* planes_out);  // hf_state_mfma.hip
size_t absorb_mfma_workspace_bytes(const hf_config& c, int n);

static bool absorb_uses_mfma(const hf_config& c) { return c.dtype == HF_BF16 && c.head_dim == 128; }

size_t absorb_workspace_bytes(const hf_config& c, int n) {
  return absorb_uses_mfma(c) ? absorb_mfma_workspace_bytes(c, n) : 0;
}

// planes_out != NULL (bf16, head_dim 128 only; the caller checks): the bf16 planes of the updated state as well
int launch_absorb(const hf_config& c, float* state, const void* K, const void* V, int n, int head_stride,
                  const float* cosv, const float* sinv, void* workspace, size_t workspace_bytes,
                  hipStream_t s, void* planes_out) {
  if (c.dtype == HF_F32) {
    return c.head_dim == 128 ? launch_absorb_fma<float, 128>(c, state, K, V, n, head_stride, cosv, sinv, s)
                             : launch_absorb_fma<float, 64>(c, state, K, V, n, head_stride, cosv, sinv, s);
  }
  if (absorb_uses_mfma(c))
    return launch_absorb_mfma(c, state, K, V, n, head_stride, cosv, sinv, workspace, workspace_bytes, s, planes_out);
  return launch_absorb_fma<bf16_t, 64>(c, state, K, V, n, head_stride, cosv, sinv, s);
}

// ---------------------------------------------------------------------------------------------
// Window compaction after an eviction: tokens [src, src + len) of every head move to [dst, dst + len)
// in K_win and V_win (16-byte pieces; blockIdx.z picks K or V).  The caller issues non-overlapping
// pieces in ascending order, so a launch never reads what it writes.
__global__ __launch_bounds__(256) void window_shift_kernel(uint4* __restrict__ K, uint4* __restrict__ V,
                                                           size_t head_stride16, size_t src16, size_t dst16,
                                                           size_t len16) {
  uint4* X = (blockIdx.z ? V : K) + (size_t)blockIdx.y * head_stride16;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < len16; i += (size_t)gridDim.x * 256)
    X[dst16 + i] = X[src16 + i];
}

int launch_window_shift(const hf_config& c, void* K, void* V, int n_kv, int first, int n_evict, hipStream_t s) {
  const int BH = c.batch * c.heads;
  const size_t row16 = (size_t)c.head_dim * (c.dtype == HF_BF16 ? 2 : 4) / 16;  // 16-byte pieces per token
  const int keep = n_kv - first - n_evict;  // tokens behind the evicted run move down to `first`
  // pieces of at most n_evict tokens: source [t + n_evict, ...) and destination [t, ...) never overlap
  for (int t = 0; t < keep; t += n_evict) {
    const int len = min(n_evict, keep - t);
    const size_t len16 = (size_t)len * row16;
    unsigned blocks = (unsigned)((len16 + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(window_shift_kernel, dim3(blocks, BH, 2), dim3(256), 0, s, static_cast<uint4*>(K),
                       static_cast<uint4*>(V), (size_t)kv_stride_of(c, n_kv) * row16,
                       (size_t)(first + t + n_evict) * row16, (size_t)(first + t) * row16, len16);
    const int rc = check_launch("hf_window_advance(shift)");
    if (rc != HF_OK) return rc;
  }
  return HF_OK;
}

}  // namespace hf
