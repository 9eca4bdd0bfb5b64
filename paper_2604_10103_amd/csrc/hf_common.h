// Shared host/device helpers of the gfx950 hybrid-attention library (internal).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "hf.h"

namespace hf {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kMaxSelectBlocks = 2048;  // largest T_n the selection kernel ranks in LDS

typedef uint16_t bf16_t;  // storage type of a bfloat16 value

__device__ __forceinline__ float bf16_to_f32(bf16_t x) {
  return __uint_as_float(static_cast<uint32_t>(x) << 16);
}

// round-to-nearest-even; maps to v_cvt_pk_bf16_f32 on gfx950
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  __bf16 b = static_cast<__bf16>(f);
  return __builtin_bit_cast(bf16_t, b);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPer16B = 4;
  __device__ static __forceinline__ float load(const float* p) { return *p; }
  __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kPer16B = 8;
  __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// 16-byte vector load of consecutive elements into fp32 registers
template <typename T> __device__ __forceinline__ void load16B(const T* p, float* out);
template <> __device__ __forceinline__ void load16B<float>(const float* p, float* out) {
  const float4 v = *reinterpret_cast<const float4*>(p);
  out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
template <> __device__ __forceinline__ void load16B<bf16_t>(const bf16_t* p, float* out) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(w[i] << 16);
    out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}

// feature map of the linear branch (Eq. 2, 3): ReLU or elu(x)+1
__device__ __forceinline__ float phi_apply(float x, int kind) {
  if (kind == HF_PHI_RELU) return fmaxf(x, 0.0f);
  return x > 0.0f ? x + 1.0f : __expf(x);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// ---- host side -------------------------------------------------------------------------
void set_error(const char* fmt, ...);
int check_launch(const char* what);

// More than 64 KB of dynamic LDS has to be granted per kernel and device.  One object per kernel (static
// storage, zero-initialised); the grant is idempotent, so threads that race here at worst both ask for it.
struct LdsGrant {
  static constexpr int kDevices = 64;
  std::atomic<int> granted[kDevices];
};
int grant_lds(LdsGrant& g, const void* kernel, int bytes, const char* what);

// Per-call tag (48 bits) of the arrival counters that kernels keep in caller workspaces: a process-wide sequence
// from a random start, so that neither an earlier call's counters nor the uninitialised contents of a fresh
// workspace pass for this call's.  A counter word is (tag << 16) | count.
unsigned long long next_call_tag();

struct Dims {
  int B, H, D, BH;
  int n_q, n_kv, bq, bkv, t_m, t_n;
};

// tokens between the heads of K_win / V_win: the cache buffer's capacity, or the window length when packed
inline int kv_stride_of(const hf_config& c, int n_kv) { return c.kv_capacity > 0 ? c.kv_capacity : n_kv; }

// Launchers implemented in the .hip files.  All pointers are device pointers.
int launch_fill_zero(float* p, size_t n, hipStream_t s);
int launch_fold_linear(const hf_config& c, const float* state_in, const float* W, float* state_out, hipStream_t s);
int launch_absorb(const hf_config& c, float* state, const void* K, const void* V, int n, int head_stride,
                  const float* cosv, const float* sinv, void* workspace, size_t workspace_bytes,
                  hipStream_t s, void* planes_out = nullptr);
int launch_window_shift(const hf_config& c, void* K, void* V, int n_kv, int first, int n_evict, hipStream_t s);
size_t absorb_workspace_bytes(const hf_config& c, int n);
// pools every query block and the KV blocks [kv_first, kv_end); the other KV blocks keep what kbar_t holds
int launch_pool_both(const hf_config& c, const void* Q, int n_q, int t_m, const void* K, int n_kv, int t_n,
                     int kv_first, int kv_end, float* qbar, float* kbar_t, hipStream_t s);
int launch_score_select(const hf_config& c, const float* qbar, const float* kbar_t, int t_m, int t_n,
                        int k, int32_t* idx, float* scores, hipStream_t s);
int launch_attn(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                const int32_t* idx, int k, void* O_local, hipStream_t s);
int launch_readout(const hf_config& c, const void* Q, int n_q, const void* O_local,
                   const float* state, const float* cosq, const float* sinq, void* planes, void* O,
                   hipStream_t s);
size_t readout_planes_bytes(const hf_config& c);  // scratch for the bf16 planes of the state
int launch_state_planes(const hf_config& c, const float* state, void* planes, hipStream_t s);
bool attn_mfma_fused_supported(const hf_config& c);
int launch_attn_mfma_fused(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                           const int32_t* idx, int k, const void* planes, const float* zvec, const float* cosq,
                           const float* sinq, const void* Q_hist, void* O, hipStream_t s, float* lse2_out = nullptr,
                           void* olocal_out = nullptr,    // by-products for hf_hybrid_attn_bwd_saved, each optional
                           const float* kbar_t = nullptr, int32_t* idx_out = nullptr, float* scores_out = nullptr);
// kbar_t given (idx NULL): every workgroup selects its KV blocks itself (Eq. 4) and writes its list to idx_out
int launch_attn_mfma_select(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv, int k,
                            const float* kbar_t, int32_t* idx_out, float* scores_out, void* O_local, hipStream_t s);
constexpr int kMaxFusedSelectBlocks = 1024;   // largest T_n the attention kernel ranks in its tile space
// the selecting launch with workgroups of their own that absorb n_ev tokens of another chunk (Eq. 2; ReLU, no
// rotation) into state_out / planes_out = state_in + their contribution; planes NULL: no history term in O
size_t step_absorb_workspace_bytes(const hf_config& c, int n_q, int n_ev);
int launch_attn_mfma_step(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv, int k,
                          const float* kbar_t, int32_t* idx_out, float* scores_out, const void* planes,
                          const float* zvec, const float* cosq, const float* sinq, const void* Q_hist, void* O,
                          const void* K_ev, const void* V_ev, int n_ev, int ev_stride, const float* state_in,
                          float* state_out, void* planes_out, void* workspace, hipStream_t s);
int launch_attn_mfma_lse(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                         const int32_t* idx, int k, void* O_local, float* lse2_out, hipStream_t s);
// backward pass (training algorithm): lse2 = per-row log2 of the softmax denominator in the scaled-logit domain
int launch_attn_generic(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                        const int32_t* idx, int k, void* O_local, hipStream_t s, float* lse2, const void* dO,
                        float* Dv);  // lse2 given: writes lse2 and Dv = dO . O_local instead of O_local
int launch_attn_mfma_stats(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                           const int32_t* idx, int k, const void* dO, float* lse2, float* dvec, hipStream_t s);
int launch_row_dot(const hf_config& c, const void* A, const void* B, long long rows, float* out, hipStream_t s);
bool bwd_mfma_supported(const hf_config& c);
size_t bwd_planes_bytes(const hf_config& c);
int launch_bwd_mfma(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                    const int32_t* idx, int k, const void* dO, const float* lse2, const float* Dv,
                    const int32_t* inv_cnt, const int32_t* inv_list, int32_t* dkv_order, const float* state,
                    const float* cosq, const float* sinq, const void* Q_hist, void* planes, void* dQ, void* dQ_hist,
                    void* dK, void* dV, hipStream_t s);
int launch_invert_index(const hf_config& c, const int32_t* idx, int k, int t_m, int t_n, int32_t* inv_cnt,
                        int32_t* inv_list, hipStream_t s);
int launch_bwd_generic(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                       const int32_t* idx, int k, const void* dO, const float* lse2, const float* Dv,
                       const int32_t* inv_cnt, const int32_t* inv_list, const float* dqh32, void* dQ, void* dK,
                       void* dV, hipStream_t s);
int launch_bwd_hist_generic(const hf_config& c, const void* Q_hist, const void* dO, const float* state, int n_q,
                            const float* cosq, const float* sinq, void* out, bool out_f32, hipStream_t s);
int launch_rope_tables(const int32_t* frame_idx, int n_frames, int height, int width, int pairs_t, int pairs_h,
                       int pairs_w, double theta, int temporal_only, float* cosv, float* sinv, hipStream_t s);
int launch_rope_apply(const hf_config& c, const void* X, int n, const float* cosv, const float* sinv, void* Y,
                      hipStream_t s);
// the chunk's new keys rotated (tables NULL: copied) into the window at token `first`, the KV blocks they touch pooled
int launch_rope_append_pool(const hf_config& c, const void* X, int n_new, const float* cosv, const float* sinv, void* Kwin,
                            int first, int n_kv, float* kbar_t, hipStream_t s);

}  // namespace hf
