// C-ABI entry points: host-side argument checks and kernel dispatch.  No device allocation,
// no synchronisation; everything is enqueued on the caller's stream.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

#include <random>

#include "hf_common.h"

// Scratch of hf_block_select_static (pooled block means), one copy per GPU the library runs on, held until the
// process ends.  In host code this name is only a handle: the memory's device address comes from
// hipGetSymbolAddress (static_scratch() below) and that pointer is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[HF_STATIC_SCRATCH_BYTES];

namespace hf {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("%s: %s", what, hipGetErrorString(e));
    return HF_ERR_HIP;
  }
  return HF_OK;
}

int grant_lds(LdsGrant& g, const void* kernel, int bytes, const char* what) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); dev = -1; }
  const bool tracked = dev >= 0 && dev < LdsGrant::kDevices;
  if (tracked && g.granted[dev].load(std::memory_order_acquire)) return HF_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) {
    (void)hipGetLastError();
    set_error("cannot reserve %d bytes of LDS for %s", bytes, what);
    return HF_ERR_HIP;
  }
  if (tracked) g.granted[dev].store(1, std::memory_order_release);
  return HF_OK;
}

unsigned long long next_call_tag() {
  static std::atomic<unsigned long long> seq{0};
  unsigned long long cur = seq.load(std::memory_order_relaxed);
  if (cur == 0) {
    std::random_device rd;
    unsigned long long start = (((unsigned long long)rd() << 32) ^ rd()) | 1ull;
    seq.compare_exchange_strong(cur, start, std::memory_order_relaxed);   // (one thread's start wins)
  }
  return seq.fetch_add(1, std::memory_order_relaxed) & 0xffffffffffffull;
}

static int check_cfg(const hf_config* c) {
  if (!c) { set_error("cfg is NULL"); return HF_ERR_NULL; }
  if (c->batch < 1 || c->heads < 1) { set_error("batch and heads must be >= 1"); return HF_ERR_SHAPE; }
  if ((int64_t)c->batch * c->heads > 65535) { set_error("batch*heads must be <= 65535"); return HF_ERR_SHAPE; }
  if (c->head_dim != 64 && c->head_dim != 128) { set_error("head_dim must be 64 or 128, got %d", c->head_dim); return HF_ERR_SHAPE; }
  if (c->dtype != HF_BF16 && c->dtype != HF_F32) { set_error("unknown dtype %d", c->dtype); return HF_ERR_DTYPE; }
  if (c->phi != HF_PHI_RELU && c->phi != HF_PHI_ELU1) { set_error("unknown phi %d", c->phi); return HF_ERR_DTYPE; }
  if (c->block_q < 1 || c->block_kv < 1) { set_error("block sizes must be >= 1"); return HF_ERR_SHAPE; }
  if (c->block_q > 1024 || c->block_kv > 1024) { set_error("block sizes must be <= 1024"); return HF_ERR_SHAPE; }
  if (c->keep_k < 0) { set_error("keep_k must be >= 0"); return HF_ERR_SHAPE; }
  if (c->kv_capacity < 0 || c->kv_capacity > (1 << 24)) { set_error("kv_capacity must be in [0, 2^24]"); return HF_ERR_SHAPE; }
  if (c->keep_k == 0 && !(c->keep_ratio > 0.0f && c->keep_ratio <= 1.0f)) {
    set_error("keep_ratio must be in (0, 1]"); return HF_ERR_SHAPE;
  }
  if (c->flags & ~(HF_FLAG_READOUT_KERNEL | HF_FLAG_HISTORY_TWO_PLANES | HF_FLAG_BWD_FP32_KERNELS | HF_FLAG_DKV_INDEX_ORDER)) {
    set_error("unknown bits in flags: 0x%x", (unsigned)c->flags); return HF_ERR_SHAPE;
  }
  if (!(c->eps >= 0.0f) || !isfinite(c->z_scale) || !(c->softmax_scale >= 0.0f)) {
    set_error("eps, z_scale or softmax_scale is invalid"); return HF_ERR_SHAPE;
  }
  return HF_OK;
}

static int check_ptr(const void* p, const char* name, bool required) {
  if (!p) {
    if (!required) return HF_OK;
    set_error("%s is NULL", name);
    return HF_ERR_NULL;
  }
  if (reinterpret_cast<uintptr_t>(p) & 15u) { set_error("%s is not 16-byte aligned", name); return HF_ERR_ALIGN; }
  return HF_OK;
}

static int check_tokens(int32_t n, const char* name) {
  // 2^24 tokens keeps every element offset within one head below 2^31
  if (n < 1 || n > (1 << 24)) { set_error("%s must be in [1, 2^24], got %d", name, n); return HF_ERR_SHAPE; }
  return HF_OK;
}

static int check_window_len(const hf_config* c, int32_t n_kv) {
  if (c->kv_capacity > 0 && n_kv > c->kv_capacity) {
    set_error("n_kv=%d exceeds kv_capacity=%d", n_kv, c->kv_capacity);
    return HF_ERR_SHAPE;
  }
  return HF_OK;
}

static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

static int select_k_of(const hf_config* c, int t_n) {
  if (c->keep_k > 0) return c->keep_k;
  // keep_ratio is a float: its representation error (up to 6e-8 relative) would exceed the 1e-9 slack whenever
  // ratio * T_n is an integer (0.1f * 10 = 1.0000000149).  The ratio is therefore read to 7 significant decimal
  // digits, which recovers the decimal value the caller wrote.
  char digits[32];
  snprintf(digits, sizeof(digits), "%.7g", (double)c->keep_ratio);
  int k = (int)ceil(strtod(digits, nullptr) * (double)t_n - 1e-9);
  if (k < 1) k = 1;
  if (k > t_n) k = t_n;
  return k;
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static inline size_t esize(const hf_config* c) { return c->dtype == HF_BF16 ? 2 : 4; }

struct WorkspaceLayout {
  size_t qbar, kbar, olocal, planes, total;  // byte offsets
};

static WorkspaceLayout workspace_layout(const hf_config* c, int n_q, int n_kv) {
  const size_t bh = (size_t)c->batch * c->heads, d = c->head_dim;
  const size_t t_m = cdiv(n_q, c->block_q), t_n = cdiv(n_kv, c->block_kv);
  WorkspaceLayout w;
  w.qbar = 0;
  w.kbar = align256(bh * t_m * d * 4);
  w.olocal = w.kbar + align256(bh * t_n * d * 4);
  w.planes = w.olocal + align256(bh * (size_t)n_q * d * esize(c));
  w.total = w.planes + align256(readout_planes_bytes(*c));
  return w;
}

struct BwdLayout {
  size_t lse2, dvec, dqh32, inv_cnt, inv_list, order, planes, total;  // byte offsets
};

static BwdLayout bwd_layout(const hf_config* c, int n_q, int n_kv) {
  const size_t bh = (size_t)c->batch * c->heads, d = c->head_dim;
  const size_t t_m = cdiv(n_q, c->block_q), t_n = cdiv(n_kv, c->block_kv);
  BwdLayout w;
  w.lse2 = 0;
  w.dvec = align256(bh * n_q * 4);
  w.dqh32 = w.dvec + align256(bh * n_q * 4);
  w.inv_cnt = w.dqh32 + align256(bh * (size_t)n_q * d * 4);
  w.inv_list = w.inv_cnt + align256(bh * t_n * 4);
  w.order = w.inv_list + align256(bh * t_n * t_m * 4);   // launch order of the dK/dV workgroups (64 keys each):
  w.planes = w.order + align256(bh * t_n * cdiv(c->block_kv, 64) * 8 * 4);   // records of 8 words
  w.total = w.planes + align256(bwd_planes_bytes(*c));
  return w;
}

}  // namespace hf

using namespace hf;

#define HF_TRY(expr) do { int _r = (expr); if (_r != HF_OK) return _r; } while (0)

extern "C" {

const char* hf_last_error(void) { return g_err; }
const char* hf_version(void) { return "hf-gfx950 0.1"; }

int hf_state_bytes(const hf_config* cfg, size_t* bytes_out) {
  HF_TRY(check_cfg(cfg));
  if (!bytes_out) { set_error("bytes_out is NULL"); return HF_ERR_NULL; }
  const size_t d = cfg->head_dim;
  *bytes_out = (size_t)cfg->batch * cfg->heads * (d * d + d) * sizeof(float);
  return HF_OK;
}

int hf_state_init(const hf_config* cfg, void* state, void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ptr(state, "state", true));
  const size_t d = cfg->head_dim;
  return launch_fill_zero(static_cast<float*>(state), (size_t)cfg->batch * cfg->heads * (d * d + d),
                          static_cast<hipStream_t>(stream));
}

int hf_state_fold_linear(const hf_config* cfg, const void* state_in, const float* W, void* state_out,
                         void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ptr(state_in, "state_in", true));
  HF_TRY(check_ptr(W, "W", true));
  HF_TRY(check_ptr(state_out, "state_out", true));
  const size_t d = cfg->head_dim;
  const size_t bytes = (size_t)cfg->batch * cfg->heads * (d * d + d) * sizeof(float);
  const char* a = static_cast<const char*>(state_in);
  const char* b = static_cast<const char*>(state_out);
  if (a < b + bytes && b < a + bytes) { set_error("state_out overlaps state_in"); return HF_ERR_SHAPE; }
  return launch_fold_linear(*cfg, static_cast<const float*>(state_in), W, static_cast<float*>(state_out),
                            static_cast<hipStream_t>(stream));
}

int hf_absorb_workspace_bytes(const hf_config* cfg, int32_t n_tokens, size_t* bytes_out) {
  HF_TRY(check_cfg(cfg));
  if (!bytes_out) { set_error("bytes_out is NULL"); return HF_ERR_NULL; }
  HF_TRY(check_tokens(n_tokens, "n_tokens"));
  *bytes_out = absorb_workspace_bytes(*cfg, n_tokens);
  return HF_OK;
}

static int check_planes_cfg(const hf_config* cfg, const void* planes, const char* what) {
  if (!attn_mfma_fused_supported(*cfg)) {
    set_error("state planes exist for bf16, head_dim 128, block_q 64 or 128 only (elsewhere the attention call converts)");
    return HF_ERR_SHAPE;
  }
  HF_TRY(check_ptr(planes, what, true));
  if (reinterpret_cast<uintptr_t>(planes) & 255u) { set_error("%s is not 256-byte aligned", what); return HF_ERR_ALIGN; }
  return HF_OK;
}

int hf_state_planes_bytes(const hf_config* cfg, size_t* bytes_out) {
  HF_TRY(check_cfg(cfg));
  if (!bytes_out) { set_error("bytes_out is NULL"); return HF_ERR_NULL; }
  *bytes_out = attn_mfma_fused_supported(*cfg) ? readout_planes_bytes(*cfg) : 0;
  return HF_OK;
}

int hf_state_planes(const hf_config* cfg, const void* state, void* planes_out, void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ptr(state, "state", true));
  HF_TRY(check_planes_cfg(cfg, planes_out, "planes_out"));
  return launch_state_planes(*cfg, static_cast<const float*>(state), planes_out, static_cast<hipStream_t>(stream));
}

static int absorb_impl(const hf_config* cfg, void* state, const void* K_ev, const void* V_ev, int32_t n_tokens,
                       const float* rope_cos, const float* rope_sin, void* workspace, size_t workspace_bytes,
                       void* planes_out, void* stream);

int hf_absorb_evicted(const hf_config* cfg, void* state, const void* K_ev, const void* V_ev,
                      int32_t n_tokens, const float* rope_cos, const float* rope_sin, void* workspace,
                      size_t workspace_bytes, void* stream) {
  return absorb_impl(cfg, state, K_ev, V_ev, n_tokens, rope_cos, rope_sin, workspace, workspace_bytes, nullptr, stream);
}

int hf_absorb_evicted_planes(const hf_config* cfg, void* state, const void* K_ev, const void* V_ev,
                             int32_t n_tokens, const float* rope_cos, const float* rope_sin, void* workspace,
                             size_t workspace_bytes, void* planes_out, void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_planes_cfg(cfg, planes_out, "planes_out"));
  if (planes_out == state || planes_out == workspace) { set_error("planes_out aliases another argument"); return HF_ERR_SHAPE; }
  return absorb_impl(cfg, state, K_ev, V_ev, n_tokens, rope_cos, rope_sin, workspace, workspace_bytes, planes_out, stream);
}

static int absorb_impl(const hf_config* cfg, void* state, const void* K_ev, const void* V_ev, int32_t n_tokens,
                       const float* rope_cos, const float* rope_sin, void* workspace, size_t workspace_bytes,
                       void* planes_out, void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ptr(state, "state", true));
  HF_TRY(check_ptr(K_ev, "K_ev", true));
  HF_TRY(check_ptr(V_ev, "V_ev", true));
  HF_TRY(check_tokens(n_tokens, "n_tokens"));
  if ((rope_cos == nullptr) != (rope_sin == nullptr)) {
    set_error("rope_cos and rope_sin must both be given or both be NULL");
    return HF_ERR_NULL;
  }
  HF_TRY(check_ptr(rope_cos, "rope_cos", false));
  HF_TRY(check_ptr(rope_sin, "rope_sin", false));
  if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) {
    set_error("workspace is not 256-byte aligned");
    return HF_ERR_ALIGN;
  }
  return launch_absorb(*cfg, static_cast<float*>(state), K_ev, V_ev, n_tokens, n_tokens, rope_cos, rope_sin,
                       workspace, workspace ? workspace_bytes : 0, static_cast<hipStream_t>(stream), planes_out);
}

int hf_window_advance(const hf_config* cfg, void* K_win, void* V_win, int32_t n_kv, int32_t n_evict, void* state,
                      const float* rope_cos, const float* rope_sin, void* workspace, size_t workspace_bytes,
                      void* stream) {
  return hf_window_evict(cfg, K_win, V_win, n_kv, 0, n_evict, state, rope_cos, rope_sin, workspace, workspace_bytes,
                         stream);
}

int hf_window_evict(const hf_config* cfg, void* K_win, void* V_win, int32_t n_kv, int32_t n_sink, int32_t n_evict,
                    void* state, const float* rope_cos, const float* rope_sin, void* workspace,
                    size_t workspace_bytes, void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ptr(K_win, "K_win", true));
  HF_TRY(check_ptr(V_win, "V_win", true));
  HF_TRY(check_ptr(state, "state", true));
  HF_TRY(check_tokens(n_kv, "n_kv"));
  HF_TRY(check_tokens(n_evict, "n_evict"));
  HF_TRY(check_window_len(cfg, n_kv));
  if (n_sink < 0 || n_sink > n_kv) { set_error("n_sink=%d outside [0, n_kv]", n_sink); return HF_ERR_SHAPE; }
  if (n_evict > n_kv - n_sink) {
    set_error("n_evict=%d exceeds the %d tokens of the window behind its %d sink tokens", n_evict, n_kv - n_sink, n_sink);
    return HF_ERR_SHAPE;
  }
  if ((rope_cos == nullptr) != (rope_sin == nullptr)) {
    set_error("rope_cos and rope_sin must both be given or both be NULL");
    return HF_ERR_NULL;
  }
  HF_TRY(check_ptr(rope_cos, "rope_cos", false));
  HF_TRY(check_ptr(rope_sin, "rope_sin", false));
  if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) {
    set_error("workspace is not 256-byte aligned");
    return HF_ERR_ALIGN;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  // the oldest n_evict tokens behind the sink of every head go into the state ...
  const size_t skip = (size_t)n_sink * cfg->head_dim * esize(cfg);
  HF_TRY(launch_absorb(*cfg, static_cast<float*>(state), static_cast<char*>(K_win) + skip,
                       static_cast<char*>(V_win) + skip, n_evict, kv_stride_of(*cfg, n_kv), rope_cos, rope_sin,
                       workspace, workspace ? workspace_bytes : 0, s));
  // ... and the rest of the window moves down to the sink
  if (n_sink + n_evict == n_kv) return HF_OK;
  return launch_window_shift(*cfg, K_win, V_win, n_kv, n_sink, n_evict, s);
}

int hf_select_k(const hf_config* cfg, int32_t n_kv, int32_t* k_out) {
  HF_TRY(check_cfg(cfg));
  if (!k_out) { set_error("k_out is NULL"); return HF_ERR_NULL; }
  HF_TRY(check_tokens(n_kv, "n_kv"));
  const int t_n = cdiv(n_kv, cfg->block_kv);
  const int k = select_k_of(cfg, t_n);
  if (k > t_n) { set_error("keep_k=%d exceeds the %d KV blocks of the window", k, t_n); return HF_ERR_SHAPE; }
  *k_out = k;
  return HF_OK;
}

int hf_workspace_bytes(const hf_config* cfg, int32_t n_q, int32_t n_kv, size_t* bytes_out) {
  HF_TRY(check_cfg(cfg));
  if (!bytes_out) { set_error("bytes_out is NULL"); return HF_ERR_NULL; }
  HF_TRY(check_tokens(n_q, "n_q"));
  HF_TRY(check_tokens(n_kv, "n_kv"));
  *bytes_out = workspace_layout(cfg, n_q, n_kv).total;
  return HF_OK;
}

int hf_block_select(const hf_config* cfg, const void* Q, int32_t n_q, const void* K_win, int32_t n_kv,
                    int32_t* block_idx, float* scores_or_null, void* workspace, size_t workspace_bytes,
                    void* stream) {
  return hf_block_select_cached(cfg, Q, n_q, K_win, n_kv, 0, block_idx, scores_or_null, workspace, workspace_bytes,
                                stream);
}

// argument checks of the selection calls; k_out = blocks kept per row
static int check_select_args(const hf_config* cfg, const void* Q, int32_t n_q, const void* K_win, int32_t n_kv,
                             int32_t n_cached_kv_blocks, const int32_t* block_idx, const float* scores_or_null,
                             int* k_out) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ptr(Q, "Q", true));
  HF_TRY(check_ptr(K_win, "K_win", true));
  HF_TRY(check_ptr(block_idx, "block_idx", true));
  HF_TRY(check_ptr(scores_or_null, "scores", false));
  HF_TRY(check_tokens(n_q, "n_q"));
  HF_TRY(check_tokens(n_kv, "n_kv"));
  HF_TRY(check_window_len(cfg, n_kv));
  const int t_m = cdiv(n_q, cfg->block_q), t_n = cdiv(n_kv, cfg->block_kv);
  if (t_n > kMaxSelectBlocks) {
    set_error("window has %d KV blocks; the selection kernel ranks at most %d", t_n, kMaxSelectBlocks);
    return HF_ERR_SHAPE;
  }
  if (n_cached_kv_blocks < 0 || n_cached_kv_blocks > n_kv / cfg->block_kv) {
    set_error("n_cached_kv_blocks=%d outside [0, %d] (whole KV blocks of the window)", n_cached_kv_blocks,
              n_kv / cfg->block_kv);
    return HF_ERR_SHAPE;
  }
  const int k = select_k_of(cfg, t_n);
  if (k > t_n) { set_error("keep_k=%d exceeds the %d KV blocks of the window", k, t_n); return HF_ERR_SHAPE; }
  (void)t_m;
  *k_out = k;
  return HF_OK;
}

// the two launches of a selection call; qbar / kbar = pooled means [BH, T_m, d] and (feature-group-major) [BH, d/4, T_n, 4]
static int select_launches(const hf_config* cfg, const void* Q, int32_t n_q, const void* K_win, int32_t n_kv,
                           int32_t n_cached_kv_blocks, int k, int32_t* block_idx, float* scores_or_null, float* qbar,
                           float* kbar, hipStream_t s, int kv_end = -1) {
  const int t_m = cdiv(n_q, cfg->block_q), t_n = cdiv(n_kv, cfg->block_kv);
  HF_TRY(launch_pool_both(*cfg, Q, n_q, t_m, K_win, n_kv, t_n, n_cached_kv_blocks, kv_end < 0 ? t_n : kv_end, qbar, kbar, s));
  return launch_score_select(*cfg, qbar, kbar, t_m, t_n, k, block_idx, scores_or_null, s);
}

int hf_block_select_cached(const hf_config* cfg, const void* Q, int32_t n_q, const void* K_win, int32_t n_kv,
                           int32_t n_cached_kv_blocks, int32_t* block_idx, float* scores_or_null, void* workspace,
                           size_t workspace_bytes, void* stream) {
  int k = 0;
  HF_TRY(check_select_args(cfg, Q, n_q, K_win, n_kv, n_cached_kv_blocks, block_idx, scores_or_null, &k));
  const WorkspaceLayout w = workspace_layout(cfg, n_q, n_kv);
  if (!workspace || workspace_bytes < w.total) {
    set_error("workspace of %zu bytes needed, %zu given", w.total, workspace ? workspace_bytes : (size_t)0);
    return HF_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) { set_error("workspace is not 256-byte aligned"); return HF_ERR_ALIGN; }
  char* ws = static_cast<char*>(workspace);
  return select_launches(cfg, Q, n_q, K_win, n_kv, n_cached_kv_blocks, k, block_idx, scores_or_null,
                         reinterpret_cast<float*>(ws + w.qbar), reinterpret_cast<float*>(ws + w.kbar),
                         static_cast<hipStream_t>(stream));
}

// device address of this GPU's copy of `scratch`, looked up once per device (each GPU holds its own copy at its
// own address) with that device current
static int static_scratch(unsigned char** ptr_out) {
  constexpr int kDevices = 64;
  static std::atomic<unsigned char*> known[kDevices];   // zero-initialised
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    set_error("hipGetDevice: %s", hipGetErrorString(hipGetLastError()));
    return HF_ERR_HIP;
  }
  if (dev < 0 || dev >= kDevices) { set_error("device index %d outside [0, %d)", dev, kDevices); return HF_ERR_HIP; }
  unsigned char* p = known[dev].load(std::memory_order_acquire);
  if (!p) {
    const hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      (void)hipGetLastError();
      set_error("hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
      return HF_ERR_HIP;
    }
    known[dev].store(p, std::memory_order_release);   // racing threads look up the same address
  }
  *ptr_out = p;
  return HF_OK;
}

int hf_block_select_static(const hf_config* cfg, const void* Q, int32_t n_q, const void* K_win, int32_t n_kv,
                           int32_t* block_idx, float* scores_or_null, void* stream) {
  int k = 0;
  HF_TRY(check_select_args(cfg, Q, n_q, K_win, n_kv, 0, block_idx, scores_or_null, &k));
  // the pooled means are all the selection kernels need of the workspace
  const size_t bh = (size_t)cfg->batch * cfg->heads, d = cfg->head_dim;
  const size_t qbar_bytes = align256(bh * cdiv(n_q, cfg->block_q) * d * 4);
  const size_t kbar_bytes = align256(bh * cdiv(n_kv, cfg->block_kv) * d * 4);
  if (qbar_bytes + kbar_bytes > (size_t)HF_STATIC_SCRATCH_BYTES) {
    set_error("hf_block_select_static: these sizes need %zu bytes of scratch, the built-in buffer holds %zu "
              "(use hf_block_select with a workspace)", qbar_bytes + kbar_bytes, (size_t)HF_STATIC_SCRATCH_BYTES);
    return HF_ERR_WORKSPACE;
  }
  unsigned char* base = nullptr;
  HF_TRY(static_scratch(&base));
  // nothing has to start at zero: the pooling kernel writes every mean before the ranking kernel reads it
  return select_launches(cfg, Q, n_q, K_win, n_kv, 0, k, block_idx, scores_or_null, reinterpret_cast<float*>(base),
                         reinterpret_cast<float*>(base + qbar_bytes), static_cast<hipStream_t>(stream));
}

int hf_hybrid_attn_fwd(const hf_config* cfg, const void* Q, int32_t n_q, const void* K_win,
                       const void* V_win, int32_t n_kv, const int32_t* block_idx, int32_t k,
                       const void* state_or_null, const float* rope_cos_q, const float* rope_sin_q,
                       void* O, void* workspace, size_t workspace_bytes, void* stream) {
  return hf_hybrid_attn_fwd_split(cfg, Q, Q, n_q, K_win, V_win, n_kv, block_idx, k, state_or_null, rope_cos_q,
                                  rope_sin_q, O, workspace, workspace_bytes, stream);
}

// the forward call; save = the training forward, which also writes O_local and the softmax row statistic
static int fwd_impl(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q, const void* K_win,
                    const void* V_win, int32_t n_kv, const int32_t* block_idx, int32_t k, const void* state_or_null,
                    const float* rope_cos_q, const float* rope_sin_q, void* O, bool save, void* O_local_out,
                    float* lse2_out, void* workspace, size_t workspace_bytes, void* stream,
                    const void* planes_in = nullptr);

int hf_hybrid_attn_fwd_split(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q,
                             const void* K_win, const void* V_win, int32_t n_kv, const int32_t* block_idx,
                             int32_t k, const void* state_or_null, const float* rope_cos_q,
                             const float* rope_sin_q, void* O, void* workspace, size_t workspace_bytes,
                             void* stream) {
  return fwd_impl(cfg, Q, Q_hist, n_q, K_win, V_win, n_kv, block_idx, k, state_or_null, rope_cos_q, rope_sin_q, O,
                  false, nullptr, nullptr, workspace, workspace_bytes, stream);
}

int hf_hybrid_attn_fwd_planes(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q,
                              const void* K_win, const void* V_win, int32_t n_kv, const int32_t* block_idx,
                              int32_t k, const void* state, const void* planes, const float* rope_cos_q,
                              const float* rope_sin_q, void* O, void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ptr(state, "state", true));
  HF_TRY(check_planes_cfg(cfg, planes, "planes"));
  if (planes == O) { set_error("planes aliases O"); return HF_ERR_SHAPE; }
  return fwd_impl(cfg, Q, Q_hist, n_q, K_win, V_win, n_kv, block_idx, k, state, rope_cos_q, rope_sin_q, O, false,
                  nullptr, nullptr, nullptr, 0, stream, planes);
}

int hf_pooled_keys_bytes(const hf_config* cfg, int32_t n_kv, size_t* bytes_out) {
  HF_TRY(check_cfg(cfg));
  if (!bytes_out) { set_error("bytes_out is NULL"); return HF_ERR_NULL; }
  HF_TRY(check_tokens(n_kv, "n_kv"));
  *bytes_out = align256((size_t)cfg->batch * cfg->heads * cdiv(n_kv, cfg->block_kv) * cfg->head_dim * 4);
  return HF_OK;
}

int hf_pool_keys(const hf_config* cfg, const void* K_win, int32_t n_kv, int32_t n_cached_kv_blocks, void* pooled_K,
                 void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ptr(K_win, "K_win", true));
  HF_TRY(check_ptr(pooled_K, "pooled_K", true));
  HF_TRY(check_tokens(n_kv, "n_kv"));
  HF_TRY(check_window_len(cfg, n_kv));
  if (reinterpret_cast<uintptr_t>(pooled_K) & 255u) { set_error("pooled_K is not 256-byte aligned"); return HF_ERR_ALIGN; }
  if (n_cached_kv_blocks < 0 || n_cached_kv_blocks > n_kv / cfg->block_kv) {
    set_error("n_cached_kv_blocks=%d outside [0, %d] (whole KV blocks of the window)", n_cached_kv_blocks,
              n_kv / cfg->block_kv);
    return HF_ERR_SHAPE;
  }
  const int t_n = cdiv(n_kv, cfg->block_kv);
  if (n_cached_kv_blocks == t_n) return HF_OK;   // nothing new to pool
  // the pooling kernel with no query blocks: KV blocks [n_cached_kv_blocks, T_n)
  return launch_pool_both(*cfg, nullptr, 0, 0, K_win, n_kv, t_n, n_cached_kv_blocks, t_n, nullptr,
                          static_cast<float*>(pooled_K), static_cast<hipStream_t>(stream));
}

// the selecting launch; K_ev given: with workgroups that absorb those tokens into state_out / planes_out
static int select_attn_impl(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q, const void* K_win,
                            const void* V_win, int32_t n_kv, const void* pooled_K, const void* state_or_null,
                            const void* planes, const float* rope_cos_q, const float* rope_sin_q, void* O,
                            int32_t* block_idx_out, float* scores_or_null, const void* K_ev, const void* V_ev,
                            int32_t n_ev, int32_t ev_stride, void* state_out, void* planes_out, void* workspace,
                            size_t workspace_bytes, void* stream) {
  HF_TRY(check_cfg(cfg));
  if (!attn_mfma_fused_supported(*cfg)) {
    set_error("selection inside the attention launch covers bf16, head_dim 128, block_q 64 or 128 "
              "(use hf_block_select + hf_hybrid_attn_fwd)");
    return HF_ERR_SHAPE;
  }
  HF_TRY(check_ptr(Q, "Q", true));
  if (!Q_hist) Q_hist = Q;
  HF_TRY(check_ptr(Q_hist, "Q_hist", true));
  HF_TRY(check_ptr(K_win, "K_win", true));
  HF_TRY(check_ptr(V_win, "V_win", true));
  HF_TRY(check_ptr(pooled_K, "pooled_K", true));
  HF_TRY(check_ptr(rope_cos_q, "rope_cos_q", false));
  HF_TRY(check_ptr(rope_sin_q, "rope_sin_q", false));
  HF_TRY(check_ptr(O, "O", true));
  HF_TRY(check_ptr(block_idx_out, "block_idx_out", true));
  HF_TRY(check_ptr(scores_or_null, "scores", false));
  HF_TRY(check_tokens(n_q, "n_q"));
  HF_TRY(check_tokens(n_kv, "n_kv"));
  HF_TRY(check_window_len(cfg, n_kv));
  if (reinterpret_cast<uintptr_t>(pooled_K) & 255u) { set_error("pooled_K is not 256-byte aligned"); return HF_ERR_ALIGN; }
  if (O == Q || O == Q_hist || O == K_win || O == V_win || O == pooled_K || static_cast<void*>(block_idx_out) == O) {
    set_error("O / block_idx_out alias another argument");
    return HF_ERR_SHAPE;
  }
  if ((rope_cos_q == nullptr) != (rope_sin_q == nullptr)) {
    set_error("rope_cos_q and rope_sin_q must both be given or both be NULL");
    return HF_ERR_NULL;
  }
  const int t_n = cdiv(n_kv, cfg->block_kv);
  if (t_n > kMaxFusedSelectBlocks) {
    set_error("window has %d KV blocks; the attention kernel selects among at most %d (use hf_block_select)", t_n,
              kMaxFusedSelectBlocks);
    return HF_ERR_SHAPE;
  }
  const int k = select_k_of(cfg, t_n);
  if (k > t_n) { set_error("keep_k=%d exceeds the %d KV blocks of the window", k, t_n); return HF_ERR_SHAPE; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const float* kbar = static_cast<const float*>(pooled_K);
  const float* st = static_cast<const float*>(state_or_null);
  const size_t d = cfg->head_dim, bh = (size_t)cfg->batch * cfg->heads;
  if (st) {
    HF_TRY(check_planes_cfg(cfg, planes, "planes"));
    if (planes == O) { set_error("planes aliases O"); return HF_ERR_SHAPE; }
  }
  if (!K_ev) {
    if (!st) return launch_attn_mfma_select(*cfg, Q, n_q, K_win, V_win, n_kv, k, kbar, block_idx_out, scores_or_null, O, s);
    return launch_attn_mfma_fused(*cfg, Q, n_q, K_win, V_win, n_kv, nullptr, k, planes, st + bh * d * d, rope_cos_q,
                                  rope_sin_q, Q_hist, O, s, nullptr, nullptr, kbar, block_idx_out, scores_or_null);
  }
  // ---- with the absorbing workgroups
  HF_TRY(check_ptr(V_ev, "V_ev", true));
  HF_TRY(check_ptr(state_out, "state_out", true));
  HF_TRY(check_tokens(n_ev, "n_ev"));
  if (cfg->phi != HF_PHI_RELU) {
    set_error("hf_step_fwd absorbs with phi = ReLU and no rotation only (use hf_absorb_evicted)");
    return HF_ERR_SHAPE;
  }
  if (ev_stride == 0) ev_stride = n_ev;
  if (ev_stride < n_ev) { set_error("ev_stride=%d is less than n_ev=%d", ev_stride, n_ev); return HF_ERR_SHAPE; }
  if ((size_t)n_ev * d * 2 >= (1ull << 31)) { set_error("n_ev=%d tokens per head exceed the 2 GiB a descriptor spans", n_ev); return HF_ERR_SHAPE; }
  if (planes_out) HF_TRY(check_planes_cfg(cfg, planes_out, "planes_out"));
  const size_t state_bytes = bh * (d * d + d) * sizeof(float), planes_bytes = readout_planes_bytes(*cfg);
  auto overlap = [](const void* a, size_t an, const void* b, size_t bn) {
    const char* x = static_cast<const char*>(a);
    const char* y = static_cast<const char*>(b);
    return a && b && x < y + bn && y < x + an;
  };
  if (overlap(state_out, state_bytes, state_or_null, state_bytes) || overlap(planes_out, planes_bytes, planes, planes_bytes) ||
      overlap(state_out, state_bytes, planes, planes_bytes) || overlap(planes_out, planes_bytes, state_or_null, state_bytes) ||
      overlap(state_out, state_bytes, planes_out, planes_bytes) || state_out == O || planes_out == O ||
      state_out == workspace || planes_out == workspace) {
    set_error("state_out / planes_out overlap another argument (the attention of this launch still reads the old state)");
    return HF_ERR_SHAPE;
  }
  const size_t need = step_absorb_workspace_bytes(*cfg, n_q, n_ev);
  if (!workspace || workspace_bytes < need) {
    set_error("workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
    return HF_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) { set_error("workspace is not 256-byte aligned"); return HF_ERR_ALIGN; }
  const float* st_in = st;
  if (!st_in) {
    // no state yet: the absorbed tokens start from zero
    HF_TRY(launch_fill_zero(static_cast<float*>(state_out), bh * (d * d + d), s));
    st_in = static_cast<const float*>(state_out);   // (every element is read and written by the same thread)
  }
  return launch_attn_mfma_step(*cfg, Q, n_q, K_win, V_win, n_kv, k, kbar, block_idx_out, scores_or_null,
                               st ? planes : nullptr, st ? st + bh * d * d : nullptr, rope_cos_q, rope_sin_q, Q_hist, O,
                               K_ev, V_ev, n_ev, ev_stride, st_in, static_cast<float*>(state_out), planes_out, workspace, s);
}

int hf_select_attn_fwd(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q, const void* K_win,
                       const void* V_win, int32_t n_kv, const void* pooled_K, const void* state_or_null,
                       const void* planes, const float* rope_cos_q, const float* rope_sin_q, void* O,
                       int32_t* block_idx_out, float* scores_or_null, void* stream) {
  return select_attn_impl(cfg, Q, Q_hist, n_q, K_win, V_win, n_kv, pooled_K, state_or_null, planes, rope_cos_q, rope_sin_q,
                          O, block_idx_out, scores_or_null, nullptr, nullptr, 0, 0, nullptr, nullptr, nullptr, 0, stream);
}

int hf_step_workspace_bytes(const hf_config* cfg, int32_t n_q, int32_t n_ev, size_t* bytes_out) {
  HF_TRY(check_cfg(cfg));
  if (!bytes_out) { set_error("bytes_out is NULL"); return HF_ERR_NULL; }
  HF_TRY(check_tokens(n_q, "n_q"));
  HF_TRY(check_tokens(n_ev, "n_ev"));
  *bytes_out = attn_mfma_fused_supported(*cfg) ? step_absorb_workspace_bytes(*cfg, n_q, n_ev) : 0;
  return HF_OK;
}

int hf_step_fwd(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q, const void* K_win,
                const void* V_win, int32_t n_kv, const void* pooled_K, const void* state_in, const void* planes,
                const float* rope_cos_q, const float* rope_sin_q, void* O, int32_t* block_idx_out,
                float* scores_or_null, const void* K_ev, const void* V_ev, int32_t n_ev, int32_t ev_stride,
                void* state_out, void* planes_out, void* workspace, size_t workspace_bytes, void* stream) {
  HF_TRY(check_ptr(K_ev, "K_ev", true));
  return select_attn_impl(cfg, Q, Q_hist, n_q, K_win, V_win, n_kv, pooled_K, state_in, planes, rope_cos_q, rope_sin_q, O,
                          block_idx_out, scores_or_null, K_ev, V_ev, n_ev, ev_stride, state_out, planes_out, workspace,
                          workspace_bytes, stream);
}

int hf_hybrid_attn_fwd_save(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q,
                            const void* K_win, const void* V_win, int32_t n_kv, const int32_t* block_idx,
                            int32_t k, const void* state_or_null, const float* rope_cos_q,
                            const float* rope_sin_q, void* O, void* O_local_out, float* lse2_out, void* workspace,
                            size_t workspace_bytes, void* stream) {
  return fwd_impl(cfg, Q, Q_hist, n_q, K_win, V_win, n_kv, block_idx, k, state_or_null, rope_cos_q, rope_sin_q, O,
                  true, O_local_out, lse2_out, workspace, workspace_bytes, stream);
}

static int fwd_impl(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q, const void* K_win,
                    const void* V_win, int32_t n_kv, const int32_t* block_idx, int32_t k, const void* state_or_null,
                    const float* rope_cos_q, const float* rope_sin_q, void* O, bool save, void* O_local_out,
                    float* lse2_out, void* workspace, size_t workspace_bytes, void* stream, const void* planes_in) {
  HF_TRY(check_cfg(cfg));
  if (save) {
    HF_TRY(check_ptr(O_local_out, "O_local_out", true));
    HF_TRY(check_ptr(lse2_out, "lse2_out", true));
    if (!attn_mfma_fused_supported(*cfg)) {
      set_error("the saving forward covers bf16, head_dim 128, block_q 64 or 128 (hf_hybrid_attn_bwd recomputes instead)");
      return HF_ERR_SHAPE;
    }
    if (O_local_out == O || O_local_out == Q || O_local_out == Q_hist || O_local_out == K_win || O_local_out == V_win ||
        static_cast<void*>(lse2_out) == O || static_cast<void*>(lse2_out) == O_local_out) {
      set_error("O_local_out / lse2_out alias another argument");
      return HF_ERR_SHAPE;
    }
  }
  HF_TRY(check_ptr(Q, "Q", true));
  if (!Q_hist) Q_hist = Q;
  HF_TRY(check_ptr(Q_hist, "Q_hist", true));
  HF_TRY(check_ptr(K_win, "K_win", true));
  HF_TRY(check_ptr(V_win, "V_win", true));
  HF_TRY(check_ptr(O, "O", true));
  HF_TRY(check_ptr(block_idx, "block_idx", false));
  HF_TRY(check_ptr(state_or_null, "state", false));
  HF_TRY(check_tokens(n_q, "n_q"));
  HF_TRY(check_tokens(n_kv, "n_kv"));
  HF_TRY(check_window_len(cfg, n_kv));
  if (O == Q || O == Q_hist || O == K_win || O == V_win) { set_error("O must not alias an input"); return HF_ERR_SHAPE; }
  if ((rope_cos_q == nullptr) != (rope_sin_q == nullptr)) {
    set_error("rope_cos_q and rope_sin_q must both be given or both be NULL");
    return HF_ERR_NULL;
  }
  HF_TRY(check_ptr(rope_cos_q, "rope_cos_q", false));
  HF_TRY(check_ptr(rope_sin_q, "rope_sin_q", false));
  const int t_n = cdiv(n_kv, cfg->block_kv);
  if (block_idx) {
    if (k < 1 || k > t_n) { set_error("k=%d must be in [1, %d]", k, t_n); return HF_ERR_SHAPE; }
  } else {
    k = t_n;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!state_or_null) {
    // no history yet: O = O_local, written directly
    if (!save) return launch_attn(*cfg, Q, n_q, K_win, V_win, n_kv, block_idx, k, O, s);
    HF_TRY(launch_attn_mfma_lse(*cfg, Q, n_q, K_win, V_win, n_kv, block_idx, k, O, lse2_out, s));
    const size_t bytes = (size_t)cfg->batch * cfg->heads * n_q * cfg->head_dim * esize(cfg);
    if (hipMemcpyAsync(O_local_out, O, bytes, hipMemcpyDeviceToDevice, s) != hipSuccess) {
      set_error("copy of O into O_local_out: %s", hipGetErrorString(hipGetLastError()));
      return HF_ERR_HIP;
    }
    return HF_OK;
  }
  if (planes_in) {
    // the caller keeps the bf16 planes of the state (hf_absorb_evicted_planes): nothing to convert, no workspace
    const float* st = static_cast<const float*>(state_or_null);
    const size_t d = cfg->head_dim;
    return launch_attn_mfma_fused(*cfg, Q, n_q, K_win, V_win, n_kv, block_idx, k, planes_in,
                                  st + (size_t)cfg->batch * cfg->heads * d * d, rope_cos_q, rope_sin_q, Q_hist, O, s);
  }
  const WorkspaceLayout w = workspace_layout(cfg, n_q, n_kv);
  if (!workspace || workspace_bytes < w.total) {
    set_error("workspace of %zu bytes needed, %zu given", w.total, workspace ? workspace_bytes : (size_t)0);
    return HF_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) { set_error("workspace is not 256-byte aligned"); return HF_ERR_ALIGN; }
  if (attn_mfma_fused_supported(*cfg) && (save || !(cfg->flags & HF_FLAG_READOUT_KERNEL))) {
    // MFMA shapes: the history term is added in the attention kernel's epilogue
    char* planes = static_cast<char*>(workspace) + w.planes;
    const float* st = static_cast<const float*>(state_or_null);
    const size_t d = cfg->head_dim;
    HF_TRY(launch_state_planes(*cfg, st, planes, s));
    return launch_attn_mfma_fused(*cfg, Q, n_q, K_win, V_win, n_kv, block_idx, k, planes,
                                  st + (size_t)cfg->batch * cfg->heads * d * d, rope_cos_q, rope_sin_q, Q_hist, O, s,
                                  save ? lse2_out : nullptr, save ? O_local_out : nullptr);
  }
  void* o_local = static_cast<char*>(workspace) + w.olocal;
  HF_TRY(launch_attn(*cfg, Q, n_q, K_win, V_win, n_kv, block_idx, k, o_local, s));
  return launch_readout(*cfg, Q_hist, n_q, o_local, static_cast<const float*>(state_or_null), rope_cos_q,
                        rope_sin_q, static_cast<char*>(workspace) + w.planes, O, s);
}

int hf_stream_open_chunk(const hf_config* cfg, hf_window* win, int32_t n_chunk, void* K_win, void* V_win,
                         void* state, const float* rope_cos_ev, const float* rope_sin_ev, void* workspace,
                         size_t workspace_bytes, int32_t* first_out, int32_t* n_evicted_out, void* stream) {
  HF_TRY(check_cfg(cfg));
  if (!win) { set_error("win is NULL"); return HF_ERR_NULL; }
  if (cfg->kv_capacity < 1) { set_error("a stream needs cfg->kv_capacity"); return HF_ERR_SHAPE; }
  if (win->n_sink < 0 || win->n_tokens < win->n_sink || win->n_tokens > cfg->kv_capacity) {
    set_error("window bookkeeping out of range: n_sink=%d n_tokens=%d capacity=%d", win->n_sink, win->n_tokens,
              cfg->kv_capacity);
    return HF_ERR_SHAPE;
  }
  HF_TRY(check_tokens(n_chunk, "n_chunk"));
  if (n_chunk > cfg->kv_capacity - win->n_sink) {
    set_error("a chunk of %d tokens does not fit behind %d sink tokens in %d", n_chunk, win->n_sink, cfg->kv_capacity);
    return HF_ERR_SHAPE;
  }
  const int32_t over = win->n_tokens + n_chunk - cfg->kv_capacity;
  if (over > 0) {
    // "KV cache is full": pop the oldest tokens behind the sink and update the linear state with them
    HF_TRY(hf_window_evict(cfg, K_win, V_win, win->n_tokens, win->n_sink, over, state, rope_cos_ev, rope_sin_ev,
                           workspace, workspace_bytes, stream));
    win->n_tokens -= over;
  }
  if (first_out) *first_out = win->n_tokens;
  if (n_evicted_out) *n_evicted_out = over > 0 ? over : 0;
  win->n_tokens += n_chunk;
  return HF_OK;
}

// One denoising step of a streaming driver where the attention kernel can select for itself (bf16, head_dim 128,
// block_q 64 or 128, at most kMaxFusedSelectBlocks KV blocks, default flags): the KV blocks [kv_first, kv_end) are
// pooled into the workspace (the others keep the means of the chunk's earlier steps), the state's planes are
// converted on the chunk's first step and reused afterwards, and ONE launch selects, attends and adds the history
// term.  Returns HF_OK with *done = false where this path does not apply (the caller takes the separate calls).
static int step_one_launch(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q, const void* K,
                           const void* V, int32_t n_kv, int kv_first, int kv_end, int32_t step_in_chunk,
                           int32_t* block_idx, const void* state_or_null, const float* rope_cos_q,
                           const float* rope_sin_q, void* O, void* workspace, size_t workspace_bytes, void* stream,
                           bool* done) {
  *done = false;
  const int t_m = cdiv(n_q, cfg->block_q), t_n = cdiv(n_kv, cfg->block_kv);
  (void)t_m;
  if (!attn_mfma_fused_supported(*cfg) || (cfg->flags & HF_FLAG_READOUT_KERNEL) || t_n > kMaxFusedSelectBlocks) return HF_OK;
  int k = 0;
  HF_TRY(check_select_args(cfg, Q, n_q, K, n_kv, 0, block_idx, nullptr, &k));
  HF_TRY(check_ptr(V, "V_win", true));
  HF_TRY(check_ptr(O, "O", true));
  if (!Q_hist) Q_hist = Q;
  if (O == Q || O == Q_hist || O == K || O == V) { set_error("O must not alias an input"); return HF_ERR_SHAPE; }
  if ((rope_cos_q == nullptr) != (rope_sin_q == nullptr)) {
    set_error("rope_cos_q and rope_sin_q must both be given or both be NULL");
    return HF_ERR_NULL;
  }
  const WorkspaceLayout w = workspace_layout(cfg, n_q, n_kv);
  if (!workspace || workspace_bytes < w.total) {
    set_error("workspace of %zu bytes needed, %zu given", w.total, workspace ? workspace_bytes : (size_t)0);
    return HF_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) { set_error("workspace is not 256-byte aligned"); return HF_ERR_ALIGN; }
  char* ws = static_cast<char*>(workspace);
  float* kbar = reinterpret_cast<float*>(ws + w.kbar);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (kv_end > kv_first)
    HF_TRY(launch_pool_both(*cfg, nullptr, 0, 0, K, n_kv, t_n, kv_first, kv_end, nullptr, kbar, s));
  *done = true;
  if (!state_or_null) return launch_attn_mfma_select(*cfg, Q, n_q, K, V, n_kv, k, kbar, block_idx, nullptr, O, s);
  const float* st = static_cast<const float*>(state_or_null);
  const size_t d = cfg->head_dim;
  // the state is frozen during a chunk's denoising steps: its planes are converted on the first and stay here
  if (step_in_chunk == 0) HF_TRY(launch_state_planes(*cfg, st, ws + w.planes, s));
  return launch_attn_mfma_fused(*cfg, Q, n_q, K, V, n_kv, nullptr, k, ws + w.planes,
                                st + (size_t)cfg->batch * cfg->heads * d * d, rope_cos_q, rope_sin_q, Q_hist, O, s, nullptr,
                                nullptr, kbar, block_idx, nullptr);
}

int hf_stream_step(const hf_config* cfg, const hf_window* win, const void* Q, const void* Q_hist, int32_t n_q,
                   const void* K_win, const void* V_win, int32_t step_in_chunk, int32_t* block_idx,
                   const void* state_or_null, const float* rope_cos_q, const float* rope_sin_q, void* O,
                   void* workspace, size_t workspace_bytes, void* stream) {
  HF_TRY(check_cfg(cfg));
  if (!win) { set_error("win is NULL"); return HF_ERR_NULL; }
  if (win->n_tokens < n_q || n_q < 1) {
    set_error("the window holds %d tokens, fewer than the chunk's %d", win->n_tokens, n_q);
    return HF_ERR_SHAPE;
  }
  if (step_in_chunk < 0) { set_error("step_in_chunk must be >= 0"); return HF_ERR_SHAPE; }
  const int32_t n_kv = win->n_tokens;
  // the chunk's own keys are the last n_q tokens; whole blocks before them are as the chunk's first step left them
  const int32_t reuse = step_in_chunk > 0 ? (n_kv - n_q) / cfg->block_kv : 0;
  HF_TRY(check_tokens(n_kv, "n_kv"));
  HF_TRY(check_window_len(cfg, n_kv));
  bool done = false;
  HF_TRY(step_one_launch(cfg, Q, Q_hist, n_q, K_win, V_win, n_kv, reuse, cdiv(n_kv, cfg->block_kv), step_in_chunk, block_idx,
                         state_or_null, rope_cos_q, rope_sin_q, O, workspace, workspace_bytes, stream, &done));
  if (done) return HF_OK;
  HF_TRY(hf_block_select_cached(cfg, Q, n_q, K_win, n_kv, reuse, block_idx, nullptr, workspace, workspace_bytes,
                                stream));
  const int32_t k = select_k_of(cfg, cdiv(n_kv, cfg->block_kv));
  if (step_in_chunk > 0 && state_or_null && attn_mfma_fused_supported(*cfg) && !(cfg->flags & HF_FLAG_READOUT_KERNEL)) {
    // the state is frozen during a chunk's denoising steps: its bf16 planes are as the chunk's first step left them
    // in this workspace (which hf_block_select_cached has just checked for size and alignment)
    const WorkspaceLayout w = workspace_layout(cfg, n_q, n_kv);
    return fwd_impl(cfg, Q, Q_hist, n_q, K_win, V_win, n_kv, block_idx, k, state_or_null, rope_cos_q, rope_sin_q, O,
                    false, nullptr, nullptr, nullptr, 0, stream, static_cast<char*>(workspace) + w.planes);
  }
  return hf_hybrid_attn_fwd_split(cfg, Q, Q_hist, n_q, K_win, V_win, n_kv, block_idx, k, state_or_null, rope_cos_q,
                                  rope_sin_q, O, workspace, workspace_bytes, stream);
}

static int check_ring(const hf_config* cfg, const hf_ring* r) {
  if (!r) { set_error("ring is NULL"); return HF_ERR_NULL; }
  if (cfg->kv_capacity < 1) { set_error("a ring needs cfg->kv_capacity"); return HF_ERR_SHAPE; }
  if (r->n_sink < 0 || r->n_chunk < 1 || r->n_sink + r->n_chunk > cfg->kv_capacity ||
      (cfg->kv_capacity - r->n_sink) % r->n_chunk != 0) {
    set_error("ring: kv_capacity - n_sink = %d must be a positive multiple of n_chunk = %d", cfg->kv_capacity - r->n_sink,
              r->n_chunk);
    return HF_ERR_SHAPE;
  }
  const int slots = (cfg->kv_capacity - r->n_sink) / r->n_chunk;
  if (r->n_filled < 0 || r->n_filled > slots || r->next_slot < 0 || r->next_slot >= slots || r->cur_slot < -1 ||
      r->cur_slot >= slots || (r->n_filled < slots && r->next_slot != r->n_filled) ||
      (r->absorbed_ahead != 0 && r->absorbed_ahead != 1)) {
    set_error("ring bookkeeping out of range: n_filled=%d next_slot=%d cur_slot=%d of %d slots", r->n_filled, r->next_slot,
              r->cur_slot, slots);
    return HF_ERR_SHAPE;
  }
  return HF_OK;
}

int hf_ring_open_chunk(const hf_config* cfg, hf_ring* ring, void* K_cache, void* V_cache, void* state,
                       const float* rope_cos_ev, const float* rope_sin_ev, void* workspace, size_t workspace_bytes,
                       int32_t* first_out, int32_t* n_evicted_out, void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ring(cfg, ring));
  HF_TRY(check_ptr(K_cache, "K_cache", true));
  HF_TRY(check_ptr(V_cache, "V_cache", true));
  const int slots = (cfg->kv_capacity - ring->n_sink) / ring->n_chunk;
  const int32_t first = ring->n_sink + ring->next_slot * ring->n_chunk;
  int32_t evicted = 0;
  if (ring->n_filled == slots && ring->absorbed_ahead) {
    // the last step of the chunk before has absorbed the slot's chunk already (hf_ring_last_step)
    ring->absorbed_ahead = 0;
    evicted = ring->n_chunk;
  } else if (ring->n_filled == slots) {
    // "KV cache is full": the chunk in the slot about to be reused is the oldest; it goes into the linear state
    // where it lies, and nothing else in the cache moves
    HF_TRY(check_ptr(state, "state", true));
    if ((rope_cos_ev == nullptr) != (rope_sin_ev == nullptr)) {
      set_error("rope_cos_ev and rope_sin_ev must both be given or both be NULL");
      return HF_ERR_NULL;
    }
    HF_TRY(check_ptr(rope_cos_ev, "rope_cos_ev", false));
    HF_TRY(check_ptr(rope_sin_ev, "rope_sin_ev", false));
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u)) {
      set_error("workspace is not 256-byte aligned");
      return HF_ERR_ALIGN;
    }
    const size_t skip = (size_t)first * cfg->head_dim * esize(cfg);
    HF_TRY(launch_absorb(*cfg, static_cast<float*>(state), static_cast<char*>(K_cache) + skip,
                         static_cast<char*>(V_cache) + skip, ring->n_chunk, cfg->kv_capacity, rope_cos_ev, rope_sin_ev,
                         workspace, workspace ? workspace_bytes : 0, static_cast<hipStream_t>(stream)));
    evicted = ring->n_chunk;
  } else {
    ring->n_filled += 1;
  }
  ring->cur_slot = ring->next_slot;
  ring->next_slot = (ring->next_slot + 1) % slots;
  if (first_out) *first_out = first;
  if (n_evicted_out) *n_evicted_out = evicted;
  return HF_OK;
}

int hf_ring_step(const hf_config* cfg, const hf_ring* ring, const void* Q, const void* Q_hist, const void* K_cache,
                 const void* V_cache, int32_t step_in_chunk, int32_t* block_idx, const void* state_or_null,
                 const float* rope_cos_q, const float* rope_sin_q, void* O, void* workspace, size_t workspace_bytes,
                 void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ring(cfg, ring));
  if (ring->cur_slot < 0) { set_error("no chunk is open (hf_ring_open_chunk first)"); return HF_ERR_SHAPE; }
  if (step_in_chunk < 0) { set_error("step_in_chunk must be >= 0"); return HF_ERR_SHAPE; }
  const int32_t n_q = ring->n_chunk, n_kv = ring->n_sink + ring->n_filled * ring->n_chunk;
  int k = 0;
  HF_TRY(check_select_args(cfg, Q, n_q, K_cache, n_kv, 0, block_idx, nullptr, &k));
  const WorkspaceLayout w = workspace_layout(cfg, n_q, n_kv);
  if (!workspace || workspace_bytes < w.total) {
    set_error("workspace of %zu bytes needed, %zu given", w.total, workspace ? workspace_bytes : (size_t)0);
    return HF_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) { set_error("workspace is not 256-byte aligned"); return HF_ERR_ALIGN; }
  // after the chunk's first step only the KV blocks that touch the chunk's own slot are pooled again
  const int t_n = cdiv(n_kv, cfg->block_kv);
  const int first = ring->n_sink + ring->cur_slot * ring->n_chunk;
  int kv_first = 0, kv_end = t_n;
  if (step_in_chunk > 0) {
    kv_first = first / cfg->block_kv;
    kv_end = cdiv(first + ring->n_chunk, cfg->block_kv);
    if (kv_end > t_n) kv_end = t_n;
  }
  bool done = false;
  HF_TRY(step_one_launch(cfg, Q, Q_hist, n_q, K_cache, V_cache, n_kv, kv_first, kv_end, step_in_chunk, block_idx,
                         state_or_null, rope_cos_q, rope_sin_q, O, workspace, workspace_bytes, stream, &done));
  if (done) return HF_OK;
  char* ws = static_cast<char*>(workspace);
  HF_TRY(select_launches(cfg, Q, n_q, K_cache, n_kv, kv_first, k, block_idx, nullptr, reinterpret_cast<float*>(ws + w.qbar),
                         reinterpret_cast<float*>(ws + w.kbar), static_cast<hipStream_t>(stream), kv_end));
  if (step_in_chunk > 0 && state_or_null && attn_mfma_fused_supported(*cfg) && !(cfg->flags & HF_FLAG_READOUT_KERNEL)) {
    // the state is frozen during a chunk's steps: its bf16 planes are as the chunk's first step left them here
    return fwd_impl(cfg, Q, Q_hist, n_q, K_cache, V_cache, n_kv, block_idx, k, state_or_null, rope_cos_q, rope_sin_q, O,
                    false, nullptr, nullptr, nullptr, 0, stream, ws + w.planes);
  }
  return hf_hybrid_attn_fwd_split(cfg, Q, Q_hist, n_q, K_cache, V_cache, n_kv, block_idx, k, state_or_null, rope_cos_q,
                                  rope_sin_q, O, workspace, workspace_bytes, stream);
}

int hf_ring_last_step(const hf_config* cfg, hf_ring* ring, const void* Q, const void* Q_hist, const void* K_cache,
                      const void* V_cache, int32_t step_in_chunk, int32_t* block_idx, const void* state_or_null,
                      const float* rope_cos_q, const float* rope_sin_q, void* O, void* workspace, size_t workspace_bytes,
                      void* state_out, const float* rope_cos_ev, const float* rope_sin_ev, void* step_workspace,
                      size_t step_workspace_bytes, int32_t* absorbed_out, void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ring(cfg, ring));
  if (ring->cur_slot < 0) { set_error("no chunk is open (hf_ring_open_chunk first)"); return HF_ERR_SHAPE; }
  if (absorbed_out) *absorbed_out = 0;
  const int slots = (cfg->kv_capacity - ring->n_sink) / ring->n_chunk;
  if (ring->n_filled < slots || ring->absorbed_ahead) {
    // a slot is still free (or the chunk is in the state already): the next chunk evicts nothing more
    return hf_ring_step(cfg, ring, Q, Q_hist, K_cache, V_cache, step_in_chunk, block_idx, state_or_null, rope_cos_q,
                        rope_sin_q, O, workspace, workspace_bytes, stream);
  }
  HF_TRY(check_ptr(state_out, "state_out", true));
  HF_TRY(check_ptr(K_cache, "K_cache", true));
  HF_TRY(check_ptr(V_cache, "V_cache", true));
  if ((rope_cos_ev == nullptr) != (rope_sin_ev == nullptr)) {
    set_error("rope_cos_ev and rope_sin_ev must both be given or both be NULL");
    return HF_ERR_NULL;
  }
  if (step_workspace && (reinterpret_cast<uintptr_t>(step_workspace) & 255u)) {
    set_error("step_workspace is not 256-byte aligned");
    return HF_ERR_ALIGN;
  }
  const int32_t n_q = ring->n_chunk, n_kv = ring->n_sink + ring->n_filled * ring->n_chunk;
  const size_t d = cfg->head_dim, bh = (size_t)cfg->batch * cfg->heads;
  const size_t state_bytes = bh * (d * d + d) * sizeof(float);
  {
    const char* a = static_cast<const char*>(state_out);
    const char* b = static_cast<const char*>(state_or_null);
    if (b && a < b + state_bytes && b < a + state_bytes) { set_error("state_out overlaps state"); return HF_ERR_SHAPE; }
  }
  // the chunk that the next hf_ring_open_chunk evicts: slot next_slot, where it lies
  const size_t skip = ((size_t)ring->n_sink + (size_t)ring->next_slot * ring->n_chunk) * d * esize(cfg);
  const char* K_ev = static_cast<const char*>(K_cache) + skip;
  const char* V_ev = static_cast<const char*>(V_cache) + skip;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int t_n = cdiv(n_kv, cfg->block_kv);
  const bool fused = attn_mfma_fused_supported(*cfg) && !(cfg->flags & HF_FLAG_READOUT_KERNEL) && t_n <= kMaxFusedSelectBlocks &&
                     cfg->phi == HF_PHI_RELU && !rope_cos_ev;
  if (fused) {
    // as step_one_launch (pool what changed, planes of the frozen state on the chunk's first step), then the
    // launch that selects, attends, adds the history term and absorbs
    int k = 0;
    HF_TRY(check_select_args(cfg, Q, n_q, K_cache, n_kv, 0, block_idx, nullptr, &k));
    const WorkspaceLayout w = workspace_layout(cfg, n_q, n_kv);
    if (!workspace || workspace_bytes < w.total) {
      set_error("workspace of %zu bytes needed, %zu given", w.total, workspace ? workspace_bytes : (size_t)0);
      return HF_ERR_WORKSPACE;
    }
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) { set_error("workspace is not 256-byte aligned"); return HF_ERR_ALIGN; }
    char* ws = static_cast<char*>(workspace);
    float* kbar = reinterpret_cast<float*>(ws + w.kbar);
    const int first = ring->n_sink + ring->cur_slot * ring->n_chunk;
    int kv_first = 0, kv_end = t_n;
    if (step_in_chunk > 0) {
      kv_first = first / cfg->block_kv;
      kv_end = cdiv(first + ring->n_chunk, cfg->block_kv);
      if (kv_end > t_n) kv_end = t_n;
    }
    // (argument checks of the fused call first: nothing is launched if it is going to refuse)
    const size_t need = step_absorb_workspace_bytes(*cfg, n_q, ring->n_chunk);
    if (!step_workspace || step_workspace_bytes < need) {
      set_error("step_workspace of %zu bytes needed, %zu given", need, step_workspace ? step_workspace_bytes : (size_t)0);
      return HF_ERR_WORKSPACE;
    }
    HF_TRY(launch_pool_both(*cfg, nullptr, 0, 0, K_cache, n_kv, t_n, kv_first, kv_end, nullptr, kbar, s));
    if (state_or_null && step_in_chunk == 0)
      HF_TRY(launch_state_planes(*cfg, static_cast<const float*>(state_or_null), ws + w.planes, s));
    HF_TRY(select_attn_impl(cfg, Q, Q_hist, n_q, K_cache, V_cache, n_kv, kbar, state_or_null,
                            state_or_null ? ws + w.planes : nullptr, rope_cos_q, rope_sin_q, O, block_idx, nullptr, K_ev, V_ev,
                            ring->n_chunk, cfg->kv_capacity, state_out, nullptr, step_workspace, step_workspace_bytes, stream));
  } else {
    HF_TRY(hf_ring_step(cfg, ring, Q, Q_hist, K_cache, V_cache, step_in_chunk, block_idx, state_or_null, rope_cos_q,
                        rope_sin_q, O, workspace, workspace_bytes, stream));
    // the state is copied and the chunk absorbed into the copy, behind the step
    if (state_or_null) {
      if (hipMemcpyAsync(state_out, state_or_null, state_bytes, hipMemcpyDeviceToDevice, s) != hipSuccess) {
        set_error("copy of the state: %s", hipGetErrorString(hipGetLastError()));
        return HF_ERR_HIP;
      }
    } else {
      HF_TRY(launch_fill_zero(static_cast<float*>(state_out), bh * (d * d + d), s));
    }
    HF_TRY(launch_absorb(*cfg, static_cast<float*>(state_out), K_ev, V_ev, ring->n_chunk, cfg->kv_capacity, rope_cos_ev,
                         rope_sin_ev, step_workspace, step_workspace ? step_workspace_bytes : 0, s));
  }
  ring->absorbed_ahead = 1;
  if (absorbed_out) *absorbed_out = 1;
  return HF_OK;
}

int hf_bwd_workspace_bytes(const hf_config* cfg, int32_t n_q, int32_t n_kv, size_t* bytes_out) {
  HF_TRY(check_cfg(cfg));
  if (!bytes_out) { set_error("bytes_out is NULL"); return HF_ERR_NULL; }
  HF_TRY(check_tokens(n_q, "n_q"));
  HF_TRY(check_tokens(n_kv, "n_kv"));
  *bytes_out = bwd_layout(cfg, n_q, n_kv).total;
  return HF_OK;
}

// the backward call; saved = O_local and lse2 of hf_hybrid_attn_fwd_save instead of a recomputed forward pass
static int bwd_impl(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q, const void* K_win,
                    const void* V_win, int32_t n_kv, const int32_t* block_idx, int32_t k, const void* state_or_null,
                    const float* rope_cos_q, const float* rope_sin_q, const void* dO, bool saved, const void* O_local,
                    const float* lse2_saved, void* dQ, void* dQ_hist, void* dK, void* dV, void* workspace,
                    size_t workspace_bytes, void* stream);

int hf_hybrid_attn_bwd(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q, const void* K_win,
                       const void* V_win, int32_t n_kv, const int32_t* block_idx, int32_t k,
                       const void* state_or_null, const float* rope_cos_q, const float* rope_sin_q, const void* dO,
                       void* dQ, void* dQ_hist, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                       void* stream) {
  return bwd_impl(cfg, Q, Q_hist, n_q, K_win, V_win, n_kv, block_idx, k, state_or_null, rope_cos_q, rope_sin_q, dO,
                  false, nullptr, nullptr, dQ, dQ_hist, dK, dV, workspace, workspace_bytes, stream);
}

int hf_hybrid_attn_bwd_saved(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q,
                             const void* K_win, const void* V_win, int32_t n_kv, const int32_t* block_idx,
                             int32_t k, const void* state_or_null, const float* rope_cos_q,
                             const float* rope_sin_q, const void* dO, const void* O_local, const float* lse2,
                             void* dQ, void* dQ_hist, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                             void* stream) {
  return bwd_impl(cfg, Q, Q_hist, n_q, K_win, V_win, n_kv, block_idx, k, state_or_null, rope_cos_q, rope_sin_q, dO,
                  true, O_local, lse2, dQ, dQ_hist, dK, dV, workspace, workspace_bytes, stream);
}

static int bwd_impl(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q, const void* K_win,
                    const void* V_win, int32_t n_kv, const int32_t* block_idx, int32_t k, const void* state_or_null,
                    const float* rope_cos_q, const float* rope_sin_q, const void* dO, bool saved, const void* O_local,
                    const float* lse2_saved, void* dQ, void* dQ_hist, void* dK, void* dV, void* workspace,
                    size_t workspace_bytes, void* stream) {
  HF_TRY(check_cfg(cfg));
  if (saved) {
    HF_TRY(check_ptr(O_local, "O_local", true));
    HF_TRY(check_ptr(lse2_saved, "lse2", true));
    if (!bwd_mfma_supported(*cfg)) {
      set_error("saved statistics cover bf16, head_dim 128, block_q 64 or 128 (hf_hybrid_attn_bwd recomputes instead)");
      return HF_ERR_SHAPE;
    }
  }
  HF_TRY(check_ptr(Q, "Q", true));
  if (!Q_hist) Q_hist = Q;
  HF_TRY(check_ptr(Q_hist, "Q_hist", true));
  HF_TRY(check_ptr(K_win, "K_win", true));
  HF_TRY(check_ptr(V_win, "V_win", true));
  HF_TRY(check_ptr(dO, "dO", true));
  HF_TRY(check_ptr(dQ, "dQ", true));
  HF_TRY(check_ptr(dK, "dK", true));
  HF_TRY(check_ptr(dV, "dV", true));
  HF_TRY(check_ptr(block_idx, "block_idx", false));
  HF_TRY(check_ptr(state_or_null, "state", false));
  HF_TRY(check_tokens(n_q, "n_q"));
  HF_TRY(check_tokens(n_kv, "n_kv"));
  HF_TRY(check_window_len(cfg, n_kv));
  const bool split = Q_hist != Q;
  if (split && !dQ_hist) { set_error("dQ_hist is required when Q_hist is a tensor of its own"); return HF_ERR_NULL; }
  if (!split && dQ_hist) { set_error("dQ_hist must be NULL when one tensor feeds both branches"); return HF_ERR_SHAPE; }
  HF_TRY(check_ptr(dQ_hist, "dQ_hist", false));
  const void* ins[] = {Q, Q_hist, K_win, V_win, dO, O_local, lse2_saved};
  void* outs[] = {dQ, dK, dV, dQ_hist};
  for (int a = 0; a < 4; ++a) {
    if (!outs[a]) continue;
    for (const void* in : ins)
      if (outs[a] == in) { set_error("an output aliases an input"); return HF_ERR_SHAPE; }
    for (int b = a + 1; b < 4; ++b)
      if (outs[a] == outs[b]) { set_error("two outputs alias"); return HF_ERR_SHAPE; }
  }
  if ((rope_cos_q == nullptr) != (rope_sin_q == nullptr)) {
    set_error("rope_cos_q and rope_sin_q must both be given or both be NULL");
    return HF_ERR_NULL;
  }
  HF_TRY(check_ptr(rope_cos_q, "rope_cos_q", false));
  HF_TRY(check_ptr(rope_sin_q, "rope_sin_q", false));
  const int t_m = cdiv(n_q, cfg->block_q), t_n = cdiv(n_kv, cfg->block_kv);
  if (block_idx) {
    if (k < 1 || k > t_n) { set_error("k=%d must be in [1, %d]", k, t_n); return HF_ERR_SHAPE; }
  } else {
    k = t_n;
  }
  const BwdLayout w = bwd_layout(cfg, n_q, n_kv);
  if (!workspace || workspace_bytes < w.total) {
    set_error("workspace of %zu bytes needed, %zu given", w.total, workspace ? workspace_bytes : (size_t)0);
    return HF_ERR_WORKSPACE;
  }
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) { set_error("workspace is not 256-byte aligned"); return HF_ERR_ALIGN; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  float* lse2 = reinterpret_cast<float*>(ws + w.lse2);
  float* dvec = reinterpret_cast<float*>(ws + w.dvec);
  float* dqh32 = reinterpret_cast<float*>(ws + w.dqh32);
  int32_t* inv_cnt = block_idx ? reinterpret_cast<int32_t*>(ws + w.inv_cnt) : nullptr;
  int32_t* inv_list = block_idx ? reinterpret_cast<int32_t*>(ws + w.inv_list) : nullptr;
  const float* st = static_cast<const float*>(state_or_null);

  const bool mfma = bwd_mfma_supported(*cfg) && (saved || !(cfg->flags & HF_FLAG_BWD_FP32_KERNELS));
  if (split && !st) {
    const size_t bytes = (size_t)cfg->batch * cfg->heads * n_q * cfg->head_dim * esize(cfg);
    HF_TRY(launch_fill_zero(static_cast<float*>(dQ_hist), bytes / 4, s));
  }
  if (block_idx) HF_TRY(launch_invert_index(*cfg, block_idx, k, t_m, t_n, inv_cnt, inv_list, s));
  if (mfma) {
    // row statistics of the softmax and D = dO . O_local (unrounded) from a recomputed forward pass; the history
    // branch rides in the dQ kernel's epilogue
    const float* lse2_in = lse2;
    if (saved) {
      // D = dO . O_local from the saved (once rounded) O_local; the row statistic as saved
      HF_TRY(launch_row_dot(*cfg, dO, O_local, (long long)cfg->batch * cfg->heads * n_q, dvec, s));
      lse2_in = lse2_saved;
    } else {
      HF_TRY(launch_attn_mfma_stats(*cfg, Q, n_q, K_win, V_win, n_kv, block_idx, k, dO, lse2, dvec, s));
    }
    return launch_bwd_mfma(*cfg, Q, n_q, K_win, V_win, n_kv, block_idx, k, dO, lse2_in, dvec, inv_cnt, inv_list,
                           reinterpret_cast<int32_t*>(ws + w.order), st, rope_cos_q, rope_sin_q, Q_hist, ws + w.planes,
                           dQ, dQ_hist, dK, dV, s);
  }
  // history branch first: its gradient either is an output of its own or joins dQ before dQ's one rounding
  const float* add_to_dq = nullptr;
  if (st) {
    if (split) {
      HF_TRY(launch_bwd_hist_generic(*cfg, Q_hist, dO, st, n_q, rope_cos_q, rope_sin_q, dQ_hist, false, s));
    } else {
      HF_TRY(launch_bwd_hist_generic(*cfg, Q_hist, dO, st, n_q, rope_cos_q, rope_sin_q, dqh32, true, s));
      add_to_dq = dqh32;
    }
  }
  HF_TRY(launch_attn_generic(*cfg, Q, n_q, K_win, V_win, n_kv, block_idx, k, nullptr, s, lse2, dO, dvec));
  return launch_bwd_generic(*cfg, Q, n_q, K_win, V_win, n_kv, block_idx, k, dO, lse2, dvec, inv_cnt, inv_list,
                            add_to_dq, dQ, dK, dV, s);
}

int hf_rope_window_indices(int32_t i_newest, int32_t n_frames, int32_t t0, int32_t* idx_out) {
  if (!idx_out) { set_error("idx_out is NULL"); return HF_ERR_NULL; }
  if (n_frames < 1) { set_error("n_frames must be >= 1"); return HF_ERR_SHAPE; }
  const int64_t newest = i_newest <= t0 ? i_newest : t0;
  if (newest - (n_frames - 1) < INT32_MIN) { set_error("index out of range"); return HF_ERR_SHAPE; }
  for (int32_t delta = 0; delta < n_frames; ++delta) idx_out[n_frames - 1 - delta] = (int32_t)(newest - delta);
  return HF_OK;
}

int hf_rope_tables(const int32_t* frame_idx, int32_t n_frames, int32_t height, int32_t width, int32_t pairs_t,
                   int32_t pairs_h, int32_t pairs_w, double theta, int32_t temporal_only, float* cos_out,
                   float* sin_out, void* stream) {
  if (!frame_idx) { set_error("frame_idx is NULL"); return HF_ERR_NULL; }
  if (n_frames < 1 || n_frames > HF_ROPE_MAX_FRAMES) {
    set_error("n_frames must be in [1, %d], got %d", HF_ROPE_MAX_FRAMES, n_frames); return HF_ERR_SHAPE;
  }
  if (height < 1 || width < 1 || (int64_t)n_frames * height * width > (1 << 24)) {
    set_error("height and width must be >= 1 and n_frames*height*width <= 2^24"); return HF_ERR_SHAPE;
  }
  if (pairs_t < 0 || pairs_h < 0 || pairs_w < 0 || pairs_t + (int64_t)pairs_h + pairs_w < 1 ||
      pairs_t + (int64_t)pairs_h + pairs_w > HF_ROPE_MAX_PAIRS) {
    set_error("pairs_t + pairs_h + pairs_w must be in [1, %d]", HF_ROPE_MAX_PAIRS); return HF_ERR_SHAPE;
  }
  if (!(theta > 0.0) || !isfinite(theta)) { set_error("theta must be positive and finite"); return HF_ERR_SHAPE; }
  HF_TRY(check_ptr(cos_out, "cos_out", true));
  HF_TRY(check_ptr(sin_out, "sin_out", true));
  return launch_rope_tables(frame_idx, n_frames, height, width, pairs_t, pairs_h, pairs_w, theta, temporal_only,
                            cos_out, sin_out, static_cast<hipStream_t>(stream));
}

int hf_rope_append_keys(const hf_config* cfg, const void* K_new, int32_t n_new, const float* rope_cos,
                        const float* rope_sin, void* K_win, int32_t first, int32_t n_kv, void* pooled_K, void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ptr(K_new, "K_new", true));
  HF_TRY(check_ptr(K_win, "K_win", true));
  HF_TRY(check_ptr(pooled_K, "pooled_K", true));
  if ((rope_cos == nullptr) != (rope_sin == nullptr)) {
    set_error("rope_cos and rope_sin must both be given or both be NULL");
    return HF_ERR_NULL;
  }
  HF_TRY(check_ptr(rope_cos, "rope_cos", false));
  HF_TRY(check_ptr(rope_sin, "rope_sin", false));
  HF_TRY(check_tokens(n_new, "n_new"));
  HF_TRY(check_tokens(n_kv, "n_kv"));
  HF_TRY(check_window_len(cfg, n_kv));
  if (first < 0 || (long long)first + n_new > n_kv) {
    set_error("tokens %d .. %d lie outside the window of %d", first, first + n_new - 1, n_kv);
    return HF_ERR_SHAPE;
  }
  if (reinterpret_cast<uintptr_t>(pooled_K) & 255u) { set_error("pooled_K is not 256-byte aligned"); return HF_ERR_ALIGN; }
  const size_t bh = (size_t)cfg->batch * cfg->heads, row = (size_t)cfg->head_dim * esize(cfg);
  const char* a = static_cast<const char*>(K_new);
  const char* b = static_cast<const char*>(K_win);
  if (a < b + bh * kv_stride_of(*cfg, n_kv) * row && b < a + bh * n_new * row) {
    set_error("K_new overlaps K_win");
    return HF_ERR_SHAPE;
  }
  return launch_rope_append_pool(*cfg, K_new, n_new, rope_cos, rope_sin, K_win, first, n_kv, static_cast<float*>(pooled_K),
                                 static_cast<hipStream_t>(stream));
}

int hf_rope_apply(const hf_config* cfg, const void* X, int32_t n_tokens, const float* rope_cos,
                  const float* rope_sin, void* Y, void* stream) {
  HF_TRY(check_cfg(cfg));
  HF_TRY(check_ptr(X, "X", true));
  HF_TRY(check_ptr(Y, "Y", true));
  HF_TRY(check_ptr(rope_cos, "rope_cos", true));
  HF_TRY(check_ptr(rope_sin, "rope_sin", true));
  HF_TRY(check_tokens(n_tokens, "n_tokens"));
  if (X != Y) {
    const size_t bytes = (size_t)cfg->batch * cfg->heads * n_tokens * cfg->head_dim * esize(cfg);
    const char* a = static_cast<const char*>(X);
    const char* b = static_cast<const char*>(Y);
    if (a < b + bytes && b < a + bytes) { set_error("Y overlaps X without being X"); return HF_ERR_SHAPE; }
  }
  return launch_rope_apply(*cfg, X, n_tokens, rope_cos, rope_sin, Y, static_cast<hipStream_t>(stream));
}

}  // extern "C"
