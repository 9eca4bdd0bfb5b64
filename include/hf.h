/*
 * hf.h — C ABI of the MI355X (gfx950) hybrid-attention library.
 *
 * One per-chunk hybrid attention of the Hybrid Forcing streaming video transformer
 * (Sec. 3.2 of the paper): block-sparse softmax attention of the chunk's queries over
 * the sliding-window KV cache (Eq. 4, 5), a linear-attention readout from a compact
 * per-head state (Eq. 3), their sum (Eq. 6), and the absorption of tokens evicted from
 * the window into that state (Eq. 2; the eviction step of the rolling-KV-cache
 * inference algorithm in the supplement).
 *
 * Conventions shared by every call
 * --------------------------------
 *  - Every data pointer is a DEVICE pointer on the current HIP device unless it says
 *    "host".  `cfg`, `bytes_out`, `k_out` are HOST pointers.
 *  - The caller owns every buffer (inputs, outputs, state, workspace).  The library
 *    allocates nothing on the device, reads no environment variable and keeps no global
 *    state except a thread-local error string and once-per-device kernel attributes.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call
 *    only enqueues kernels on that stream: no call synchronises, none allocates.
 *  - Tensors are contiguous, head-major [batch, heads, tokens, head_dim] with head_dim
 *    innermost; dtype of Q, K, V, O is cfg->dtype (bf16 or fp32).  The linear state is
 *    ALWAYS fp32.  Data pointers must be 16-byte aligned.
 *  - Blocks are consecutive runs of block_q / block_kv tokens counted from token 0 of the
 *    buffer; the last block may be short (it is pooled over its real length and only its
 *    real keys take part).  T_m = ceil(n_q / block_q), T_n = ceil(n_kv / block_kv).
 *  - The window buffer holds [older cached tokens ... | current chunk]; sink frames are
 *    ordinary leading tokens.  There is no causal mask inside the window.
 *  - Return value: HF_OK (0) or a negative HF_ERR_* code; on error nothing was enqueued
 *    and hf_last_error() describes the problem.  No C++ exception crosses this boundary.
 *
 * State layout (fp32), for batch b and head h, with d = head_dim:
 *     L[b][h][i][j]   i = key feature, j = value feature     B*H*d*d floats
 *     z[b][h][i]      normaliser (the paper's H)             B*H*d floats, after all of L
 */
#ifndef HF_H_
#define HF_H_

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define HF_API __attribute__((visibility("default")))
#else
#define HF_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

enum { HF_BF16 = 0, HF_F32 = 1 };            /* hf_config.dtype */
enum { HF_PHI_RELU = 0, HF_PHI_ELU1 = 1 };   /* hf_config.phi: max(x,0) | elu(x)+1 */

/* hf_config.flags: choices between kernels that compute the same thing.  0 is the fast default; the other
 * settings exist so that every kernel can be reached, timed and checked through this interface (the library
 * reads no environment variable). */
enum {
  HF_FLAG_READOUT_KERNEL = 1,      /* history term (Eq. 3, 6) by a readout kernel of its own behind the attention
                                      kernel, instead of in that kernel's epilogue (bf16, head_dim 128, block_q
                                      64 / 128; elsewhere that is the only path anyway) */
  HF_FLAG_HISTORY_TWO_PLANES = 2,  /* the fused epilogue multiplies with both bf16 planes of L (high part and
                                      remainder, ~2^-17 relative) instead of the high plane alone (2^-9) */
  HF_FLAG_BWD_FP32_KERNELS = 4,    /* hf_hybrid_attn_bwd through the fp32-arithmetic kernels also where the
                                      matrix-core kernels apply */
  HF_FLAG_DKV_INDEX_ORDER = 8      /* dK / dV workgroups in index order instead of longest list first */
};

enum {
  HF_OK = 0,
  HF_ERR_NULL = -1,       /* a required pointer is NULL */
  HF_ERR_SHAPE = -2,      /* unsupported or inconsistent sizes */
  HF_ERR_DTYPE = -3,      /* unknown dtype / phi */
  HF_ERR_ALIGN = -4,      /* a data pointer is not 16-byte aligned */
  HF_ERR_WORKSPACE = -5,  /* workspace missing or too small */
  HF_ERR_HIP = -6         /* a kernel launch failed; text from the HIP runtime */
};

/* Problem statement of the paper's hybrid-attention algorithm: per-head Q, K, V in
 * R^{N x d}, state L in R^{d x d} and H in R^{1 x d}, block sizes b_q, b_kv, sparse Top K. */
typedef struct hf_config {
  int32_t batch;          /* >= 1 */
  int32_t heads;          /* >= 1 */
  int32_t head_dim;       /* 64 or 128 */
  int32_t dtype;          /* HF_BF16 | HF_F32: storage type of Q, K, V, O */
  int32_t block_q;        /* b_q  >= 1 */
  int32_t block_kv;       /* b_kv >= 1 */
  float   keep_ratio;     /* in (0, 1]; 1.0 keeps every block (dense window attention).  Read to 7 significant
                             decimal digits, so that 0.1f means 0.1 (and 0.1 * 10 blocks keeps 1, not 2) */
  int32_t keep_k;         /* > 0 overrides keep_ratio; 0: k = clamp(ceil(keep_ratio*T_n - 1e-9), 1, T_n) */
  int32_t phi;            /* HF_PHI_RELU (default) | HF_PHI_ELU1 */
  float   eps;            /* added to the readout denominator (Eq. 3); e.g. 1e-6 */
  float   z_scale;        /* multiplies phi(q).z at readout; 1.0 = plain sum normaliser */
  float   softmax_scale;  /* 0 means 1/sqrt(head_dim) (Eq. 5) */
  int32_t kv_capacity;    /* 0: the heads of K_win, V_win are packed, n_kv tokens apart.  > 0: they are the
                             heads of a cache buffer [B, H, kv_capacity, d] whose first n_kv <= kv_capacity
                             tokens are valid.  Applies to every K_win / V_win argument, to nothing else. */
  int32_t flags;          /* bitwise OR of HF_FLAG_*; 0 = defaults */
} hf_config;

/* Size in bytes of the linear state: batch*heads*(d*d + d)*4.  Host-only. */
HF_API int hf_state_bytes(const hf_config* cfg, size_t* bytes_out);

/* "Initialize Linear State cache" of the inference algorithm: L = 0, z = 0.
 * Uses a fill kernel (not a memset node), so it is safe to capture in a HIP graph. */
HF_API int hf_state_init(const hf_config* cfg, void* state, void* stream);

/* Linear map of the history branch (Eq. 3), read as a per-head d x d matrix W without bias acting
 * on the value features (out = x W).  The row-wise division of Eq. 3 commutes with it, so it is
 * folded into a copy of the state once per chunk:
 *     L'[b,h] = L[b,h] W[h]      z' = z
 * and hf_hybrid_attn_fwd on state_out then returns O_local + Linear(history term) at no cost on
 * the per-step path.  fp32 arithmetic.
 *   state_in   fp32 state (read-only)        state_out  fp32 state, must not alias state_in
 *   W          fp32 [H, d, d] device, row = input feature, column = output feature, shared by batch */
HF_API int hf_state_fold_linear(const hf_config* cfg, const void* state_in, const float* W,
                         void* state_out, void* stream);

/* Bytes of scratch that let hf_absorb_evicted combine its per-slice partial sums without
 * atomics (0 when the configuration has no such path).  Host-only. */
HF_API int hf_absorb_workspace_bytes(const hf_config* cfg, int32_t n_tokens, size_t* bytes_out);

/* Eq. 2, incremental form used at cache eviction: for every (b, h)
 *     L += sum_t R_t(phi(k_t))^T v_t      z += sum_t phi(k_t)
 * over the n_tokens evicted tokens K_ev, V_ev [B, H, n_tokens, d] (read-only).
 * rope_cos / rope_sin: fp32 [n_tokens, d/2] per-token rotation of adjacent feature pairs
 * (2p, 2p+1), shared by heads and batch, applied after phi to the L term only; both NULL =
 * identity.  The state is updated in place (fp32 accumulation; concurrent calls on the same
 * state from different streams are allowed only if the caller orders them).
 * workspace: optional scratch of >= hf_absorb_workspace_bytes(...) bytes, 256-byte aligned;
 * with it the partial sums of a head's token slices meet there and are added in a fixed order
 * (fast path: one launch for bf16, head_dim 128, ReLU, no rotation; results do not vary from run
 * to run), with NULL (or too small a buffer) they are added to the state with float atomics.
 * Same result up to fp32 summation order.  The workspace needs no initialisation; two calls that
 * may overlap in time must not share one. */
HF_API int hf_absorb_evicted(const hf_config* cfg, void* state,
                      const void* K_ev, const void* V_ev, int32_t n_tokens,
                      const float* rope_cos, const float* rope_sin,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---- The state's bf16 planes, kept by the caller (bf16, head_dim 128, block_q 64 or 128 only) ----------
 * The history term of Eq. 3 is evaluated on the matrix cores from two bf16 planes of L (high part and
 * remainder, transposed).  hf_hybrid_attn_fwd derives them from the state on every call; the state changes
 * only when tokens are absorbed (Eq. 2), so a caller may keep the planes next to the state instead:
 * hf_absorb_evicted_planes writes them from the kernel that writes the state, hf_hybrid_attn_fwd_planes
 * reads them.  Outputs are bit-identical to the ordinary calls.  The caller owns the buffer and the
 * invariant: whatever else writes the state (hf_state_init, hf_state_fold_linear, hf_window_evict, a
 * copy) must be followed by hf_state_planes before the planes are used again. */

/* Bytes of the planes buffer (0 for configurations without this path).  Host-only. */
HF_API int hf_state_planes_bytes(const hf_config* cfg, size_t* bytes_out);

/* planes_out (device, 256-byte aligned, hf_state_planes_bytes bytes) = the planes of state (read-only). */
HF_API int hf_state_planes(const hf_config* cfg, const void* state, void* planes_out, void* stream);

/* hf_absorb_evicted (Eq. 2; every argument as there) that also writes the planes of the UPDATED state into
 * planes_out.  With a workspace they leave the kernel that sums the slices; without, a conversion launch
 * follows the atomics. */
HF_API int hf_absorb_evicted_planes(const hf_config* cfg, void* state,
                      const void* K_ev, const void* V_ev, int32_t n_tokens,
                      const float* rope_cos, const float* rope_sin,
                      void* workspace, size_t workspace_bytes, void* planes_out, void* stream);

/* Cache eviction of the inference algorithm of the supplement ("pop(0)" of the KV cache followed by
 * the update of the linear state) on the window buffers themselves: the oldest n_evict tokens of
 * K_win, V_win [B, H, n_kv, d] are absorbed into the state exactly as hf_absorb_evicted does
 * (rope tables [n_evict, d/2] or both NULL; workspace as for hf_absorb_evicted with n_evict
 * tokens), then tokens [n_evict, n_kv) of every head move to [0, n_kv - n_evict), in place.  The
 * last n_evict token slots keep stale data: the caller writes the next chunk's K, V there.
 * Both steps are enqueued on the stream; 0 < n_evict <= n_kv. */
HF_API int hf_window_advance(const hf_config* cfg, void* K_win, void* V_win, int32_t n_kv, int32_t n_evict,
                      void* state, const float* rope_cos, const float* rope_sin,
                      void* workspace, size_t workspace_bytes, void* stream);

/* hf_window_advance for a cache that keeps sink frames: the first n_sink tokens of the window stay where
 * they are, the n_evict tokens behind them are absorbed into the state, tokens [n_sink + n_evict, n_kv)
 * move down to n_sink.  0 <= n_sink, 0 < n_evict <= n_kv - n_sink; the rest as hf_window_advance. */
HF_API int hf_window_evict(const hf_config* cfg, void* K_win, void* V_win, int32_t n_kv, int32_t n_sink,
                    int32_t n_evict, void* state, const float* rope_cos, const float* rope_sin,
                    void* workspace, size_t workspace_bytes, void* stream);

/* Bookkeeping of the rolling KV cache of the inference algorithm of the supplement, kept by the caller
 * on the host; the cache buffers K_win, V_win [B, H, cfg->kv_capacity, d] are the caller's too. */
typedef struct hf_window {
  int32_t n_sink;     /* leading tokens that are never evicted (sink frames) */
  int32_t n_tokens;   /* valid tokens now: sink, cached chunks and, once opened, the current chunk */
} hf_window;

/* Start of a chunk ("if KV cache is full: pop(0), update the linear state" followed by the append, done
 * ahead of the chunk so that its own K, V have their slot during all of its denoising steps): if
 * win->n_tokens + n_chunk exceeds cfg->kv_capacity, the overflow is evicted from behind the sink into the
 * state (hf_window_evict; rope_*_ev are tables for exactly that many tokens or NULL, workspace as for
 * hf_absorb_evicted).  Then the chunk's slot is reserved: *first_out = token offset at which the caller
 * writes the chunk's K, V (before each hf_stream_step, and the clean ones after the last step),
 * *n_evicted_out = tokens evicted (both HOST, may be NULL), and win->n_tokens grows by n_chunk.
 * The overflow is max(0, win->n_tokens + n_chunk - cfg->kv_capacity): the caller can size the tables
 * before the call. */
HF_API int hf_stream_open_chunk(const hf_config* cfg, hf_window* win, int32_t n_chunk, void* K_win, void* V_win,
                         void* state, const float* rope_cos_ev, const float* rope_sin_ev,
                         void* workspace, size_t workspace_bytes,
                         int32_t* first_out, int32_t* n_evicted_out, void* stream);

/* One denoising step of the current chunk (the hybrid attention inside g_theta of the inference
 * algorithm): hf_block_select_cached over the win->n_tokens valid tokens of the cache (on steps after the
 * chunk's first, step_in_chunk > 0, the pooled keys of the whole blocks before the chunk's own n_q
 * tokens are reused, and so are the bf16 planes of the state that the first step left in the workspace:
 * the state must not change between the steps of a chunk, as in the inference algorithm, where it is
 * updated only when a chunk opens) followed by hf_hybrid_attn_fwd_split.  Where the attention kernel can
 * select for itself (bf16, head_dim 128, block_q 64 or 128, at most 1024 KV blocks, default flags) the step is
 * hf_pool_keys over the blocks that changed plus ONE launch that selects, attends and adds the history term
 * (hf_select_attn_fwd); same outputs to the same bounds.  block_idx: scratch and output,
 * int32 [B, H, T_m, k] for this window length; workspace >= hf_workspace_bytes(cfg, n_q, win->n_tokens),
 * the same buffer on every step of a chunk, written by nothing else in between.  The other arguments as
 * in those two calls. */
HF_API int hf_stream_step(const hf_config* cfg, const hf_window* win, const void* Q, const void* Q_hist, int32_t n_q,
                   const void* K_win, const void* V_win, int32_t step_in_chunk, int32_t* block_idx,
                   const void* state_or_null, const float* rope_cos_q, const float* rope_sin_q,
                   void* O, void* workspace, size_t workspace_bytes, void* stream);

/* ---- The same cache as a ring: eviction moves nothing -------------------------------------------------
 * The cache buffers [B, H, cfg->kv_capacity, d] hold n_sink sink tokens in front and, behind them,
 * (kv_capacity - n_sink) / n_chunk chunk slots of n_chunk tokens each, written round-robin.  "pop(0)" of the
 * inference algorithm is then the slot about to be overwritten: hf_ring_open_chunk absorbs it into the linear
 * state where it lies and hands the slot to the new chunk; no token of the cache is copied.
 * The window that Eq. 4 and Eq. 5 see is the buffer in STORAGE order (sink, then the slots): softmax attention
 * does not depend on the order of its keys, and the KV blocks of Eq. 4 are runs of block_kv tokens of the buffer,
 * so that at most one block spans the seam between the newest and the oldest chunk (with the compacting cache
 * above, blocks follow the temporal order instead).  Rotation tables are per token and therefore the caller's to
 * lay out in storage order. */
typedef struct hf_ring {
  int32_t n_sink;      /* leading tokens that are never evicted */
  int32_t n_chunk;     /* tokens per chunk slot; kv_capacity - n_sink must be a positive multiple of it */
  int32_t n_filled;    /* slots that hold a chunk (the open one included); starts at 0 */
  int32_t next_slot;   /* slot the next chunk goes to; starts at 0 */
  int32_t cur_slot;    /* slot of the open chunk; starts at -1 */
  int32_t absorbed_ahead;  /* set by hf_ring_last_step: the chunk in slot next_slot is in the state already; starts at 0 */
} hf_ring;

/* Start of a chunk: if every slot is taken, the chunk in slot next_slot (the oldest) is absorbed into the state
 * (Eq. 2; rope_*_ev: tables for its n_chunk tokens or both NULL; workspace as for hf_absorb_evicted; nothing is
 * absorbed if hf_ring_last_step has done so already, ring->absorbed_ahead, which is cleared) and
 * *n_evicted_out = n_chunk, else 0.  *first_out = token offset of the slot: the caller writes the chunk's K, V
 * there before each hf_ring_step (and the clean ones after the last).  Both outputs HOST, may be NULL. */
HF_API int hf_ring_open_chunk(const hf_config* cfg, hf_ring* ring, void* K_cache, void* V_cache, void* state,
                       const float* rope_cos_ev, const float* rope_sin_ev,
                       void* workspace, size_t workspace_bytes,
                       int32_t* first_out, int32_t* n_evicted_out, void* stream);

/* One denoising step of the open chunk, as hf_stream_step: selection over the n_sink + n_filled * n_chunk valid
 * tokens (after the chunk's first step only the KV blocks that touch the chunk's own slot are pooled again; the
 * state's bf16 planes of the first step are reused) and hf_hybrid_attn_fwd_split.  Q, Q_hist: [B, H, n_chunk, d];
 * block_idx: int32 [B, H, T_m, k] for that window length; workspace >= hf_workspace_bytes(cfg, n_chunk, n_kv),
 * the same buffer on every step of a chunk. */
HF_API int hf_ring_step(const hf_config* cfg, const hf_ring* ring, const void* Q, const void* Q_hist,
                 const void* K_cache, const void* V_cache, int32_t step_in_chunk, int32_t* block_idx,
                 const void* state_or_null, const float* rope_cos_q, const float* rope_sin_q,
                 void* O, void* workspace, size_t workspace_bytes, void* stream);

/* hf_ring_step for the LAST denoising step of the open chunk, together with the eviction that the next
 * hf_ring_open_chunk would carry out: if every slot is taken, the oldest chunk (slot next_slot, whose keys and values
 * are final) is absorbed into state_out = state + its contribution (Eq. 2) while this step still attends with
 * `state`; ring->absorbed_ahead is set, *absorbed_out = 1, and the next hf_ring_open_chunk, which is to be given
 * state_out as the state from then on, absorbs nothing.  While a slot is still free the next chunk evicts nothing:
 * state_out is not written and *absorbed_out = 0 (the caller keeps `state`).
 * Where hf_step_fwd applies (bf16, head_dim 128, block_q 64 or 128, ReLU, no rotation of the absorbed keys, default
 * flags) the absorb runs in workgroups of the attention launch; elsewhere the state is copied and the chunk absorbed
 * by launches of their own behind the step.  state_or_null NULL with a full ring: the chunk starts a state from zero.
 *   state_out        fp32 state buffer, must not overlap `state` or any other argument
 *   rope_*_ev        tables for the n_chunk absorbed tokens or both NULL (as hf_ring_open_chunk)
 *   step_workspace   >= max(hf_step_workspace_bytes(cfg, n_chunk, n_chunk), hf_absorb_workspace_bytes(cfg, n_chunk))
 *                    bytes, 256-byte aligned
 *   absorbed_out     HOST, may be NULL
 * Every other argument as hf_ring_step. */
HF_API int hf_ring_last_step(const hf_config* cfg, hf_ring* ring, const void* Q, const void* Q_hist,
                 const void* K_cache, const void* V_cache, int32_t step_in_chunk, int32_t* block_idx,
                 const void* state_or_null, const float* rope_cos_q, const float* rope_sin_q,
                 void* O, void* workspace, size_t workspace_bytes,
                 void* state_out, const float* rope_cos_ev, const float* rope_sin_ev,
                 void* step_workspace, size_t step_workspace_bytes, int32_t* absorbed_out, void* stream);

/* k of "sparse Top K" for a window of n_kv tokens (see keep_k / keep_ratio).  Host-only. */
HF_API int hf_select_k(const hf_config* cfg, int32_t n_kv, int32_t* k_out);

/* Bytes of scratch hf_block_select and hf_hybrid_attn_fwd need for these sizes.  Host-only. */
HF_API int hf_workspace_bytes(const hf_config* cfg, int32_t n_q, int32_t n_kv, size_t* bytes_out);

/* Eq. 4 and the Top-K mask: per (b, h) mean-pool Q and K_win per block,
 * A[i][j] = mean(q_i) . mean(k_j) (raw dot product), and for each query-block row i keep
 * the k largest A[i][:] (ties: lower j).  Row-wise softmax and the 1/sqrt(d) factor of the
 * algorithm listing are monotone per row and do not change the kept set.
 *   Q      [B, H, n_q, d], K_win [B, H, n_kv, d]                      read-only
 *   block_idx   out int32 [B, H, T_m, k], ascending within a row
 *   scores_or_null   out fp32 [B, H, T_m, T_n] raw scores, or NULL
 *   workspace   >= hf_workspace_bytes(...) bytes, 256-byte aligned */
HF_API int hf_block_select(const hf_config* cfg, const void* Q, int32_t n_q,
                    const void* K_win, int32_t n_kv,
                    int32_t* block_idx, float* scores_or_null,
                    void* workspace, size_t workspace_bytes, void* stream);

/* hf_block_select for the denoising steps after a chunk's first (inference algorithm of the
 * supplement: the older part of the window does not change between the steps of a chunk):
 * the pooled means of the first n_cached_kv_blocks KV blocks are taken from the workspace as
 * the previous hf_block_select / hf_block_select_cached call on the SAME workspace, cfg, n_q
 * and n_kv left them; only the remaining blocks of K_win are read and pooled again.  The
 * caller guarantees that the tokens of the reused blocks are unchanged and that nothing else
 * wrote the workspace's pooled-key region in between (hf_hybrid_attn_fwd does not).
 * 0 <= n_cached_kv_blocks <= floor(n_kv / block_kv) (whole blocks only); 0 = hf_block_select.
 * Same outputs, bit for bit, as hf_block_select on the same K_win. */
HF_API int hf_block_select_cached(const hf_config* cfg, const void* Q, int32_t n_q,
                    const void* K_win, int32_t n_kv, int32_t n_cached_kv_blocks,
                    int32_t* block_idx, float* scores_or_null,
                    void* workspace, size_t workspace_bytes, void* stream);

/* hf_block_select for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same outputs bit for bit; the
 * pooled block means live in a buffer built into the library (HF_STATIC_SCRATCH_BYTES per GPU, held until the
 * process ends) instead of a workspace.  The call allocates nothing and frees nothing.
 *   - sizes whose pooled means, B*H*(T_m + T_n)*d*4 bytes (each part rounded up to 256), exceed the buffer
 *     are refused with HF_ERR_WORKSPACE (use hf_block_select);
 *   - every call on a GPU shares that GPU's buffer: calls that may overlap in time on one GPU (different
 *     streams, different threads) race and must be ordered by the caller; calls on different GPUs do not
 *     interact;
 *   - the first call on a device looks the buffer's address up (no stream work; do it once outside a graph
 *     capture). */
#define HF_STATIC_SCRATCH_BYTES (8u << 20)
HF_API int hf_block_select_static(const hf_config* cfg, const void* Q, int32_t n_q,
                    const void* K_win, int32_t n_kv,
                    int32_t* block_idx, float* scores_or_null, void* stream);

/* Eq. 5 + Eq. 3 + Eq. 6 for one chunk:
 *   O_local = softmax over the keys of the selected blocks of (Q K^T * scale) times V
 *             (online softmax, fp32 statistics and accumulation);
 *   O_hist  = R_q(phi(q)) L / (z_scale * phi(q).z + eps)          (no Linear map);
 *   O       = O_local + O_hist.
 *   block_idx  int32 [B, H, T_m, k] from hf_block_select (entries in [0, T_n), distinct
 *              within a row); NULL = every block (dense sliding-window attention), k ignored.
 *   state_or_null   the fp32 state, or NULL for O_hist = 0.
 *   rope_cos_q / rope_sin_q  fp32 [n_q, d/2] for the numerator of Eq. 3, or both NULL.
 *   O          out [B, H, n_q, d], must not alias an input.
 *   workspace  >= hf_workspace_bytes(...) bytes, 256-byte aligned. */
HF_API int hf_hybrid_attn_fwd(const hf_config* cfg, const void* Q, int32_t n_q,
                       const void* K_win, const void* V_win, int32_t n_kv,
                       const int32_t* block_idx, int32_t k,
                       const void* state_or_null,
                       const float* rope_cos_q, const float* rope_sin_q,
                       void* O, void* workspace, size_t workspace_bytes, void* stream);

/* hf_hybrid_attn_fwd for a model that rotates q and k for the softmax branch as well (Sec. 3.3):
 * Q_local (already rotated, e.g. by hf_rope_apply) feeds Eq. 5, Q_hist (un-rotated) feeds phi of
 * Eq. 3, whose numerator is then rotated by rope_cos_q / rope_sin_q.  Both [B, H, n_q, d];
 * Q_hist == Q_local or NULL is hf_hybrid_attn_fwd.  Everything else as there. */
HF_API int hf_hybrid_attn_fwd_split(const hf_config* cfg, const void* Q_local, const void* Q_hist, int32_t n_q,
                       const void* K_win, const void* V_win, int32_t n_kv,
                       const int32_t* block_idx, int32_t k,
                       const void* state_or_null,
                       const float* rope_cos_q, const float* rope_sin_q,
                       void* O, void* workspace, size_t workspace_bytes, void* stream);

/* hf_hybrid_attn_fwd_split (Eq. 5 + Eq. 3 + Eq. 6; every argument as there, Q_hist NULL = Q_local) with the
 * state's planes supplied by the caller (see hf_state_planes above): state must not be NULL, planes must
 * be the planes of exactly this state; no workspace is needed.  HF_ERR_SHAPE for configurations without
 * this path. */
HF_API int hf_hybrid_attn_fwd_planes(const hf_config* cfg, const void* Q_local, const void* Q_hist, int32_t n_q,
                       const void* K_win, const void* V_win, int32_t n_kv,
                       const int32_t* block_idx, int32_t k,
                       const void* state, const void* planes,
                       const float* rope_cos_q, const float* rope_sin_q,
                       void* O, void* stream);

/* ---- Selection inside the attention launch (bf16, head_dim 128, block_q 64 or 128, T_n <= 1024) --------
 * Eq. 4 scores a query block against the pooled keys of the whole window, but needs of Q only that block's own
 * rows, which the attention workgroup of the block reads anyway.  So the Top-K of the "Hybrid Attention"
 * algorithm can run in the prologue of that workgroup: hf_pool_keys pools K_win once (the only pass that has to
 * finish before any block can choose), hf_select_attn_fwd does the rest in ONE launch: pooled query, Eq. 4,
 * Top-K (ties to the lower index), Eq. 5 over the chosen blocks, Eq. 3 and Eq. 6 in the epilogue.  The scores
 * and lists meet the same oracle bounds as hf_block_select's (fp32 sums in another order: not bit-identical to it).
 *
 * hf_pooled_keys_bytes: bytes of the pooled-key buffer for a window of n_kv tokens (host only).
 * hf_pool_keys: pooled_K [B*H][d/4][T_n][4] fp32 (means over the real length of every KV block, 16-byte feature
 *   groups outermost), 256-byte aligned, written for the KV blocks n_cached_kv_blocks .. T_n-1; the blocks before
 *   keep what the buffer holds (the older part of the window does not change between the denoising steps of a
 *   chunk; 0 <= n_cached_kv_blocks <= floor(n_kv / block_kv)).  Any dtype / head_dim the selection supports.
 * hf_select_attn_fwd: arguments as hf_hybrid_attn_fwd_planes (Q_hist NULL = Q_local), except
 *   pooled_K        from hf_pool_keys for exactly this K_win and n_kv
 *   state_or_null   NULL: O = O_local and planes is ignored; else planes must be this state's planes
 *   block_idx_out   out int32 [B, H, T_m, k], k = hf_select_k(cfg, n_kv): the list every query block chose,
 *                   ascending (the kernel also reads it back)
 *   scores_or_null  out fp32 [B, H, T_m, T_n] raw scores of Eq. 4, or NULL
 * HF_ERR_SHAPE for configurations without this path (use hf_block_select + hf_hybrid_attn_fwd there). */
HF_API int hf_pooled_keys_bytes(const hf_config* cfg, int32_t n_kv, size_t* bytes_out);
HF_API int hf_pool_keys(const hf_config* cfg, const void* K_win, int32_t n_kv, int32_t n_cached_kv_blocks,
                 void* pooled_K, void* stream);
HF_API int hf_select_attn_fwd(const hf_config* cfg, const void* Q_local, const void* Q_hist, int32_t n_q,
                       const void* K_win, const void* V_win, int32_t n_kv, const void* pooled_K,
                       const void* state_or_null, const void* planes,
                       const float* rope_cos_q, const float* rope_sin_q,
                       void* O, int32_t* block_idx_out, float* scores_or_null, void* stream);

/* ---- A whole step in one launch: hf_select_attn_fwd with Eq. 2 in workgroups of their own ------------
 * The attending workgroups of one launch seldom fill every slot of the chip (888 workgroups on 1024 slots at the
 * 832x480 shape) and the state update of Eq. 2 is independent of the attention that runs beside it if it goes to
 * another buffer.  In the inference algorithm the chunk evicted NEXT is known during a chunk's last denoising step
 * (the oldest chunk of the window): hf_step_fwd absorbs it while that step attends,
 *     state_out = state_in + sum_t phi(k_t)^T v_t, sum_t phi(k_t)   over K_ev, V_ev        (Eq. 2)
 *     planes_out = the bf16 planes of state_out (NULL: not written),
 * and state_out / planes_out become the state of the next chunk's steps.  The attention reads state_in / planes
 * exactly as hf_select_attn_fwd does (state_in NULL: O = O_local; the absorbed tokens then start from a zero
 * state).  phi = ReLU and no rotation of the absorbed keys (else HF_ERR_SHAPE: use hf_absorb_evicted).
 *   K_ev, V_ev   [B, H, ev_stride, d], the first n_ev tokens of every head are absorbed (ev_stride 0 = n_ev,
 *                packed; a slice of the window cache itself may be passed with its head stride)
 *   state_out, planes_out   must not overlap state_in / planes or any other argument
 *   workspace    >= hf_step_workspace_bytes(cfg, n_q, n_ev) bytes, 256-byte aligned, no initialisation needed;
 *                two launches that may overlap in time must not share one
 * Every other argument as hf_select_attn_fwd. */
HF_API int hf_step_workspace_bytes(const hf_config* cfg, int32_t n_q, int32_t n_ev, size_t* bytes_out);
HF_API int hf_step_fwd(const hf_config* cfg, const void* Q_local, const void* Q_hist, int32_t n_q,
                const void* K_win, const void* V_win, int32_t n_kv, const void* pooled_K,
                const void* state_in, const void* planes,
                const float* rope_cos_q, const float* rope_sin_q,
                void* O, int32_t* block_idx_out, float* scores_or_null,
                const void* K_ev, const void* V_ev, int32_t n_ev, int32_t ev_stride,
                void* state_out, void* planes_out,
                void* workspace, size_t workspace_bytes, void* stream);

/* ---- Backward pass (training algorithm of the supplement) ------------------------------------------- */

/* hf_hybrid_attn_fwd_split as the training algorithm's forward pass of the one denoising step per chunk that
 * carries gradients: the same O, plus two by-products that spare hf_hybrid_attn_bwd_saved the recomputed
 * forward pass:
 *   O_local_out  out [B, H, n_q, d] of cfg->dtype: the sparse branch's output alone (Eq. 5), rounded once
 *                (equal to O when state_or_null is NULL)
 *   lse2_out     out float [B*H, n_q]: log2 of the softmax denominator of every query row, logits scaled by
 *                softmax_scale * log2(e); +inf for a row without a single real key
 * Covers bf16, head_dim 128, block_q 64 or 128; HF_ERR_SHAPE for any other configuration (use
 * hf_hybrid_attn_fwd_split and hf_hybrid_attn_bwd there).  Neither output may alias another argument. */
HF_API int hf_hybrid_attn_fwd_save(const hf_config* cfg, const void* Q_local, const void* Q_hist, int32_t n_q,
                       const void* K_win, const void* V_win, int32_t n_kv,
                       const int32_t* block_idx, int32_t k,
                       const void* state_or_null,
                       const float* rope_cos_q, const float* rope_sin_q,
                       void* O, void* O_local_out, float* lse2_out,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of scratch hf_hybrid_attn_bwd needs for these sizes.  Host-only. */
HF_API int hf_bwd_workspace_bytes(const hf_config* cfg, int32_t n_q, int32_t n_kv, size_t* bytes_out);

/* Gradients of O = O_local + O_hist (Eq. 5, 3, 6) for the step of the training algorithm that runs with
 * gradients enabled.  That algorithm builds the KV cache and the linear state with gradients disabled, so
 * the state, the index lists of the Top-K mask and the rotation tables are constants here; the
 * differentiable inputs are the queries and the window's keys and values.  Needs only the forward call's
 * inputs and dO: the row statistics of the softmax are recomputed.
 *   Q, Q_hist, K_win, V_win, block_idx, k, state_or_null, rope_cos_q / rope_sin_q: exactly what the forward
 *        call (hf_hybrid_attn_fwd_split) was given; Q_hist == Q or NULL means one tensor fed both branches
 *   dO       [B, H, n_q, d] of cfg->dtype, gradient of the loss with respect to O        read-only
 *   dQ       out [B, H, n_q, d]: gradient with respect to Q (the softmax branch, plus the history branch
 *            when one tensor fed both)
 *   dQ_hist  out [B, H, n_q, d]: gradient with respect to Q_hist; required when Q_hist is a tensor of its
 *            own, must be NULL otherwise.  With state_or_null == NULL it is filled with zeros.
 *   dK, dV   out, laid out like K_win, V_win (heads kv_capacity tokens apart if cfg->kv_capacity is set;
 *            only the first n_kv tokens of a head are written): gradients with respect to every key and
 *            value of the window; keys of blocks that no query block selected get zeros.
 *   workspace >= hf_bwd_workspace_bytes(...) bytes, 256-byte aligned.
 * fp32 arithmetic on the recomputed probabilities, one rounding to cfg->dtype per output element.
 * Outputs must not alias inputs or each other. */
HF_API int hf_hybrid_attn_bwd(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q,
                       const void* K_win, const void* V_win, int32_t n_kv,
                       const int32_t* block_idx, int32_t k, const void* state_or_null,
                       const float* rope_cos_q, const float* rope_sin_q, const void* dO,
                       void* dQ, void* dQ_hist, void* dK, void* dV,
                       void* workspace, size_t workspace_bytes, void* stream);

/* hf_hybrid_attn_bwd from the by-products of hf_hybrid_attn_fwd_save instead of a recomputed forward pass:
 *   O_local, lse2   exactly what that call wrote (for the same inputs, index lists and state)    read-only
 * D = dO . O_local is formed from the once-rounded O_local (the recomputing call uses the unrounded one: the
 * two calls agree to the rounding of O_local).  Same configurations as hf_hybrid_attn_fwd_save; everything
 * else as hf_hybrid_attn_bwd, the same workspace size included. */
HF_API int hf_hybrid_attn_bwd_saved(const hf_config* cfg, const void* Q, const void* Q_hist, int32_t n_q,
                       const void* K_win, const void* V_win, int32_t n_kv,
                       const int32_t* block_idx, int32_t k,
                       const void* state_or_null,
                       const float* rope_cos_q, const float* rope_sin_q,
                       const void* dO, const void* O_local, const float* lse2,
                       void* dQ, void* dQ_hist, void* dK, void* dV,
                       void* workspace, size_t workspace_bytes, void* stream);

/* ---- Relative RoPE (Sec. 3.3) ------------------------------------------------------------------ */
#define HF_ROPE_MAX_FRAMES 64    /* frames one hf_rope_tables call covers */
#define HF_ROPE_MAX_PAIRS 128    /* feature pairs (head_dim / 2) of a table row */

/* Eq. 7 and the re-basing of the KV cache, host-only: temporal indices of the last n_frames latent
 * frames up to and including the frame with running index i_newest (cached frames first, the
 * current chunk last).  The newest frame takes min(i_newest, t0) (the index stops at the cap t0 of
 * the pretrained model), every other frame keeps its offset to it:
 *     idx_out[n_frames - 1 - delta] = min(i_newest, t0) - delta.
 * idx_out: HOST int32 [n_frames], 1 <= n_frames. */
HF_API int hf_rope_window_indices(int32_t i_newest, int32_t n_frames, int32_t t0, int32_t* idx_out);

/* cos / sin tables of the three-axis rotary embedding for n_frames * height * width tokens ordered
 * frame-major, then row, then column: of the pairs_t + pairs_h + pairs_w adjacent feature pairs of
 * a token the first pairs_t turn by frame_idx[frame] * w, the next pairs_h by row * w, the last
 * pairs_w by column * w radians, with w = theta^(-p / pairs_axis) for pair p of its axis.  The paper
 * fixes only the temporal indices (Eq. 7; spatial coordinates unchanged); the split and theta are
 * those of the pretrained model (head_dim 128: 22 + 21 + 21 pairs, theta 10000).
 *   frame_idx  HOST int32 [n_frames] (copied into the launch), 1 <= n_frames <= HF_ROPE_MAX_FRAMES;
 *              negative values allowed
 *   temporal_only != 0: spatial angles are zero; such a table moves tokens that already carry
 *              their rotation by frame_idx frames (re-basing cached keys by an offset)
 *   cos_out, sin_out  out fp32 [n_frames * height * width, pairs_t + pairs_h + pairs_w]
 * Angles and their sine / cosine are computed in fp64 and rounded once to fp32. */
HF_API int hf_rope_tables(const int32_t* frame_idx, int32_t n_frames, int32_t height, int32_t width,
                   int32_t pairs_t, int32_t pairs_h, int32_t pairs_w, double theta, int32_t temporal_only,
                   float* cos_out, float* sin_out, void* stream);

/* Rotation of adjacent feature pairs (2p, 2p+1) of every token by its own angle:
 *     y[2p] = x[2p] cos - x[2p+1] sin,   y[2p+1] = x[2p] sin + x[2p+1] cos
 * for X [B, H, n_tokens, d] of cfg->dtype with tables fp32 [n_tokens, d/2] shared by heads and
 * batch; fp32 arithmetic, one rounding to cfg->dtype.  Y may be X (in place) but must not overlap
 * it otherwise. */
HF_API int hf_rope_apply(const hf_config* cfg, const void* X, int32_t n_tokens,
                  const float* rope_cos, const float* rope_sin, void* Y, void* stream);

/* The chunk's keys enter the window and are pooled in the pass that already reads them: K_new [B, H, n_new, d]
 * (un-rotated, of cfg->dtype) is rotated like hf_rope_apply (tables fp32 [n_new, d/2] for exactly these tokens; both
 * NULL: copied as it is) and written to tokens first .. first + n_new - 1 of every head of the window buffer K_win
 * ([B, H, n_kv, d], or [B, H, cfg->kv_capacity, d] with n_kv valid tokens), and the pooled keys of hf_pool_keys are
 * written for the KV blocks that those tokens touch, as means of the STORED values over each block's real length
 * (tokens of such a block outside the new range are read from K_win as they stand).  Every other block of pooled_K
 * keeps its value: with the cached part of the window pooled once per chunk, a denoising step needs no pooling
 * launch (inference algorithm: only the chunk's own keys change between the steps of a chunk).
 *   0 <= first, 1 <= n_new, first + n_new <= n_kv; K_new must not overlap K_win; pooled_K 256-byte aligned. */
HF_API int hf_rope_append_keys(const hf_config* cfg, const void* K_new, int32_t n_new,
                        const float* rope_cos, const float* rope_sin,
                        void* K_win, int32_t first, int32_t n_kv, void* pooled_K, void* stream);

/* ---- Measurement helper (no part of the method) ------------------------------------------------ */

/* Enqueues a kernel in which 2048 wavefronts (two per SIMD of a 256-unit chip) each issue iters * 16 independent
 * v_mfma_f32_32x32x16_bf16, the MFMA of the attention kernels, on non-trivial operands and nothing else:
 * timed by the caller (events on `stream`), *flops_out / time is the rate the matrix cores sustain at the clock
 * the chip holds under such a load, a practical ceiling to quote next to the nominal peak.
 *   iters      in [1, 2^20]
 *   scratch4   device, >= 4 bytes (never written in practice; keeps the products alive)
 *   flops_out  HOST, may be NULL: floating-point operations of the launch */
HF_API int hf_probe_mfma_bf16(int32_t iters, void* scratch4, double* flops_out, void* stream);

/* Last error message of the calling thread (static storage, never NULL). */
HF_API const char* hf_last_error(void);

/* Library version string, e.g. "hf-gfx950 0.1". */
HF_API const char* hf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HF_H_ */
