// Block-sparse flash forward (Eq. 5) on bf16 MFMA for gfx950: head_dim 128, block_q 64 or 128.
//
// One workgroup owns one query block; each of its wavefronts owns 32 query rows and walks the
// block's selected KV blocks in tiles of 64 keys.  The products are formed TRANSPOSED so that
// every softmax statistic is private to a lane:
//
//   S^T (keys x queries) = K_tile (A operand, from LDS)  x  Q^T (B operand, registers)
//   O^T (d x queries)   += V_tile^T (A operand, LDS transpose read)  x  P^T (B operand, registers)
//
// With the 32x32x16 MFMA a lane then holds, for ONE query, 16 keys of each 32-key sub-tile:
// row max and row sum are in-lane reductions plus one exchange with lane^32, the rescale
// factor is a per-lane scalar, and the exp'd accumulators of S^T are, after rounding to bf16,
// already the B operand of the second product (the k index of that MFMA is bound to the keys
// the lane holds; V^T fragments are fetched with the matching key order by two
// ds_read_b64_tr_b16 each).  K and V tiles are staged in LDS in their memory layout
// (key-major), the next tile travels global -> registers while the current one is consumed.
#include "hf_common.h"

namespace hf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

namespace {

constexpr int D = 128;
constexpr int TK = 64;      // keys per tile
constexpr int KSTR = 272;   // bytes per key row of the K tile in LDS (256 + 16: conflict-free 16-byte operand reads)
constexpr int VSTR = 320;   // bytes per key row of the V tile in LDS (256 + 64: conflict-free transpose reads)

typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;

template <int NW>
__global__ __launch_bounds__(64 * NW, 2) void attn_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const int32_t* __restrict__ idx, int k, int n_q, int n_kv, int bkv, int t_m, int t_n, int items_per_xcd,
    int total_items, float c_scale, bf16_t* __restrict__ O) {
  constexpr int NT = 64 * NW;
  constexpr int BQ = 32 * NW;
  constexpr int CPT = (TK * D * 2 / 16) / NT;  // 16-byte chunks of a tile per thread
  __shared__ __attribute__((aligned(16))) char sK[TK * KSTR];
  __shared__ __attribute__((aligned(16))) char sV[TK * VSTR];

  // consecutive workgroup ids go to consecutive XCDs: give every XCD one contiguous run of
  // (head, query block) items so that its L2 sees few heads
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int item = xcd * items_per_xcd + slot;
  if (slot >= items_per_xcd || item >= total_items) return;
  const int bh = item / t_m, qb = item % t_m;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  const bf16_t* Qh = Q + (size_t)bh * n_q * D;
  const bf16_t* Kh = K + (size_t)bh * n_kv * D;
  const bf16_t* Vh = V + (size_t)bh * n_kv * D;
  bf16_t* Oh = O + (size_t)bh * n_q * D;
  const int32_t* row_idx = idx ? idx + ((size_t)bh * t_m + qb) * k : nullptr;
  const int nsel = idx ? k : t_n;
  const int subs = (bkv + TK - 1) / TK;
  const int ntiles = nsel * subs;

  // ---- this lane's query row as B-operand fragments (d = 16 s + 8 h .. +8)
  const int q_row = qb * BQ + 32 * wave + l32;
  bf16x8 qf[8];
  {
    const bf16_t* qp = Qh + (size_t)min(q_row, n_q - 1) * D + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
  }

  f32x16 o[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;

  uint4 kreg[CPT], vreg[CPT];
  auto gload = [&](int t) -> int {
    const int s = t / subs, sub = t - s * subs;
    const int jb = row_idx ? row_idx[s] : s;
    int start = 0, valid = 0;
    if ((unsigned)jb < (unsigned)t_n) {  // an out-of-range block index contributes nothing
      start = jb * bkv + TK * sub;
      valid = max(0, min(TK, min(n_kv, (jb + 1) * bkv) - start));
    }
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + NT * i, row = c >> 4, col = c & 15;
      if (row < valid) {
        const size_t off = (size_t)(start + row) * D + col * 8;
        kreg[i] = *reinterpret_cast<const uint4*>(Kh + off);
        vreg[i] = *reinterpret_cast<const uint4*>(Vh + off);
      } else {
        kreg[i] = make_uint4(0, 0, 0, 0);
        vreg[i] = make_uint4(0, 0, 0, 0);
      }
    }
    return valid;
  };
  auto lstore = [&]() {
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
      const int c = tid + NT * i, row = c >> 4, col = c & 15;
      *reinterpret_cast<uint4*>(sK + row * KSTR + col * 16) = kreg[i];
      *reinterpret_cast<uint4*>(sV + row * VSTR + col * 16) = vreg[i];
    }
  };

  // per-lane LDS offsets
  const int k_off = l32 * KSTR + 16 * h;                                   // + 32*kt*KSTR + 32*s
  const int g = lane >> 4, i16 = lane & 15;
  // transpose read: lane i of a 16-lane group points at key (i>>2), 4 features from 4*(i&3);
  // it receives keys 0..3 of feature i.  Group g serves features 16*(g&1).., keys 4*(g>>1)..
  const int v_off = (4 * (g >> 1) + (i16 >> 2)) * VSTR + (16 * (g & 1) + 4 * (i16 & 3)) * 2;

  int valid_cur = gload(0);
  lstore();
  __syncthreads();

  for (int t = 0; t < ntiles; ++t) {
    int valid_next = 0;
    if (t + 1 < ntiles) valid_next = gload(t + 1);

    // ---- S^T = K Q^T : 2 sub-tiles of 32 keys, 8 steps over d
    f32x16 sacc[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[kt][r] = 0.0f;
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(sK + k_off + 32 * kt * KSTR + 32 * s);
        sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s], sacc[kt], 0, 0, 0);
      }
    if (valid_cur < TK) {  // short last block: keys that do not exist never contribute
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = 32 * kt + 8 * (r >> 2) + 4 * h + (r & 3);
          if (key >= valid_cur) sacc[kt][r] = -INFINITY;
        }
    }

    // ---- online softmax in the exp2 domain; statistics are per lane (= per query)
    float mx = sacc[0][0];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kt][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    const float m_new = fmaxf(m_run, mx * c_scale);
    const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;  // nothing seen yet: keep exp2 finite
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    m_run = m_new;
    float psum = 0.0f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kt][r], c_scale, -m_use));
        psum += p;
        pf[kt][r >> 3][r & 7] = static_cast<__bf16>(p);
      }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;

    // ---- O^T += V^T P^T : 4 steps of 16 keys, 4 tiles of 32 features
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        const int key0 = 32 * kt + 16 * t2;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const char* p0 = sV + v_off + key0 * VSTR + 64 * dt;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p0));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p0 + 8 * VSTR));
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf[kt][t2], o[dt], 0, 0, 0);
        }
      }

    __syncthreads();  // every wavefront is done with this tile
    if (t + 1 < ntiles) lstore();
    __syncthreads();
    valid_cur = valid_next;
  }

  // ---- normalise and store: lane holds query l32, features 32 dt + 8 (r/4) + 4 h + (r%4)
  const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
  const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
  if (q_row < n_q) {
    bf16_t* op = Oh + (size_t)q_row * D + 4 * h;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        uint2 w;
        w.x = (uint32_t)f32_to_bf16(o[dt][4 * rq] * inv) | ((uint32_t)f32_to_bf16(o[dt][4 * rq + 1] * inv) << 16);
        w.y = (uint32_t)f32_to_bf16(o[dt][4 * rq + 2] * inv) | ((uint32_t)f32_to_bf16(o[dt][4 * rq + 3] * inv) << 16);
        *reinterpret_cast<uint2*>(op + 32 * dt + 8 * rq) = w;
      }
  }
}

}  // namespace

bool attn_mfma_supported(const hf_config& c) {
  return c.dtype == HF_BF16 && c.head_dim == 128 && (c.block_q == 64 || c.block_q == 128);
}

int launch_attn_mfma(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                     const int32_t* idx, int k, void* O_local, hipStream_t s) {
  const int BH = c.batch * c.heads;
  const int t_m = (n_q + c.block_q - 1) / c.block_q, t_n = (n_kv + c.block_kv - 1) / c.block_kv;
  const long long total = (long long)BH * t_m;
  if (total > (1ll << 30)) { set_error("too many query blocks"); return HF_ERR_SHAPE; }
  const int per_xcd = (int)((total + 7) / 8);
  const float scale = c.softmax_scale > 0.0f ? c.softmax_scale : 1.0f / sqrtf((float)c.head_dim);
  const float c_scale = scale * 1.4426950408889634f;
  const dim3 grid(8 * per_xcd);
  const bf16_t* q = static_cast<const bf16_t*>(Q);
  const bf16_t* kk = static_cast<const bf16_t*>(K);
  const bf16_t* v = static_cast<const bf16_t*>(V);
  bf16_t* o = static_cast<bf16_t*>(O_local);
  if (c.block_q == 64) {
    hipLaunchKernelGGL((attn_mfma_kernel<2>), grid, dim3(128), 0, s, q, kk, v, idx, k, n_q, n_kv, c.block_kv, t_m,
                       t_n, per_xcd, (int)total, c_scale, o);
  } else {
    hipLaunchKernelGGL((attn_mfma_kernel<4>), grid, dim3(256), 0, s, q, kk, v, idx, k, n_q, n_kv, c.block_kv, t_m,
                       t_n, per_xcd, (int)total, c_scale, o);
  }
  return check_launch("hf_hybrid_attn_fwd(attention)");
}

}  // namespace hf
