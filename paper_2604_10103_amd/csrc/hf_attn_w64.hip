// Block-sparse flash forward (Eq. 5) on bf16 MFMA for gfx950, one wavefront per 64 query rows.
//
// head_dim 128, block_q a multiple of 64.  Each wavefront is its own workgroup: it owns 64
// query rows, keeps private K / V tiles of 32 keys in LDS (no workgroup barrier anywhere) and
// walks the selected KV blocks of its query block.  Both products are formed transposed,
//
//   S^T (32 keys x 64 queries)  = K_tile (A, LDS)       x  Q^T (B, registers)
//   O^T (128 d   x 64 queries) += V_tile^T (A, LDS)     x  P^T (B, registers)
//
// so every LDS operand fragment feeds two MFMAs (two 32-query halves) and all softmax
// statistics are per-lane scalars: with the 32x32x16 MFMA a lane holds, for each of its two
// queries, 16 of the tile's 32 scores; the exp'd, bf16-rounded scores are directly the B
// operand of the second product.  The k index of that MFMA is thereby bound to the order in
// which a lane holds keys, so V is transposed on its way into LDS with the keys stored in
// that order: a V^T fragment is then one conflict-free 16-byte read.
//
// Software pipeline per tile t (all in one wavefront; MFMA issue is asynchronous, so the
// vector ALU works on softmax(t) while the matrix core works on S(t+1)):
//   A  S(t+1) = K(t+1) Q^T                 ||  softmax of S(t): max, exp2, sum, bf16 pack
//   B  K(t+2): registers -> LDS, K(t+3): global -> registers
//   C  O^T += V(t)^T P(t)^T                (after a rescale only when the running max moved a lot)
//   D  V(t+1): registers -> LDS (transposing), V(t+2): global -> registers
#include "hf_common.h"

namespace hf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int D = 128;
constexpr int TK = 32;            // keys per tile
constexpr int KSTR = 272;         // bytes per key row of the K tile (256 + 16: conflict-free 16-byte reads)
constexpr int VSTRD = 36;         // dwords per feature row of the V^T tile (16 key pairs used, rotated within 32)
constexpr int OSTR = 272;         // bytes per query row of the staged output
constexpr float kRescaleThreshold = 8.0f;  // log2 units: rescale only when the max grew by more than 2^8

struct Cursor {  // position in the list of 32-key tiles of this query block
  int s;         // index into the selected-block list
  int sub;       // 32-key tile within the block
};

template <bool kDense>
__global__ __launch_bounds__(64, 1) void attn_w64_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const int32_t* __restrict__ idx, int k, int n_q, int n_kv, int kv_stride, int bq, int bkv, int t_m, int t_n,
    int items_per_xcd, int total_items, float c_scale, bf16_t* __restrict__ O) {
  __shared__ __attribute__((aligned(16))) char sK[TK * KSTR];
  __shared__ __attribute__((aligned(16))) uint32_t sVt[D * VSTRD];

  // consecutive workgroup ids go to consecutive XCDs: every XCD gets one contiguous run of
  // (head, query block, 64-row part) items so that its L2 sees few heads
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int item = xcd * items_per_xcd + slot;
  if (slot >= items_per_xcd || item >= total_items) return;
  const int parts = bq >> 6;
  const int part = item % parts, qb = (item / parts) % t_m, bh = item / (parts * t_m);

  const int lane = threadIdx.x, l32 = lane & 31, h = lane >> 5;
  const bf16_t* Qh = Q + (size_t)bh * n_q * D;
  const bf16_t* Kh = K + (size_t)bh * kv_stride * D;
  const bf16_t* Vh = V + (size_t)bh * kv_stride * D;
  bf16_t* Oh = O + (size_t)bh * n_q * D;
  const int32_t* row_idx = kDense ? nullptr : idx + ((size_t)bh * t_m + qb) * k;
  const int nsel = kDense ? t_n : k;
  const int subs = (bkv + TK - 1) / TK;
  const int ntiles = nsel * subs;
  const int q0 = qb * bq + 64 * part;
  const int q_end = min(n_q, (qb + 1) * bq);
  if (q0 >= q_end) return;

  // tile -> first key and number of real keys; branch-free.  Tiles past the end of the list and
  // out-of-range block indices give (0, 0): such a tile reads real rows and is masked entirely.
  auto tile_of = [&](const Cursor& c, int& start, int& valid) {
    const int sc = min(c.s, nsel - 1);
    const int jb = kDense ? sc : row_idx[sc];
    const bool ok = (c.s < nsel) && ((unsigned)jb < (unsigned)t_n);
    const int st = jb * bkv + TK * c.sub;
    start = ok ? st : 0;
    valid = ok ? max(0, min(TK, min(n_kv, (jb + 1) * bkv) - st)) : 0;
  };
  auto advance = [&](Cursor& c) {
    if (++c.sub == subs) { c.sub = 0; ++c.s; }
  };

  // ---- Q^T fragments: lane owns queries q0 + l32 and q0 + 32 + l32, features 16 s + 8 h .. +8
  bf16x8 qf[2][8];
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const bf16_t* qp = Qh + (size_t)min(q0 + 32 * qt + l32, n_q - 1) * D + 8 * h;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[qt][s] = *reinterpret_cast<const bf16x8*>(qp + 16 * s);
  }

  // ---- staging registers and their LDS images
  // K tile: 32 rows x 256 B; lane loads rows (lane>>4) + 4 i, 16-byte group lane & 15
  // V tile: loads i = 2 j + u fetch key 16 t2 + 8 x + 4 hh + 2 y + u with j = 2 t2 + hh, (x, y) = (lane>>5, (lane>>4)&1)
  // Loads go through buffer resources that end at the head's last key: rows past n_kv (the only
  // rows of a tile that can be missing) read as zero without any branch; every offset is in the
  // vector operand, which is what the hardware range check looks at.
  u32x4 kreg[8], vreg[8];
  const int ld_row = lane >> 4, ld_grp = lane & 15;
  const __amdgpu_buffer_rsrc_t k_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(Kh), 0, n_kv * (D * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t v_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(Vh), 0, n_kv * (D * 2), 0x00020000);
  const int k_ld_off = ld_row * (D * 2) + ld_grp * 16;
  auto gload_k = [&](const Cursor& c) {
    int start, valid;
    tile_of(c, start, valid);
    const int base = k_ld_off + start * (D * 2);
#pragma unroll
    for (int i = 0; i < 8; ++i) kreg[i] = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, base + 4 * i * (D * 2), 0, 0);
  };
  const int v_ld_off = (8 * (lane >> 5) + 2 * ((lane >> 4) & 1)) * (D * 2) + ld_grp * 16;
  auto gload_v = [&](const Cursor& c) {
    int start, valid;
    tile_of(c, start, valid);
    const int base = v_ld_off + start * (D * 2);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int j = i >> 1, u = i & 1;
      const int row = 16 * (j >> 1) + 4 * (j & 1) + u;
      vreg[i] = __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, base + row * (D * 2), 0, 0);
    }
  };
  auto store_k = [&]() {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      *reinterpret_cast<u32x4*>(sK + (ld_row + 4 * i) * KSTR + ld_grp * 16) = kreg[i];
  };
  // V^T image: row = feature, dword column = key pair in MFMA order 8 t2 + 4 hh + 2 x + y, rotated
  // by 4 dwords per 16 features (keeps the dword stores of a wavefront on distinct banks)
  const int vt_rot = 4 * ((ld_grp >> 1) & 7);
  const int vt_col_lane = 2 * (lane >> 5) + ((lane >> 4) & 1);
  auto store_v = [&]() {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = (4 * j + vt_col_lane + vt_rot) & 31;
      const u32x4 a = vreg[2 * j], b = vreg[2 * j + 1];  // rows key and key + 1
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int f = 8 * ld_grp + 2 * p;
        sVt[f * VSTRD + col] = __builtin_amdgcn_perm(b[p], a[p], 0x05040100u);        // (key, key+1) of feature f
        sVt[(f + 1) * VSTRD + col] = __builtin_amdgcn_perm(b[p], a[p], 0x07060302u);  // ... of feature f + 1
      }
    }
  };

  // per-lane LDS read offsets
  const char* k_rd = sK + l32 * KSTR + 16 * h;   // + 32 s
  // feature row 32 dt + l32, columns 8 t2 + 4 h .. +3, rotated like the stores
  int v_row[4], v_rot[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    v_row[dt] = (32 * dt + l32) * VSTRD;
    v_rot[dt] = 4 * ((2 * dt + (l32 >> 4)) & 7);
  }

  auto compute_s = [&](f32x16 (&sacc)[2]) {
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[qt][r] = 0.0f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(k_rd + 32 * s);
      sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][s], sacc[0], 0, 0, 0);
      sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][s], sacc[1], 0, 0, 0);
    }
  };
  auto mask_s = [&](f32x16 (&sacc)[2], int valid) {  // keys of a short last block that do not exist
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = 8 * (r >> 2) + 4 * h + (r & 3);
      if (key >= valid) {
        sacc[0][r] = -INFINITY;
        sacc[1][r] = -INFINITY;
      }
    }
  };

  f32x16 o[4][2];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][qt][r] = 0.0f;
  float m_ref[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.0f, 0.0f};

  // ---- prologue
  Cursor ck = {0, 0}, cv = {0, 0}, cs = {0, 0};
  int start_s, valid_s;
  gload_k(ck); advance(ck);
  gload_v(cv); advance(cv);
  store_k();
  gload_k(ck); advance(ck);
  store_v();
  gload_v(cv); advance(cv);
  f32x16 s_cur[2], s_next[2];
  compute_s(s_cur);
  tile_of(cs, start_s, valid_s); advance(cs);
  if (valid_s < TK) mask_s(s_cur, valid_s);
  store_k();
  gload_k(ck); advance(ck);

  for (int t = 0; t < ntiles; ++t) {
    // ---- A: S(t+1) on the matrix core, softmax(t) on the vector ALU
    compute_s(s_next);

    float mx[2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      float a = fmaxf(s_cur[qt][0], s_cur[qt][1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) a = fmaxf(a, fmaxf(s_cur[qt][r], s_cur[qt][r + 1]));
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(a), false, false);
      mx[qt] = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * c_scale;  // both lanes of a query agree
    }
    // lazy rescale: keep the reference max unless some query's max grew by more than the threshold
    const bool grow = (mx[0] > m_ref[0] + kRescaleThreshold) || (mx[1] > m_ref[1] + kRescaleThreshold);
    float alpha[2] = {1.0f, 1.0f};
    const bool rescale = __any(grow);
    if (rescale) {
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
        const float m_new = fmaxf(m_ref[qt], mx[qt]);
        const float m_use = (m_new == -INFINITY) ? 0.0f : m_new;
        alpha[qt] = __builtin_amdgcn_exp2f(m_ref[qt] - m_use);
        l_run[qt] *= alpha[qt];
        m_ref[qt] = m_new;
      }
    }
    bf16x8 pf[2][2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
      const float m_use = (m_ref[qt] == -INFINITY) ? 0.0f : m_ref[qt];
      float psum = 0.0f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s_cur[qt][r], c_scale, -m_use));
        psum += p;
        pf[qt][r >> 3][r & 7] = static_cast<__bf16>(p);
      }
      l_run[qt] += psum;
    }
    tile_of(cs, start_s, valid_s); advance(cs);
    if (valid_s < TK) mask_s(s_next, valid_s);

    // ---- B: K(t+2) into LDS, K(t+3) on its way
    store_k();
    gload_k(ck); advance(ck);

    if (rescale) {
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dt][qt][r] *= alpha[qt];
    }

    // ---- C: O^T += V(t)^T P(t)^T
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        // column (8 t2 + 4 h + rotation) mod 32; the rotation is a multiple of 4, so the 4 dwords stay together
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&sVt[v_row[dt] + ((8 * t2 + 4 * h + v_rot[dt]) & 31)]);
        o[dt][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[0][t2], o[dt][0], 0, 0, 0);
        o[dt][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[1][t2], o[dt][1], 0, 0, 0);
      }

    // ---- D: V(t+1) into LDS, V(t+2) on its way
    store_v();
    gload_v(cv); advance(cv);

#pragma unroll
    for (int qt = 0; qt < 2; ++qt) s_cur[qt] = s_next[qt];
  }

  // ---- normalise, transpose through LDS (reusing the V^T tile) and store coalesced
  char* stage = reinterpret_cast<char*>(sVt);
  static_assert(64 * OSTR <= D * VSTRD * 4, "staged output must fit in the V^T tile");
#pragma unroll
  for (int qt = 0; qt < 2; ++qt) {
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run[qt]), __float_as_uint(l_run[qt]), false, false);
    const float l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    const float inv = l_tot > 0.0f ? 1.0f / l_tot : 0.0f;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        uint2 w;
        w.x = (uint32_t)f32_to_bf16(o[dt][qt][4 * rq] * inv) | ((uint32_t)f32_to_bf16(o[dt][qt][4 * rq + 1] * inv) << 16);
        w.y = (uint32_t)f32_to_bf16(o[dt][qt][4 * rq + 2] * inv) | ((uint32_t)f32_to_bf16(o[dt][qt][4 * rq + 3] * inv) << 16);
        *reinterpret_cast<uint2*>(stage + (32 * qt + l32) * OSTR + (32 * dt + 8 * rq + 4 * h) * 2) = w;
      }
  }
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int c = lane + 64 * i, row = c >> 4, col = c & 15;
    if (q0 + row < q_end)
      *reinterpret_cast<uint4*>(Oh + (size_t)(q0 + row) * D + col * 8) =
          *reinterpret_cast<const uint4*>(stage + row * OSTR + col * 16);
  }
}

}  // namespace

bool attn_w64_supported(const hf_config& c) {
  return c.dtype == HF_BF16 && c.head_dim == 128 && c.block_q % 64 == 0;
}

// byte offsets inside one head are 32-bit in the buffer loads
constexpr int kW64MaxKeys = 1 << 23;

int launch_attn_w64(const hf_config& c, const void* Q, int n_q, const void* K, const void* V, int n_kv,
                    const int32_t* idx, int k, void* O_local, hipStream_t s) {
  if (n_kv >= kW64MaxKeys) { set_error("window longer than %d keys", kW64MaxKeys); return HF_ERR_SHAPE; }
  const int BH = c.batch * c.heads;
  const int t_m = (n_q + c.block_q - 1) / c.block_q, t_n = (n_kv + c.block_kv - 1) / c.block_kv;
  const long long total = (long long)BH * t_m * (c.block_q / 64);
  if (total > (1ll << 30)) { set_error("too many query blocks"); return HF_ERR_SHAPE; }
  const int per_xcd = (int)((total + 7) / 8);
  const float scale = c.softmax_scale > 0.0f ? c.softmax_scale : 1.0f / sqrtf((float)c.head_dim);
  const float c_scale = scale * 1.4426950408889634f;
  const dim3 grid(8 * per_xcd), block(64);
  const bf16_t* q = static_cast<const bf16_t*>(Q);
  const bf16_t* kk = static_cast<const bf16_t*>(K);
  const bf16_t* v = static_cast<const bf16_t*>(V);
  bf16_t* o = static_cast<bf16_t*>(O_local);
  if (idx)
    hipLaunchKernelGGL((attn_w64_kernel<false>), grid, block, 0, s, q, kk, v, idx, k, n_q, n_kv, kv_stride_of(c, n_kv), c.block_q,
                       c.block_kv, t_m, t_n, per_xcd, (int)total, c_scale, o);
  else
    hipLaunchKernelGGL((attn_w64_kernel<true>), grid, block, 0, s, q, kk, v, idx, k, n_q, n_kv, kv_stride_of(c, n_kv), c.block_q,
                       c.block_kv, t_m, t_n, per_xcd, (int)total, c_scale, o);
  return check_launch("hf_hybrid_attn_fwd(attention)");
}

}  // namespace hf
