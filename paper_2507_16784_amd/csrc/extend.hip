// Extend attention: the attention half of re-encoding the repositioned tokens (the paper's
// own way of reassigning positions, Eq. 1).  After a flush, each survivor behind the first
// pruned token attends causally to everything up to and including itself in the compacted
// cache.  Many queries share each key, so unlike decode this kernel reuses every loaded
// K/V tile for 32 (token, head) query rows per wave and is bounded by the matrix cores
// and L2 rather than by HBM.
//
// Decomposition.  grid = (kv_heads, tiles of 32 extended tokens).  A block's four waves
// take 8 tokens each: two sets of 16 query rows (4 tokens x the 4 heads of the group).
// Per pair of key pages a wave loads K and V exactly like the decode kernel and runs, per
// set, S^T = K . Q^T (K tile as A operand, the 16 query rows as B columns) and
// O += P . V with the probabilities staying in their lanes and V transposed in registers
// once for both sets.  The four waves of a block walk the same pages at the same time, so
// the CU's vector L1 serves three of the four reads.  Causality is a mask on the pages at
// the diagonal only.  One lazy reference maximum per query row, as in decode.
#include "tim_internal.h"

#define EX_THREADS 256
#define EX_TILE_TOKENS 32
#define EX_WAVE_TOKENS 8
#define EX_NEG_BIG (-1.0e30f)
#define EX_LAZY_MAX 8.0f

typedef __bf16 ex_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 ex_bf16x2 __attribute__((ext_vector_type(2)));
typedef float ex_f32x4 __attribute__((ext_vector_type(4)));
typedef float ex_f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t ex_pack_bf16(float lo, float hi) {
  ex_f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, ex_bf16x2));
}
__device__ __forceinline__ ex_bf16x8 ex_as_bf16x8(const uint4 &u) { return __builtin_bit_cast(ex_bf16x8, u); }

template <bool OUT_BF16>
__global__ void __launch_bounds__(EX_THREADS, 2)
tim_extend_attn_kernel(tim_config cfg, tim_state st, tim_plan pl, int n_seqs, int layer, const uint4 *__restrict__ q_ext,
                       void *__restrict__ out_ext, int n_ext_total, float scale_log2) {
  // workgroup ids run over the kv heads first: with 8 heads each XCD keeps one head's K/V in
  // its L2 for all query tiles.  Tiles are taken last-first: under the causal mask the late
  // tiles of a sequence are the long ones, and starting them first shortens the tail.
  const int kvh = blockIdx.x;
  if (!pl.totals[TIM_TOT_OK] || (int)blockIdx.y >= pl.totals[TIM_TOT_EXT_TILES]) return;
  const int tile = pl.totals[TIM_TOT_EXT_TILES] - 1 - blockIdx.y;
  // flushed sequence of this tile: last e with EXT_TILE_OFF[e] <= tile (n_seqs is small)
  int lo = 0, hi = n_seqs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (pl.hdr[(int64_t)mid * TIM_PLAN_HDR + TIM_HDR_EXT_TILE_OFF] <= tile) lo = mid; else hi = mid - 1;
  }
  const int32_t *hdr = pl.hdr + (int64_t)lo * TIM_PLAN_HDR;
  if (hdr[TIM_HDR_BAD]) return;
  const int b = hdr[TIM_HDR_SEQ], m = hdr[TIM_HDR_N_KEPT], f = hdr[TIM_HDR_FIRST_PRUNED];
  const int ext = hdr[TIM_HDR_EXT], ext_off = hdr[TIM_HDR_EXT_OFF];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, g = lane >> 4, n = lane & 15;
  const int tok0 = (tile - hdr[TIM_HDR_EXT_TILE_OFF]) * EX_TILE_TOKENS + w * EX_WAVE_TOKENS;
  if (tok0 >= ext) return;  // this wave has no token; the kernel has no block-wide sync

  // B operands of the score product: the wave's query rows.  Column n of set s is
  // (token tok0 + 4s + n/4, head n%4), dims 32*step + 8g .. +8.
  uint4 qb[2][4];
  int pos[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int tl = tok0 + 4 * s + (n >> 2);
    const bool ok = tl < ext && ext_off + tl < n_ext_total;
    pos[s] = ok ? f + tl : -1;  // a column without a token sees no key at all
#pragma unroll
    for (int step = 0; step < 4; ++step) {
      qb[s][step] = make_uint4(0, 0, 0, 0);
      if (ok) qb[s][step] = q_ext[((int64_t)(ext_off + tl) * cfg.q_heads + kvh * TIM_G + (n & 3)) * 16 + 4 * step + g];
    }
  }
  const int first_pos = f + tok0;                                   // smallest query position of the wave
  const int last_pos = f + min(tok0 + EX_WAVE_TOKENS, ext) - 1;      // largest
  const int last_page = last_pos / TIM_PS;

  float m_ref[2] = {EX_NEG_BIG, EX_NEG_BIG}, l_part[2] = {0.f, 0.f};
  ex_f32x4 acc[2][8];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int mf = 0; mf < 8; ++mf) acc[s][mf] = (ex_f32x4){0.f, 0.f, 0.f, 0.f};

  const uint4 *kpool = reinterpret_cast<const uint4 *>(st.k_pool);
  const uint4 *vpool = reinterpret_cast<const uint4 *>(st.v_pool);
  const int32_t *ptab = st.page_table + (int64_t)b * cfg.max_pages_per_seq;
  const int64_t layer_base = (int64_t)layer * cfg.num_pages;

  for (int pg = 0; pg <= last_page; pg += 2) {
    const bool has_b = pg + 1 <= last_page;
    int phys_a = __builtin_amdgcn_readfirstlane(ptab[pg]);
    int phys_b = __builtin_amdgcn_readfirstlane(ptab[has_b ? pg + 1 : pg]);
    if (phys_a < 0 || phys_a >= cfg.num_pages || phys_b < 0 || phys_b >= cfg.num_pages) {
      tim_set_status(st.status, TIM_ERR_INVALID_ARG);  // never dereference a bad page id
      phys_a = phys_b = 0;
    }
    const int64_t tile_a = ((layer_base + phys_a) * cfg.kv_heads + kvh) * (TIM_TILE_BYTES / 16);
    const int64_t tile_b = ((layer_base + phys_b) * cfg.kv_heads + kvh) * (TIM_TILE_BYTES / 16);
    uint4 ka[4], kb[4], va[4], vb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) ka[s] = kpool[tile_a + n * 16 + 4 * s + g];
#pragma unroll
    for (int s = 0; s < 4; ++s) kb[s] = kpool[tile_b + n * 16 + 4 * s + g];
#pragma unroll
    for (int i = 0; i < 4; ++i) va[i] = vpool[tile_a + (4 * g + i) * 16 + n];
#pragma unroll
    for (int i = 0; i < 4; ++i) vb[i] = vpool[tile_b + (4 * g + i) * 16 + n];

    // keys of this lane: page A rows 4g..4g+3, page B rows 4g..4g+3
    const int key_a = pg * TIM_PS + 4 * g, key_b = key_a + TIM_PS;
    // pages wholly below every query of the wave need no mask
    const bool diag = !has_b || key_b - 4 * g + TIM_PS - 1 > first_pos;
    if (diag) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {  // rows past the sequence may hold anything
        if (key_a + r >= m) va[r] = make_uint4(0, 0, 0, 0);
        if (!has_b || key_b + r >= m) vb[r] = make_uint4(0, 0, 0, 0);
      }
    }

    uint4 pw[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      ex_f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int step = 0; step < 4; ++step)
        sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ex_as_bf16x8(ka[step]), ex_as_bf16x8(qb[s][step]), sa, 0, 0, 0);
#pragma unroll
      for (int step = 0; step < 4; ++step)
        sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ex_as_bf16x8(kb[step]), ex_as_bf16x8(qb[s][step]), sb, 0, 0, 0);
      float t[8];
      if (!diag) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          t[r] = sa[r] * scale_log2;
          t[4 + r] = sb[r] * scale_log2;
        }
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {  // causal: key index <= query position (select on the product)
          t[r] = key_a + r <= pos[s] ? sa[r] * scale_log2 : -INFINITY;
          t[4 + r] = (has_b && key_b + r <= pos[s]) ? sb[r] * scale_log2 : -INFINITY;
        }
      }
      const float lm = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])), fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
      if (__any(lm > m_ref[s] + EX_LAZY_MAX)) {
        float x = lm;
        x = fmaxf(x, __shfl_xor(x, 16, 64));
        x = fmaxf(x, __shfl_xor(x, 32, 64));
        const float m_new = fmaxf(m_ref[s], x);
        const float alpha = __builtin_amdgcn_exp2f(m_ref[s] - m_new);
        l_part[s] *= alpha;
        m_ref[s] = m_new;
        // accumulator rows 4g..4g+3 of this lane are query rows whose factor sits in lanes 4g+r
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float ar = __shfl(alpha, 4 * g + r, 64);
#pragma unroll
          for (int mf = 0; mf < 8; ++mf) acc[s][mf][r] *= ar;
        }
      }
      float p[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = __builtin_amdgcn_exp2f(t[e] - m_ref[s]);
        l_part[s] += p[e];
      }
      pw[s].x = ex_pack_bf16(p[0], p[1]);
      pw[s].y = ex_pack_bf16(p[2], p[3]);
      pw[s].z = ex_pack_bf16(p[4], p[5]);
      pw[s].w = ex_pack_bf16(p[6], p[7]);
    }

    // 8x8 transpose of 16-bit elements (rows = the lane's 8 keys, columns = dims 8n..8n+7),
    // one column per MFMA, used by both sets
    const uint32_t *ra[8] = {&va[0].x, &va[1].x, &va[2].x, &va[3].x, &vb[0].x, &vb[1].x, &vb[2].x, &vb[3].x};
#pragma unroll
    for (int mf = 0; mf < 8; ++mf) {
      uint4 col;
      uint32_t *cw = &col.x;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t x0 = ra[2 * u][mf >> 1], x1 = ra[2 * u + 1][mf >> 1];
        cw[u] = (mf & 1) ? __builtin_amdgcn_perm(x1, x0, 0x07060302u) : __builtin_amdgcn_perm(x1, x0, 0x05040100u);
      }
#pragma unroll
      for (int s = 0; s < 2; ++s)
        acc[s][mf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ex_as_bf16x8(pw[s]), ex_as_bf16x8(col), acc[s][mf], 0, 0, 0);
    }
  }

  // normalise and store: lane (g, c) holds query rows 4g+r = (token tok0 + 4s + g, head r), dims 8c + mf
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    float lt = l_part[s];
    lt += __shfl_xor(lt, 16, 64);
    lt += __shfl_xor(lt, 32, 64);
    const int tl = tok0 + 4 * s + g;
    const bool ok = tl < ext && ext_off + tl < n_ext_total;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float inv = 1.f / __shfl(lt, 4 * g + r, 64);
      if (!ok) continue;
      const int64_t o = ((int64_t)(ext_off + tl) * cfg.q_heads + kvh * TIM_G + r) * TIM_D + 8 * n;
      if (OUT_BF16) {
        uint4 v;
        v.x = ex_pack_bf16(acc[s][0][r] * inv, acc[s][1][r] * inv);
        v.y = ex_pack_bf16(acc[s][2][r] * inv, acc[s][3][r] * inv);
        v.z = ex_pack_bf16(acc[s][4][r] * inv, acc[s][5][r] * inv);
        v.w = ex_pack_bf16(acc[s][6][r] * inv, acc[s][7][r] * inv);
        *reinterpret_cast<uint4 *>(reinterpret_cast<__bf16 *>(out_ext) + o) = v;
      } else {
        float *dst = reinterpret_cast<float *>(out_ext) + o;
        *reinterpret_cast<float4 *>(dst) = make_float4(acc[s][0][r] * inv, acc[s][1][r] * inv, acc[s][2][r] * inv, acc[s][3][r] * inv);
        *reinterpret_cast<float4 *>(dst + 4) = make_float4(acc[s][4][r] * inv, acc[s][5][r] * inv, acc[s][6][r] * inv, acc[s][7][r] * inv);
      }
    }
  }
}

// ---- LDS-staged variant ----------------------------------------------------------------
// The four waves of a block need the same K and V tiles.  Instead of each wave pulling them
// through the vector L1, each wave fetches one of the pair's four 4 KiB tiles (K page A, K page
// B, V page A, V page B) with fully coalesced loads and parks it in LDS; all waves then read
// their MFMA operands from LDS.  Two LDS buffers: the global loads of the next pair are in
// flight while this pair is multiplied, and one barrier per pair separates readers from the
// next writer.
//
// Bank conflicts.  Measured on this chip: a 16-byte-per-lane LDS read is served 16 lanes at a
// time, and the lanes served together are not consecutive: of lanes 0..31 they are
// {0-3, 12-15, 20-23, 24-27} and {4-7, 8-11, 16-19, 28-31} (same for 32..63); such a group is
// conflict-free when its 16-byte slots differ modulo 256 bytes.  A V tile is read as "row
// 4g+i, chunk n": plain 256-byte rows already give every lane of a group its own slot.  A K
// tile is read as "row n, chunk 4s+g": chunk c of row r is stored at slot c ^ r, which makes
// the slots of each group a permutation of 0..15.  (Rows padded to 272 bytes, the usual
// remedy, collide two-way under this grouping: measured 1.7 times slower.)
#define EXL_TILE_BYTES TIM_TILE_BYTES
#define EXL_BUF_BYTES (4 * EXL_TILE_BYTES)

template <bool OUT_BF16>
__global__ void __launch_bounds__(256, 2)
tim_extend_attn_lds_kernel(tim_config cfg, tim_state st, tim_plan pl, int n_seqs, int layer,
                           const uint4 *__restrict__ q_ext, void *__restrict__ out_ext, int n_ext_total,
                           float scale_log2) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * EXL_BUF_BYTES];
  const int kvh = blockIdx.x;
  if (!pl.totals[TIM_TOT_OK] || (int)blockIdx.y >= pl.totals[TIM_TOT_EXT_TILES]) return;
  const int tile = pl.totals[TIM_TOT_EXT_TILES] - 1 - blockIdx.y;
  int lo = 0, hi = n_seqs - 1;  // flushed sequence of this tile: last e with EXT_TILE_OFF[e] <= tile
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (pl.hdr[(int64_t)mid * TIM_PLAN_HDR + TIM_HDR_EXT_TILE_OFF] <= tile) lo = mid; else hi = mid - 1;
  }
  const int32_t *hdr = pl.hdr + (int64_t)lo * TIM_PLAN_HDR;
  if (hdr[TIM_HDR_BAD]) return;  // uniform for the block
  const int b = hdr[TIM_HDR_SEQ], m = hdr[TIM_HDR_N_KEPT], f = hdr[TIM_HDR_FIRST_PRUNED];
  const int ext = hdr[TIM_HDR_EXT], ext_off = hdr[TIM_HDR_EXT_OFF];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, g = lane >> 4, n = lane & 15;
  const int blk_tok0 = (tile - hdr[TIM_HDR_EXT_TILE_OFF]) * EX_TILE_TOKENS;
  const int tok0 = blk_tok0 + w * EX_WAVE_TOKENS;
  const bool active = tok0 < ext;  // a wave without a token still fetches and meets the barriers

  uint4 qb[2][4];
  int pos[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int tl = tok0 + 4 * s + (n >> 2);
    const bool ok = tl < ext && ext_off + tl < n_ext_total;
    pos[s] = ok ? f + tl : -1;
#pragma unroll
    for (int step = 0; step < 4; ++step) {
      qb[s][step] = make_uint4(0, 0, 0, 0);
      if (ok) qb[s][step] = q_ext[((int64_t)(ext_off + tl) * cfg.q_heads + kvh * TIM_G + (n & 3)) * 16 + 4 * step + g];
    }
  }
  const int first_pos = f + tok0;
  const int last_pos = f + min(tok0 + EX_WAVE_TOKENS, ext) - 1;            // this wave's largest position
  const int last_page = (f + min(blk_tok0 + EX_TILE_TOKENS, ext) - 1) / TIM_PS;  // the block's last key page

  float m_ref[2] = {EX_NEG_BIG, EX_NEG_BIG}, l_part[2] = {0.f, 0.f};
  ex_f32x4 acc[2][8];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int mf = 0; mf < 8; ++mf) acc[s][mf] = (ex_f32x4){0.f, 0.f, 0.f, 0.f};

  const uint4 *kpool = reinterpret_cast<const uint4 *>(st.k_pool);
  const uint4 *vpool = reinterpret_cast<const uint4 *>(st.v_pool);
  const int32_t *ptab = st.page_table + (int64_t)b * cfg.max_pages_per_seq;
  const int64_t layer_base = (int64_t)layer * cfg.num_pages;

  // this wave's share of a pair: tile w (0: K page A, 1: K page B, 2: V page A, 3: V page B)
  const uint4 *tile_pool = w < 2 ? kpool : vpool;
  // 16-byte unit i * 64 + lane of the tile is chunk lane % 16 of row 4 i + lane / 16
  const int park_row = lane >> 4, park_chunk = lane & 15, park_swz = w < 2 ? 15 : 0;
  unsigned char *park_base = lds + w * EXL_TILE_BYTES + park_row * 256;
  uint4 stage0, stage1, stage2, stage3;
  // The page id of a tile is read one pair before the tile itself, so that its latency is not in the way.
#define EXL_PAGE_ID(pg_) ptab[min((pg_) + (w & 1), last_page)]
#define EXL_FETCH(pid_)                                                                                         \
  {                                                                                                             \
    int phys_ = __builtin_amdgcn_readfirstlane(pid_);                                                           \
    if (phys_ < 0 || phys_ >= cfg.num_pages) {                                                                  \
      tim_set_status(st.status, TIM_ERR_INVALID_ARG); /* never dereference a bad page id */                     \
      phys_ = 0;                                                                                                \
    }                                                                                                           \
    const uint4 *src_ = tile_pool + ((layer_base + phys_) * cfg.kv_heads + kvh) * (TIM_TILE_BYTES / 16) + lane; \
    stage0 = src_[0];                                                                                           \
    stage1 = src_[64];                                                                                          \
    stage2 = src_[128];                                                                                         \
    stage3 = src_[192];                                                                                         \
  }
#define EXL_PARK(buf_)                                                                  \
  {                                                                                     \
    unsigned char *dst_ = park_base + (buf_) * EXL_BUF_BYTES;                           \
    *reinterpret_cast<uint4 *>(dst_ + ((park_chunk ^ (park_row & park_swz)) << 4)) = stage0;                \
    *reinterpret_cast<uint4 *>(dst_ + 4 * 256 + ((park_chunk ^ ((park_row + 4) & park_swz)) << 4)) = stage1;  \
    *reinterpret_cast<uint4 *>(dst_ + 8 * 256 + ((park_chunk ^ ((park_row + 8) & park_swz)) << 4)) = stage2;  \
    *reinterpret_cast<uint4 *>(dst_ + 12 * 256 + ((park_chunk ^ ((park_row + 12) & park_swz)) << 4)) = stage3; \
  }

  int pid_next = EXL_PAGE_ID(0);
  EXL_FETCH(pid_next);
  pid_next = EXL_PAGE_ID(2);
  EXL_PARK(0);
  __syncthreads();
  for (int pg = 0, it = 0; pg <= last_page; pg += 2, ++it) {
    const bool more = pg + 2 <= last_page;
    if (more) {
      EXL_FETCH(pid_next);
      pid_next = EXL_PAGE_ID(pg + 4);
    }
    if (active && pg * TIM_PS <= last_pos) {
      const unsigned char *buf = lds + (it & 1) * EXL_BUF_BYTES;
      const bool has_b = pg + 1 <= last_page;
      uint4 ka[4], kb[4], va[4], vb[4];
#pragma unroll
      for (int step = 0; step < 4; ++step) {
        ka[step] = *reinterpret_cast<const uint4 *>(buf + n * 256 + (((4 * step + g) ^ n) << 4));
        kb[step] = *reinterpret_cast<const uint4 *>(buf + EXL_TILE_BYTES + n * 256 + (((4 * step + g) ^ n) << 4));
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        va[i] = *reinterpret_cast<const uint4 *>(buf + 2 * EXL_TILE_BYTES + (4 * g + i) * 256 + n * 16);
        vb[i] = *reinterpret_cast<const uint4 *>(buf + 3 * EXL_TILE_BYTES + (4 * g + i) * 256 + n * 16);
      }
      const int key_a = pg * TIM_PS + 4 * g, key_b = key_a + TIM_PS;
      const bool diag = !has_b || (pg + 2) * TIM_PS - 1 > first_pos;
      if (diag) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {  // rows past the sequence may hold anything
          if (key_a + r >= m) va[r] = make_uint4(0, 0, 0, 0);
          if (!has_b || key_b + r >= m) vb[r] = make_uint4(0, 0, 0, 0);
        }
      }
      uint4 pw[2];
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        ex_f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int step = 0; step < 4; ++step)
          sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ex_as_bf16x8(ka[step]), ex_as_bf16x8(qb[s][step]), sa, 0, 0, 0);
#pragma unroll
        for (int step = 0; step < 4; ++step)
          sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ex_as_bf16x8(kb[step]), ex_as_bf16x8(qb[s][step]), sb, 0, 0, 0);
        float t[8];
        if (!diag) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            t[r] = sa[r] * scale_log2;
            t[4 + r] = sb[r] * scale_log2;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            t[r] = key_a + r <= pos[s] ? sa[r] * scale_log2 : -INFINITY;
            t[4 + r] = (has_b && key_b + r <= pos[s]) ? sb[r] * scale_log2 : -INFINITY;
          }
        }
        const float lm = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])), fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
        if (__any(lm > m_ref[s] + EX_LAZY_MAX)) {
          float x = lm;
          x = fmaxf(x, __shfl_xor(x, 16, 64));
          x = fmaxf(x, __shfl_xor(x, 32, 64));
          const float m_new = fmaxf(m_ref[s], x);
          const float alpha = __builtin_amdgcn_exp2f(m_ref[s] - m_new);
          l_part[s] *= alpha;
          m_ref[s] = m_new;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float ar = __shfl(alpha, 4 * g + r, 64);
#pragma unroll
            for (int mf = 0; mf < 8; ++mf) acc[s][mf][r] *= ar;
          }
        }
        float pr[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          pr[e] = __builtin_amdgcn_exp2f(t[e] - m_ref[s]);
          l_part[s] += pr[e];
        }
        pw[s].x = ex_pack_bf16(pr[0], pr[1]);
        pw[s].y = ex_pack_bf16(pr[2], pr[3]);
        pw[s].z = ex_pack_bf16(pr[4], pr[5]);
        pw[s].w = ex_pack_bf16(pr[6], pr[7]);
      }
      const uint32_t *ra[8] = {&va[0].x, &va[1].x, &va[2].x, &va[3].x, &vb[0].x, &vb[1].x, &vb[2].x, &vb[3].x};
#pragma unroll
      for (int mf = 0; mf < 8; ++mf) {
        uint4 col;
        uint32_t *cw = &col.x;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t x0 = ra[2 * u][mf >> 1], x1 = ra[2 * u + 1][mf >> 1];
          cw[u] = (mf & 1) ? __builtin_amdgcn_perm(x1, x0, 0x07060302u) : __builtin_amdgcn_perm(x1, x0, 0x05040100u);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s)
          acc[s][mf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ex_as_bf16x8(pw[s]), ex_as_bf16x8(col), acc[s][mf], 0, 0, 0);
      }
    }
    if (more) EXL_PARK((it + 1) & 1);
    __syncthreads();
  }
#undef EXL_PAGE_ID
#undef EXL_FETCH
#undef EXL_PARK
  if (!active) return;

#pragma unroll
  for (int s = 0; s < 2; ++s) {
    float lt = l_part[s];
    lt += __shfl_xor(lt, 16, 64);
    lt += __shfl_xor(lt, 32, 64);
    const int tl = tok0 + 4 * s + g;
    const bool ok = tl < ext && ext_off + tl < n_ext_total;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float inv = 1.f / __shfl(lt, 4 * g + r, 64);
      if (!ok) continue;
      const int64_t o = ((int64_t)(ext_off + tl) * cfg.q_heads + kvh * TIM_G + r) * TIM_D + 8 * n;
      if (OUT_BF16) {
        uint4 v;
        v.x = ex_pack_bf16(acc[s][0][r] * inv, acc[s][1][r] * inv);
        v.y = ex_pack_bf16(acc[s][2][r] * inv, acc[s][3][r] * inv);
        v.z = ex_pack_bf16(acc[s][4][r] * inv, acc[s][5][r] * inv);
        v.w = ex_pack_bf16(acc[s][6][r] * inv, acc[s][7][r] * inv);
        *reinterpret_cast<uint4 *>(reinterpret_cast<__bf16 *>(out_ext) + o) = v;
      } else {
        float *dst = reinterpret_cast<float *>(out_ext) + o;
        *reinterpret_cast<float4 *>(dst) = make_float4(acc[s][0][r] * inv, acc[s][1][r] * inv, acc[s][2][r] * inv, acc[s][3][r] * inv);
        *reinterpret_cast<float4 *>(dst + 4) = make_float4(acc[s][4][r] * inv, acc[s][5][r] * inv, acc[s][6][r] * inv, acc[s][7][r] * inv);
      }
    }
  }
}

extern "C" int tim_extend_attn(tim_ctx *ctx, int32_t layer, const tim_plan *plan, const void *q_ext, void *out_ext,
                               int32_t n_ext_total, float sm_scale, int32_t out_dtype, tim_stream stream) {
  if (!ctx || !ctx->bound || !plan || !plan->hdr || !plan->totals || plan->n_seqs <= 0 ||
      plan->n_seqs > plan->max_seqs || layer < 0 || layer >= ctx->cfg.layers || n_ext_total < 0 ||
      ctx->cfg.page_size != TIM_PS ||  // the extend kernel reads 16-token pages only
      (out_dtype != TIM_OUT_F32 && out_dtype != TIM_OUT_BF16))
    return TIM_ERR_INVALID_ARG;
  if (n_ext_total == 0) return TIM_OK;
  if (!q_ext || !out_ext) return TIM_ERR_INVALID_ARG;
  // every sequence adds at most one partly filled tile
  const int tiles = (n_ext_total + EX_TILE_TOKENS - 1) / EX_TILE_TOKENS + plan->n_seqs;
  dim3 grid(ctx->cfg.kv_heads, tiles);
  const float scale_log2 = sm_scale * 1.4426950408889634f;
  const uint4 *q4 = reinterpret_cast<const uint4 *>(q_ext);
  if (ctx->extend_lds) {
    if (out_dtype == TIM_OUT_BF16)
      hipLaunchKernelGGL((tim_extend_attn_lds_kernel<true>), grid, dim3(EX_THREADS), 0, tim_hs(stream), ctx->cfg, ctx->st,
                         *plan, plan->n_seqs, layer, q4, out_ext, n_ext_total, scale_log2);
    else
      hipLaunchKernelGGL((tim_extend_attn_lds_kernel<false>), grid, dim3(EX_THREADS), 0, tim_hs(stream), ctx->cfg, ctx->st,
                         *plan, plan->n_seqs, layer, q4, out_ext, n_ext_total, scale_log2);
  } else if (out_dtype == TIM_OUT_BF16)
    hipLaunchKernelGGL((tim_extend_attn_kernel<true>), grid, dim3(EX_THREADS), 0, tim_hs(stream), ctx->cfg, ctx->st, *plan,
                       plan->n_seqs, layer, reinterpret_cast<const uint4 *>(q_ext), out_ext, n_ext_total, scale_log2);
  else
    hipLaunchKernelGGL((tim_extend_attn_kernel<false>), grid, dim3(EX_THREADS), 0, tim_hs(stream), ctx->cfg, ctx->st, *plan,
                       plan->n_seqs, layer, reinterpret_cast<const uint4 *>(q_ext), out_ext, n_ext_total, scale_log2);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}
