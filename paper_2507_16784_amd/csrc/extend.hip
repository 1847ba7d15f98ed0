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
#include <type_traits>

#define EX_THREADS 256
#define EX_TILE_TOKENS 32
#define EX_WAVE_TOKENS 8
#define EX_NEG_BIG (-1.0e30f)
#define EX_LAZY_MAX 8.0f
#define EX_LAZY_LIMIT 256.0f  // 2^EX_LAZY_MAX

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
// through the vector L1, each wave copies one of the pair's four 4 KiB tiles (K page A, K page
// B, V page A, V page B) from global memory straight into LDS, and all waves read their MFMA
// operands from there.  Two LDS buffers: the copies of the next pair are in flight while this
// pair is multiplied, and one barrier per pair separates readers from the next writer.
//
// Matrix instruction.  The 32x32x16 bf16 MFMA, not the 16x16x32 one of the decode kernel:
// a loop of nothing but independent MFMAs sustains 1.8-2.1 PFLOP/s with the former and
// 1.36 PFLOP/s with the latter on this chip (measured; nominal peak 2.5).  A wave's 32 query
// rows (8 tokens x 4 heads) are exactly one 32-wide operand, a pair of pages the other.
//
// Operands.  Lane l = 32 h + j.  Scores S^T = K . Q^T: A operand = K, lane (h, j) reads key j
// of the pair (page j / 16, row j % 16), 16-byte chunk 2 t + h for step t of 8; B operand =
// Q, the lane's own query row j, same chunk.  The result has, in register r of lane (h, j),
// the score of row j against key 8 (r / 4) + 4 h + r % 4: a query row's 16 scores per half
// wave sit in one lane, so the softmax arithmetic is lane-local and the weights, packed, are
// directly the A operand of the output product (registers 0..7: page A, 8..15: page B).
// Its B operand, V, is read with the transposing LDS load: each group of 16 lanes points at
// four rows x 16 dims, and lane (h, j) receives V[4 h + x][32 c + j], x = 0..3, and with a
// second read the same of rows + 8: the 8 keys that the weights' registers hold.  No
// transposition in registers.  Output O: register r of lane (h, j) holds row
// 8 (r / 4) + 4 h + r % 4, dim 32 c + j of block c.
//
// Bank conflicts.  Measured on this chip: a 16-byte-per-lane LDS read is served 16 lanes at a
// time, and the lanes served together are not consecutive: of lanes 0..31 they are
// {0-3, 12-15, 20-23, 24-27} and {4-7, 8-11, 16-19, 28-31} (same for 32..63); such a group is
// conflict-free when its 16-byte slots differ modulo 256 bytes.  For K, chunk c of row r is
// stored at slot c ^ r, which makes the slots of each group a permutation of 0..15.  (Rows
// padded to 272 bytes, the usual remedy, collide two-way under this grouping.)  For V, the
// 64-byte unit u of row r is stored at unit u ^ (r % 4): the four rows that a transposing
// read touches per half-wave then lie in four different 64-byte bank groups.  The copy into LDS writes
// 1 KiB (4 rows) per instruction in lane order, so the swizzle is applied on the global
// side: each lane fetches the chunk that belongs in its slot.
//
// The copies are issued from inline assembly: the compiler, seeing its own builtin for the
// same instruction, makes every LDS read of the kernel wait for all copies in flight (it
// cannot tell the two buffers apart), which would serialise copy and compute.  The wait for
// the copies is therefore written by hand before each barrier.
#define EXL_TILE_BYTES TIM_TILE_BYTES
#define EXL_PAIR_BYTES (2 * EXL_TILE_BYTES)  // one pair of pages of K, or of V
#define EXL_RING 3                           // pairs of K, and of V, in LDS: one in use, two on their way

typedef __attribute__((address_space(3))) unsigned char *exl_lds_ptr;
typedef short exl_s16x4 __attribute__((ext_vector_type(4)));
typedef float exl_f32x16 __attribute__((ext_vector_type(16)));

// 16 bytes per lane from global memory into LDS at lds_base + 16 * lane (lds_base is wave-uniform)
__device__ __forceinline__ void exl_copy16(const void *src, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(src) : "memory");
}
__device__ __forceinline__ void exl_wait_copies() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// all but the four youngest copies of this wave (memory operations complete in order)
__device__ __forceinline__ void exl_wait_older_copies() { asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); }

typedef unsigned int exl_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 exl_read16(exl_lds_ptr p) {
  return __builtin_bit_cast(uint4, *(const __attribute__((address_space(3))) exl_u32x4 *)p);
}
// transposing read: see the operand note above
__device__ __forceinline__ uint2 exl_read_tr(exl_lds_ptr p) {
  return __builtin_bit_cast(uint2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) exl_s16x4 *)p));
}

template <bool OUT_BF16>
__global__ void __launch_bounds__(EX_THREADS, 2)
tim_extend_attn_lds_kernel(tim_config cfg, tim_state st, tim_plan pl, int n_seqs, int layer,
                           const uint4 *__restrict__ q_ext, void *__restrict__ out_ext, int n_ext_total,
                           float scale_log2) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * EXL_RING * EXL_PAIR_BYTES];
  const int kvh = blockIdx.x;
  if (!pl.totals[TIM_TOT_OK] || (int)blockIdx.y >= pl.totals[TIM_TOT_EXT_TILES]) return;
  const int tile = pl.totals[TIM_TOT_EXT_TILES] - 1 - blockIdx.y;
  int lo = 0, hi = n_seqs - 1;  // flushed sequence of this tile: last e with EXT_TILE_OFF[e] <= tile
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (pl.hdr[(int64_t)mid * TIM_PLAN_HDR + TIM_HDR_EXT_TILE_OFF] <= tile) lo = mid; else hi = mid - 1;
  }
  const int32_t *hdr = pl.hdr + (int64_t)lo * TIM_PLAN_HDR;
  if (hdr[TIM_HDR_BAD]) return;  // uniform for the block, like every exit before the barriers
  const int b = hdr[TIM_HDR_SEQ], m = hdr[TIM_HDR_N_KEPT], f = hdr[TIM_HDR_FIRST_PRUNED];
  const int ext = hdr[TIM_HDR_EXT], ext_off = hdr[TIM_HDR_EXT_OFF];
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, h = lane >> 5, j = lane & 31;
  const int blk_tok0 = (tile - hdr[TIM_HDR_EXT_TILE_OFF]) * EX_TILE_TOKENS;
  const int tok0 = blk_tok0 + w * EX_WAVE_TOKENS;
  const bool active = tok0 < ext;  // a wave without a token still copies and meets the barriers

  // B operands of the score product: this lane's query row j = (token j / 4, head j % 4), chunks 2 t + h.
  // A negative scale is applied as |scale| to -q, which is exact.
  const uint32_t q_flip = scale_log2 < 0.f ? 0x80008000u : 0u;
  const float scale_abs = fabsf(scale_log2);
  uint4 qb[8];
  int pos;  // position of the lane's query row; -1: no such row
  {
    const int tl = tok0 + (j >> 2);
    const bool ok = tl < ext && ext_off + tl < n_ext_total;
    pos = ok ? f + tl : -1;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      uint4 q = make_uint4(0, 0, 0, 0);
      if (ok) q = q_ext[((int64_t)(ext_off + tl) * cfg.q_heads + kvh * TIM_G + (j & 3)) * 16 + 2 * t + h];
      qb[t] = make_uint4(q.x ^ q_flip, q.y ^ q_flip, q.z ^ q_flip, q.w ^ q_flip);
    }
  }
  const int blk_first_pos = f + blk_tok0;
  // block-uniform: the pairs of pages the block walks, and how many of them lie wholly at or
  // before its first position (no mask, no stale row, both pages present)
  const int last_page = (f + min(blk_tok0 + EX_TILE_TOKENS, ext) - 1) / TIM_PS;
  const int n_pairs = last_page / 2 + 1;
  const int n_full = min(n_pairs, (blk_first_pos + 1) / (2 * TIM_PS));

  float m_ref = EX_NEG_BIG, l_part = 0.f;  // of the lane's row j; l_part covers the keys of this half wave
  exl_f32x16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;

  const uint4 *kpool = reinterpret_cast<const uint4 *>(st.k_pool);
  const uint4 *vpool = reinterpret_cast<const uint4 *>(st.v_pool);
  const int32_t *ptab = st.page_table + (int64_t)b * cfg.max_pages_per_seq;
  const int64_t layer_base = (int64_t)layer * cfg.num_pages;

  // ---- LDS: a ring of EXL_RING pairs of K tiles and one of V tiles, 8 KiB (page A, page B) per pair;
  // pair q lives in slot q % EXL_RING of each.  While pair p is weighted, K holds pairs p + 1 (read),
  // p + 2 (arrived or arriving) and p + 3 (requested now), V holds p, p + 1, p + 2 likewise: a copy has
  // two trips of the loop to arrive.
  // ---- the copy side: waves 0 and 1 bring K pages A and B, waves 2 and 3 bring V pages A and B
  const int ws = __builtin_amdgcn_readfirstlane(w);
  const bool k_wave = ws < 2;
  const uint4 *tile_pool = k_wave ? kpool : vpool;
  int src_unit[4];  // which 16-byte unit of the tile lane l fetches with copy i (slot l % 16 of row 4 i + l / 16)
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 4 * i + (lane >> 4), slot = lane & 15;
    src_unit[i] = r * 16 + (k_wave ? slot ^ r : slot ^ ((r & 3) << 2));
  }
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)lds);
  const uint32_t copy_base = lds_base + (k_wave ? 0 : EXL_RING * EXL_PAIR_BYTES) + (ws & 1) * EXL_TILE_BYTES;
  // Page ids: lane l of pid_vec holds the id of this wave's page of pair pid_base + l; one load per 64 pairs
  // keeps the loop free of global loads (whose waits would also wait for the copies in flight).
  auto load_pids = [&](int base) { return ptab[min(2 * (base + lane) + (ws & 1), last_page)]; };
  int pid_base = 0;
  int pid_vec = load_pids(0);
  auto copy_tile = [&](int pair_, int slot) {  // pair_ in [pid_base, pid_base + 64)
    int phys = __builtin_amdgcn_readlane(pid_vec, pair_ - pid_base);
    if (phys < 0 || phys >= cfg.num_pages) {
      tim_set_status(st.status, TIM_ERR_INVALID_ARG);  // never dereference a bad page id
      phys = 0;
    }
    const uint4 *src = tile_pool + ((layer_base + phys) * cfg.kv_heads + kvh) * (TIM_TILE_BYTES / 16);
    const uint32_t dst = copy_base + slot * EXL_PAIR_BYTES;
    exl_copy16(src + src_unit[0], dst);
    exl_copy16(src + src_unit[1], dst + 1024);
    exl_copy16(src + src_unit[2], dst + 2048);
    exl_copy16(src + src_unit[3], dst + 3072);
  };

  // ---- the read side: LDS offsets of this lane's operands within a pair's 8 KiB
  const exl_lds_ptr lds3 = (exl_lds_ptr)lds;
  // K: key j = (page j / 16, row j % 16), chunk (2 t + h) ^ row.  The step is three address bits of their
  // own (5..7), so the offset of step t is k_off0 ^ (t << 5).
  const int k_off0 = (j >> 4) * EXL_TILE_BYTES + (j & 15) * 256 + ((h ^ (j & 15)) << 4);
  // V: the 16 lanes of group G = lane / 16 point at rows 4 h + jj / 4 (jj = lane % 16), dims
  // 32 c + 16 (G % 2) + 4 (jj % 4) .. + 3, i.e. 64-byte unit c of the row, stored at unit c ^ (row % 4).
  // The unit is two address bits of their own (6..7): offset of block c = v_off0 ^ (c << 6).
  const int v_row = 4 * h + ((lane & 15) >> 2);
  const int v_off0 = EXL_RING * EXL_PAIR_BYTES + v_row * 256 + ((v_row & 3) << 6) + 32 * ((lane >> 4) & 1) + 8 * (lane & 3);

  // The A operands of a pair's score product, from the given slot of the K ring.
  auto read_k = [&](int slot, uint4 (&ka)[8]) {
    const exl_lds_ptr buf = lds3 + slot * EXL_PAIR_BYTES;
#pragma unroll
    for (int t = 0; t < 8; ++t) ka[t] = exl_read16(buf + (k_off0 ^ (t << 5)));
  };
  // scores, raw (unscaled, unmasked): raw[r] = row j against key 8 (r / 4) + 4 h + r % 4 of the pair
  auto scores = [&](const uint4 (&ka)[8], float (&raw)[16]) {
    exl_f32x16 sc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t)
      sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ex_as_bf16x8(ka[t]), ex_as_bf16x8(qb[t]), sc, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 16; ++r) raw[r] = sc[r];
  };

  // One trip of the pipeline, pair p, s0 = p % EXL_RING: the scores of pair p + 1 go through the matrix
  // cores while the vector units turn the scores of pair p (in `cur`) into weights; then the products of
  // pair p.  K of pair p + 3 and V of pair p + 2 are requested.  DIAG: pair p may hold keys beyond some
  // row's own position, rows past the sequence, or no second page (the DIAG instance is also correct for
  // any other pair, only slower).
  //
  // Lazy reference maximum, checked on the weights: they are first computed against the current
  // reference; only if one of them exceeds 2^EX_LAZY_MAX (always on the first pair: every weight is then
  // infinite) is the reference renewed from the scores, the accumulators rescaled and the weights redone.
  auto trip = [&](int p, int s0, auto diag_c, float (&cur)[16], float (&nxt)[16]) {
    constexpr bool DIAG = decltype(diag_c)::value;
    const int s1 = s0 == EXL_RING - 1 ? 0 : s0 + 1, s2 = s1 == EXL_RING - 1 ? 0 : s1 + 1;
    // The operands are fetched from LDS as early as the code allows, in basic blocks of their own, because the
    // compiler otherwise puts each read right in front of its use: K of pair p + 1 here, V of pair p before
    // the check of the maximum.  (Past the last pair this reads stale tiles; the scores are not used.)
    uint4 ka[8];
    read_k(s1, ka);
    // K of pair p + 3 takes the slot of pair p, V of pair p + 2 that of pair p - 1: every wave left both
    // at the last barrier
    const int cp = p + (k_wave ? 3 : 2);
    const bool copied = cp < n_pairs;
    if (copied) {
      if (cp - pid_base == 64) {
        pid_base = cp;
        pid_vec = load_pids(cp);
      }
      copy_tile(cp, k_wave ? s0 : s2);
    }
    if (active) {
      const int key0 = 2 * p * TIM_PS + 4 * h;  // key of register r: key0 + 8 (r / 4) + r % 4
      const bool has_b = !DIAG || 2 * p + 1 <= last_page;
      scores(ka, nxt);
      // weights of the lane's row against the current reference, packed: pw[u] covers page u; returns the largest
      uint4 pw[2];
      auto weights = [&]() {
        float pe[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) pe[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[r], scale_abs, -m_ref));
        const float top = fmaxf(fmaxf(fmaxf(fmaxf(pe[0], pe[1]), fmaxf(pe[2], pe[3])), fmaxf(fmaxf(pe[4], pe[5]), fmaxf(pe[6], pe[7]))),
                                fmaxf(fmaxf(fmaxf(pe[8], pe[9]), fmaxf(pe[10], pe[11])), fmaxf(fmaxf(pe[12], pe[13]), fmaxf(pe[14], pe[15]))));
        if (DIAG) {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (key0 + 8 * (r >> 2) + (r & 3) > pos || (r >= 8 && !has_b)) pe[r] = 0.f;
        }
        const float sum = (((pe[0] + pe[1]) + (pe[2] + pe[3])) + ((pe[4] + pe[5]) + (pe[6] + pe[7]))) +
                          (((pe[8] + pe[9]) + (pe[10] + pe[11])) + ((pe[12] + pe[13]) + (pe[14] + pe[15])));
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          pw[u].x = ex_pack_bf16(pe[8 * u + 0], pe[8 * u + 1]);
          pw[u].y = ex_pack_bf16(pe[8 * u + 2], pe[8 * u + 3]);
          pw[u].z = ex_pack_bf16(pe[8 * u + 4], pe[8 * u + 5]);
          pw[u].w = ex_pack_bf16(pe[8 * u + 6], pe[8 * u + 7]);
        }
        return make_float2(top, sum);
      };
      if (DIAG) {
#pragma unroll
        for (int r = 0; r < 16; ++r)  // a masked score is a large negative finite number: it survives a zero scale
          if (key0 + 8 * (r >> 2) + (r & 3) > pos || (r >= 8 && !has_b)) cur[r] = EX_NEG_BIG;
      }
      const exl_lds_ptr vbuf = lds3 + s0 * EXL_PAIR_BYTES;
      uint4 col[4][2];
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const exl_lds_ptr at = vbuf + u * EXL_TILE_BYTES + (v_off0 ^ (c << 6));
          const uint2 ta = exl_read_tr(at), tb = exl_read_tr(at + 8 * 256);
          col[c][u] = make_uint4(ta.x, ta.y, tb.x, tb.y);
        }
      float2 ts = weights();
      if (__any(ts.x > EX_LAZY_LIMIT)) {
        float x = cur[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) x = fmaxf(x, cur[r]);
        x *= scale_abs;
        x = fmaxf(x, __shfl_xor(x, 32, 64));  // the other half of the row's keys
        const float m_new = fmaxf(m_ref, x);
        const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
        m_ref = m_new;
        l_part *= alpha;
#pragma unroll
        for (int r = 0; r < 16; ++r) {  // the accumulators hold other rows than the lane's own
          const float ar = __shfl(alpha, 8 * (r >> 2) + 4 * h + (r & 3), 64);
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[c][r] *= ar;
        }
        ts = weights();
      }
      l_part += ts.y;
      uint4 live[2] = {make_uint4(~0u, ~0u, ~0u, ~0u), make_uint4(~0u, ~0u, ~0u, ~0u)};
      if (DIAG) {  // rows past the sequence may hold anything: their V is cleared (element e of the operand:
                   // key 16 u + 8 (e / 4) + 4 h + e % 4 of the pair)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int k = key0 + 16 * u;
          const bool pg_ok = u == 0 || has_b;
          live[u].x = (pg_ok && k + 0 < m ? 0x0000FFFFu : 0u) | (pg_ok && k + 1 < m ? 0xFFFF0000u : 0u);
          live[u].y = (pg_ok && k + 2 < m ? 0x0000FFFFu : 0u) | (pg_ok && k + 3 < m ? 0xFFFF0000u : 0u);
          live[u].z = (pg_ok && k + 8 < m ? 0x0000FFFFu : 0u) | (pg_ok && k + 9 < m ? 0xFFFF0000u : 0u);
          live[u].w = (pg_ok && k + 10 < m ? 0x0000FFFFu : 0u) | (pg_ok && k + 11 < m ? 0xFFFF0000u : 0u);
        }
      }
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          uint4 x = col[c][u];
          if (DIAG) x = make_uint4(x.x & live[u].x, x.y & live[u].y, x.z & live[u].z, x.w & live[u].w);
          acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ex_as_bf16x8(pw[u]), ex_as_bf16x8(x), acc[c], 0, 0, 0);
        }
    }
    // what the next trip reads was requested one trip ago: only this trip's four copies may still be under way
    if (copied) exl_wait_older_copies();
    else exl_wait_copies();
    __syncthreads();
  };

  // fill the pipeline: K of pairs 0, 1 and 2, V of pairs 0 and 1; scores of pair 0
  for (int q = 0; q < (k_wave ? 3 : 2); ++q)
    if (q < n_pairs) copy_tile(q, q);
  exl_wait_copies();
  __syncthreads();
  float raw_even[16], raw_odd[16];  // scores waiting to be weighted: of even pairs, of odd pairs (hot loop)
  if (active) {
    uint4 ka[8];
    read_k(0, ka);
    scores(ka, raw_even);
  }
  __syncthreads();  // the first trip overwrites the K tiles just read
  // All bounds are the same for the whole block.
  int p = 0, s0 = 0;  // s0 = p % EXL_RING
  auto advance = [&]() {
    ++p;
    s0 = s0 == EXL_RING - 1 ? 0 : s0 + 1;
  };
  while (p + 2 <= n_full) {  // two pairs per trip of the loop: the two score arrays swap roles without copies
    trip(p, s0, std::false_type{}, raw_even, raw_odd);
    advance();
    trip(p, s0, std::false_type{}, raw_odd, raw_even);
    advance();
  }
  while (p < n_pairs) {  // the last of the full pairs, if their number is odd, and the pairs at the diagonal
    trip(p, s0, std::true_type{}, raw_even, raw_odd);
    advance();
#pragma unroll
    for (int r = 0; r < 16; ++r) raw_even[r] = raw_odd[r];
  }
  if (!active) return;

  // register r of lane (h, j) holds row i = 8 (r / 4) + 4 h + r % 4 = (token i / 4, head i % 4), dim 32 c + j;
  // the row's denominator is the sum of the two partial ones in lanes i and i + 32
  const float l_row = l_part + __shfl_xor(l_part, 32, 64);
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = 8 * (r >> 2) + 4 * h + (r & 3);
    const float inv = 1.f / __shfl(l_row, i, 64);
    const int tl = tok0 + (i >> 2);
    if (!(tl < ext && ext_off + tl < n_ext_total)) continue;
    const int64_t o = ((int64_t)(ext_off + tl) * cfg.q_heads + kvh * TIM_G + (i & 3)) * TIM_D + j;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float y = acc[c][r] * inv;
      if (OUT_BF16) reinterpret_cast<__bf16 *>(out_ext)[o + 32 * c] = (__bf16)y;
      else reinterpret_cast<float *>(out_ext)[o + 32 * c] = y;
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
  if (ctx->extend_lds) {  // (the kernel's LDS array is the only one, so its offset in LDS is 0 and 1 KiB-aligned)
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
