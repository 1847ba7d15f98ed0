// Extend attention: the attention half of re-encoding the repositioned tokens (the paper's
// own way of reassigning positions, Eq. 1).  After a flush, each survivor behind the first
// pruned token attends causally to everything up to and including itself in the compacted
// cache.  Many queries share each key, so unlike decode this kernel reuses every K/V tile
// for 128 (token, head) query rows per block and is bounded by the matrix cores, not by HBM.
//
// Decomposition.  grid = (kv_heads, tiles of 32 extended tokens); workgroup ids run over
// the kv heads first, so that with 8 heads each XCD keeps one head's K/V in its L2 for all
// query tiles, and tiles are taken last-first (under the causal mask the late tiles of a
// sequence are the long ones; starting them first shortens the tail).  A block's four
// waves take 8 tokens each: two sets of 16 query rows (4 tokens x the 4 heads of the
// group).  Per pair of key pages and per set a wave runs S^T = K . Q^T (K tile as A
// operand, the 16 query rows as B columns) and O += P . V with the weights staying in
// their lanes.  Causality is a mask on the pairs at the diagonal only.  One lazy reference
// maximum per query row.
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

// Staging.  The four waves of a block need the same K and V tiles.  Instead of each wave
// pulling them through the vector L1, each wave copies one of a pair's four 4 KiB tiles (K
// page A, K page B, V page A, V page B) from global memory straight into LDS, and all waves
// read their MFMA operands from there.  K and V each have a ring of three pairs in LDS: one
// being read, one arrived or arriving, one requested; a copy has two trips of the loop to
// land, and one barrier per pair separates the readers of a slot from its next writer.
//
// Pipeline.  The scores run one pair ahead of the weights and products: in one trip the
// matrix cores take K(p + 1) . Q^T while the vector units turn the scores of pair p into
// weights; then P(p) . V(p).  The softmax denominators come from the matrix cores as well
// (P times a column of ones).  The weights are computed speculatively against the current
// reference maximum and only redone when one of them exceeds 2^8.
//
// Operands.  K (A operand of the score product) is read as "row n, 16-byte chunk 4 s + g".
// V (B operand of the output product) is read with the transposing LDS load: lanes (g, j)
// point at row 4 g + j / 4, dims 16 mf + 4 (j % 4) .. +3, and lane (g, n) receives
// V[4 g + e][16 mf + n], e = 0..3, which together with the same read of the second page is
// the B operand for output columns 16 mf .. 16 mf + 15.  No transposition in registers.
//
// Bank conflicts.  Measured on this chip: a 16-byte-per-lane LDS read is served 16 lanes at a
// time, and the lanes served together are not consecutive: of lanes 0..31 they are
// {0-3, 12-15, 20-23, 24-27} and {4-7, 8-11, 16-19, 28-31} (same for 32..63); such a group is
// conflict-free when its 16-byte slots differ modulo 256 bytes.  For K, chunk c of row r is
// stored at slot c ^ r, which makes the slots of each group a permutation of 0..15.  (Rows
// padded to 272 bytes, the usual remedy, collide two-way under this grouping.)  For V, the
// 32-byte unit u of row r is stored at unit u ^ (r % 8): the eight rows that a transposing
// read touches per half-wave then lie in eight different 32-byte bank groups (measured
// conflict-free; unswizzled the same read is 3.5 times slower).  The copy into LDS writes
// 1 KiB (4 rows) per instruction in lane order, so the swizzle is applied on the global
// side: each lane fetches the chunk that belongs in its slot.
//
// The copies are issued from inline assembly: the compiler, seeing its own builtin for the
// same instruction, makes every LDS read of the kernel wait for all copies in flight (it
// cannot tell the slots apart), which would serialise copy and compute.  The wait for the
// copies is therefore written by hand before each barrier, and the loop itself holds no
// other global load (page ids are fetched 64 pairs at a time), whose wait would be a wait
// for the copies too.
//
// Matrix instruction.  16x16x32 bf16.  A loop of nothing but independent MFMAs sustains
// 1.36 PFLOP/s with it and 1.8-2.1 PFLOP/s with the 32x32x16 form on this chip (nominal
// 2.5; the shader clock falls to 1.9-2.0 GHz under matrix load).  A 32x32x16 version of
// this kernel (a wave's 32 rows as one operand, weights lane-local, same staging) was
// measured at 835-866 TFLOP/s against 908 for this one: here neither pipe is saturated
// (matrix cores 40-45 % busy, vector units about the same, LDS 25-40 %), the time goes
// into their imperfect overlap within the two waves per SIMD that the registers allow.
#define EXL_TILE_BYTES TIM_TILE_BYTES
#define EXL_PAIR_BYTES (2 * EXL_TILE_BYTES)  // one pair of pages of K, or of V
#define EXL_RING 3                           // pairs of K, and of V, in LDS: one in use, two on their way

typedef __attribute__((address_space(3))) unsigned char *exl_lds_ptr;
typedef short exl_s16x4 __attribute__((ext_vector_type(4)));

// 16 bytes per lane from global memory into LDS at lds_base + 16 * lane (lds_base is wave-uniform).
// The statement overwrites m0 and says so: the compiler sets m0 itself before each of its own uses
// (LDS-DMA builtins, indexed register moves, messages) and merges such settings when it sees no
// write between them, so an undeclared write here could leave a later use with this address.  m0 is
// a reserved register, for which clang prints a generic caution; that is the one diagnostic silenced.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void exl_copy16(const void *src, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(src) : "memory", "m0");
}
#pragma clang diagnostic pop
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
tim_extend_attn_kernel(tim_config cfg, tim_state st, tim_plan pl, int n_seqs, int layer,
                           const uint4 *__restrict__ q_ext, void *__restrict__ out_ext, int n_ext_total,
                           float scale_log2) {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * EXL_RING * EXL_PAIR_BYTES];
  const int kvh = blockIdx.x;
  if (!pl.totals[TIM_TOT_OK]) return;
  if (n_ext_total < pl.totals[TIM_TOT_EXT]) {  // the caller's buffers hold fewer rows than the plan extends: nothing is written
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) tim_set_status(st.status, TIM_ERR_INVALID_ARG);
    return;
  }
  if ((int)blockIdx.y >= pl.totals[TIM_TOT_EXT_TILES]) return;
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
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, g = lane >> 4, n = lane & 15;
  const int blk_tok0 = (tile - hdr[TIM_HDR_EXT_TILE_OFF]) * EX_TILE_TOKENS;
  const int tok0 = blk_tok0 + w * EX_WAVE_TOKENS;
  const bool active = tok0 < ext;  // a wave without a token still copies and meets the barriers

  // B operands of the score product: column n of set s is (token 4 s + n / 4, head n % 4).
  // A negative scale is applied as |scale| to -q, which is exact.
  const uint32_t q_flip = scale_log2 < 0.f ? 0x80008000u : 0u;
  const float scale_abs = fabsf(scale_log2);
  uint4 qb[2][4];
  int pos[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int tl = tok0 + 4 * s + (n >> 2);
    const bool ok = tl < ext && ext_off + tl < n_ext_total;
    pos[s] = ok ? f + tl : -1;
#pragma unroll
    for (int step = 0; step < 4; ++step) {
      uint4 q = make_uint4(0, 0, 0, 0);
      if (ok) q = q_ext[((int64_t)(ext_off + tl) * cfg.q_heads + kvh * TIM_G + (n & 3)) * 16 + 4 * step + g];
      qb[s][step] = make_uint4(q.x ^ q_flip, q.y ^ q_flip, q.z ^ q_flip, q.w ^ q_flip);
    }
  }
  const int blk_first_pos = f + blk_tok0;
  const int last_pos = f + min(tok0 + EX_WAVE_TOKENS, ext) - 1;  // this wave's largest position
  // block-uniform: the pairs of pages the block walks, and how many of them lie wholly at or
  // before its first position (no mask, no stale row, both pages present)
  const int last_page = (f + min(blk_tok0 + EX_TILE_TOKENS, ext) - 1) / TIM_PS;
  const int n_pairs = last_page / 2 + 1;
  const int n_full = min(n_pairs, (blk_first_pos + 1) / (2 * TIM_PS));

  // The softmax denominators come from the matrix cores too: P times a column of ones, in the
  // same layout (row 4 g + r in register r) as the output accumulators.
  const uint4 ones = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
  float m_ref[2] = {EX_NEG_BIG, EX_NEG_BIG};
  ex_f32x4 lsum[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  ex_f32x4 acc[2][8];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int mf = 0; mf < 8; ++mf) acc[s][mf] = (ex_f32x4){0.f, 0.f, 0.f, 0.f};

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
    src_unit[i] = r * 16 + (k_wave ? slot ^ r : slot ^ ((r & 7) << 1));
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
  int k_off[4];
#pragma unroll
  for (int step = 0; step < 4; ++step) k_off[step] = n * 256 + (((4 * step + g) ^ n) << 4);
  // V: row r = 4 g + n / 4, unit mf ^ (r % 8), piece n % 4; the unit is three address bits of their own,
  // so the offset for column block mf is v_off0 ^ (mf << 5)
  const int v_off0 = EXL_RING * EXL_PAIR_BYTES + (4 * g + (n >> 2)) * 256 + (((4 * g + (n >> 2)) & 7) << 5) + 8 * (n & 3);

  // scores of the pair whose K lies in the given slot of the K ring: both row sets, raw (unscaled, unmasked)
  auto scores = [&](int slot, float (&raw)[2][8]) {
    const exl_lds_ptr buf = lds3 + slot * EXL_PAIR_BYTES;
    ex_f32x4 sa[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}}, sb[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int step = 0; step < 4; ++step) {  // four independent accumulation chains; K operands live one step only
      // LDS reads may not be moved up across this point (everything else may): otherwise all eight K
      // operands are fetched first and the kernel runs out of registers
      if (step == 2) __builtin_amdgcn_sched_barrier(0x7F);
      const uint4 ka = exl_read16(buf + k_off[step]), kb = exl_read16(buf + EXL_TILE_BYTES + k_off[step]);
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        sa[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ex_as_bf16x8(ka), ex_as_bf16x8(qb[s][step]), sa[s], 0, 0, 0);
        sb[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ex_as_bf16x8(kb), ex_as_bf16x8(qb[s][step]), sb[s], 0, 0, 0);
      }
    }
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        raw[s][r] = sa[s][r];
        raw[s][4 + r] = sb[s][r];
      }
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
  auto trip = [&](int p, int s0, auto diag_c, float (&cur)[2][8], float (&nxt)[2][8]) {
    constexpr bool DIAG = decltype(diag_c)::value;
    const int s1 = s0 == EXL_RING - 1 ? 0 : s0 + 1, s2 = s1 == EXL_RING - 1 ? 0 : s1 + 1;
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
      const int pg = 2 * p;
      const bool has_b = !DIAG || pg + 1 <= last_page;
      const int key_a = pg * TIM_PS + 4 * g, key_b = key_a + TIM_PS;
      scores(s1, nxt);  // past the last pair this reads stale tiles; unused
      // weights of set s against the current reference, packed; returns their largest
      auto weights = [&](int s, uint4 &packed) {
        float pe[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) pe[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[s][e], scale_abs, -m_ref[s]));
        const float top = fmaxf(fmaxf(fmaxf(pe[0], pe[1]), fmaxf(pe[2], pe[3])), fmaxf(fmaxf(pe[4], pe[5]), fmaxf(pe[6], pe[7])));
        if (DIAG) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (key_a + r > pos[s]) pe[r] = 0.f;
            if (!has_b || key_b + r > pos[s]) pe[4 + r] = 0.f;
          }
        }
        packed.x = ex_pack_bf16(pe[0], pe[1]);
        packed.y = ex_pack_bf16(pe[2], pe[3]);
        packed.z = ex_pack_bf16(pe[4], pe[5]);
        packed.w = ex_pack_bf16(pe[6], pe[7]);
        return top;
      };
      if (DIAG) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
          for (int r = 0; r < 4; ++r) {  // a masked score is a large negative finite number: it survives a zero scale
            if (key_a + r > pos[s]) cur[s][r] = EX_NEG_BIG;
            if (!has_b || key_b + r > pos[s]) cur[s][4 + r] = EX_NEG_BIG;
          }
      }
      uint4 pw[2];
      const float pmax = fmaxf(weights(0, pw[0]), weights(1, pw[1]));
      if (__any(pmax > EX_LAZY_LIMIT)) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
          float x = scale_abs * fmaxf(fmaxf(fmaxf(cur[s][0], cur[s][1]), fmaxf(cur[s][2], cur[s][3])),
                                      fmaxf(fmaxf(cur[s][4], cur[s][5]), fmaxf(cur[s][6], cur[s][7])));
          x = fmaxf(x, __shfl_xor(x, 16, 64));
          x = fmaxf(x, __shfl_xor(x, 32, 64));
          const float m_new = fmaxf(m_ref[s], x);
          const float alpha = __builtin_amdgcn_exp2f(m_ref[s] - m_new);
          m_ref[s] = m_new;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float ar = __shfl(alpha, 4 * g + r, 64);
            lsum[s][r] *= ar;
#pragma unroll
            for (int mf = 0; mf < 8; ++mf) acc[s][mf][r] *= ar;
          }
          weights(s, pw[s]);
        }
      }
#pragma unroll
      for (int s = 0; s < 2; ++s)
        lsum[s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ex_as_bf16x8(pw[s]), ex_as_bf16x8(ones), lsum[s], 0, 0, 0);
      uint4 live = make_uint4(~0u, ~0u, ~0u, ~0u);  // rows past the sequence may hold anything: their V is cleared
      if (DIAG) {
        live.x = (key_a + 0 < m ? 0x0000FFFFu : 0u) | (key_a + 1 < m ? 0xFFFF0000u : 0u);
        live.y = (key_a + 2 < m ? 0x0000FFFFu : 0u) | (key_a + 3 < m ? 0xFFFF0000u : 0u);
        live.z = has_b ? (key_b + 0 < m ? 0x0000FFFFu : 0u) | (key_b + 1 < m ? 0xFFFF0000u : 0u) : 0u;
        live.w = has_b ? (key_b + 2 < m ? 0x0000FFFFu : 0u) | (key_b + 3 < m ? 0xFFFF0000u : 0u) : 0u;
      }
      const exl_lds_ptr vbuf = lds3 + s0 * EXL_PAIR_BYTES;
#pragma unroll
      for (int mf = 0; mf < 8; ++mf) {
        const int v_off = v_off0 ^ (mf << 5);
        const uint2 ta = exl_read_tr(vbuf + v_off), tb = exl_read_tr(vbuf + EXL_TILE_BYTES + v_off);
        uint4 col = make_uint4(ta.x, ta.y, tb.x, tb.y);
        if (DIAG) col = make_uint4(col.x & live.x, col.y & live.y, col.z & live.z, col.w & live.w);
#pragma unroll
        for (int s = 0; s < 2; ++s)
          acc[s][mf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ex_as_bf16x8(pw[s]), ex_as_bf16x8(col), acc[s][mf], 0, 0, 0);
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
  float raw_even[2][8], raw_odd[2][8];  // scores waiting to be weighted: of even pairs, of odd pairs (hot loop)
  if (active) scores(0, raw_even);
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
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int e = 0; e < 8; ++e) raw_even[s][e] = raw_odd[s][e];
  }
  if (!active) return;

  // lane (g, n) holds, for row (token 4 s + g, head r), output columns 16 mf + n
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int tl = tok0 + 4 * s + g;
    if (!(tl < ext && ext_off + tl < n_ext_total)) continue;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float inv = 1.f / lsum[s][r];
      const int64_t o = ((int64_t)(ext_off + tl) * cfg.q_heads + kvh * TIM_G + r) * TIM_D + n;
#pragma unroll
      for (int mf = 0; mf < 8; ++mf) {
        const float y = acc[s][mf][r] * inv;
        if (OUT_BF16) reinterpret_cast<__bf16 *>(out_ext)[o + 16 * mf] = (__bf16)y;
        else reinterpret_cast<float *>(out_ext)[o + 16 * mf] = y;
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
  if (n_ext_total > 0 && (!tim_rows_ok(q_ext) || !tim_rows_ok(out_ext))) return TIM_ERR_INVALID_ARG;  // (with no rows the kernel only checks the plan)
  // every sequence adds at most one partly filled tile
  const int tiles = (n_ext_total + EX_TILE_TOKENS - 1) / EX_TILE_TOKENS + plan->n_seqs;
  dim3 grid(ctx->cfg.kv_heads, tiles);
  const float scale_log2 = sm_scale * 1.4426950408889634f;
  const uint4 *q4 = reinterpret_cast<const uint4 *>(q_ext);
  if (out_dtype == TIM_OUT_BF16)
    hipLaunchKernelGGL((tim_extend_attn_kernel<true>), grid, dim3(EX_THREADS), 0, tim_hs(stream), ctx->cfg, ctx->st, *plan,
                       plan->n_seqs, layer, q4, out_ext, n_ext_total, scale_log2);
  else
    hipLaunchKernelGGL((tim_extend_attn_kernel<false>), grid, dim3(EX_THREADS), 0, tim_hs(stream), ctx->cfg, ctx->st, *plan,
                       plan->n_seqs, layer, q4, out_ext, n_ext_total, scale_log2);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}
