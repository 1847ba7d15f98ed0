// Split-K paged GQA decode attention (HBM-bound: 4096 B per live token per layer).
//
// Work decomposition.  One block per (sequence, kv head, slot).  A sequence's pages are cut
// into chunks of AT_CHUNK_PAGES pages; a sequence uses one slot per `cpb` chunks, and block
// `slot` takes chunks slot, slot + used, ... and accumulates them into one partial
// (m, l, o[128]) per query head of its group.  Inside a chunk each of the four waves
// streams its own run of pages.  Fixed-size chunks keep a batch of very unequal lengths
// balanced: a long sequence simply occupies more blocks.  Which blocks are launched, and in
// which order, is at_take_work's business (a static grid, or the list tim_attn_schedule wrote).
//
// Wave mapping for one (page, kv head) tile of 16 rows x 256 B, K and V alike: load j
// (j = 0..3) is one 16-byte load per lane covering 1 KiB of the tile contiguously, so
// lane (g, c) = (lane / 16, lane % 16) holds dims 8c..8c+7 of row 4j + g.  The dot product
// with the four query heads of the group is finished by a rotate-add over the 16 lanes
// of a DPP row.  Each lane row g keeps its own online-softmax state over the rows it
// sees (4j + g), so the page loop has no cross-row traffic; rows, waves and chunks are
// merged once at the end (log-sum-exp algebra), then a small kernel merges the slots.
#include <hip/hip_ext.h>

#include <mutex>

#include "tim_internal.h"

#define AT_THREADS 256
#define AT_WAVES 4
#define AT_CHUNK_PAGES 16
#define AT_PAGES_PER_WAVE (AT_CHUNK_PAGES / AT_WAVES)
#define AT_MAX_SLOTS 128
#define AT_BLOCKS_PER_CU 3  // of the matrix-core kernel: what its registers allow
#define AT_GRADE_MIN_ROUNDS 3
#define AT_MAX_CPB 64  // tim_tuning.chunks_per_block is at most this
#define AT_SCHED_STAGE 4096  // largest batch that is scheduled: the schedule kernel keeps four words per sequence in LDS
#define AT_NEG_BIG (-1.0e30f)

__device__ __forceinline__ float at_bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float at_bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

template <int CTRL>
__device__ __forceinline__ float at_dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// sum over the 16 lanes of a DPP row; every lane ends with the total
__device__ __forceinline__ float at_row_sum(float v) {
  v += at_dpp<0x128>(v);  // row_ror:8
  v += at_dpp<0x124>(v);  // row_ror:4
  v += at_dpp<0x122>(v);  // row_ror:2
  v += at_dpp<0x121>(v);  // row_ror:1
  return v;
}

__device__ __forceinline__ void at_unpack(const uint4 &u, float (&f)[8]) {
  f[0] = at_bf_lo(u.x); f[1] = at_bf_hi(u.x);
  f[2] = at_bf_lo(u.y); f[3] = at_bf_hi(u.y);
  f[4] = at_bf_lo(u.z); f[5] = at_bf_hi(u.z);
  f[6] = at_bf_lo(u.w); f[7] = at_bf_hi(u.w);
}

struct AttnWs {
  float *ml;             // [B][Hkv][slots][4 heads][m, l]: the 32 bytes one block writes are contiguous
  float *o;              // [B][Hkv][slots][4 heads][128] (fp32, or bf16 in half the bytes): 2 KiB or 1 KiB per block, contiguous
  const int32_t *sched;  // work list written by tim_attn_schedule, or nullptr (see at_take_work)
};
#define AT_SCHED_HDR 4  // words before the items: [0] = number of items; an item is {sequence, slot, length, slots used}

template <bool OUT_BF16>
__device__ __forceinline__ void at_store_out(void *out, int64_t idx, float v) {
  if (OUT_BF16) {
    reinterpret_cast<__bf16 *>(out)[idx] = (__bf16)v;
  } else {
    reinterpret_cast<float *>(out)[idx] = v;
  }
}


typedef __attribute__((address_space(3))) void *at_lds_ptr;
typedef __bf16 at_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 at_bf16x2 __attribute__((ext_vector_type(2)));
typedef float at_f32x4 __attribute__((ext_vector_type(4)));
typedef float at_f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t at_pack_bf16(float lo, float hi) {
  at_f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, at_bf16x2));
}
__device__ __forceinline__ at_bf16x8 at_as_bf16x8(const uint4 &u) { return __builtin_bit_cast(at_bf16x8, u); }

// Partials.  The few KB a block writes cost far more than their size: measured on a uniform 4.3 GB launch, the
// kernel runs at 6.80 TB/s without them and at 6.46 TB/s with 2 KiB per block of ordinary stores into the
// workspace (not the stores' latency: the same stores into one small hot region cost nothing; the cost is
// proportional to the bytes that reach memory while the read stream is running).  So they are kept small and
// written through (agent-scope stores, 6.58 TB/s): with bf16 output a slot's partial output is stored
// normalised (o / l) in bf16, 1 KiB per block; with fp32 output unnormalised in fp32.  m and l are fp32.
__device__ __forceinline__ void at_store_through(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void at_store_through(uint32_t *p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void at_store_through(float4 *p, const float4 &v) {
  const at_f32x4 x = {v.x, v.y, v.z, v.w};
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(x) : "memory");
}

// Block epilogue shared by both variants.  The NS (m, l, o) states the block holds in LDS
// are merged (log-sum-exp algebra).  If the block is the sequence's only one, the result is
// final; otherwise it becomes this slot's partial for the merge kernel.  (Merging in the
// last block to finish, behind an agent-scope counter, was measured and rejected: the
// release/acquire fences it needs write back and invalidate the XCD's whole L2 per block
// and cost 6x the kernel's run time.)
template <int NS, int NT, bool OUT_BF16>  // NS states in LDS, NT threads in the block
__device__ __forceinline__ void at_finish(const tim_config &cfg, const AttnWs &ws, void *out, const float *red_m,
                                          const float *red_l, const float *red_o, int b, int kvh, int slot, int slots,
                                          int used) {
  const int tid = threadIdx.x;
  // the NS states in LDS merged for one (head, dim): returns o, sets m and l
  auto merged = [&](int h, int dim, float &mx, float &lt) {
    mx = AT_NEG_BIG;
#pragma unroll
    for (int s2 = 0; s2 < NS; ++s2) mx = fmaxf(mx, red_m[s2 * TIM_G + h]);
    float ot = 0.f;
    lt = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < NS; ++s2) {
      const float sc = __builtin_amdgcn_exp2f(red_m[s2 * TIM_G + h] - mx);
      lt = fmaf(red_l[s2 * TIM_G + h], sc, lt);
      ot = fmaf(red_o[(s2 * TIM_G + h) * TIM_D + dim], sc, ot);
    }
    return ot;
  };
  // m and l of the block's four heads: one thread, two 16-byte stores into one 32-byte record (four 8-byte
  // stores from four waves, each a partial line reaching memory on its own, cost 0.3 % of the whole kernel)
  auto store_ml = [&]() {
    float v[2 * TIM_G];
#pragma unroll
    for (int h = 0; h < TIM_G; ++h) {
      float mx = AT_NEG_BIG, lt = 0.f;
#pragma unroll
      for (int s2 = 0; s2 < NS; ++s2) mx = fmaxf(mx, red_m[s2 * TIM_G + h]);
#pragma unroll
      for (int s2 = 0; s2 < NS; ++s2) lt = fmaf(red_l[s2 * TIM_G + h], __builtin_amdgcn_exp2f(red_m[s2 * TIM_G + h] - mx), lt);
      v[2 * h] = mx;
      v[2 * h + 1] = lt;
    }
    float4 *dst = reinterpret_cast<float4 *>(ws.ml + (((int64_t)b * cfg.kv_heads + kvh) * slots + slot) * (2 * TIM_G));
    at_store_through(dst, make_float4(v[0], v[1], v[2], v[3]));
    at_store_through(dst + 1, make_float4(v[4], v[5], v[6], v[7]));
  };
  if (OUT_BF16 && used > 1) {
    // bf16 partial: thread -> head tid / 64, dims 2 (tid % 64) and the next one, one 32-bit word
    static_assert(NT >= TIM_G * TIM_D / 2, "one pair of dims per thread");
    if (tid < TIM_G * TIM_D / 2) {
      const int h = tid >> 6, d0 = 2 * (tid & 63);
      float mx, lt, mx1, lt1;
      const float o0 = merged(h, d0, mx, lt), o1 = merged(h, d0 + 1, mx1, lt1);
      const float inv = lt > 0.f ? 1.f / lt : 0.f;  // (a slot whose tokens are all hidden has l = 0)
      const int64_t pi = (((int64_t)b * cfg.kv_heads + kvh) * slots + slot) * TIM_G + h;  // a block's four rows are contiguous
      at_store_through(reinterpret_cast<uint32_t *>(ws.o) + (pi * TIM_D + d0) / 2, at_pack_bf16(o0 * inv, o1 * inv));
      if (tid == 0) store_ml();
    }
    return;
  }
#pragma unroll
  for (int idx = tid; idx < TIM_G * TIM_D; idx += NT) {  // idx = (h, dim)
    const int h = idx >> 7, dim = idx & 127, hq = kvh * TIM_G + h;
    float mx, lt;
    const float ot = merged(h, dim, mx, lt);
    if (used == 1) {
      // (in-forward variant: a working memory whose tokens are all hidden has l = 0; its output is defined as zero)
      at_store_out<OUT_BF16>(out, ((int64_t)b * cfg.q_heads + hq) * TIM_D + dim, lt > 0.f ? ot / lt : 0.f);
    } else {
      const int64_t pi = (((int64_t)b * cfg.kv_heads + kvh) * slots + slot) * TIM_G + h;
      at_store_through(ws.o + pi * TIM_D + dim, ot);
      if (idx == 0) store_ml();
    }
  }
}

// A sequence with no tokens has no block that computes; slot 0 defines its output as zero.
template <bool OUT_BF16>
__device__ __forceinline__ void at_empty_out(const tim_config &cfg, void *out, int b, int kvh) {
  for (int idx = threadIdx.x; idx < TIM_G * TIM_D; idx += blockDim.x)
    at_store_out<OUT_BF16>(out, ((int64_t)b * cfg.q_heads + kvh * TIM_G) * TIM_D + idx, 0.f);
}

// Slots a sequence of n tokens occupies: one per `cpb` chunks, at most `slots`.
__device__ __forceinline__ int at_slots_used(int n, int cpb, int slots) {
  const int n_pages = (n + TIM_PS - 1) / TIM_PS;
  const int nchunks = (n_pages + AT_CHUNK_PAGES - 1) / AT_CHUNK_PAGES;
  return min(slots, (nchunks + cpb - 1) / cpb);
}

// Which (sequence, kv head, slot) this workgroup takes; false = none (uniform for the block).
//
// Without a schedule the grid is (batch * kv_heads, slots) with `slots` sized for the host's bound on the
// longest sequence: consecutive workgroup ids run over (sequence, kv head) first and are dealt round-robin
// to the 8 XCDs, so every XCD gets the same share of every sequence (with 8 kv heads: one head per XCD).
// Slots beyond a sequence's need exit at once.  That is fine for batches of similar lengths.  Next to
// one 32K-token sequence, 63 sequences of 2.5K tokens leave 14 of 16 slots idle, and the long sequence's
// last slots are the last workgroups of the grid, behind all the idle ones: measured 161 us for a launch
// whose bytes take 117 us.
//
// With a schedule (tim_attn_schedule: one small kernel per decode step, after the lengths are final) the
// grid is one-dimensional and workgroup i takes kv head i % kv_heads of item i / kv_heads of a list that
// holds only the slots in use, longest sequence first.  Workgroups beyond the list retire after two scalar
// loads, at the end of the grid, while the last busy ones still run.
struct AtWork {
  int b, kvh, slot, n, used;
};
template <bool OUT_BF16>
__device__ __forceinline__ bool at_take_work(const tim_config &cfg, const tim_state &st, const AttnWs &ws, void *out,
                                             int slots, int cpb, AtWork &wk) {
  // Everything here is wave-uniform and must stay on the scalar path: a vector load issued by a new
  // workgroup queues behind the tile loads its CU already has in flight (measured: 2.5 us more per idle
  // workgroup).  Hence no store or atomic before the last of these loads - the compiler would then no
  // longer trust the scalar cache - and the stale-schedule check waits until the block's end (at_check_live).
  wk.kvh = blockIdx.x % cfg.kv_heads;
  if (ws.sched != nullptr) {
    const int item = blockIdx.x / cfg.kv_heads;  // below batch * slots, the list's capacity
    const int total = ws.sched[0];
    int4 e = reinterpret_cast<const int4 *>(ws.sched + AT_SCHED_HDR)[item];
    // both loads are on their way before either is used: one round trip, as without a schedule
    asm("" : "+s"(e.x), "+s"(e.y), "+s"(e.z), "+s"(e.w) : "s"(total));
    if (item >= total || (unsigned)e.x >= (unsigned)cfg.max_batch) return false;  // (the list lies in caller-owned memory)
    wk.b = e.x;
    wk.slot = e.y;
    wk.n = e.z;
    wk.used = e.w;
  } else {
    wk.b = blockIdx.x / cfg.kv_heads;
    wk.slot = blockIdx.y;
    wk.n = st.seq_len[wk.b];
    wk.used = at_slots_used(wk.n, cpb, slots);
    if (wk.slot >= max(wk.used, 1)) return false;
  }
  if (wk.n <= 0) {  // a sequence without tokens has one workgroup per kv head, which defines its output as zero
    at_empty_out<OUT_BF16>(cfg, out, wk.b, wk.kvh);
    return false;
  }
  return true;
}
// A length that changed since the schedule was written is reported; the stale one was used (every page id is
// checked before it is dereferenced, so the worst outcome is a wrong output).
__device__ __forceinline__ void at_check_live(const tim_state &st, const AttnWs &ws, int b, int n) {
  if (ws.sched != nullptr && st.seq_len[b] != n) tim_set_status(st.status, TIM_ERR_INVALID_ARG);
}

template <bool OUT_BF16>
__global__ void __launch_bounds__(AT_THREADS)
tim_attn_partial_kernel(tim_config cfg, tim_state st, AttnWs ws, int layer, const uint4 *__restrict__ q,
                        void *__restrict__ out, float scale_log2, int cpb, int slots, const uint4 *__restrict__,
                        const uint4 *__restrict__) {
  __shared__ float red_m[AT_WAVES * 4][TIM_G];
  __shared__ float red_l[AT_WAVES * 4][TIM_G];
  __shared__ float red_o[AT_WAVES * 4][TIM_G][TIM_D];

  AtWork wk;
  if (!at_take_work<OUT_BF16>(cfg, st, ws, out, slots, cpb, wk)) return;
  const int b = wk.b, kvh = wk.kvh, slot = wk.slot, n = wk.n, used = wk.used;
  const int n_pages = (n + TIM_PS - 1) / TIM_PS;
  const int nchunks = (n_pages + AT_CHUNK_PAGES - 1) / AT_CHUNK_PAGES;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, g = lane >> 4, c = lane & 15;

  // the group's four query rows, dims 8c..8c+7, pre-scaled so that exp2 gives softmax
  float qf[TIM_G][8];
#pragma unroll
  for (int h = 0; h < TIM_G; ++h) {
    const uint4 u = q[((int64_t)b * cfg.q_heads + kvh * TIM_G + h) * 16 + c];
    at_unpack(u, qf[h]);
#pragma unroll
    for (int e2 = 0; e2 < 8; ++e2) qf[h][e2] *= scale_log2;
  }

  float m[TIM_G], l[TIM_G], acc[TIM_G][8];
#pragma unroll
  for (int h = 0; h < TIM_G; ++h) {
    m[h] = AT_NEG_BIG;
    l[h] = 0.f;
#pragma unroll
    for (int e2 = 0; e2 < 8; ++e2) acc[h][e2] = 0.f;
  }

  const uint4 *kpool = reinterpret_cast<const uint4 *>(st.k_pool);
  const uint4 *vpool = reinterpret_cast<const uint4 *>(st.v_pool);
  const int32_t *ptab = st.page_table + (int64_t)b * cfg.max_pages_per_seq;
  const int64_t layer_base = (int64_t)layer * cfg.num_pages;

  for (int chunk = slot; chunk < nchunks; chunk += used) {
    const int pg0 = chunk * AT_CHUNK_PAGES + w * AT_PAGES_PER_WAVE;
    const int pg1 = min(pg0 + AT_PAGES_PER_WAVE, n_pages);
    for (int pg = pg0; pg < pg1; ++pg) {
      int phys = __builtin_amdgcn_readfirstlane(ptab[pg]);
      if (phys < 0 || phys >= cfg.num_pages) {  // never dereference a bad page id
        tim_set_status(st.status, TIM_ERR_INVALID_ARG);
        phys = 0;
      }
      const int64_t tile = ((layer_base + phys) * cfg.kv_heads + kvh) * (TIM_TILE_BYTES / 16);
      uint4 kk[4], vv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) kk[j] = tim_load_stream(kpool + tile + j * 64 + lane);
#pragma unroll
      for (int j = 0; j < 4; ++j) vv[j] = tim_load_stream(vpool + tile + j * 64 + lane);
      const int left = n - pg * TIM_PS;  // rows of this page that exist (>= 1)

      float s[TIM_G][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float kf[8];
        at_unpack(kk[j], kf);
        const bool valid = 4 * j + g < left;
#pragma unroll
        for (int h = 0; h < TIM_G; ++h) {
          float d = 0.f;
#pragma unroll
          for (int e2 = 0; e2 < 8; ++e2) d = fmaf(qf[h][e2], kf[e2], d);
          d = at_row_sum(d);
          s[h][j] = valid ? d : -INFINITY;
        }
        if (!valid) vv[j] = make_uint4(0, 0, 0, 0);  // stale rows may hold anything
      }
      float p[TIM_G][4];
#pragma unroll
      for (int h = 0; h < TIM_G; ++h) {
        const float mn = fmaxf(fmaxf(m[h], fmaxf(s[h][0], s[h][1])), fmaxf(s[h][2], s[h][3]));
        const float alpha = __builtin_amdgcn_exp2f(m[h] - mn);
        float ps = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          p[h][j] = __builtin_amdgcn_exp2f(s[h][j] - mn);
          ps += p[h][j];
        }
        l[h] = fmaf(l[h], alpha, ps);
        m[h] = mn;
#pragma unroll
        for (int e2 = 0; e2 < 8; ++e2) acc[h][e2] *= alpha;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float vf[8];
        at_unpack(vv[j], vf);
#pragma unroll
        for (int h = 0; h < TIM_G; ++h)
#pragma unroll
          for (int e2 = 0; e2 < 8; ++e2) acc[h][e2] = fmaf(p[h][j], vf[e2], acc[h][e2]);
      }
    }
  }

  // merge the 16 (wave, row) states of the block
  const int sidx = w * 4 + g;
#pragma unroll
  for (int h = 0; h < TIM_G; ++h) {
    if (c == 0) {
      red_m[sidx][h] = m[h];
      red_l[sidx][h] = l[h];
    }
#pragma unroll
    for (int e2 = 0; e2 < 8; ++e2) red_o[sidx][h][8 * c + e2] = acc[h][e2];
  }
  __syncthreads();
  at_check_live(st, ws, b, n);
  at_finish<AT_WAVES * 4, AT_THREADS, OUT_BF16>(cfg, ws, out, &red_m[0][0], &red_l[0][0], &red_o[0][0][0], b, kvh, slot, slots,
                                    used);
}

// ---- MFMA variant ---------------------------------------------------------------------
// Same decomposition, but the two contractions run on the matrix cores
// (v_mfma_f32_16x16x32_bf16: A[i][k] in lane i + 16*(k/8), element k%8; B[k][j] in lane
// j + 16*(k/8); D[i][j] in lane j + 16*(i/4), register i%4).  A wave takes two pages
// (32 tokens) per iteration.
//   scores  S^T[token][head] = K[token][:] . Q[head][:]   A = K tile (16 tokens x 32 dims per
//           step, 4 steps), B = Q^T with heads 4..15 zero.  Lane (g, j) = (lane/16, lane%16)
//           loads 16 B of row j at dims 32s + 8g: each instruction reads 64 contiguous bytes
//           of 16 rows, the four steps together the whole tile.  Lane (g, j<4) ends up with
//           the scores of tokens 4g..4g+3 for head j, of both pages.
//   values  O[head][dim] = P[head][token] . V[token][dim]   A = P: the eight probabilities a
//           lane just computed are exactly its eight k-entries (k = 8g + e: page A tokens
//           4g..4g+3, then page B's), so P never crosses lanes.  B = V: lane (g, c) loads the
//           same eight token rows at dims 8c..8c+7 (full 256-byte rows per 16 lanes) and an
//           in-register 8x8 transpose of 16-bit elements gives, for each of 8 MFMAs, its
//           column "dim 8c + mf".  Output rows 0..3 (lanes 0..15) are the group's heads.
// Softmax keeps one reference maximum per head, shared by the four lane groups, and only
// renews it (cross-lane max, rescale of the accumulators) when a score exceeds it by more
// than 2^8; until then p = exp2(t - ref) <= 256 is exact enough in bf16/fp32.  The row
// sums stay per lane and are added once at the end.

#define AT_LAZY_MAX 8.0f

// WAVES = waves per block (4, 6 or 12; the host picks it so that a CU holds about twelve waves whatever the
// number of blocks, see at_shape).  The pairs of pages of a sequence are dealt round-robin over all the waves
// of all its blocks: unit u = slot * WAVES + wave takes pairs u, u + U, u + 2U, ... with U = used * WAVES, so
// the waves' shares differ by at most one pair whatever the length.
template <bool OUT_BF16, bool MASKED, bool PS1, int WAVES>
__global__ void __launch_bounds__(64 * WAVES, 12 / WAVES)
tim_attn_partial_mfma_kernel(tim_config cfg, tim_state st, AttnWs ws, int layer, const uint4 *__restrict__ q,
                             void *__restrict__ out, float scale_log2, int cpb, int slots,
                             const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new) {
  __shared__ float red_m[WAVES][TIM_G];
  __shared__ float red_l[WAVES][TIM_G];
  __shared__ float red_o[WAVES][TIM_G][TIM_D];
  // Page size 1 only: each wave's key rows of one pair of "pages" (32 tokens), copied there straight from global
  // memory as whole 256-byte rows and read back in the matrix operand's layout (see issue / process below).
  __shared__ uint4 kstage[PS1 ? WAVES : 1][PS1 ? 2 * TIM_PS : 1][16];

  AtWork wk;
  if (!at_take_work<OUT_BF16>(cfg, st, ws, out, slots, cpb, wk)) return;
  const int b = wk.b, kvh = wk.kvh, slot = wk.slot, n = wk.n, used = wk.used;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63, g = lane >> 4, j = lane & 15;
  const int wu = __builtin_amdgcn_readfirstlane(w);  // the same number where the compiler must see it is wave-uniform
  const int n_pages = (n + TIM_PS - 1) / TIM_PS;
  const int n_pairs = (n_pages + 1) >> 1;
  const int unit = slot * WAVES + w, stride = used * WAVES;  // this wave's pairs: unit, unit + stride, ...
  // Page ids run ahead of the tiles they name, so that no tile load waits for a page-id load first: lane i of
  // one load holds page 2 * (unit + (k0 + i / 2) * stride) + i % 2, the ids of 32 of the wave's pairs, and the next
  // 32 are requested when these come into use.  Entries past the sequence's end are read (the index is
  // clamped to the table's row) but never used.
  const int32_t *ptab = st.page_table + (int64_t)b * cfg.max_pages_per_seq;
  auto load_pids = [&](int k0) {
    const int64_t pg_ = 2 * ((int64_t)unit + (int64_t)(k0 + (lane >> 1)) * stride) + (lane & 1);
    return ptab[(int)min(pg_, (int64_t)cfg.max_pages_per_seq - 1)];
  };
  int my_pid = 0, next_pid = 0;
  if (!PS1) next_pid = load_pids(0);

  // B operand of the score product: Q^T, head j (zero for j >= 4), dims 32s + 8g .. +8
  uint4 qb[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    qb[s] = make_uint4(0, 0, 0, 0);
    if (j < TIM_G) qb[s] = q[((int64_t)b * cfg.q_heads + kvh * TIM_G + j) * 16 + 4 * s + g];
  }
  const float lane_bias = j < TIM_G ? 0.f : -INFINITY;  // padded heads never contribute

  float m_ref = AT_NEG_BIG, l_part = 0.f;
  at_f32x4 acc[8];
#pragma unroll
  for (int mf = 0; mf < 8; ++mf) acc[mf] = (at_f32x4){0.f, 0.f, 0.f, 0.f};

  const uint4 *kpool = reinterpret_cast<const uint4 *>(st.k_pool);
  const uint4 *vpool = reinterpret_cast<const uint4 *>(st.v_pool);
  const int64_t layer_base = (int64_t)layer * cfg.num_pages;

  // Page size 1: a "page" below is a run of 16 tokens and every row has its own page id.  The ids of a pair's
  // 32 tokens are one load (lane l holds token 32 * pair + l % 32), requested one pair ahead like the page
  // ids above, and handed to the lanes that need them by cross-lane reads.
  struct __attribute__((aligned(4))) RowIds { int a[4], b[4]; };  // ids of tokens 4g .. 4g+3 of page A and of page B
  auto load_row_ids = [&](int pr_) __attribute__((always_inline)) -> RowIds {
    RowIds r;
    const int base = pr_ * (2 * TIM_PS) + 4 * g;
    if (pr_ * (2 * TIM_PS) + 2 * TIM_PS <= cfg.max_pages_per_seq) {  // the whole pair lies inside the table's row: two 16-byte loads
      struct __attribute__((aligned(4))) I4 { int v[4]; };
      const I4 x = *reinterpret_cast<const I4 *>(ptab + base), y = *reinterpret_cast<const I4 *>(ptab + base + TIM_PS);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        r.a[i] = x.v[i];
        r.b[i] = y.v[i];
      }
    } else {  // the row's last, ragged pair: entry by entry, clamped to the row
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        r.a[i] = ptab[min(base + i, cfg.max_pages_per_seq - 1)];
        r.b[i] = ptab[min(base + TIM_PS + i, cfg.max_pages_per_seq - 1)];
      }
    }
    return r;
  };
  RowIds next_ids = {};
  if (PS1) next_ids = load_row_ids(min(unit, n_pairs - 1));

  // One pair of pages in registers: the K and V tiles of pages A and B, where they start in the pools (16-byte
  // units; page size 1: unused) and, in the in-forward variant, the visibility of the pair's 32 tokens.
  // (handed over by value: through references the compiler kept the tiles in scratch memory)
  struct Tiles {
    uint4 ka[4], kb[4], va[4], vb[4];
    int64_t row_a, row_b;
    uint32_t vis;
  };

  // Moves the page-id pipeline on to pair `pr`, the wave's k-th pair; called once per pair, in order, also for a
  // pair that is then skipped.
  RowIds my_ids = {};
  auto advance_ids = [&](int pr, int k) __attribute__((always_inline)) {
    if (!PS1 && (k & 31) == 0) {  // the ids of this and the next 31 pairs arrive; those of the 32 after them are requested
      my_pid = next_pid;
      if ((int64_t)pr + 32 * (int64_t)stride < n_pairs) next_pid = load_pids(k + 32);
    }
    my_ids = next_ids;
    if (PS1) next_ids = load_row_ids(min(pr + stride, n_pairs - 1));
  };
  // In-forward variant: visibility of the pair's 32 tokens; a pair without a visible token is not read at all.
  auto visibility = [&](int pr) __attribute__((always_inline)) -> uint32_t {
    if (!MASKED) return 0xffffffffu;
    return __builtin_amdgcn_readfirstlane(st.keep_mask[(int64_t)b * tim_mask_words(cfg) + pr]);
  };

  // Requests the tiles of pair `pr`, the wave's k-th pair, after advance_ids(pr, k).
  auto issue = [&](int pr, int k, uint32_t vis_) __attribute__((always_inline)) -> Tiles {
    Tiles t;
    uint4 (&t_ka)[4] = t.ka, (&t_kb)[4] = t.kb, (&t_va)[4] = t.va, (&t_vb)[4] = t.vb;
    int64_t &t_row_a = t.row_a, &t_row_b = t.row_b;
    const int pg = 2 * pr;
    const bool has_b = pg + 1 < n_pages;
    t.vis = vis_;
    t_row_a = t_row_b = 0;
    if (PS1) {
      // One page per token: every row brings its own id.  The operand layout of the score product wants lane
      // (g, j) to hold 16 bytes of row j, which read straight from memory touches sixteen rows in 64-byte pieces
      // per instruction (that needed the L1 and measured 5.98 TB/s against 6.42 with 16-token pages).  Instead both
      // K and V are fetched as whole rows, 256 bytes per 16 lanes, non-temporally: lane (g, c) takes chunk c of
      // token 4g + i with load i.  V stays in registers (that is its operand layout).  K goes directly into the
      // wave's LDS stage (lane order: position 4i + g holds token 4g + i; chunk c sits in slot c ^ position, so
      // that the operand reads below are free of bank conflicts) and is read back from there in process().
      int64_t rows[8];  // 16-byte units: start of the row of token 4g + i of page A (i < 4) and of page B
      bool bad = false;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        // a token past the sequence's end has no page (its table entry may hold anything): row 0 stands in, masked below
        const int tok = pg * TIM_PS + (i >> 2) * TIM_PS + 4 * g + (i & 3);
        int id = i < 4 ? my_ids.a[i] : my_ids.b[i - 4];
        if (tok >= n) id = 0;
        if (id < 0 || id >= cfg.num_pages) {  // never dereference a bad page id
          bad = true;
          id = 0;
        }
        rows[i] = ((layer_base + id) * cfg.kv_heads + kvh) * 16;
      }
      if (bad) tim_set_status(st.status, TIM_ERR_INVALID_ARG);
#pragma unroll
      for (int i = 0; i < 8; ++i) {  // copy i fills positions 4 (i % 4) .. + 3 of page i / 4 of the stage, 1 KiB in lane order
        const int pos = 4 * (i & 3) + g;
        __builtin_amdgcn_global_load_lds(kpool + rows[i] + (j ^ pos), (at_lds_ptr)&kstage[wu][TIM_PS * (i >> 2) + 4 * (i & 3)][0], 16, 0,
                                         2 /* non-temporal */);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) t_va[i] = tim_load_stream(vpool + rows[i] + j);
#pragma unroll
      for (int i = 0; i < 4; ++i) t_vb[i] = tim_load_stream(vpool + rows[4 + i] + j);
    } else {
      int phys_a = __builtin_amdgcn_readlane(my_pid, 2 * (k & 31));
      int phys_b = __builtin_amdgcn_readlane(my_pid, 2 * (k & 31) + (has_b ? 1 : 0));
      if (phys_a < 0 || phys_a >= cfg.num_pages || phys_b < 0 || phys_b >= cfg.num_pages) {
        tim_set_status(st.status, TIM_ERR_INVALID_ARG);  // never dereference a bad page id
        phys_a = phys_b = 0;
      }
      t_row_a = ((layer_base + phys_a) * cfg.kv_heads + kvh) * (TIM_TILE_BYTES / 16);
      t_row_b = ((layer_base + phys_b) * cfg.kv_heads + kvh) * (TIM_TILE_BYTES / 16);
#pragma unroll
      for (int s = 0; s < 4; ++s) t_ka[s] = tim_load_stream(kpool + t_row_a + j * 16 + 4 * s + g);
#pragma unroll
      for (int s = 0; s < 4; ++s) t_kb[s] = tim_load_stream(kpool + t_row_b + j * 16 + 4 * s + g);
#pragma unroll
      for (int i = 0; i < 4; ++i) t_va[i] = tim_load_stream(vpool + t_row_a + (4 * g + i) * 16 + j);
#pragma unroll
      for (int i = 0; i < 4; ++i) t_vb[i] = tim_load_stream(vpool + t_row_b + (4 * g + i) * 16 + j);
    }
    return t;
  };

  // Scores, weights and output products of pair `pr`, whose tiles `issue` requested.
  auto process = [&](int pr, Tiles t) __attribute__((always_inline)) {
    uint4 (&t_ka)[4] = t.ka, (&t_kb)[4] = t.kb, (&t_va)[4] = t.va, (&t_vb)[4] = t.vb;
    const int64_t t_row_a = t.row_a, t_row_b = t.row_b;
    const uint32_t t_vis = t.vis;
    const int pg = 2 * pr;
    const bool has_b = pg + 1 < n_pages;
    const uint32_t vis = t_vis;
    if (PS1) {  // the K operands come out of the wave's stage: token j sits at position 4 (j % 4) + j / 4
      const int pos = 4 * (j & 3) + (j >> 2);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        t_ka[s] = kstage[wu][pos][(4 * s + g) ^ pos];
        t_kb[s] = kstage[wu][TIM_PS + pos][(4 * s + g) ^ pos];
      }
    }
    // fused append: the wave that owns the sequence's last page takes the pending token's
    // row from the caller's buffers instead of the pool, and stores it into the pool
    if (k_new != nullptr) {
      const int last_tok = n - 1, last_pg = last_tok / TIM_PS, row = last_tok % TIM_PS;
      if (pg == last_pg || (has_b && pg + 1 == last_pg)) {  // uniform for the wave
        const bool in_b = pg != last_pg;
        int64_t krow;  // 16-byte units of the row's start in the pools
        if (PS1) {
          int sid = ptab[last_tok];
          if (sid < 0 || sid >= cfg.num_pages) sid = 0;  // reported by the loads above
          krow = ((layer_base + sid) * cfg.kv_heads + kvh) * 16;
        } else {
          krow = (in_b ? t_row_b : t_row_a) + row * 16;
        }
        const int64_t src = ((int64_t)b * cfg.kv_heads + kvh) * 16;
        if (j == row) {
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            const uint4 x = k_new[src + 4 * s + g];
            if (in_b) t_kb[s] = x;
            if (!in_b) t_ka[s] = x;
            const_cast<uint4 *>(kpool)[krow + 4 * s + g] = x;
          }
        }
        if ((row >> 2) == g) {
          const uint4 x = v_new[src + j];
          // (written as selects on every slot: an index computed at run time would move the tiles to scratch memory)
          auto pick = [](bool c, const uint4 &a2, const uint4 &b2) { return make_uint4(c ? a2.x : b2.x, c ? a2.y : b2.y, c ? a2.z : b2.z, c ? a2.w : b2.w); };
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const bool hit = i == (row & 3);
            t_va[i] = pick(hit && !in_b, x, t_va[i]);
            t_vb[i] = pick(hit && in_b, x, t_vb[i]);
          }
          const_cast<uint4 *>(vpool)[krow + j] = x;
        }
      }
    }

    // rows that exist: page A has left_a >= 1 rows, page B left_b (0 if absent)
    const int left_a = n - pg * TIM_PS;
    const int left_b = has_b ? n - (pg + 1) * TIM_PS : 0;
    const bool full = left_b >= TIM_PS && vis == 0xffffffffu;  // then page A is full as well

    at_f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(at_as_bf16x8(t_ka[s]), at_as_bf16x8(qb[s]), sa, 0, 0, 0);
#pragma unroll
    for (int s = 0; s < 4; ++s) sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(at_as_bf16x8(t_kb[s]), at_as_bf16x8(qb[s]), sb, 0, 0, 0);

    float tt[8];
    if (full) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        tt[r] = fmaf(sa[r], scale_log2, lane_bias);
        tt[4 + r] = fmaf(sb[r], scale_log2, lane_bias);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const bool ok_a = 4 * g + r < left_a && ((vis >> (4 * g + r)) & 1u);
        const bool ok_b = 4 * g + r < left_b && ((vis >> (16 + 4 * g + r)) & 1u);
        // the select is on the product: a stale row may hold anything, also NaN or Inf
        tt[r] = ok_a ? fmaf(sa[r], scale_log2, lane_bias) : -INFINITY;
        tt[4 + r] = ok_b ? fmaf(sb[r], scale_log2, lane_bias) : -INFINITY;
        if (!ok_a) t_va[r] = make_uint4(0, 0, 0, 0);
        if (!ok_b) t_vb[r] = make_uint4(0, 0, 0, 0);
      }
    }
    float lm = fmaxf(fmaxf(fmaxf(tt[0], tt[1]), fmaxf(tt[2], tt[3])), fmaxf(fmaxf(tt[4], tt[5]), fmaxf(tt[6], tt[7])));
    if (__any(lm > m_ref + AT_LAZY_MAX)) {
      // renew the reference: maximum over the four lane groups of each head column
      float x = lm;
      x = fmaxf(x, __shfl_xor(x, 16, 64));
      x = fmaxf(x, __shfl_xor(x, 32, 64));
      const float m_new = fmaxf(m_ref, x);
      const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
      l_part *= alpha;
      m_ref = m_new;
      // accumulator row r (head r) lives in lanes 0..15; its factor sits in lane r
      float ar[TIM_G];
#pragma unroll
      for (int r = 0; r < TIM_G; ++r) ar[r] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(alpha), r));
#pragma unroll
      for (int mf = 0; mf < 8; ++mf)
#pragma unroll
        for (int r = 0; r < TIM_G; ++r) acc[mf][r] *= ar[r];
    }
    float p[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = __builtin_amdgcn_exp2f(tt[e] - m_ref);
      l_part += p[e];
    }
    uint4 pw;
    pw.x = at_pack_bf16(p[0], p[1]);
    pw.y = at_pack_bf16(p[2], p[3]);
    pw.z = at_pack_bf16(p[4], p[5]);
    pw.w = at_pack_bf16(p[6], p[7]);
    const at_bf16x8 pa = at_as_bf16x8(pw);

    // 8x8 transpose of 16-bit elements: rows = token slots (A0..A3, B0..B3), columns = dims
    auto word = [&](int r, int c) -> uint32_t {  // 32-bit word c of token slot r (constants once unrolled)
      const uint4 &x = r < 4 ? t_va[r & 3] : t_vb[r & 3];
      return c == 0 ? x.x : c == 1 ? x.y : c == 2 ? x.z : x.w;
    };
#pragma unroll
    for (int mf = 0; mf < 8; ++mf) {
      uint32_t cw[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const uint32_t x0 = word(2 * u, mf >> 1), x1 = word(2 * u + 1, mf >> 1);
        cw[u] = (mf & 1) ? __builtin_amdgcn_perm(x1, x0, 0x07060302u) : __builtin_amdgcn_perm(x1, x0, 0x05040100u);
      }
      acc[mf] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, at_as_bf16x8(make_uint4(cw[0], cw[1], cw[2], cw[3])), acc[mf], 0, 0, 0);
    }
  };

  // (Requesting a wave's next pair before working on the current one was measured twice and rejected.  With two
  // register sets that swap roles the compiler spills about 50 of 256 registers inside the loop and a CU holds 8
  // waves instead of 12: 35.4 against 50.5 decode steps/s on long working memories, 37.8 against 26.1 us per
  // launch on short ones.  At 12 waves per CU, with the next pair's V tiles copied straight into a per-wave LDS
  // stage and its K tiles loaded into the registers the score products have just freed (no extra registers, both
  // requests in flight during the weights and output products): 50.79 against 50.60 steps/s on long working
  // memories, 1,005 against 1,017 on short ones in a small batch, same box, alternating.  Twelve waves per CU
  // already keep the memory system as busy as it gets; the wave's own wait is not what limits the kernel.)
  int k = 0;
  for (int pr = unit; pr < n_pairs; pr += stride, ++k) {
    advance_ids(pr, k);
    const uint32_t vis = visibility(pr);
    if (MASKED && vis == 0) continue;
    process(pr, issue(pr, k, vis));
  }

  // row sums: add the four lane groups of each head column
  l_part += __shfl_xor(l_part, 16, 64);
  l_part += __shfl_xor(l_part, 32, 64);
  if (lane < TIM_G) {
    red_m[w][lane] = m_ref;
    red_l[w][lane] = l_part;
  }
  if (lane < 16) {
#pragma unroll
    for (int r = 0; r < TIM_G; ++r)
#pragma unroll
      for (int mf = 0; mf < 8; ++mf) red_o[w][r][8 * lane + mf] = acc[mf][r];
  }
  __syncthreads();
  at_check_live(st, ws, b, n);
  at_finish<WAVES, 64 * WAVES, OUT_BF16>(cfg, ws, out, &red_m[0][0], &red_l[0][0], &red_o[0][0][0], b, kvh, slot, slots,
                                         used);
}

// Log-sum-exp merge of the slot partials: one block of 128 threads per (sequence, query
// head).  Thread s first turns slot s's (m, l) into a weight 2^(m_s - max) held in LDS;
// then thread d sums the weighted o_s[d] over the slots with independent, unrolled loads.
__device__ __forceinline__ float at_wave_max(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
  return v;
}
__device__ __forceinline__ float at_wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

template <bool OUT_BF16>
__global__ void __launch_bounds__(TIM_D)
tim_attn_merge_kernel(tim_config cfg, tim_state st, AttnWs ws, void *__restrict__ out, int slots, int cpb) {
  __shared__ float wgt[AT_MAX_SLOTS];
  __shared__ float red[4];
  const int bh = blockIdx.x, b = bh / cfg.q_heads, tid = threadIdx.x;
  const int n = st.seq_len[b];
  const int n_pages = (n + TIM_PS - 1) / TIM_PS;
  const int nchunks = (n_pages + AT_CHUNK_PAGES - 1) / AT_CHUNK_PAGES;
  const int used = ws.sched != nullptr ? ws.sched[AT_SCHED_HDR + 4 * (int64_t)cfg.max_batch * AT_MAX_SLOTS + b]
                                       : min(slots, (nchunks + cpb - 1) / cpb);
  if (used == 1) return;  // written by the partial kernel
  if (used == 0) {        // empty working memory: defined as zero
    at_store_out<OUT_BF16>(out, (int64_t)bh * TIM_D + tid, 0.f);
    return;
  }
  // partial outputs: [B][Hkv][slots][4 heads][128]; slot s of this head is row p0 + s * TIM_G
  const int64_t p0 = ((int64_t)b * cfg.kv_heads + (bh % cfg.q_heads) / TIM_G) * slots * TIM_G + (bh % cfg.q_heads) % TIM_G;
  float m = AT_NEG_BIG, l = 0.f;
  if (tid < used) {
    const int hq = bh % cfg.q_heads;
    const int64_t rec = (((int64_t)b * cfg.kv_heads + hq / TIM_G) * slots + tid) * (2 * TIM_G) + 2 * (hq % TIM_G);
    m = ws.ml[rec];
    l = ws.ml[rec + 1];
  }
  const float wm = at_wave_max(m);
  if ((tid & 63) == 0) red[tid >> 6] = wm;
  __syncthreads();
  const float mx = fmaxf(red[0], red[1]);
  const float w = tid < used ? __builtin_amdgcn_exp2f(m - mx) : 0.f;
  wgt[tid] = OUT_BF16 ? w * l : w;  // a bf16 partial is stored normalised: its weight carries l
  const float ws_l = at_wave_sum(w * l);
  if ((tid & 63) == 0) red[2 + (tid >> 6)] = ws_l;
  __syncthreads();
  const float lt = red[2] + red[3];
  float acc = 0.f;
  int s = 0;
  if (OUT_BF16) {
    const uint16_t *o = reinterpret_cast<const uint16_t *>(ws.o) + p0 * TIM_D + tid;
    for (; s + 8 <= used; s += 8) {
      uint16_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = o[(int64_t)(s + u) * (TIM_G * TIM_D)];
#pragma unroll
      for (int u = 0; u < 8; ++u) acc = fmaf(__uint_as_float((uint32_t)v[u] << 16), wgt[s + u], acc);
    }
    for (; s < used; ++s) acc = fmaf(__uint_as_float((uint32_t)o[(int64_t)s * (TIM_G * TIM_D)] << 16), wgt[s], acc);
  } else {
    const float *o = ws.o + p0 * TIM_D + tid;
    for (; s + 8 <= used; s += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = o[(int64_t)(s + u) * (TIM_G * TIM_D)];
#pragma unroll
      for (int u = 0; u < 8; ++u) acc = fmaf(v[u], wgt[s + u], acc);
    }
    for (; s < used; ++s) acc = fmaf(o[(int64_t)s * (TIM_G * TIM_D)], wgt[s], acc);
  }
  at_store_out<OUT_BF16>(out, (int64_t)bh * TIM_D + tid, lt > 0.f ? acc / lt : 0.f);  // all tokens hidden: zero
}

// words of the workspace that hold the partials; the schedule follows them
static int64_t at_partials_words(const tim_config &cfg) {
  return (int64_t)cfg.max_batch * cfg.q_heads * AT_MAX_SLOTS * (TIM_D + 2);
}

extern "C" int64_t tim_attn_ws_bytes(const tim_config *cfg) {
  if (!cfg) return 0;
  return at_partials_words(*cfg) * (int64_t)sizeof(float) +
         (AT_SCHED_HDR + (4 * (int64_t)AT_MAX_SLOTS + 1) * cfg->max_batch) * (int64_t)sizeof(int32_t);
}

// Launch shape for a bound on the longest sequence: chunks per block, slots, and waves per block.
// Blocks have 4 waves, three to a CU, and a sequence is cut into as many of them as it takes to fill the chip.
// One case is treated differently: a launch whose longest sequence fits one block anyway and which has at most
// one or two (sequence, kv head) rows per CU - short working memories in a small batch, the regime right after
// the flushes.  Cutting those rows further to fill the CUs' wave slots costs a second kernel for the partial
// results (measured: 31-34 us against 26 us per launch on 256 rows of about 900 tokens); instead the blocks are
// made wider, 12 waves for one row per CU and 6 for two, so that a CU still holds twelve waves and every
// sequence stays in one block: no partial, no merge launch.
static void at_shape(const tim_ctx *ctx, int32_t max_seq_len, int *cpb_out, int *slots_out, int *waves_out) {
  const tim_config &cfg = ctx->cfg;
  const int full = cfg.max_pages_per_seq * cfg.page_size;
  const int bound = (max_seq_len == 0 || max_seq_len > full) ? full : max_seq_len;
  const int max_pages = (bound + TIM_PS - 1) / TIM_PS;
  const int nchunks = (max_pages + AT_CHUNK_PAGES - 1) / AT_CHUNK_PAGES;
  const int64_t rows = (int64_t)cfg.max_batch * cfg.kv_heads;
  int cpb = ctx->attn_cpb;
  int waves = ctx->block_waves;
  if (waves == 0) {
    waves = AT_WAVES;
    if (ctx->attn_impl == TIM_ATTN_MFMA && nchunks <= cpb && rows <= 2 * (int64_t)ctx->n_cu) {
      const int wide = rows <= ctx->n_cu ? 12 : 6;
      if (rows * wide >= ctx->attn_fill * (int64_t)AT_WAVES * ctx->n_cu) waves = wide;  // else too few rows: cut them after all
    }
  }
  // chunks per block: as many as still leave `fill` blocks' worth of waves (4 each) per CU
  while (cpb > 1 && rows * ((nchunks + cpb - 1) / cpb) * waves < ctx->attn_fill * (int64_t)AT_WAVES * ctx->n_cu) --cpb;
  int slots = (nchunks + cpb - 1) / cpb;
  if (slots > AT_MAX_SLOTS) slots = AT_MAX_SLOTS;
  if (slots < 1) slots = 1;
  *cpb_out = cpb;
  *slots_out = slots;
  *waves_out = waves;
}

// The work list of at_take_work.  One block; thread b (and b + blockDim.x, ...) handles sequence b; quadratic in
// the batch, which is a few thousand at most.  Order: longest sequence first (ties: lower index first).
// Block sizes are graded along the list when it holds at least AT_GRADE_MIN_ROUNDS rounds of work (a round =
// what the chip's resident blocks take at cpb chunks each): a sequence that starts with more than grade_big / 16
// rounds still to go gets blocks of 2 cpb chunks (fewer partial results, which cost far more than their size),
// one that starts within the last grade_small / 16 rounds gets blocks of cpb / 2 (the launch ends on small
// blocks), the rest cpb.
// sched: [0] = number of items, items from word AT_SCHED_HDR on, then the slots each sequence uses
// (the merge kernel's view of the same decision).
__device__ __forceinline__ int at_chunks_of(int n) {
  const int n_pages = (n + TIM_PS - 1) / TIM_PS;
  return n > 0 ? (n_pages + AT_CHUNK_PAGES - 1) / AT_CHUNK_PAGES : 0;
}
__global__ void __launch_bounds__(1024)
tim_attn_schedule_kernel(tim_config cfg, tim_state st, int32_t *__restrict__ sched, int slots, int cpb, int grade_big,
                         int grade_small, int round_chunks, int short_per) {
  int32_t *used_of = sched + AT_SCHED_HDR + 4 * (int64_t)cfg.max_batch * AT_MAX_SLOTS;
  // A list of under AT_GRADE_MIN_ROUNDS rounds is not graded; its one block size is chosen so that the blocks
  // spread evenly over the CUs.  A CU streams at the same rate whether it holds two blocks or three, so a launch
  // of equal blocks lasts as long as the CU with the most of them: with `per` chunks per block the list holds
  // items(per) blocks per kv head, the fullest CU gets ceil(items / (CUs / kv_heads)) of them, and the launch
  // takes that many times `per`.  (Measured after the flushes of the batch-64 workload, 64 working memories of
  // 1.6-3.6K tokens on 256 CUs: blocks of 6 chunks, 4.2 per CU, run at 5.53 TB/s; of 4 chunks, 6.0 per CU: 5.79;
  // of 3: 5.70; of 8: 5.36; whole sequences: 5.0-5.6.)  Where several sizes cost the same, sequences of one
  // length take the largest (fewer partial results: 64 x 2,500 tokens, 102 us per launch whole against 104 in
  // halves), unequal ones the smallest (the even spread the model assumes needs many small blocks: 5.76-5.79
  // TB/s at 3 or 4 chunks against 5.53 at 6 in the measurement above, all three tied at 24 in the model).
  //
  // One block; every pass reads the lengths and slot counts from LDS, and the two passes that compare every
  // sequence with every other one are spread over all threads (P threads per sequence, joined by LDS atomics):
  // the kernel runs once per decode step in front of the step's attention launches, alone on the chip, so its
  // length is latency, not work.  (As first written - one thread per sequence, every pass re-reading the lengths
  // from global memory, one atomic per sequence and candidate size - it took 39 us for 64 sequences.)
  __shared__ int s_items[2 * AT_MAX_CPB + 1];
  __shared__ int s_per, s_cmin, s_cmax, s_work_total, s_items_total;
  __shared__ unsigned long long s_best;
  __shared__ int s_len[AT_SCHED_STAGE], s_used[AT_SCHED_STAGE], s_work_before[AT_SCHED_STAGE], s_before[AT_SCHED_STAGE];
  const int B = cfg.max_batch, T = blockDim.x, tid = threadIdx.x;  // B <= AT_SCHED_STAGE (checked by the host)
  int P = 1;  // threads per sequence in the all-pairs passes: a power of two, at most T / B
  while (2 * P * B <= T) P *= 2;
  const int part = tid % P, seqs_per_pass = T / P;
  const int per_lo = max(cpb / 2, 1), per_hi = 2 * cpb, cu_items = max(round_chunks / cpb / AT_BLOCKS_PER_CU, 1);
  for (int i = tid; i <= 2 * AT_MAX_CPB; i += T) s_items[i] = 0;
  if (tid == 0) {
    s_cmin = INT32_MAX;
    s_cmax = s_work_total = s_items_total = 0;
    s_best = ~0ull;
  }
  __syncthreads();
  {
    int cmin = INT32_MAX, cmax = 0, csum = 0;  // (chunks of the whole batch: at most num_pages / 16)
    for (int b = tid; b < B; b += T) {
      const int n = st.seq_len[b], c = at_chunks_of(n);
      s_len[b] = n;
      s_work_before[b] = s_before[b] = 0;
      csum += c;
      if (c > 0) {
        cmin = min(cmin, c);
        cmax = max(cmax, c);
      }
    }
    if (cmax > 0) {
      atomicMin(&s_cmin, cmin);
      atomicMax(&s_cmax, cmax);
      atomicAdd(&s_work_total, csum);
    }
  }
  __syncthreads();
  // blocks per candidate size: thread (group, candidate) sums over every 'groups'-th sequence
  {
    const int lanes = 16, groups = T / lanes, group = tid / lanes;
    for (int per = per_lo + tid % lanes; per <= per_hi; per += lanes) {
      int sum = 0;
#pragma unroll 4
      for (int b = group; b < B; b += groups) sum += max(min(slots, (at_chunks_of(s_len[b]) + per - 1) / per), 1);
      atomicAdd(&s_items[per], sum);
    }
  }
  // work in front of each sequence in the list's order (longest first, ties: lower index first)
  for (int b = tid / P; b < B; b += seqs_per_pass) {
    const int n = s_len[b];
    int before = 0;
#pragma unroll 4
    for (int o = part; o < B; o += P) {
      const int no = s_len[o];
      if (no > n || (no == n && o < b)) before += at_chunks_of(no);
    }
    if (before > 0) atomicAdd(&s_work_before[b], before);
  }
  __syncthreads();
  // the cheapest size: one thread per candidate, joined by a minimum over (cost, tie order, size)
  for (int per = per_lo + tid; per <= per_hi; per += T) {
    const unsigned long long cost = (unsigned long long)((s_items[per] + cu_items - 1) / cu_items) * per;
    const unsigned tie = s_cmin >= s_cmax ? 255u - per : (unsigned)per;  // equal lengths: the largest; else the smallest
    atomicMin(&s_best, (cost << 16) | (tie << 8) | (unsigned)per);
  }
  __syncthreads();
  if (tid == 0) s_per = short_per > 0 ? min(max(short_per, per_lo), per_hi) : (int)(s_best & 255u);
  __syncthreads();
  {
    const int64_t work_total = s_work_total;
    int my_items = 0;
    for (int b = tid; b < B; b += T) {
      const int c = at_chunks_of(s_len[b]);
      int per = s_per;
      const int64_t to_go = work_total - s_work_before[b];
      if (work_total >= (int64_t)AT_GRADE_MIN_ROUNDS * round_chunks) {
        per = cpb;
        if (to_go * 16 > (int64_t)grade_big * round_chunks) per = 2 * cpb;
        else if (to_go * 16 <= (int64_t)grade_small * round_chunks) per = max(cpb / 2, 1);
      }
      const int used = min(slots, (c + per - 1) / per);
      used_of[b] = used;
      s_used[b] = used;
      my_items += max(used, 1);
    }
    if (my_items > 0) atomicAdd(&s_items_total, my_items);
  }
  __syncthreads();
  // items in front of each sequence, then its own
  for (int b = tid / P; b < B; b += seqs_per_pass) {
    const int n = s_len[b];
    int before = 0;
#pragma unroll 4
    for (int o = part; o < B; o += P) {
      const int no = s_len[o];
      if (no > n || (no == n && o < b)) before += max(s_used[o], 1);
    }
    if (before > 0) atomicAdd(&s_before[b], before);
  }
  __syncthreads();
  if (tid == 0) sched[0] = s_items_total;
  int4 *items = reinterpret_cast<int4 *>(sched + AT_SCHED_HDR);
  for (int b = tid / P; b < B; b += seqs_per_pass) {
    const int n = s_len[b], used = s_used[b], before = s_before[b];
    for (int s2 = part; s2 < max(used, 1); s2 += P) items[before + s2] = make_int4(b, s2, n, used);
  }
}

extern "C" int tim_attn_schedule(tim_ctx *ctx, int32_t max_seq_len, tim_stream stream) {
  if (!ctx || !ctx->bound || max_seq_len < 0 || !ctx->st.attn_ws) return TIM_ERR_INVALID_ARG;
  at_shape(ctx, max_seq_len, &ctx->sched_cpb, &ctx->sched_slots, &ctx->sched_waves);
  // Nothing to gain when every block of the bound's grid is resident at once (idle blocks then cost nothing,
  // and on configuration 4, 117 MB per launch, the list's order paired blocks on CUs worse than the grid's:
  // 29.5 vs 27.0 us per launch), or when there is one sequence: the calls then run unscheduled.
  ctx->sched_valid = false;
  if (ctx->cfg.max_batch > AT_SCHED_STAGE) return TIM_OK;  // beyond what the schedule kernel holds in LDS
  if (ctx->round_items == 0 &&
      (ctx->cfg.max_batch == 1 ||
       (int64_t)ctx->cfg.max_batch * ctx->cfg.kv_heads * ctx->sched_slots <= (int64_t)AT_BLOCKS_PER_CU * ctx->n_cu))
    return TIM_OK;
  if (ctx->grade_small > 0 && ctx->sched_cpb > 1) {  // the smallest blocks decide how many slots a sequence may need
    const int per = ctx->sched_cpb / 2;
    ctx->sched_slots = (ctx->sched_slots * ctx->sched_cpb + per - 1) / per;
    if (ctx->sched_slots > AT_MAX_SLOTS) ctx->sched_slots = AT_MAX_SLOTS;
  }
  // (a caller-set round of a few items lets small shapes reach all three block sizes)
  const int round_chunks =
      (ctx->round_items > 0 ? ctx->round_items : AT_BLOCKS_PER_CU * ctx->n_cu / ctx->cfg.kv_heads) * ctx->sched_cpb;
  int32_t *sched = reinterpret_cast<int32_t *>(ctx->st.attn_ws + at_partials_words(ctx->cfg));
  const int threads = ctx->cfg.max_batch <= 64 ? 256 : 1024;
  hipLaunchKernelGGL(tim_attn_schedule_kernel, dim3(1), dim3(threads), 0, tim_hs(stream), ctx->cfg, ctx->st, sched,
                     ctx->sched_slots, ctx->sched_cpb, ctx->grade_big, ctx->grade_small, round_chunks > 0 ? round_chunks : 1,
                     ctx->short_per);
  TIM_LAUNCH_CHECK();
  ctx->sched_valid = true;
  return TIM_OK;
}

template <int IMPL, bool OUT_BF16>  // 0 = vector ALU, 1 = matrix cores, 2 = matrix cores with visibility mask
static void at_launch(dim3 grid, hipStream_t s, tim_ctx *ctx, const AttnWs &ws, int layer, const void *q, void *out,
                      float scale_log2, int cpb, int slots, int waves, const void *k_new, const void *v_new) {
  const bool ps1 = ctx->cfg.page_size == 1;
  typedef void (*kernel_t)(tim_config, tim_state, AttnWs, int, const uint4 *, void *, float, int, int, const uint4 *,
                           const uint4 *);
  kernel_t kernel;
  constexpr bool M = IMPL == 2;
  if (IMPL == 0) {
    kernel = tim_attn_partial_kernel<OUT_BF16>;
    waves = AT_WAVES;
  } else if (waves == 12) {
    kernel = ps1 ? tim_attn_partial_mfma_kernel<OUT_BF16, M, true, 12> : tim_attn_partial_mfma_kernel<OUT_BF16, M, false, 12>;
  } else if (waves == 8) {
    kernel = ps1 ? tim_attn_partial_mfma_kernel<OUT_BF16, M, true, 8> : tim_attn_partial_mfma_kernel<OUT_BF16, M, false, 8>;
  } else if (waves == 6) {
    kernel = ps1 ? tim_attn_partial_mfma_kernel<OUT_BF16, M, true, 6> : tim_attn_partial_mfma_kernel<OUT_BF16, M, false, 6>;
  } else {
    kernel = ps1 ? tim_attn_partial_mfma_kernel<OUT_BF16, M, true, 4> : tim_attn_partial_mfma_kernel<OUT_BF16, M, false, 4>;
    waves = 4;
  }
  const dim3 block(64 * waves);
  const uint4 *q4 = reinterpret_cast<const uint4 *>(q);
  const uint4 *kn = reinterpret_cast<const uint4 *>(k_new), *vn = reinterpret_cast<const uint4 *>(v_new);
  if (ctx->timing_on && ctx->timing_n < (int)ctx->ev_start.size()) {
    // events attached to the dispatch itself: the kernel's own begin/end, no extra barrier
    const int i = ctx->timing_n++;
    hipExtLaunchKernelGGL(kernel, grid, block, 0, s, ctx->ev_start[i], ctx->ev_stop[i], 0, ctx->cfg, ctx->st,
                          ws, layer, q4, out, scale_log2, cpb, slots, kn, vn);
  } else {
    hipLaunchKernelGGL(kernel, grid, block, 0, s, ctx->cfg, ctx->st, ws, layer, q4, out, scale_log2, cpb,
                       slots, kn, vn);
  }
}

extern "C" int tim_timing_begin(tim_ctx *ctx, int32_t max_launches) {
  if (!ctx || max_launches <= 0 || ctx->timing_on) return TIM_ERR_INVALID_ARG;
  ctx->ev_start.resize(max_launches);
  ctx->ev_stop.resize(max_launches);
  for (int i = 0; i < max_launches; ++i) {
    TIM_HIP_CHECK(hipEventCreate(&ctx->ev_start[i]));
    TIM_HIP_CHECK(hipEventCreate(&ctx->ev_stop[i]));
  }
  ctx->timing_n = 0;
  ctx->timing_on = true;
  return TIM_OK;
}

extern "C" int tim_timing_end(tim_ctx *ctx, float *ms_out, int32_t *n_out) {
  if (!ctx || !ctx->timing_on || !ms_out || !n_out) return TIM_ERR_INVALID_ARG;
  int rc = TIM_OK;
  for (int i = 0; i < ctx->timing_n; ++i) {
    if (hipEventSynchronize(ctx->ev_stop[i]) != hipSuccess ||
        hipEventElapsedTime(&ms_out[i], ctx->ev_start[i], ctx->ev_stop[i]) != hipSuccess)
      rc = TIM_ERR_HIP;
  }
  *n_out = ctx->timing_n;
  for (size_t i = 0; i < ctx->ev_start.size(); ++i) {
    (void)hipEventDestroy(ctx->ev_start[i]);
    (void)hipEventDestroy(ctx->ev_stop[i]);
  }
  ctx->ev_start.clear();
  ctx->ev_stop.clear();
  ctx->timing_on = false;
  ctx->timing_n = 0;
  return rc;
}

// ---- split partials in memory the library itself holds -----------------------------------------------
// For callers that cannot hand over a workspace they allocated (code under graph capture, serving loops
// and harnesses that forbid allocation): the partial results of tim_decode_attn_noalloc pass through this
// file-scope device array instead of tim_state.attn_ws.  Each GPU the library runs on holds its own copy
// of the array, at its own address, until the process ends.  In host code the array's name is only a
// handle: the address a kernel may use comes from hipGetSymbolAddress, asked once per device with that
// device current, and is kept per device.
static __device__ __align__(256) unsigned char tim_noalloc_scratch[TIM_NOALLOC_SCRATCH_BYTES];

#define AT_MAX_DEVICES 64
static std::mutex at_scratch_mutex;
static void *at_scratch_ptr[AT_MAX_DEVICES];  // per device, nullptr = not asked yet

static int at_noalloc_scratch(float **out) {
  int dev = -1;
  TIM_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= AT_MAX_DEVICES) return TIM_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(at_scratch_mutex);
  if (!at_scratch_ptr[dev]) {
    void *p = nullptr;
    TIM_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(tim_noalloc_scratch)));
    if (!p) return TIM_ERR_HIP;
    at_scratch_ptr[dev] = p;
  }
  *out = reinterpret_cast<float *>(at_scratch_ptr[dev]);
  return TIM_OK;
}

// Called by tim_ctx_create with the context's device current, so that a first attention call made under graph
// capture finds the address already known.  Without a usable device (a host-only build check) it does nothing
// and the entry point asks on its first call.
void tim_noalloc_scratch_init() {
  float *unused = nullptr;
  (void)at_noalloc_scratch(&unused);
  (void)hipGetLastError();  // a failure here is not the caller's: the entry point will report it if it persists
}

static int at_decode(tim_ctx *ctx, int32_t layer, const void *q, void *out, float sm_scale, int32_t out_dtype,
                     int32_t max_seq_len, tim_stream stream, bool masked, const void *k_new = nullptr,
                     const void *v_new = nullptr, bool own_scratch = false) {
  if (!ctx || !ctx->bound || !tim_rows_ok(q) || !tim_rows_ok(out) || !tim_aligned(k_new, 16) || !tim_aligned(v_new, 16) ||
      layer < 0 || layer >= ctx->cfg.layers || (!own_scratch && !ctx->st.attn_ws) ||
      (out_dtype != TIM_OUT_F32 && out_dtype != TIM_OUT_BF16) || max_seq_len < 0 || (masked && !ctx->st.keep_mask) ||
      (ctx->cfg.page_size == 1 && ctx->attn_impl != 1 && !masked))  // page size 1 exists for the matrix-core kernels only
    return TIM_ERR_INVALID_ARG;
  const tim_config &cfg = ctx->cfg;
  int cpb, slots, waves;
  AttnWs ws;
  ws.ml = ws.o = nullptr;
  ws.sched = nullptr;
  if (!own_scratch) {
    ws.ml = ctx->st.attn_ws;
    ws.o = ws.ml + (int64_t)cfg.max_batch * cfg.q_heads * AT_MAX_SLOTS * 2;
  }
  dim3 grid;
  if (own_scratch) {
    // Unscheduled (a schedule lives in the caller's workspace), and with as many slots as the library's own
    // array holds partials for: records [B][Hkv][slots][4 heads] of (m, l), then of o[128], all fp32-sized.
    // Fewer slots than the bound asks for only mean larger blocks: a block strides over its sequence's chunks.
    const int64_t per_slot = (int64_t)cfg.max_batch * cfg.q_heads * (TIM_D + 2) * (int64_t)sizeof(float);
    if (per_slot > (int64_t)TIM_NOALLOC_SCRATCH_BYTES) return TIM_ERR_TOO_LARGE;
    float *base = nullptr;
    const int rc = at_noalloc_scratch(&base);
    if (rc != TIM_OK) return rc;
    at_shape(ctx, max_seq_len, &cpb, &slots, &waves);
    const int fit = (int)((int64_t)TIM_NOALLOC_SCRATCH_BYTES / per_slot);
    if (slots > fit) slots = fit;
    ws.ml = base;
    ws.o = base + (int64_t)cfg.max_batch * cfg.q_heads * slots * 2;
    grid = dim3(cfg.max_batch * cfg.kv_heads, slots);
  } else if (ctx->sched_valid) {  // the schedule's shape, not this call's bound: the merge must see the same slots
    cpb = ctx->sched_cpb;
    slots = ctx->sched_slots;
    waves = ctx->sched_waves;
    ws.sched = reinterpret_cast<const int32_t *>(ctx->st.attn_ws + at_partials_words(cfg));
    grid = dim3(cfg.max_batch * cfg.kv_heads * slots);  // an upper bound on the list's length
  } else {
    at_shape(ctx, max_seq_len, &cpb, &slots, &waves);
    grid = dim3(cfg.max_batch * cfg.kv_heads, slots);
  }
  const float scale_log2 = sm_scale * 1.4426950408889634f;
  hipStream_t s = tim_hs(stream);
  const bool bf = out_dtype == TIM_OUT_BF16;
  if (masked) {
    if (bf) at_launch<2, true>(grid, s, ctx, ws, layer, q, out, scale_log2, cpb, slots, waves, k_new, v_new);
    else at_launch<2, false>(grid, s, ctx, ws, layer, q, out, scale_log2, cpb, slots, waves, k_new, v_new);
  } else if (ctx->attn_impl == 1) {
    if (bf) at_launch<1, true>(grid, s, ctx, ws, layer, q, out, scale_log2, cpb, slots, waves, k_new, v_new);
    else at_launch<1, false>(grid, s, ctx, ws, layer, q, out, scale_log2, cpb, slots, waves, k_new, v_new);
  } else {
    if (bf) at_launch<0, true>(grid, s, ctx, ws, layer, q, out, scale_log2, cpb, slots, waves, k_new, v_new);
    else at_launch<0, false>(grid, s, ctx, ws, layer, q, out, scale_log2, cpb, slots, waves, k_new, v_new);
  }
  TIM_LAUNCH_CHECK();
  if (slots > 1) {  // with one slot every block has already written its final output
    dim3 mgrid(cfg.max_batch * cfg.q_heads);
    if (bf) hipLaunchKernelGGL((tim_attn_merge_kernel<true>), mgrid, dim3(TIM_D), 0, s, cfg, ctx->st, ws, out, slots, cpb);
    else hipLaunchKernelGGL((tim_attn_merge_kernel<false>), mgrid, dim3(TIM_D), 0, s, cfg, ctx->st, ws, out, slots, cpb);
    TIM_LAUNCH_CHECK();
  }
  return TIM_OK;
}

extern "C" int tim_decode_attn(tim_ctx *ctx, int32_t layer, const void *q, void *out, float sm_scale,
                               int32_t out_dtype, int32_t max_seq_len, tim_stream stream) {
  return at_decode(ctx, layer, q, out, sm_scale, out_dtype, max_seq_len, stream, false);
}

extern "C" int tim_decode_attn_noalloc(tim_ctx *ctx, int32_t layer, const void *q, void *out, float sm_scale,
                                       int32_t out_dtype, int32_t max_seq_len, tim_stream stream) {
  return at_decode(ctx, layer, q, out, sm_scale, out_dtype, max_seq_len, stream, false, nullptr, nullptr, true);
}

extern "C" int tim_decode_attn_masked(tim_ctx *ctx, int32_t layer, const void *q, void *out, float sm_scale,
                                      int32_t out_dtype, int32_t max_seq_len, tim_stream stream) {
  return at_decode(ctx, layer, q, out, sm_scale, out_dtype, max_seq_len, stream, true);
}

extern "C" int tim_decode_attn_append(tim_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new,
                                      void *out, float sm_scale, int32_t out_dtype, int32_t max_seq_len,
                                      tim_stream stream) {
  if (!k_new || !v_new) return TIM_ERR_INVALID_ARG;
  if (ctx && ctx->bound && ctx->attn_impl != 1) {  // the vector-ALU variant has no fused path: two launches
    const int rc = tim_kv_append(ctx, layer, k_new, v_new, stream);
    if (rc != TIM_OK) return rc;
    return at_decode(ctx, layer, q, out, sm_scale, out_dtype, max_seq_len, stream, false);
  }
  return at_decode(ctx, layer, q, out, sm_scale, out_dtype, max_seq_len, stream, false, k_new, v_new);
}
