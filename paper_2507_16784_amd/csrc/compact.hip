// KV compaction with RoPE re-rotation: gathers the planned survivors into their fresh
// pages.  HBM-bound: 4096 B read + 4096 B written per moved token per layer.
//
// Mapping.  One block of 128 threads owns one destination page (16 tokens) for a group
// of layers and all KV heads.  Thread (t, c) = (tid / 8, tid % 8) owns token t and the
// eight rotation pairs (8c+k, 64+8c+k): two 16-byte pieces of the K row, 128 B apart, and
// the same two pieces of the V row.  Eight neighbouring threads cover 128 contiguous
// bytes, so every access is a full line of a 256-byte row; rows of one source run are
// adjacent in memory.  The cos/sin of the token's position change are computed once per
// thread (angle in fp64, reduced to [-pi, pi], then fp32 sincos) and reused for every
// head and layer of the group, which keeps the kernel on the bandwidth roof.
//
// With the interleaved pairing (pairs (2i, 2i+1)) the same thread owns the same two pieces; each 32-bit word then
// is one pair, the first piece holds pairs 4c..4c+3 and the second pairs 32+4c..32+4c+3, and only the angles and
// the arithmetic between registers differ (template parameter IL): addresses and traffic are the same.
//
// No tile passes through LDS: a thread holds both halves of its rotation pairs in registers, so there is nothing
// to exchange.  A variant that did stage the key tile through LDS (256 threads per page, whole 256-byte rows per 16
// lanes on the way in, the 4 KiB destination tile written linearly, the partner half read from LDS under an XOR
// swizzle) produced identical bits and measured 6.28 ms against 6.13 ms for all 64 big flushes of the batch-64
// workload (6.01 against 6.16 TB/s read + write, same box, alternating): the line-sized accesses here already coalesce.
#include "tim_internal.h"

#define CP_THREADS 128
#define CP_LAYERS_PER_BLOCK 4

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// two floats -> packed bf16 pair, round to nearest even (hardware conversion on gfx950)
__device__ __forceinline__ uint32_t bf_pack(float lo, float hi) {
  float2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, b);
}

// cos / sin of the thread's eight angles for a position change d.  Half-split: pairs 8c..8c+7 (theta_step =
// theta_8).  Interleaved: pairs 4c..4c+3, then 32+4c..32+4c+3 (theta_step = theta_4).  theta_i is built by fp64
// multiplication from theta_1 (relative error ~1e-15, far below the fp32 sincos); the angle is reduced to
// [-pi, pi] in fp64 with a two-term 2 pi.
template <bool IL>
__device__ __forceinline__ void cp_angles(int d, int c, double theta1, double theta_step, double theta32, float (&cs)[8],
                                          float (&sn)[8]) {
  double th0 = 1.0;
  for (int q = 0; q < c; ++q) th0 *= theta_step;
  const double two_pi_hi = 6.283185307179586232e+00, two_pi_lo = 2.449293598294706414e-16;
  const double inv_two_pi = 1.591549430918953456e-01;
  double th = th0;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    if (IL && k == 4) th = th0 * theta32;
    const double a = (double)d * th;
    const double n2 = rint(a * inv_two_pi);
    double r = fma(-n2, two_pi_hi, a);
    r = fma(-n2, two_pi_lo, r);
    sincosf((float)r, &sn[k], &cs[k]);
    th *= theta1;
  }
}

// Rotates the thread's two 16-byte pieces of one key row (lo = dims 8c..8c+7, hi = the same + 64) in fp32.
template <bool IL>
__device__ __forceinline__ void cp_rotate(uint4 &lo, uint4 &hi, const float (&cs)[8], const float (&sn)[8]) {
  uint32_t *a = reinterpret_cast<uint32_t *>(&lo);
  uint32_t *b = reinterpret_cast<uint32_t *>(&hi);
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    if (IL) {  // each word is a pair: (dims 8c+2w, 8c+2w+1) in lo, the same + 64 in hi
      const float x = bf_lo(a[w]), y = bf_hi(a[w]);
      const float u = bf_lo(b[w]), v = bf_hi(b[w]);
      a[w] = bf_pack(fmaf(x, cs[w], -(y * sn[w])), fmaf(y, cs[w], x * sn[w]));
      b[w] = bf_pack(fmaf(u, cs[4 + w], -(v * sn[4 + w])), fmaf(v, cs[4 + w], u * sn[4 + w]));
    } else {
      const float x0 = bf_lo(a[w]), x1 = bf_hi(a[w]);  // dims 8c+2w, 8c+2w+1
      const float y0 = bf_lo(b[w]), y1 = bf_hi(b[w]);  // their partners at +64
      const float c0 = cs[2 * w], s0 = sn[2 * w], c1 = cs[2 * w + 1], s1 = sn[2 * w + 1];
      const float rx0 = fmaf(x0, c0, -(y0 * s0)), ry0 = fmaf(y0, c0, x0 * s0);
      const float rx1 = fmaf(x1, c1, -(y1 * s1)), ry1 = fmaf(y1, c1, x1 * s1);
      a[w] = bf_pack(rx0, rx1);
      b[w] = bf_pack(ry0, ry1);
    }
  }
}

// Work items are (destination page, layer group) pairs.  The destination pages of a flush
// are exactly its fresh pages, numbered 0..total_need-1 in (sequence, page) order, so item
// i belongs to the sequence whose PAGE_OFF range contains i; no work list is materialised
// and the host never needs to know how much moved: a fixed grid strides over the items.
template <bool IL>
__device__ __forceinline__ void tim_compact_item(const tim_config &cfg, const tim_state &st, const tim_plan &pl,
                                                 int n_seqs, int item, int l0, int l1, double theta1,
                                                 double theta_step, double theta32) {
  // sequence of this fresh page: last e with PAGE_OFF[e] <= item (n_seqs is small)
  int lo = 0, hi = n_seqs - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (pl.hdr[(int64_t)mid * TIM_PLAN_HDR + TIM_HDR_PAGE_OFF] <= item) lo = mid; else hi = mid - 1;
  }
  const int e = lo;
  const int32_t *hdr = pl.hdr + (int64_t)e * TIM_PLAN_HDR;
  const int m = hdr[TIM_HDR_N_KEPT], keep = hdr[TIM_HDR_KEEP_PAGES];
  const int p = keep + (item - hdr[TIM_HDR_PAGE_OFF]);
  const int tid = threadIdx.x, t = tid >> 3, c = tid & 7;
  const int j = p * TIM_PS + t;
  if (hdr[TIM_HDR_BAD] || j >= m) return;  // ragged last page; no block-wide sync below
  const int T = cfg.max_pages_per_seq * TIM_PS;
  const int src = pl.src_slot[(int64_t)e * T + j];
  const int dst = pl.dst_slot[(int64_t)e * T + j];
  const int d = pl.delta[(int64_t)e * T + j];
  const int64_t nslots = (int64_t)cfg.num_pages * TIM_PS;
  if (src < 0 || src >= nslots || dst < 0 || dst >= nslots) {
    tim_set_status(st.status, TIM_ERR_INVALID_ARG);
    return;
  }

  float cs[8], sn[8];
  if (d != 0) cp_angles<IL>(d, c, theta1, theta_step, theta32, cs, sn);

  const uint4 *kp = reinterpret_cast<const uint4 *>(st.k_pool);
  const uint4 *vp = reinterpret_cast<const uint4 *>(st.v_pool);
  uint4 *kw = reinterpret_cast<uint4 *>(st.k_pool);
  uint4 *vw = reinterpret_cast<uint4 *>(st.v_pool);
  const int hkv = cfg.kv_heads;
  // offsets in uint4 (16 B) units: tile = 256 units, row = 16 units
  const int64_t s_off = (int64_t)(src / TIM_PS) * hkv * 256 + (src % TIM_PS) * 16 + c;
  const int64_t d_off = (int64_t)(dst / TIM_PS) * hkv * 256 + (dst % TIM_PS) * 16 + c;
  for (int layer = l0; layer < l1; ++layer) {
    const int64_t lbase = (int64_t)layer * cfg.num_pages * hkv * 256;
    // heads go two at a time with all eight loads issued before the first store: source
    // and destination live in the same pool, so the compiler may not reorder them itself
    for (int h = 0; h < hkv; h += 2) {
      const bool two = h + 1 < hkv;
      const int64_t so = lbase + s_off + (int64_t)h * 256;
      const int64_t dof = lbase + d_off + (int64_t)h * 256;
      uint4 klo[2], khi[2], vlo[2], vhi[2];
      klo[0] = tim_load_stream(kp + so);
      khi[0] = tim_load_stream(kp + so + 8);
      vlo[0] = tim_load_stream(vp + so);
      vhi[0] = tim_load_stream(vp + so + 8);
      if (two) {
        klo[1] = tim_load_stream(kp + so + 256);
        khi[1] = tim_load_stream(kp + so + 256 + 8);
        vlo[1] = tim_load_stream(vp + so + 256);
        vhi[1] = tim_load_stream(vp + so + 256 + 8);
      }
      if (d != 0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) cp_rotate<IL>(klo[u], khi[u], cs, sn);
      }
      tim_store_stream(kw + dof, klo[0]);
      tim_store_stream(kw + dof + 8, khi[0]);
      tim_store_stream(vw + dof, vlo[0]);
      tim_store_stream(vw + dof + 8, vhi[0]);
      if (two) {
        tim_store_stream(kw + dof + 256, klo[1]);
        tim_store_stream(kw + dof + 256 + 8, khi[1]);
        tim_store_stream(vw + dof + 256, vlo[1]);
        tim_store_stream(vw + dof + 256 + 8, vhi[1]);
      }
    }
  }
}

template <bool IL>
__global__ void __launch_bounds__(CP_THREADS)
tim_compact_kernel(tim_config cfg, tim_state st, tim_plan pl, int n_seqs, int layer_begin, int layer_end,
                   double theta1, double theta_step, double theta32) {
  if (!pl.totals[TIM_TOT_OK]) return;
  const int groups = (layer_end - layer_begin + CP_LAYERS_PER_BLOCK - 1) / CP_LAYERS_PER_BLOCK;
  const int64_t n_work = (int64_t)pl.totals[TIM_TOT_NEED] * groups;
  for (int64_t w = blockIdx.x; w < n_work; w += gridDim.x) {
    const int item = (int)(w / groups), grp = (int)(w % groups);
    const int l0 = layer_begin + grp * CP_LAYERS_PER_BLOCK;
    tim_compact_item<IL>(cfg, st, pl, n_seqs, item, l0, min(l0 + CP_LAYERS_PER_BLOCK, layer_end), theta1, theta_step,
                         theta32);
  }
}

// Page size 1 (the paper's setting): survivors keep their pages, so a flush moves no row at
// all; only the keys behind the first pruned token are re-rotated where they lie (2 x 2 KiB
// per token per layer instead of 2 x 4 KiB, values untouched).  Work items are (tile of 32
// such tokens, layer group); thread (t, c) owns token t's eight rotation pairs as above and
// reads and writes the same addresses, so there is no hazard between threads.
template <bool IL>
__global__ void __launch_bounds__(CP_THREADS)
tim_rotate_inplace_kernel(tim_config cfg, tim_state st, tim_plan pl, int n_seqs, int layer_begin, int layer_end,
                          double theta1, double theta_step, double theta32) {
  if (!pl.totals[TIM_TOT_OK]) return;
  const int groups = (layer_end - layer_begin + CP_LAYERS_PER_BLOCK - 1) / CP_LAYERS_PER_BLOCK;
  const int64_t n_work = (int64_t)pl.totals[TIM_TOT_EXT_TILES] * groups;
  const int tid = threadIdx.x, t = tid >> 3, c = tid & 7;
  const int T = cfg.max_pages_per_seq * cfg.page_size;
  const int hkv = cfg.kv_heads;
  uint4 *kw = reinterpret_cast<uint4 *>(st.k_pool);
  for (int64_t w = blockIdx.x; w < n_work; w += gridDim.x) {
    const int tile = (int)(w / groups), grp = (int)(w % groups);
    int lo = 0, hi = n_seqs - 1;  // last e with EXT_TILE_OFF[e] <= tile
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (pl.hdr[(int64_t)mid * TIM_PLAN_HDR + TIM_HDR_EXT_TILE_OFF] <= tile) lo = mid; else hi = mid - 1;
    }
    const int e = lo;
    const int32_t *hdr = pl.hdr + (int64_t)e * TIM_PLAN_HDR;
    if (hdr[TIM_HDR_BAD]) continue;
    const int m = hdr[TIM_HDR_N_KEPT], f = hdr[TIM_HDR_FIRST_PRUNED];
    const int l0 = layer_begin + grp * CP_LAYERS_PER_BLOCK, l1 = min(l0 + CP_LAYERS_PER_BLOCK, layer_end);
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
      const int j = f + (tile - hdr[TIM_HDR_EXT_TILE_OFF]) * 32 + half * 16 + t;
      if (j >= m) continue;
      const int d = pl.delta[(int64_t)e * T + j];
      const int slot = pl.src_slot[(int64_t)e * T + j];
      if (d == 0) continue;
      if (slot < 0 || slot >= cfg.num_pages) {
        tim_set_status(st.status, TIM_ERR_INVALID_ARG);
        continue;
      }
      float cs[8], sn[8];
      cp_angles<IL>(d, c, theta1, theta_step, theta32, cs, sn);
      for (int layer = l0; layer < l1; ++layer) {
        const int64_t base = (((int64_t)layer * cfg.num_pages + slot) * hkv) * 16 + c;  // uint4 units, row = 16
        for (int h = 0; h < hkv; h += 2) {
          const bool two = h + 1 < hkv;
          uint4 klo[2], khi[2];
          klo[0] = kw[base + (int64_t)h * 16];
          khi[0] = kw[base + (int64_t)h * 16 + 8];
          if (two) {
            klo[1] = kw[base + (int64_t)(h + 1) * 16];
            khi[1] = kw[base + (int64_t)(h + 1) * 16 + 8];
          }
          cp_rotate<IL>(klo[0], khi[0], cs, sn);
          if (two) cp_rotate<IL>(klo[1], khi[1], cs, sn);
          kw[base + (int64_t)h * 16] = klo[0];
          kw[base + (int64_t)h * 16 + 8] = khi[0];
          if (two) {
            kw[base + (int64_t)(h + 1) * 16] = klo[1];
            kw[base + (int64_t)(h + 1) * 16 + 8] = khi[1];
          }
        }
      }
    }
  }
}

extern "C" int tim_kv_compact(tim_ctx *ctx, const tim_plan *plan, int32_t layer_begin, int32_t layer_end,
                              tim_stream stream) {
  if (!ctx || !ctx->bound || !plan || !plan->hdr || !plan->totals || !plan->src_slot || !plan->dst_slot ||
      !plan->delta || plan->n_seqs <= 0 || plan->n_seqs > plan->max_seqs || layer_begin < 0 ||
      layer_end > ctx->cfg.layers || layer_begin > layer_end)
    return TIM_ERR_INVALID_ARG;
  if (layer_begin == layer_end) return TIM_OK;
  // enough two-wave blocks to keep every CU's load queues full; they stride over the items
  dim3 grid(16 * ctx->n_cu);
  const bool il = ctx->cfg.rope_pairing == TIM_ROPE_INTERLEAVED;
  const double theta1 = ctx->inv_freq[1], theta_step = ctx->inv_freq[il ? 4 : 8], theta32 = ctx->inv_freq[32];
  auto kernel = ctx->cfg.page_size == 1 ? (il ? tim_rotate_inplace_kernel<true> : tim_rotate_inplace_kernel<false>)
                                        : (il ? tim_compact_kernel<true> : tim_compact_kernel<false>);
  hipLaunchKernelGGL(kernel, grid, dim3(CP_THREADS), 0, tim_hs(stream), ctx->cfg, ctx->st, *plan, plan->n_seqs,
                     layer_begin, layer_end, theta1, theta_step, theta32);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}
