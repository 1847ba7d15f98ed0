// Split-K paged GQA decode attention (HBM-bound: 4096 B per live token per layer).
//
// Work decomposition.  grid = (slots, kv_heads, batch).  A sequence's pages are cut into
// chunks of AT_CHUNK_PAGES pages; block `slot` takes chunks slot, slot + slots, ... and
// accumulates them into one partial (m, l, o[128]) per query head of its group.  Inside a
// chunk each of the four waves streams its own run of pages.  Fixed-size chunks keep a
// batch of very unequal lengths balanced: a long sequence simply occupies more blocks.
//
// Wave mapping for one (page, kv head) tile of 16 rows x 256 B, K and V alike: load j
// (j = 0..3) is one 16-byte load per lane covering 1 KiB of the tile contiguously, so
// lane (g, c) = (lane / 16, lane % 16) holds dims 8c..8c+7 of row 4j + g.  The dot product
// with the four query heads of the group is finished by a rotate-add over the 16 lanes
// of a DPP row.  Each lane row g keeps its own online-softmax state over the rows it
// sees (4j + g), so the page loop has no cross-row traffic; rows, waves and chunks are
// merged once at the end (log-sum-exp algebra), then a small kernel merges the slots.
#include "tim_internal.h"

#define AT_THREADS 256
#define AT_WAVES 4
#define AT_CHUNK_PAGES 16
#define AT_PAGES_PER_WAVE (AT_CHUNK_PAGES / AT_WAVES)
#define AT_MAX_SLOTS 128
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
  float *ml;  // [B][Hq][slots][2]
  float *o;   // [B][Hq][slots][128]
};

__device__ __forceinline__ int at_used_slots(int n, int slots) {
  const int n_pages = (n + TIM_PS - 1) / TIM_PS;
  const int nchunks = (n_pages + AT_CHUNK_PAGES - 1) / AT_CHUNK_PAGES;
  return min(nchunks, slots);
}

template <bool OUT_BF16>
__device__ __forceinline__ void at_store_out(void *out, int64_t idx, float v) {
  if (OUT_BF16) {
    reinterpret_cast<__bf16 *>(out)[idx] = (__bf16)v;
  } else {
    reinterpret_cast<float *>(out)[idx] = v;
  }
}

template <bool OUT_BF16>
__global__ void __launch_bounds__(AT_THREADS)
tim_attn_partial_kernel(tim_config cfg, tim_state st, AttnWs ws, int layer, const uint4 *__restrict__ q,
                        void *__restrict__ out, float scale_log2) {
  __shared__ float red_m[AT_WAVES * 4][TIM_G];
  __shared__ float red_l[AT_WAVES * 4][TIM_G];
  __shared__ float red_o[AT_WAVES * 4][TIM_G][TIM_D];

  const int slot = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z, slots = gridDim.x;
  const int n = st.seq_len[b];
  const int n_pages = (n + TIM_PS - 1) / TIM_PS;
  const int nchunks = (n_pages + AT_CHUNK_PAGES - 1) / AT_CHUNK_PAGES;
  if (slot >= nchunks) return;  // uniform for the block
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

  for (int chunk = slot; chunk < nchunks; chunk += slots) {
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
      for (int j = 0; j < 4; ++j) kk[j] = kpool[tile + j * 64 + lane];
#pragma unroll
      for (int j = 0; j < 4; ++j) vv[j] = vpool[tile + j * 64 + lane];
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
  const int used = min(nchunks, slots);
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int idx = tid + r * AT_THREADS;  // 0..511 = (h, dim)
    const int h = idx >> 7, dim = idx & 127;
    float mx = AT_NEG_BIG;
#pragma unroll
    for (int s2 = 0; s2 < AT_WAVES * 4; ++s2) mx = fmaxf(mx, red_m[s2][h]);
    float lt = 0.f, ot = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < AT_WAVES * 4; ++s2) {
      const float sc = __builtin_amdgcn_exp2f(red_m[s2][h] - mx);
      lt = fmaf(red_l[s2][h], sc, lt);
      ot = fmaf(red_o[s2][h][dim], sc, ot);
    }
    const int hq = kvh * TIM_G + h;
    if (used == 1) {  // the only partial of this sequence: finish here
      at_store_out<OUT_BF16>(out, ((int64_t)b * cfg.q_heads + hq) * TIM_D + dim, ot / lt);
    } else {
      const int64_t pi = ((int64_t)b * cfg.q_heads + hq) * slots + slot;
      ws.o[pi * TIM_D + dim] = ot;
      if (dim == 0) {
        ws.ml[pi * 2] = mx;
        ws.ml[pi * 2 + 1] = lt;
      }
    }
  }
}

// Log-sum-exp merge of the slot partials of one (sequence, query head).
template <bool OUT_BF16>
__global__ void __launch_bounds__(TIM_D)
tim_attn_merge_kernel(tim_config cfg, tim_state st, AttnWs ws, void *__restrict__ out, int slots) {
  const int bh = blockIdx.x, b = bh / cfg.q_heads, dim = threadIdx.x;
  const int n = st.seq_len[b];
  const int used = at_used_slots(n, slots);
  if (used == 1) return;  // written by the partial kernel
  if (used == 0) {        // empty working memory: defined as zero
    at_store_out<OUT_BF16>(out, (int64_t)bh * TIM_D + dim, 0.f);
    return;
  }
  const int64_t p0 = (int64_t)bh * slots;
  float mx = AT_NEG_BIG;
  for (int s = 0; s < used; ++s) mx = fmaxf(mx, ws.ml[(p0 + s) * 2]);
  float lt = 0.f, ot = 0.f;
  for (int s = 0; s < used; ++s) {
    const float sc = __builtin_amdgcn_exp2f(ws.ml[(p0 + s) * 2] - mx);
    lt = fmaf(ws.ml[(p0 + s) * 2 + 1], sc, lt);
    ot = fmaf(ws.o[(p0 + s) * TIM_D + dim], sc, ot);
  }
  at_store_out<OUT_BF16>(out, (int64_t)bh * TIM_D + dim, ot / lt);
}

extern "C" int64_t tim_attn_ws_bytes(const tim_config *cfg) {
  if (!cfg) return 0;
  return (int64_t)cfg->max_batch * cfg->q_heads * AT_MAX_SLOTS * (TIM_D + 2) * (int64_t)sizeof(float);
}

extern "C" int tim_decode_attn(tim_ctx *ctx, int32_t layer, const void *q, void *out, float sm_scale,
                               int32_t out_dtype, int32_t max_seq_len, tim_stream stream) {
  if (!ctx || !ctx->bound || !q || !out || layer < 0 || layer >= ctx->cfg.layers ||
      (out_dtype != TIM_OUT_F32 && out_dtype != TIM_OUT_BF16) || max_seq_len < 0)
    return TIM_ERR_INVALID_ARG;
  const tim_config &cfg = ctx->cfg;
  const int full = cfg.max_pages_per_seq * TIM_PS;
  const int bound = (max_seq_len == 0 || max_seq_len > full) ? full : max_seq_len;
  const int max_pages = (bound + TIM_PS - 1) / TIM_PS;
  const int nchunks = (max_pages + AT_CHUNK_PAGES - 1) / AT_CHUNK_PAGES;
  const int rows = cfg.max_batch * cfg.kv_heads;
  const int slots_occ = (8 * ctx->n_cu + rows - 1) / rows;  // enough blocks to fill the chip
  const int slots_len = (nchunks + 3) / 4;                  // at most four chunks per block
  int slots = slots_occ > slots_len ? slots_occ : slots_len;
  if (slots > nchunks) slots = nchunks;
  if (slots > AT_MAX_SLOTS) slots = AT_MAX_SLOTS;
  if (slots < 1) slots = 1;
  AttnWs ws;
  ws.ml = ctx->st.attn_ws;
  ws.o = ctx->st.attn_ws + (int64_t)cfg.max_batch * cfg.q_heads * AT_MAX_SLOTS * 2;
  const float scale_log2 = sm_scale * 1.4426950408889634f;
  hipStream_t s = tim_hs(stream);
  dim3 grid(slots, cfg.kv_heads, cfg.max_batch);
  if (out_dtype == TIM_OUT_BF16) {
    hipLaunchKernelGGL(tim_attn_partial_kernel<true>, grid, dim3(AT_THREADS), 0, s, cfg, ctx->st, ws, layer,
                       reinterpret_cast<const uint4 *>(q), out, scale_log2);
    TIM_LAUNCH_CHECK();
    hipLaunchKernelGGL(tim_attn_merge_kernel<true>, dim3(cfg.max_batch * cfg.q_heads), dim3(TIM_D), 0, s, cfg,
                       ctx->st, ws, out, slots);
  } else {
    hipLaunchKernelGGL(tim_attn_partial_kernel<false>, grid, dim3(AT_THREADS), 0, s, cfg, ctx->st, ws, layer,
                       reinterpret_cast<const uint4 *>(q), out, scale_log2);
    TIM_LAUNCH_CHECK();
    hipLaunchKernelGGL(tim_attn_merge_kernel<false>, dim3(cfg.max_batch * cfg.q_heads), dim3(TIM_D), 0, s, cfg,
                       ctx->st, ws, out, slots);
  }
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}
