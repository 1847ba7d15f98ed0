// Context object: configuration, the caller's buffer pointers, host-side constants.
#include <cmath>
#include <new>

#include "tim_internal.h"

extern "C" int tim_ctx_create(tim_ctx **out, const tim_config *cfg) {
  if (!out || !cfg) return TIM_ERR_INVALID_ARG;
  *out = nullptr;
  if (cfg->head_dim != TIM_D || (cfg->page_size != TIM_PS && cfg->page_size != 1) || cfg->kv_heads <= 0 ||
      cfg->q_heads != TIM_G * cfg->kv_heads || cfg->layers <= 0 || cfg->num_pages <= 0 || cfg->max_batch <= 0 ||
      cfg->max_pages_per_seq <= 0 || cfg->max_nodes <= 0 || !(cfg->rope_base > 1.0f) ||
      (cfg->rope_pairing != TIM_ROPE_HALF_SPLIT && cfg->rope_pairing != TIM_ROPE_INTERLEAVED))
    return TIM_ERR_INVALID_ARG;
  // slots are int32: page * 16 + row must not overflow
  if ((int64_t)cfg->num_pages * cfg->page_size > INT32_MAX || (int64_t)cfg->max_pages_per_seq * cfg->page_size > INT32_MAX / 2)
    return TIM_ERR_INVALID_ARG;
  tim_ctx *c = new (std::nothrow) tim_ctx();
  if (!c) return TIM_ERR_INVALID_ARG;
  c->cfg = *cfg;
  c->bound = false;
  c->n_cu = 256;
  c->attn_impl = TIM_ATTN_MFMA;
  c->attn_cpb = 6;  // 768 KiB of K/V per block; 5 to 8 measure within 0.5 % of each other on 16-32K-token sequences
  c->attn_fill = 2;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
    c->n_cu = prop.multiProcessorCount;
  if (hipGetDevice(&dev) == hipSuccess) tim_noalloc_scratch_init();
  for (int i = 0; i < TIM_D / 2; ++i) c->inv_freq[i] = std::pow((double)cfg->rope_base, -2.0 * i / TIM_D);
  *out = c;
  return TIM_OK;
}

extern "C" int tim_ctx_get_tuning(const tim_ctx *ctx, tim_tuning *out) {
  if (!ctx || !out) return TIM_ERR_INVALID_ARG;
  out->attn_impl = ctx->attn_impl;
  out->chunks_per_block = ctx->attn_cpb;
  out->fill = ctx->attn_fill;
  out->grade_big = ctx->grade_big;
  out->grade_small = ctx->grade_small;
  out->round_items = ctx->round_items;
  out->block_waves = ctx->block_waves;
  out->short_list_chunks = ctx->short_per;
  return TIM_OK;
}

extern "C" int tim_ctx_set_tuning(tim_ctx *ctx, const tim_tuning *t) {
  if (!ctx || !t) return TIM_ERR_INVALID_ARG;
  if ((t->attn_impl != TIM_ATTN_VALU && t->attn_impl != TIM_ATTN_MFMA) || t->chunks_per_block < 1 ||
      t->chunks_per_block > 64 || t->fill < 1 || t->fill > 64 || t->grade_small < 0 || t->grade_big < t->grade_small ||
      t->round_items < 0 || (t->block_waves != 0 && t->block_waves != 4 && t->block_waves != 6 && t->block_waves != 8 && t->block_waves != 12) ||
      t->short_list_chunks < 0 || t->short_list_chunks > 128)
    return TIM_ERR_INVALID_ARG;
  ctx->attn_impl = t->attn_impl;
  ctx->attn_cpb = t->chunks_per_block;
  ctx->attn_fill = t->fill;
  ctx->grade_big = t->grade_big;
  ctx->grade_small = t->grade_small;
  ctx->round_items = t->round_items;
  ctx->block_waves = t->block_waves;
  ctx->short_per = t->short_list_chunks;
  ctx->sched_valid = false;  // a schedule written under the old shape no longer matches the launches
  return TIM_OK;
}

extern "C" int tim_ctx_destroy(tim_ctx *ctx) {
  delete ctx;
  return TIM_OK;
}

extern "C" int tim_bind(tim_ctx *ctx, const tim_state *s) {
  if (!ctx || !s) return TIM_ERR_INVALID_ARG;
  if (!tim_rows_ok(s->k_pool) || !tim_rows_ok(s->v_pool) || !tim_ints_ok(s->page_table) || !tim_ints_ok(s->seq_len) ||
      !tim_ints_ok(s->free_stack) || !tim_ints_ok(s->free_top) || !tim_ints_ok(s->status) || !tim_ints_ok(s->node_tok_begin) ||
      !tim_ints_ok(s->node_sub_begin) || !tim_ints_ok(s->node_sub_end) || !tim_ints_ok(s->node_tok_end) ||
      !tim_ints_ok(s->node_list_order) || !tim_ints_ok(s->n_nodes) || !tim_ints_ok(s->lists_done) ||
      !tim_aligned(s->attn_ws, 16) || !tim_aligned(s->keep_mask, 4))
    return TIM_ERR_INVALID_ARG;
  // the workspace is optional (tim_decode_attn_noalloc needs none); if given it must be large enough
  if (s->attn_ws && s->attn_ws_bytes < tim_attn_ws_bytes(&ctx->cfg)) return TIM_ERR_INVALID_ARG;
  ctx->st = *s;
  ctx->bound = true;
  ctx->sched_valid = false;
  return TIM_OK;
}
