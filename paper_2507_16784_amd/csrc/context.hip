// Context object: configuration, the caller's buffer pointers, host-side constants.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "tim_internal.h"

extern "C" int tim_ctx_create(tim_ctx **out, const tim_config *cfg) {
  if (!out || !cfg) return TIM_ERR_INVALID_ARG;
  *out = nullptr;
  if (cfg->head_dim != TIM_D || (cfg->page_size != TIM_PS && cfg->page_size != 1) || cfg->kv_heads <= 0 ||
      cfg->q_heads != TIM_G * cfg->kv_heads || cfg->layers <= 0 || cfg->num_pages <= 0 || cfg->max_batch <= 0 ||
      cfg->max_pages_per_seq <= 0 || cfg->max_nodes <= 0 || !(cfg->rope_base > 1.0f))
    return TIM_ERR_INVALID_ARG;
  // slots are int32: page * 16 + row must not overflow
  if ((int64_t)cfg->num_pages * cfg->page_size > INT32_MAX || (int64_t)cfg->max_pages_per_seq * cfg->page_size > INT32_MAX / 2)
    return TIM_ERR_INVALID_ARG;
  tim_ctx *c = new (std::nothrow) tim_ctx();
  if (!c) return TIM_ERR_INVALID_ARG;
  c->cfg = *cfg;
  c->bound = false;
  c->n_cu = 256;
  c->attn_impl = 1;
  c->attn_cpb = 6;  // 768 KiB of K/V per block; 5 to 8 measure within 0.5 % of each other on 16-32K-token sequences
  c->attn_fill = 2;
  if (const char *v = std::getenv("TIM_ATTN_FILL")) {  // tuning experiments only
    const int x = std::atoi(v);
    if (x >= 1 && x <= 64) c->attn_fill = x;
  }
  if (const char *v = std::getenv("TIM_ATTN_CPB")) {  // tuning experiments only
    const int x = std::atoi(v);
    if (x >= 1 && x <= 64) c->attn_cpb = x;
  }
  if (const char *v = std::getenv("TIM_ATTN_GRADE")) {  // tuning experiments only: "big,small" in 1/16 rounds
    int a = 0, b2 = 0;
    if (std::sscanf(v, "%d,%d", &a, &b2) == 2 && a >= b2 && b2 >= 0) {
      c->grade_big = a;
      c->grade_small = b2;
    }
  }
  if (const char *v = std::getenv("TIM_ATTN_SCHED_FORCE"))  // tests: small shapes must reach the scheduled path too
    c->sched_force = std::atoi(v) != 0;
  if (const char *v = std::getenv("TIM_ATTN_IMPL"))  // debugging / A-B measurement only
    c->attn_impl = std::strcmp(v, "valu") == 0 ? 0 : 1;
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
    c->n_cu = prop.multiProcessorCount;
  for (int i = 0; i < TIM_D / 2; ++i) c->inv_freq[i] = std::pow((double)cfg->rope_base, -2.0 * i / TIM_D);
  *out = c;
  return TIM_OK;
}

extern "C" int tim_ctx_destroy(tim_ctx *ctx) {
  delete ctx;
  return TIM_OK;
}

extern "C" int tim_bind(tim_ctx *ctx, const tim_state *s) {
  if (!ctx || !s) return TIM_ERR_INVALID_ARG;
  if (!s->k_pool || !s->v_pool || !s->page_table || !s->seq_len || !s->free_stack || !s->free_top || !s->status ||
      !s->node_tok_begin || !s->node_sub_begin || !s->node_sub_end || !s->node_tok_end || !s->node_list_order ||
      !s->n_nodes || !s->lists_done || !s->attn_ws)
    return TIM_ERR_INVALID_ARG;
  if (s->attn_ws_bytes < tim_attn_ws_bytes(&ctx->cfg)) return TIM_ERR_INVALID_ARG;
  ctx->st = *s;
  ctx->bound = true;
  ctx->sched_valid = false;
  return TIM_OK;
}
