// Device page allocator (LIFO free stack), structure tracking, slot reservation and
// KV append.  All integer work; every kernel here is tiny and latency-bound.
#include "tim_internal.h"

// ---- reset ---------------------------------------------------------------------
__global__ void tim_reset_kernel(tim_config cfg, tim_state st) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t k = i; k < cfg.num_pages; k += stride) st.free_stack[k] = cfg.num_pages - 1 - (int32_t)k;
  const int64_t npt = (int64_t)cfg.max_batch * cfg.max_pages_per_seq;
  for (int64_t k = i; k < npt; k += stride) st.page_table[k] = -1;
  const int64_t nn = (int64_t)cfg.max_batch * cfg.max_nodes;
  for (int64_t k = i; k < nn; k += stride) {
    st.node_tok_begin[k] = -1;
    st.node_sub_begin[k] = -1;
    st.node_sub_end[k] = -1;
    st.node_tok_end[k] = -1;
    st.node_list_order[k] = -1;
  }
  if (st.keep_mask) {
    const int64_t nw = (int64_t)cfg.max_batch * tim_mask_words(cfg);
    for (int64_t k = i; k < nw; k += stride) st.keep_mask[k] = 0xffffffffu;
  }
  for (int64_t k = i; k < cfg.max_batch; k += stride) {
    st.seq_len[k] = 0;
    st.n_nodes[k] = 0;
    st.lists_done[k] = 0;
  }
  if (i == 0) {
    *st.free_top = cfg.num_pages;
    *st.status = 0;
  }
}

// ---- structure marks -----------------------------------------------------------------
// One thread per sequence walks the op list in order and applies its own ops, so
// completion ordinals follow array order without atomics.
__global__ void tim_mark_kernel(tim_config cfg, tim_state st, const int32_t *__restrict__ ops, int n_ops) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  // out-of-range sequence ids are reported once, by thread 0 of block 0
  if (b == 0) {
    for (int i = 0; i < n_ops; ++i) {
      const int s = ops[4 * i];
      if (s < 0 || s >= cfg.max_batch) tim_set_status(st.status, TIM_ERR_BAD_TREE);
    }
  }
  if (b >= cfg.max_batch) return;
  const int n = st.seq_len[b];
  int done = st.lists_done[b];
  int nn = st.n_nodes[b];
  const int64_t row = (int64_t)b * cfg.max_nodes;
  const int limit = cfg.max_pages_per_seq * cfg.page_size;
  for (int i = 0; i < n_ops; ++i) {
    if (ops[4 * i] != b) continue;
    const int code = ops[4 * i + 1], node = ops[4 * i + 2], at = ops[4 * i + 3];
    const int pos = at < 0 ? n : at;
    if (node < 0 || node >= cfg.max_nodes || pos > limit || code < TIM_MARK_OPEN || code > TIM_MARK_CLOSE) {
      tim_set_status(st.status, TIM_ERR_BAD_TREE);
      continue;
    }
    if (code == TIM_MARK_OPEN) {
      st.node_tok_begin[row + node] = pos;
    } else if (code == TIM_MARK_SUB_BEGIN) {
      st.node_sub_begin[row + node] = pos;
    } else if (code == TIM_MARK_SUB_END) {
      st.node_sub_end[row + node] = pos;
      st.node_list_order[row + node] = done++;
    } else {
      st.node_tok_end[row + node] = pos;
    }
    nn = max(nn, node + 1);
  }
  st.lists_done[b] = done;
  st.n_nodes[b] = nn;
}

// ---- reserve one slot per sequence ---------------------------------------------------
// Single block.  Sequences that start a new page pop in ascending id: an exclusive
// scan over the need flags gives each its depth below the top of the stack.
__global__ void __launch_bounds__(1024) tim_advance_kernel(tim_config cfg, tim_state st) {
  __shared__ int smem[17];
  __shared__ int s_bad;
  const int tid = threadIdx.x;
  if (tid == 0) s_bad = 0;
  __syncthreads();
  const int top = *st.free_top;
  // pass 1: count and validate
  int cnt = 0;
  for (int b = tid; b < cfg.max_batch; b += blockDim.x) {
    const int n = st.seq_len[b];
    if (n % cfg.page_size == 0) {
      ++cnt;
      if (n / cfg.page_size >= cfg.max_pages_per_seq) atomicOr(&s_bad, 1);
    }
  }
  int total;
  tim_block_incl_scan(cnt, smem, &total);
  __syncthreads();
  if (s_bad) {
    if (tid == 0) tim_set_status(st.status, TIM_ERR_SEQ_TOO_LONG);
    return;
  }
  if (total > top) {
    if (tid == 0) tim_set_status(st.status, TIM_ERR_OOM_PAGES);
    return;
  }
  // pass 2: assign, in chunks of blockDim sequences so ids stay ascending
  int base = 0;
  for (int b0 = 0; b0 < cfg.max_batch; b0 += blockDim.x) {
    const int b = b0 + tid;
    int need = 0, n = 0;
    if (b < cfg.max_batch) {
      n = st.seq_len[b];
      need = (n % cfg.page_size == 0) ? 1 : 0;
    }
    int chunk_total;
    const int incl = tim_block_incl_scan(need, smem, &chunk_total);
    if (b < cfg.max_batch) {
      if (need) st.page_table[(int64_t)b * cfg.max_pages_per_seq + n / cfg.page_size] = st.free_stack[top - 1 - (base + incl - 1)];
      st.seq_len[b] = n + 1;
    }
    base += chunk_total;
  }
  if (tid == 0) *st.free_top = top - total;
}

// ---- reserve several slots per sequence (tool responses) --------------------------------
// Single block, same deterministic pop order as the one-token case: sequence b needs
// ceil((n+c)/16) - ceil(n/16) pages; an exclusive scan gives its first depth below the top.
__global__ void __launch_bounds__(1024) tim_extend_kernel(tim_config cfg, tim_state st, const int32_t *__restrict__ counts) {
  __shared__ int smem[17];
  __shared__ int s_bad;
  const int tid = threadIdx.x;
  if (tid == 0) s_bad = 0;
  __syncthreads();
  const int top = *st.free_top;
  int cnt = 0;
  for (int b = tid; b < cfg.max_batch; b += blockDim.x) {
    const int n = st.seq_len[b], c = counts[b];
    if (c < 0) {
      atomicOr(&s_bad, 2);
      continue;
    }
    const int have = (n + cfg.page_size - 1) / cfg.page_size, want = (n + c + cfg.page_size - 1) / cfg.page_size;
    if (want > cfg.max_pages_per_seq) atomicOr(&s_bad, 1);
    cnt += want - have;
  }
  int total;
  tim_block_incl_scan(cnt, smem, &total);
  __syncthreads();
  if (s_bad) {
    if (tid == 0) tim_set_status(st.status, (s_bad & 2) ? TIM_ERR_INVALID_ARG : TIM_ERR_SEQ_TOO_LONG);
    return;
  }
  if (total > top) {
    if (tid == 0) tim_set_status(st.status, TIM_ERR_OOM_PAGES);
    return;
  }
  int base = 0;
  for (int b0 = 0; b0 < cfg.max_batch; b0 += blockDim.x) {
    const int b = b0 + tid;
    int need = 0, n = 0, c = 0, have = 0;
    if (b < cfg.max_batch) {
      n = st.seq_len[b];
      c = counts[b];
      have = (n + cfg.page_size - 1) / cfg.page_size;
      need = (n + c + cfg.page_size - 1) / cfg.page_size - have;
    }
    int chunk_total;
    const int incl = tim_block_incl_scan(need, smem, &chunk_total);
    if (b < cfg.max_batch) {
      const int first = base + incl - need;
      for (int k = 0; k < need; ++k)
        st.page_table[(int64_t)b * cfg.max_pages_per_seq + have + k] = st.free_stack[top - 1 - (first + k)];
      st.seq_len[b] = n + c;
    }
    base += chunk_total;
  }
  if (tid == 0) *st.free_top = top - total;
}

// ---- write the rows of the tokens just reserved ---------------------------------------------
// One thread moves 16 bytes of one (row, kv head) of K or V; the row's sequence is found by
// bisection in the prefix sums.
__global__ void tim_write_rows_kernel(tim_config cfg, tim_state st, int layer, const int32_t *__restrict__ row_off,
                                      int n_rows, const uint4 *__restrict__ k_rows, const uint4 *__restrict__ v_rows) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // over n_rows * Hkv * 16 * 2
  const int64_t per = (int64_t)n_rows * cfg.kv_heads * 16;
  if (idx >= 2 * per) return;
  const int which = (int)(idx / per);
  const int64_t r = idx % per;
  const int piece = (int)(r % 16);
  const int h = (int)((r / 16) % cfg.kv_heads);
  const int row = (int)(r / (16 * cfg.kv_heads));
  int lo = 0, hi = cfg.max_batch - 1;  // last b with row_off[b] <= row
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (row_off[mid] <= row) lo = mid; else hi = mid - 1;
  }
  const int b = lo, c = row_off[b + 1] - row_off[b];
  const int t = st.seq_len[b] - c + (row - row_off[b]);
  if (row >= row_off[cfg.max_batch] || t < 0) return;
  const int page = st.page_table[(int64_t)b * cfg.max_pages_per_seq + t / cfg.page_size];
  if (page < 0 || page >= cfg.num_pages) {
    tim_set_status(st.status, TIM_ERR_INVALID_ARG);
    return;
  }
  const int64_t tile = ((int64_t)layer * cfg.num_pages + page) * cfg.kv_heads + h;
  uint4 *pool = reinterpret_cast<uint4 *>(which ? st.v_pool : st.k_pool);
  const uint4 *src = which ? v_rows : k_rows;
  pool[tile * (cfg.page_size * 16) + (t % cfg.page_size) * 16 + piece] = src[((int64_t)row * cfg.kv_heads + h) * 16 + piece];
}

// ---- append the pending token's K/V row of one layer ------------------------------------
// One thread moves 16 bytes; 16 threads cover a 256-byte row; K and V rows of all
// (sequence, kv head) pairs are spread over the grid.
__global__ void tim_append_kernel(tim_config cfg, tim_state st, int layer, const uint4 *__restrict__ k_new,
                                  const uint4 *__restrict__ v_new) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;  // over B * Hkv * 16 * 2
  const int per = cfg.max_batch * cfg.kv_heads * 16;
  if (idx >= 2 * per) return;
  const int which = idx / per;  // 0 = K, 1 = V
  const int r = idx % per;
  const int piece = r % 16;
  const int bh = r / 16;  // b * Hkv + h
  const int b = bh / cfg.kv_heads, h = bh % cfg.kv_heads;
  const int n = st.seq_len[b];
  if (n <= 0) return;
  const int t = n - 1;
  const int page = st.page_table[(int64_t)b * cfg.max_pages_per_seq + t / cfg.page_size];
  if (page < 0 || page >= cfg.num_pages) {
    tim_set_status(st.status, TIM_ERR_INVALID_ARG);
    return;
  }
  const int64_t tile = ((int64_t)layer * cfg.num_pages + page) * cfg.kv_heads + h;
  uint4 *pool = reinterpret_cast<uint4 *>(which ? st.v_pool : st.k_pool);
  const uint4 *src = which ? v_new : k_new;
  pool[tile * (cfg.page_size * 16) + (t % cfg.page_size) * 16 + piece] = src[(int64_t)bh * 16 + piece];
}

// ---- accounting ---------------------------------------------------------------------------
// Counted from the page tables themselves, not derived from the lengths, so that a leaked or doubly
// pushed page, or a table entry that disagrees with its sequence's length, shows up on the device.
__global__ void tim_stats_clear_kernel(tim_config cfg, int32_t *out, int32_t *seen) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (int64_t)gridDim.x * blockDim.x;
  if (seen)
    for (int64_t k = i; k < cfg.num_pages; k += stride) seen[k] = 0;
  if (i < 4) out[i] = (i == 3 && !seen) ? -1 : 0;
}
__global__ void __launch_bounds__(256) tim_stats_kernel(tim_config cfg, tim_state st, int32_t *out, int32_t *seen) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (int64_t)gridDim.x * blockDim.x;
  const int top = min(max(*st.free_top, 0), cfg.num_pages);
  int entries = 0, by_len = 0, bad = 0;
  auto visit = [&](int page) {
    if (page < 0 || page >= cfg.num_pages) bad = 1;
    else if (seen && atomicAdd(&seen[page], 1) != 0) bad = 1;
  };
  for (int64_t k = i; k < top; k += stride) visit(st.free_stack[k]);
  const int64_t npt = (int64_t)cfg.max_batch * cfg.max_pages_per_seq;
  for (int64_t k = i; k < npt; k += stride) {
    const int page = st.page_table[k];
    if (page != -1) {
      ++entries;
      visit(page);
    }
  }
  for (int64_t b = i; b < cfg.max_batch; b += stride) by_len += (st.seq_len[b] + cfg.page_size - 1) / cfg.page_size;
  if (entries) atomicAdd(&out[1], entries);
  if (by_len) atomicAdd(&out[2], by_len);
  if (bad && seen) atomicOr(&out[3], 1);
  if (i == 0) out[0] = *st.free_top;
}

// ---- host entry points -----------------------------------------------------------------------
extern "C" int tim_pool_reset(tim_ctx *ctx, tim_stream stream) {
  if (!ctx || !ctx->bound) return TIM_ERR_INVALID_ARG;
  ctx->sched_valid = false;  // lengths change: an attention schedule no longer holds
  hipLaunchKernelGGL(tim_reset_kernel, dim3(256), dim3(256), 0, tim_hs(stream), ctx->cfg, ctx->st);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}

extern "C" int tim_tree_mark(tim_ctx *ctx, const int32_t *ops, int32_t n_ops, tim_stream stream) {
  if (!ctx || !ctx->bound || n_ops < 0 || (n_ops > 0 && !tim_ints_ok(ops))) return TIM_ERR_INVALID_ARG;
  if (n_ops == 0) return TIM_OK;
  const int threads = 64;
  const int blocks = (ctx->cfg.max_batch + threads - 1) / threads;
  hipLaunchKernelGGL(tim_mark_kernel, dim3(blocks), dim3(threads), 0, tim_hs(stream), ctx->cfg, ctx->st, ops, n_ops);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}

extern "C" int tim_seq_advance(tim_ctx *ctx, tim_stream stream) {
  if (!ctx || !ctx->bound) return TIM_ERR_INVALID_ARG;
  ctx->sched_valid = false;  // lengths change: an attention schedule no longer holds
  int threads = ((ctx->cfg.max_batch + 63) / 64) * 64;
  if (threads > 1024) threads = 1024;
  hipLaunchKernelGGL(tim_advance_kernel, dim3(1), dim3(threads), 0, tim_hs(stream), ctx->cfg, ctx->st);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}

extern "C" int tim_seq_extend(tim_ctx *ctx, const int32_t *counts, tim_stream stream) {
  if (!ctx || !ctx->bound || !tim_ints_ok(counts)) return TIM_ERR_INVALID_ARG;
  ctx->sched_valid = false;  // lengths change: an attention schedule no longer holds
  int threads = ((ctx->cfg.max_batch + 63) / 64) * 64;
  if (threads > 1024) threads = 1024;
  hipLaunchKernelGGL(tim_extend_kernel, dim3(1), dim3(threads), 0, tim_hs(stream), ctx->cfg, ctx->st, counts);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}

extern "C" int tim_kv_write(tim_ctx *ctx, int32_t layer, const int32_t *row_off, int32_t n_rows, const void *k_rows,
                            const void *v_rows, tim_stream stream) {
  if (!ctx || !ctx->bound || !tim_ints_ok(row_off) || n_rows < 0 || layer < 0 || layer >= ctx->cfg.layers) return TIM_ERR_INVALID_ARG;
  if (n_rows == 0) return TIM_OK;
  if (!tim_rows_ok(k_rows) || !tim_rows_ok(v_rows)) return TIM_ERR_INVALID_ARG;
  const int64_t total = 2 * (int64_t)n_rows * ctx->cfg.kv_heads * 16;
  const int threads = 256;
  hipLaunchKernelGGL(tim_write_rows_kernel, dim3((unsigned)((total + threads - 1) / threads)), dim3(threads), 0,
                     tim_hs(stream), ctx->cfg, ctx->st, layer, row_off, n_rows, reinterpret_cast<const uint4 *>(k_rows),
                     reinterpret_cast<const uint4 *>(v_rows));
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}

extern "C" int tim_kv_append(tim_ctx *ctx, int32_t layer, const void *k_new, const void *v_new, tim_stream stream) {
  if (!ctx || !ctx->bound || !tim_rows_ok(k_new) || !tim_rows_ok(v_new) || layer < 0 || layer >= ctx->cfg.layers) return TIM_ERR_INVALID_ARG;
  const int total = 2 * ctx->cfg.max_batch * ctx->cfg.kv_heads * 16;
  const int threads = 256;
  hipLaunchKernelGGL(tim_append_kernel, dim3((total + threads - 1) / threads), dim3(threads), 0, tim_hs(stream),
                     ctx->cfg, ctx->st, layer, reinterpret_cast<const uint4 *>(k_new),
                     reinterpret_cast<const uint4 *>(v_new));
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}

extern "C" int tim_pool_stats(tim_ctx *ctx, int32_t *out, int32_t *scratch, tim_stream stream) {
  if (!ctx || !ctx->bound || !tim_ints_ok(out) || !tim_aligned(scratch, 4)) return TIM_ERR_INVALID_ARG;
  hipLaunchKernelGGL(tim_stats_clear_kernel, dim3(64), dim3(256), 0, tim_hs(stream), ctx->cfg, out, scratch);
  TIM_LAUNCH_CHECK();
  hipLaunchKernelGGL(tim_stats_kernel, dim3(64), dim3(256), 0, tim_hs(stream), ctx->cfg, ctx->st, out, scratch);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}

extern "C" int tim_status(tim_ctx *ctx, tim_stream stream) {
  if (!ctx || !ctx->bound) return TIM_ERR_INVALID_ARG;
  int32_t v = 0;
  TIM_HIP_CHECK(hipStreamSynchronize(tim_hs(stream)));
  TIM_HIP_CHECK(hipMemcpy(&v, ctx->st.status, sizeof(v), hipMemcpyDeviceToHost));
  if (v != 0) {
    const int32_t zero = 0;
    TIM_HIP_CHECK(hipMemcpy(ctx->st.status, &zero, sizeof(zero), hipMemcpyHostToDevice));
  }
  return v;
}
