// Prune plan: pruning rule -> kept flags -> prefix-sum compaction -> page plan.
//
// Kernel 1 (one block per flushed sequence): the lists that left the pruning buffer
// mark their token ranges in a difference array; one pass of two chained block scans
// (coverage, then survivors) turns it into rank[], kept_idx[], new_pos[], delta[].
// Kernel 2 (one block): per-sequence page counts, two exclusive scans over the flushed
// sequences, the pool check, and the pop of all fresh pages at once.
// Kernel 3: fills the new page-table rows and the (src, dst) slot of every moved token.
// Commit: pushes replaced pages, installs rows and lengths, remaps node boundaries.
#include "tim_internal.h"

#define PLAN_THREADS 1024
#define PLAN_ITEMS 4

__global__ void __launch_bounds__(PLAN_THREADS)
tim_plan_scan_kernel(tim_config cfg, tim_state st, tim_plan pl, const int32_t *__restrict__ seq_ids, int threshold) {
  __shared__ int smem[17];
  __shared__ int s_first, s_bad;
  const int e = blockIdx.x, tid = threadIdx.x;
  const int b = seq_ids[e];
  int32_t *hdr = pl.hdr + (int64_t)e * TIM_PLAN_HDR;
  const int T = cfg.max_pages_per_seq * cfg.page_size;
  if (tid == 0) {
    s_first = 0x7fffffff;
    s_bad = 0;
    pl.seq_ids[e] = b;
  }
  __syncthreads();
  const bool seq_ok = b >= 0 && b < cfg.max_batch && (e == 0 || seq_ids[e - 1] < b);
  if (!seq_ok) {
    if (tid == 0) {
      tim_set_status(st.status, TIM_ERR_INVALID_ARG);
      for (int i = 0; i < TIM_PLAN_HDR; ++i) hdr[i] = 0;
      hdr[TIM_HDR_SEQ] = b;
      hdr[TIM_HDR_BAD] = 1;
    }
    return;
  }
  const int n = st.seq_len[b];
  int32_t *cover = pl.cover + (int64_t)e * (T + 1);
  int32_t *rank = pl.rank + (int64_t)e * (T + 1);
  int32_t *kept_idx = pl.kept_idx + (int64_t)e * T;
  int32_t *new_pos = pl.new_pos + (int64_t)e * T;
  int32_t *delta = pl.delta + (int64_t)e * T;

  for (int t = tid; t <= n; t += PLAN_THREADS) cover[t] = 0;
  __syncthreads();

  // the rule: every completed list except the `threshold` most recent ones is evicted
  const int64_t row = (int64_t)b * cfg.max_nodes;
  const int nn = min(st.n_nodes[b], cfg.max_nodes);
  const int gone_below = st.lists_done[b] - threshold;
  for (int i = tid; i < nn; i += PLAN_THREADS) {
    const int lo = st.node_list_order[row + i];
    if (lo < 0 || lo >= gone_below) continue;
    const int sb = st.node_sub_begin[row + i], se = st.node_sub_end[row + i];
    if (sb < 0 || se < sb || se > n) {
      atomicOr(&s_bad, 1);
      continue;
    }
    if (se > sb) {
      atomicAdd(&cover[sb], 1);
      atomicAdd(&cover[se], -1);
    }
  }
  __threadfence_block();
  __syncthreads();
  if (s_bad) {  // reject the tree: this sequence is left exactly as it is
    if (tid == 0) {
      tim_set_status(st.status, TIM_ERR_BAD_TREE);
      for (int i = 0; i < TIM_PLAN_HDR; ++i) hdr[i] = 0;
      hdr[TIM_HDR_SEQ] = b;
      hdr[TIM_HDR_N] = n;
      hdr[TIM_HDR_N_KEPT] = n;
      hdr[TIM_HDR_FIRST_PRUNED] = n;
      hdr[TIM_HDR_BAD] = 1;
    }
    return;
  }

  int cov_base = 0, kept_base = 0;
  for (int t0 = 0; t0 < n; t0 += PLAN_THREADS * PLAN_ITEMS) {
    const int tb = t0 + tid * PLAN_ITEMS;
    int c[PLAN_ITEMS];
    int csum = 0;
#pragma unroll
    for (int k = 0; k < PLAN_ITEMS; ++k) {
      c[k] = (tb + k < n) ? cover[tb + k] : 0;
      csum += c[k];
    }
    int ctot;
    int cexcl = tim_block_incl_scan(csum, smem, &ctot) - csum + cov_base;
    int kf[PLAN_ITEMS];
    int ksum = 0;
#pragma unroll
    for (int k = 0; k < PLAN_ITEMS; ++k) {
      cexcl += c[k];  // coverage of token tb+k (inclusive of ranges starting here)
      kf[k] = (tb + k < n && cexcl == 0) ? 1 : 0;
      ksum += kf[k];
    }
    int ktot;
    int r = tim_block_incl_scan(ksum, smem, &ktot) - ksum + kept_base;
    int first = 0x7fffffff;
#pragma unroll
    for (int k = 0; k < PLAN_ITEMS; ++k) {
      const int t = tb + k;
      if (t < n) {
        rank[t] = r;
        if (kf[k]) {
          new_pos[t] = r;
          kept_idx[r] = t;
          delta[r] = r - t;
          ++r;
        } else {
          new_pos[t] = -1;
          first = min(first, t);
        }
      }
    }
    if (first != 0x7fffffff) atomicMin(&s_first, first);
    cov_base += ctot;
    kept_base += ktot;
  }
  __syncthreads();
  if (tid == 0) {
    const int m = kept_base;
    rank[n] = m;
    const int f = s_first == 0x7fffffff ? n : s_first;
    for (int i = 0; i < TIM_PLAN_HDR; ++i) hdr[i] = 0;
    hdr[TIM_HDR_SEQ] = b;
    hdr[TIM_HDR_N] = n;
    hdr[TIM_HDR_N_KEPT] = m;
    hdr[TIM_HDR_FIRST_PRUNED] = f;
    // whole pages before the first pruned token stay in place; when only a tail was
    // pruned (m == f, which includes "nothing pruned") the boundary page stays as well
    if (cfg.page_size == 1) {
      // page size 1 (the paper's setting): a survivor keeps its page, nothing is copied; the
      // pruned tokens' pages are returned and the table is compacted as integers
      hdr[TIM_HDR_KEEP_PAGES] = f;
      hdr[TIM_HDR_NEED] = 0;
      hdr[TIM_HDR_PUSH] = n - m;
    } else {
      const int keep = (m == f) ? (f + cfg.page_size - 1) / cfg.page_size : f / cfg.page_size;
      hdr[TIM_HDR_KEEP_PAGES] = keep;
      hdr[TIM_HDR_NEED] = (m + cfg.page_size - 1) / cfg.page_size - keep;
      hdr[TIM_HDR_PUSH] = (n + cfg.page_size - 1) / cfg.page_size - keep;
    }
    hdr[TIM_HDR_EXT] = m - f;  // survivors behind the first pruned token (0 when nothing moves)
  }
}

__global__ void __launch_bounds__(1024) tim_plan_pages_kernel(tim_config cfg, tim_state st, tim_plan pl, int n_seqs) {
  __shared__ int smem[17];
  const int tid = threadIdx.x;
  int need_base = 0, push_base = 0, ext_base = 0, tile_base = 0;
  for (int e0 = 0; e0 < n_seqs; e0 += blockDim.x) {
    const int e = e0 + tid;
    int need = 0, push = 0, ext = 0;
    if (e < n_seqs) {
      need = pl.hdr[(int64_t)e * TIM_PLAN_HDR + TIM_HDR_NEED];
      push = pl.hdr[(int64_t)e * TIM_PLAN_HDR + TIM_HDR_PUSH];
      ext = pl.hdr[(int64_t)e * TIM_PLAN_HDR + TIM_HDR_EXT];
    }
    const int tiles = (ext + 31) / 32;
    int nt, pt, et, tt;
    const int ni = tim_block_incl_scan(need, smem, &nt);
    const int pi = tim_block_incl_scan(push, smem, &pt);
    const int ei = tim_block_incl_scan(ext, smem, &et);
    const int ti = tim_block_incl_scan(tiles, smem, &tt);
    if (e < n_seqs) {
      pl.hdr[(int64_t)e * TIM_PLAN_HDR + TIM_HDR_PAGE_OFF] = need_base + ni - need;
      pl.hdr[(int64_t)e * TIM_PLAN_HDR + TIM_HDR_PUSH_OFF] = push_base + pi - push;
      pl.hdr[(int64_t)e * TIM_PLAN_HDR + TIM_HDR_EXT_OFF] = ext_base + ei - ext;
      pl.hdr[(int64_t)e * TIM_PLAN_HDR + TIM_HDR_EXT_TILE_OFF] = tile_base + ti - tiles;
    }
    need_base += nt;
    push_base += pt;
    ext_base += et;
    tile_base += tt;
  }
  if (tid == 0) {
    const int top = *st.free_top;
    const int ok = need_base <= top ? 1 : 0;
    pl.totals[TIM_TOT_OK] = ok;
    pl.totals[TIM_TOT_NEED] = need_base;
    pl.totals[TIM_TOT_PUSH] = push_base;
    pl.totals[TIM_TOT_TOP_BEFORE] = top;
    pl.totals[TIM_TOT_TOP_AFTER_POP] = ok ? top - need_base : top;
    pl.totals[TIM_TOT_EXT] = ext_base;
    pl.totals[TIM_TOT_EXT_TILES] = tile_base;
    if (ok)
      *st.free_top = top - need_base;  // the fresh pages are taken now
    else
      tim_set_status(st.status, TIM_ERR_OOM_PAGES);
  }
}

__global__ void tim_plan_slots_kernel(tim_config cfg, tim_state st, tim_plan pl) {
  const int e = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (!pl.totals[TIM_TOT_OK]) return;
  const int32_t *hdr = pl.hdr + (int64_t)e * TIM_PLAN_HDR;
  if (hdr[TIM_HDR_BAD]) return;
  const int b = hdr[TIM_HDR_SEQ], m = hdr[TIM_HDR_N_KEPT];
  const int keep = hdr[TIM_HDR_KEEP_PAGES], need = hdr[TIM_HDR_NEED], off = hdr[TIM_HDR_PAGE_OFF];
  const int top = pl.totals[TIM_TOT_TOP_BEFORE];
  const int T = cfg.max_pages_per_seq * cfg.page_size;
  const int32_t *old_row = st.page_table + (int64_t)b * cfg.max_pages_per_seq;
  if (cfg.page_size == 1) {  // survivors keep their pages: the new row is the old one gathered by kept_idx
    if (j < cfg.max_pages_per_seq) {
      const int v = j < m ? old_row[pl.kept_idx[(int64_t)e * T + j]] : -1;
      pl.new_table[(int64_t)e * cfg.max_pages_per_seq + j] = v;
      if (j >= keep && j < m) pl.src_slot[(int64_t)e * T + j] = pl.dst_slot[(int64_t)e * T + j] = v;
    }
    return;
  }
  if (j < cfg.max_pages_per_seq) {
    int v = -1;
    if (j < keep)
      v = old_row[j];
    else if (j < keep + need)
      v = st.free_stack[top - 1 - (off + (j - keep))];
    pl.new_table[(int64_t)e * cfg.max_pages_per_seq + j] = v;
  }
  if (j >= keep * cfg.page_size && j < m) {
    const int src = pl.kept_idx[(int64_t)e * T + j];
    pl.src_slot[(int64_t)e * T + j] = old_row[src / cfg.page_size] * cfg.page_size + src % cfg.page_size;
    const int fresh = st.free_stack[top - 1 - (off + (j / cfg.page_size - keep))];
    pl.dst_slot[(int64_t)e * T + j] = fresh * cfg.page_size + j % cfg.page_size;
  }
}

__global__ void tim_plan_commit_kernel(tim_config cfg, tim_state st, tim_plan pl) {
  const int e = blockIdx.y;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (!pl.totals[TIM_TOT_OK]) return;
  // the new stack height is written once, whatever becomes of the first listed sequence
  if (e == 0 && i == 0) *st.free_top = pl.totals[TIM_TOT_TOP_AFTER_POP] + pl.totals[TIM_TOT_PUSH];
  const int32_t *hdr = pl.hdr + (int64_t)e * TIM_PLAN_HDR;
  if (hdr[TIM_HDR_BAD]) return;
  const int b = hdr[TIM_HDR_SEQ], n = hdr[TIM_HDR_N], m = hdr[TIM_HDR_N_KEPT];
  const int keep = hdr[TIM_HDR_KEEP_PAGES], push = hdr[TIM_HDR_PUSH], push_off = hdr[TIM_HDR_PUSH_OFF];
  const int T = cfg.max_pages_per_seq * cfg.page_size;
  if (cfg.page_size == 1) {
    if (i < cfg.max_pages_per_seq && i >= keep) {
      int32_t *slot = st.page_table + (int64_t)b * cfg.max_pages_per_seq + i;
      // a pruned token returns its page; its rank among the pruned tokens keeps the order ascending
      if (i < n && pl.new_pos[(int64_t)e * T + i] < 0)
        st.free_stack[pl.totals[TIM_TOT_TOP_AFTER_POP] + push_off + (i - pl.rank[(int64_t)e * (T + 1) + i])] = *slot;
      *slot = pl.new_table[(int64_t)e * cfg.max_pages_per_seq + i];
    }
  } else if (i < cfg.max_pages_per_seq) {
    int32_t *slot = st.page_table + (int64_t)b * cfg.max_pages_per_seq + i;
    if (i >= keep) {
      if (i < keep + push) st.free_stack[pl.totals[TIM_TOT_TOP_AFTER_POP] + push_off + (i - keep)] = *slot;
      *slot = pl.new_table[(int64_t)e * cfg.max_pages_per_seq + i];
    }
  }
  if (m != n) {  // boundaries only move when something was pruned
    const int nn = min(st.n_nodes[b], cfg.max_nodes);
    if (i < nn) {
      const int32_t *rank = pl.rank + (int64_t)e * (T + 1);
      const int64_t k = (int64_t)b * cfg.max_nodes + i;
      int x;
      x = st.node_tok_begin[k]; if (x >= 0) st.node_tok_begin[k] = rank[min(x, n)];
      x = st.node_sub_begin[k]; if (x >= 0) st.node_sub_begin[k] = rank[min(x, n)];
      x = st.node_sub_end[k];   if (x >= 0) st.node_sub_end[k] = rank[min(x, n)];
      x = st.node_tok_end[k];   if (x >= 0) st.node_tok_end[k] = rank[min(x, n)];
    }
  }
  if (i == 0) st.seq_len[b] = m;
}

// In-forward variant: same rule, but the evicted tokens are only made invisible.  One block
// per sequence: difference array -> coverage by a block scan -> one visibility flag per
// token in scratch -> packed 32 per word and AND-ed into the persistent mask.
__global__ void __launch_bounds__(PLAN_THREADS)
tim_prune_mask_kernel(tim_config cfg, tim_state st, tim_plan pl, const int32_t *__restrict__ seq_ids, int threshold) {
  __shared__ int smem[17];
  __shared__ int s_bad;
  const int e = blockIdx.x, tid = threadIdx.x;
  const int b = seq_ids[e];
  if (tid == 0) s_bad = 0;
  __syncthreads();
  if (b < 0 || b >= cfg.max_batch || (e > 0 && seq_ids[e - 1] >= b)) {
    if (tid == 0) tim_set_status(st.status, TIM_ERR_INVALID_ARG);
    return;
  }
  const int T = cfg.max_pages_per_seq * cfg.page_size;
  const int n = st.seq_len[b];
  int32_t *cover = pl.cover + (int64_t)e * (T + 1);
  int32_t *vis = pl.new_pos + (int64_t)e * T;
  for (int t = tid; t <= n; t += PLAN_THREADS) cover[t] = 0;
  __syncthreads();
  const int64_t row = (int64_t)b * cfg.max_nodes;
  const int nn = min(st.n_nodes[b], cfg.max_nodes);
  const int gone_below = st.lists_done[b] - threshold;
  for (int i = tid; i < nn; i += PLAN_THREADS) {
    const int lo = st.node_list_order[row + i];
    if (lo < 0 || lo >= gone_below) continue;
    const int sb = st.node_sub_begin[row + i], se = st.node_sub_end[row + i];
    if (sb < 0 || se < sb || se > n) {
      atomicOr(&s_bad, 1);
      continue;
    }
    if (se > sb) {
      atomicAdd(&cover[sb], 1);
      atomicAdd(&cover[se], -1);
    }
  }
  __threadfence_block();
  __syncthreads();
  if (s_bad) {
    if (tid == 0) tim_set_status(st.status, TIM_ERR_BAD_TREE);
    return;
  }
  int cov_base = 0;
  for (int t0 = 0; t0 < n; t0 += PLAN_THREADS * PLAN_ITEMS) {
    const int tb = t0 + tid * PLAN_ITEMS;
    int c[PLAN_ITEMS];
    int csum = 0;
#pragma unroll
    for (int k = 0; k < PLAN_ITEMS; ++k) {
      c[k] = (tb + k < n) ? cover[tb + k] : 0;
      csum += c[k];
    }
    int ctot;
    int cexcl = tim_block_incl_scan(csum, smem, &ctot) - csum + cov_base;
#pragma unroll
    for (int k = 0; k < PLAN_ITEMS; ++k) {
      cexcl += c[k];
      if (tb + k < n) vis[tb + k] = cexcl == 0 ? 1 : 0;
    }
    cov_base += ctot;
  }
  __threadfence_block();
  __syncthreads();
  const int words = (n + 31) / 32;
  uint32_t *mask = st.keep_mask + (int64_t)b * tim_mask_words(cfg);
  for (int w = tid; w < words; w += PLAN_THREADS) {
    uint32_t bits = 0;
    for (int k = 0; k < 32; ++k) {
      const int t = 32 * w + k;
      if (t >= n || vis[t]) bits |= 1u << k;  // tokens not decoded yet stay visible
    }
    mask[w] &= bits;
  }
}

static int plan_ok(const tim_ctx *ctx, const tim_plan *p) {
  return ctx && ctx->bound && p && tim_ints_ok(p->seq_ids) && tim_ints_ok(p->cover) && tim_ints_ok(p->rank) &&
         tim_ints_ok(p->kept_idx) && tim_ints_ok(p->new_pos) && tim_ints_ok(p->delta) && tim_ints_ok(p->src_slot) &&
         tim_ints_ok(p->dst_slot) && tim_ints_ok(p->new_table) && tim_ints_ok(p->hdr) && tim_ints_ok(p->totals);
}

extern "C" int tim_prune_plan(tim_ctx *ctx, const int32_t *seq_ids, int32_t n_seqs, int32_t threshold, tim_plan *plan,
                              tim_stream stream) {
  if (!plan_ok(ctx, plan) || !tim_ints_ok(seq_ids) || n_seqs <= 0 || n_seqs > plan->max_seqs || n_seqs > ctx->cfg.max_batch ||
      threshold < 0)
    return TIM_ERR_INVALID_ARG;
  plan->n_seqs = n_seqs;
  hipStream_t s = tim_hs(stream);
  hipLaunchKernelGGL(tim_plan_scan_kernel, dim3(n_seqs), dim3(PLAN_THREADS), 0, s, ctx->cfg, ctx->st, *plan, seq_ids,
                     threshold);
  TIM_LAUNCH_CHECK();
  hipLaunchKernelGGL(tim_plan_pages_kernel, dim3(1), dim3(n_seqs <= 64 ? 64 : 1024), 0, s, ctx->cfg, ctx->st, *plan,
                     n_seqs);
  TIM_LAUNCH_CHECK();
  const int T = ctx->cfg.max_pages_per_seq * ctx->cfg.page_size;
  hipLaunchKernelGGL(tim_plan_slots_kernel, dim3((T + 255) / 256, n_seqs), dim3(256), 0, s, ctx->cfg, ctx->st, *plan);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}

extern "C" int tim_plan_commit(tim_ctx *ctx, const tim_plan *plan, tim_stream stream) {
  if (!plan_ok(ctx, plan) || plan->n_seqs <= 0 || plan->n_seqs > plan->max_seqs) return TIM_ERR_INVALID_ARG;
  ctx->sched_valid = false;  // lengths change: an attention schedule no longer holds
  const int span = ctx->cfg.max_pages_per_seq > ctx->cfg.max_nodes ? ctx->cfg.max_pages_per_seq : ctx->cfg.max_nodes;
  hipLaunchKernelGGL(tim_plan_commit_kernel, dim3((span + 255) / 256, plan->n_seqs), dim3(256), 0, tim_hs(stream),
                     ctx->cfg, ctx->st, *plan);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}

extern "C" int tim_prune_mask(tim_ctx *ctx, const int32_t *seq_ids, int32_t n_seqs, int32_t threshold, tim_plan *plan,
                              tim_stream stream) {
  if (!ctx || !ctx->bound || !ctx->st.keep_mask || !plan || !tim_ints_ok(plan->cover) || !tim_ints_ok(plan->new_pos) ||
      !tim_ints_ok(seq_ids) || n_seqs <= 0 ||
      n_seqs > plan->max_seqs || n_seqs > ctx->cfg.max_batch || threshold < 0)
    return TIM_ERR_INVALID_ARG;
  hipLaunchKernelGGL(tim_prune_mask_kernel, dim3(n_seqs), dim3(PLAN_THREADS), 0, tim_hs(stream), ctx->cfg, ctx->st, *plan,
                     seq_ids, threshold);
  TIM_LAUNCH_CHECK();
  return TIM_OK;
}
