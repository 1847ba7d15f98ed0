/*
 * tim.h - C ABI of the working-memory decoding path for AMD MI355X (gfx950).
 *
 * The path is the GPU-side memory management of the paper's inference runtime
 * (Sec. 3.1): before a decode step, the subtask lists that left the pruning
 * buffer are evicted from the paged KV cache, their pages are recycled, the
 * surviving tokens receive contiguous positions again (Eq. 1, here in its
 * weight-free form: cached RoPE keys are re-rotated by their position change),
 * and paged grouped-query decode attention runs over the retained working
 * memory only.
 *
 * Conventions that hold for every call below
 *   - Returns TIM_OK (0) or a negative tim_error.  Errors the host can see
 *     (null pointers, shapes the kernels do not support, a HIP launch failure)
 *     are returned at once.  Errors only the device can see (page pool
 *     exhausted, a sequence outgrowing its page table, a malformed tree) are
 *     written to the sticky device word tim_state.status (first error wins) and
 *     turn the call into a no-op for the state it guards; read it with
 *     tim_status().
 *   - All pointers named "device" are device memory owned by the caller for the
 *     lifetime of the context.  The library allocates no device memory and
 *     keeps only the pointers it is given.  Pointers named "host" are ordinary
 *     host memory read during the call.
 *   - Every call is asynchronous on the given stream (a hipStream_t passed as
 *     void*; NULL is the default stream), except tim_status(), which waits.
 *     One context serves one stream at a time.
 *   - Shapes: head_dim = 128, q_heads = 4 * kv_heads, page_size = 16, or 1 (the paper's
 *     own setting, Sec. 3.1; see "Page size 1" below).  Other values are rejected with
 *     TIM_ERR_INVALID_ARG.  One pool layout (below); the rotary pairing is a field of tim_config.
 *   - bf16 is the upper half of an IEEE binary32, round-to-nearest-even.
 *   - Alignment: device pointers to K/V rows, queries and outputs (the pools, q, out, k_new,
 *     v_new, k_rows, v_rows, q_ext, out_ext, attn_ws) must be 16-byte aligned, int32 and
 *     uint32 arrays 4-byte aligned; a pointer that is not is refused with
 *     TIM_ERR_INVALID_ARG before anything is launched.
 *
 * Data layout
 *   K and V pools: bf16 [layers][num_pages][kv_heads][page_size][head_dim],
 *   so the 16 rows of one (page, kv head) are 4 KiB contiguous.  Keys are
 *   stored rotated (RoPE, pairs per tim_config.rope_pairing, theta_i = rope_base^(-2i/128)) at
 *   their current position.  A token with logical index t of sequence b lives
 *   in page page_table[b][t / 16], row t % 16.  "slot" = page * 16 + row.
 *   Where the two pools lie relative to each other is the caller's choice, and it is worth
 *   0.7 % (16-token pages) to 4.5 % (page size 1) of the attention kernel's bandwidth on MI355X:
 *   a wave requests the K and the V tile (row) of a page (token) together, and with equally
 *   aligned pools both fall on the same memory channels.  Start v_pool 4096 + 256 bytes
 *   (modulo 16 KiB) beyond k_pool's alignment; the Python binding's alloc_pools does.
 *
 * Page size 1
 *   Every token owns a page (pool [layers][num_pages][kv_heads][1][128]), so a flush moves no
 *   row: a survivor keeps its page, the page-table row is compacted as integers, the pruned
 *   tokens' pages return to the free stack in ascending logical order, and tim_kv_compact
 *   only re-rotates, in place, the keys behind the first pruned token.  tim_extend_attn and
 *   the vector-ALU attention variant do not support it.
 *
 * Order of one decode step
 *   tim_tree_mark (structure seen at this boundary)
 *   [flush:  tim_prune_plan -> tim_kv_compact -> tim_plan_commit]
 *   tim_seq_advance
 *   per layer:  tim_kv_append, tim_decode_attn
 */
#ifndef TIM_H
#define TIM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tim_ctx tim_ctx;
typedef void *tim_stream; /* hipStream_t */

typedef enum {
  TIM_OK = 0,
  TIM_ERR_INVALID_ARG = -1,
  TIM_ERR_BAD_TREE = -2,     /* mark or node span outside the sequence / tables */
  TIM_ERR_OOM_PAGES = -3,    /* free stack holds fewer pages than a batch needs */
  TIM_ERR_HIP = -4,          /* a HIP runtime call failed */
  TIM_ERR_SEQ_TOO_LONG = -5, /* a sequence needs more than max_pages_per_seq pages */
  TIM_ERR_TOO_LARGE = -6     /* the configuration exceeds what tim_decode_attn_noalloc's built-in scratch holds */
} tim_error;

/* Structural marks of the task tree (Sec. 2.1: thought, subtasks, conclusion). */
typedef enum {
  TIM_MARK_OPEN = 1,      /* the task's first token comes next */
  TIM_MARK_SUB_BEGIN = 2, /* its thought ended, its subtask list starts */
  TIM_MARK_SUB_END = 3,   /* the list is complete: it enters the pruning buffer */
  TIM_MARK_CLOSE = 4      /* its conclusion ended */
} tim_mark;

typedef enum { TIM_OUT_F32 = 0, TIM_OUT_BF16 = 1 } tim_out_dtype;

/* Which two coordinates of a key row turn together under the rotary embedding (the position
 * reassignment of Sec. 3.1 / Eq. 1 is done by turning each kept key by its position change).
 * Pair i turns by (change) * rope_base^(-2i/128) in both; only tim_kv_compact reads it. */
typedef enum {
  TIM_ROPE_HALF_SPLIT = 0,  /* pair i = (i, i + 64): the base model's family */
  TIM_ROPE_INTERLEAVED = 1  /* pair i = (2i, 2i + 1): the original rotary formulation */
} tim_rope_pairing;

typedef struct {
  int32_t layers;
  int32_t q_heads;
  int32_t kv_heads;
  int32_t head_dim;          /* 128 */
  int32_t page_size;         /* 16 */
  int32_t num_pages;         /* pages per layer in each pool */
  int32_t max_batch;         /* sequences; all of them decode every step */
  int32_t max_pages_per_seq; /* row length of page_table */
  int32_t max_nodes;         /* task-tree nodes per sequence */
  float rope_base;           /* 1e6 in the configurations */
  int32_t rope_pairing;      /* tim_rope_pairing; TIM_ROPE_HALF_SPLIT in the configurations */
} tim_config;

/* Caller-owned device buffers that make up one decoding context. */
typedef struct {
  void *k_pool;              /* device bf16, layout above */
  void *v_pool;              /* device bf16, layout above */
  int32_t *page_table;       /* device [max_batch][max_pages_per_seq], -1 = none */
  int32_t *seq_len;          /* device [max_batch], tokens in the working memory */
  int32_t *free_stack;       /* device [num_pages], free page ids, bottom first */
  int32_t *free_top;         /* device [1], number of free pages */
  int32_t *status;           /* device [1], sticky first device-side error */
  /* task tree per sequence, boundaries in current logical coordinates, -1 = unset */
  int32_t *node_tok_begin;   /* device [max_batch][max_nodes] */
  int32_t *node_sub_begin;   /* device [max_batch][max_nodes] */
  int32_t *node_sub_end;     /* device [max_batch][max_nodes] */
  int32_t *node_tok_end;     /* device [max_batch][max_nodes] */
  int32_t *node_list_order;  /* device [max_batch][max_nodes], completion ordinal of the list */
  int32_t *n_nodes;          /* device [max_batch], 1 + highest node id marked */
  int32_t *lists_done;       /* device [max_batch], lists completed so far */
  float *attn_ws;            /* device scratch for split partials, see tim_attn_ws_bytes */
  int64_t attn_ws_bytes;
  uint32_t *keep_mask;       /* device [max_batch][ceil(max_pages_per_seq * page_size / 32)], bit t%32 of word t/32 = token t is
                                visible; only the *_mask calls use it, may be NULL otherwise */
} tim_state;

/*
 * Caller-owned device scratch that carries one flush from tim_prune_plan to
 * tim_kv_compact and tim_plan_commit.  T = max_pages_per_seq * page_size.
 * Row e belongs to the e-th flushed sequence.  Contents are outputs of
 * tim_prune_plan; the caller may read them back (they are the plan).
 */
typedef struct {
  int32_t max_seqs;     /* capacity in sequences (host field) */
  int32_t n_seqs;       /* set by tim_prune_plan (host field) */
  int32_t *seq_ids;     /* device [max_seqs]   flushed sequence ids, ascending */
  int32_t *cover;       /* device [max_seqs][T+1] scratch: pruned-range difference array */
  int32_t *rank;        /* device [max_seqs][T+1] survivors before boundary t */
  int32_t *kept_idx;    /* device [max_seqs][T]   old index of new token j, j < n_kept */
  int32_t *new_pos;     /* device [max_seqs][T]   new index of old token t, -1 = pruned */
  int32_t *delta;       /* device [max_seqs][T]   j - kept_idx[j] (<= 0) */
  int32_t *src_slot;    /* device [max_seqs][T]   old slot of new token j, j in [keep_pages*16, n_kept) */
  int32_t *dst_slot;    /* device [max_seqs][T]   new slot of new token j, same range */
  int32_t *new_table;   /* device [max_seqs][max_pages_per_seq] page-table row after the flush */
  int32_t *hdr;         /* device [max_seqs][TIM_PLAN_HDR] per-sequence scalars, see below */
  int32_t *totals;      /* device [TIM_PLAN_TOTALS] */
} tim_plan;

enum {
  TIM_HDR_SEQ = 0,          /* sequence id */
  TIM_HDR_N = 1,            /* tokens before the flush */
  TIM_HDR_N_KEPT = 2,       /* m: tokens after */
  TIM_HDR_FIRST_PRUNED = 3, /* first pruned token (n if none) */
  TIM_HDR_KEEP_PAGES = 4,   /* leading pages that stay in place */
  TIM_HDR_NEED = 5,         /* fresh pages taken */
  TIM_HDR_PAGE_OFF = 6,     /* exclusive sum of NEED over earlier sequences */
  TIM_HDR_PUSH = 7,         /* old pages returned */
  TIM_HDR_PUSH_OFF = 8,     /* exclusive sum of PUSH over earlier sequences */
  TIM_HDR_BAD = 9,          /* 1 = tree rejected, sequence left untouched */
  TIM_HDR_EXT = 10,         /* survivors after the first pruned token: m - first_pruned (0 if nothing moved) */
  TIM_HDR_EXT_OFF = 11,     /* exclusive sum of EXT over earlier sequences */
  TIM_HDR_EXT_TILE_OFF = 12,/* exclusive sum of ceil(EXT / 32) over earlier sequences */
  TIM_PLAN_HDR = 16
};
enum {
  TIM_TOT_OK = 0,        /* 1 = plan valid; 0 = pool exhausted, flush is a no-op */
  TIM_TOT_NEED = 1,
  TIM_TOT_PUSH = 2,
  TIM_TOT_TOP_AFTER_POP = 3,
  TIM_TOT_TOP_BEFORE = 4,
  TIM_TOT_EXT = 5,       /* sum of EXT */
  TIM_TOT_EXT_TILES = 6, /* sum of ceil(EXT / 32) */
  TIM_PLAN_TOTALS = 8
};

/* Bytes of tim_state.attn_ws that tim_decode_attn needs for this configuration. */
int64_t tim_attn_ws_bytes(const tim_config *cfg);

/* Creates a context (host object only).  cfg is copied.  Shapes are checked. */
int tim_ctx_create(tim_ctx **out, const tim_config *cfg);
int tim_ctx_destroy(tim_ctx *ctx);

/* Attaches the caller's device buffers; all pointers must be non-null, except keep_mask (see there) and
 * attn_ws, which may be NULL (with attn_ws_bytes 0) for a caller that only attends through
 * tim_decode_attn_noalloc; the other attention calls then return TIM_ERR_INVALID_ARG. */
int tim_bind(tim_ctx *ctx, const tim_state *state);

/*
 * Launch-shape parameters of the decode-attention calls (the split-K decomposition of
 * Sec. 3.1's paged attention).  They change how the work is cut, never what is computed.
 * tim_ctx_create installs the defaults measured on MI355X; a caller (a test that wants a
 * small shape to reach every code path, an A/B measurement) reads them with
 * tim_ctx_get_tuning, changes fields and installs them with tim_ctx_set_tuning, which
 * rejects values outside the ranges given here with TIM_ERR_INVALID_ARG and lets any
 * schedule lapse.  Host objects only; nothing is read from the environment.
 */
typedef enum { TIM_ATTN_VALU = 0, TIM_ATTN_MFMA = 1 } tim_attn_impl;
typedef struct {
  int32_t attn_impl;         /* TIM_ATTN_MFMA (default): both contractions on the matrix cores;
                                TIM_ATTN_VALU: vector-ALU kernel with cross-lane reductions (16-token pages only) */
  int32_t chunks_per_block;  /* 1..64, default 6: 256-token chunks one block accumulates */
  int32_t fill;              /* 1..64, default 2: blocks shrink until the launch holds this many per CU */
  int32_t grade_big;         /* default 32: under a schedule, a sequence that starts with more than grade_big/16
                                rounds of work to go gets blocks of twice the size */
  int32_t grade_small;       /* default 8, 0 <= grade_small <= grade_big: one that starts within the last
                                grade_small/16 rounds gets blocks of half the size */
  int32_t round_items;       /* default 0: a round is what the chip's resident blocks take.  > 0: a round is
                                this many blocks, and tim_attn_schedule schedules even launches that fit the
                                chip at once or hold one sequence (small shapes then reach all block sizes) */
  int32_t block_waves;       /* default 0: waves per attention block chosen per launch (12 when the launch holds at
                                most one block per CU, 6 when at most two, else 4); 4, 6, 8 or 12 forces one */
  int32_t short_list_chunks; /* default 0: under a schedule, the one block size of a list too short to be graded is
                                chosen from the lengths; 1..128 fixes it (clamped to chunks_per_block / 2 .. x 2) */
} tim_tuning;
int tim_ctx_get_tuning(const tim_ctx *ctx, tim_tuning *out);
int tim_ctx_set_tuning(tim_ctx *ctx, const tim_tuning *tuning);

/*
 * Empties the context: free_stack[i] = num_pages-1-i (so the first pops hand out
 * pages 0, 1, 2, ...), free_top = num_pages, all sequences empty, page tables and
 * trees unset, status cleared.  The paper recycles pages of pruned tokens
 * (Sec. 1, Sec. 3.1) without fixing an order; the LIFO order here is this
 * library's, chosen so page tables are reproducible.
 */
int tim_pool_reset(tim_ctx *ctx, tim_stream stream);

/*
 * Structure tracking (Sec. 2.1, Sec. 3.1: the runtime follows the structure of
 * the reasoning while it is generated).  ops: device int32 [n_ops][4] =
 * (sequence, tim_mark, node id, boundary).  boundary = -1 stands for the
 * sequence's current length (the mark sits right before the pending token);
 * an explicit boundary serves bulk loading.  Ops of one sequence are applied in
 * array order.  TIM_MARK_SUB_END also stamps the node's list with the next
 * completion ordinal of its sequence.  Bad ids set TIM_ERR_BAD_TREE and are skipped.
 */
int tim_tree_mark(tim_ctx *ctx, const int32_t *ops, int32_t n_ops, tim_stream stream);

/*
 * Reserves the slot of each sequence's pending token (Sec. 3.1: while the cache is
 * pruned the newest token x_k is still waiting to be encoded; its state h_k then
 * joins the working memory as the last element, and the pages freed by pruning are
 * the ones reused for it): a sequence whose length is
 * a multiple of the page size pops one page (sequences served in ascending id), then every
 * length grows by one.  If the pool cannot serve the whole batch, or a page
 * table is full, nothing changes and status is set.
 */
int tim_seq_advance(tim_ctx *ctx, tim_stream stream);

/*
 * Bulk form of tim_seq_advance for tool responses, which the runtime encodes as a batch of
 * new tokens that extend the cache (Sec. 2.1 "tooluse", Sec. 3.2): sequence b grows by
 * counts[b] >= 0 tokens.  New pages are popped in ascending (sequence, logical page) order;
 * if the pool or a page table cannot take the whole batch nothing changes and status is set.
 * counts: device int32 [max_batch].
 */
int tim_seq_extend(tim_ctx *ctx, const int32_t *counts, tim_stream stream);

/*
 * Writes the keys and values of the last counts[b] tokens of every sequence for one layer
 * (positions seq_len[b]-counts[b] .. seq_len[b]-1, i.e. right after tim_seq_extend).
 * k_rows, v_rows: device bf16 [n_rows][kv_heads][128], sequences in ascending order, keys
 * rotated at their positions.  row_off: device int32 [max_batch + 1], exclusive prefix sum of
 * counts (row_off[max_batch] = n_rows); n_rows is the host's copy of that total.
 */
int tim_kv_write(tim_ctx *ctx, int32_t layer, const int32_t *row_off, int32_t n_rows, const void *k_rows,
                 const void *v_rows, tim_stream stream);

/*
 * Writes the pending token's key and value of one layer into slot seq_len-1 of
 * every sequence (Sec. 3.1, Eq. 1: h_k, the encoding of the pending token x_k, is
 * appended behind the retained and repositioned states).  k_new, v_new: device bf16 [max_batch][kv_heads][128]; the key
 * is already rotated at position seq_len-1.
 */
int tim_kv_append(tim_ctx *ctx, int32_t layer, const void *k_new, const void *v_new, tim_stream stream);

/*
 * The pruning rule and the plan that follows from it (Sec. 2.1 "Subtask
 * pruning", Sec. 3.1).  For each listed sequence every subtask list that has
 * left the pruning buffer - all completed lists but the `threshold` most recent
 * ones, i.e. the first-in-first-out buffer of the paper - loses the tokens
 * between its task's thought and conclusion.  Survivors keep their order and
 * get positions 0..m-1.  Pages that lie wholly before the first pruned token
 * stay; the rest of the survivors is planned into fresh pages popped here
 * (ascending sequence, ascending page); if only a tail is pruned nothing moves.
 * seq_ids: device int32 [n_seqs], strictly ascending.  If the pool cannot supply
 * all fresh pages the plan is marked invalid, status is set and the three flush
 * calls change nothing.
 */
int tim_prune_plan(tim_ctx *ctx, const int32_t *seq_ids, int32_t n_seqs, int32_t threshold, tim_plan *plan,
                   tim_stream stream);

/*
 * Moves the planned survivors of layers [layer_begin, layer_end): values are
 * copied bit for bit; a key with position change d != 0 is rotated by d (the
 * RoPE composition R(p+d) = R(d) R(p) applied to the stored key: the positional
 * part of Eq. 1), in fp32 with angles reduced in fp64, and rounded to bf16; a key
 * with d = 0 is copied bit for bit.  Source and destination pages are disjoint.
 */
int tim_kv_compact(tim_ctx *ctx, const tim_plan *plan, int32_t layer_begin, int32_t layer_end, tim_stream stream);

/*
 * Completes the flush (Sec. 1 and Sec. 3.1: the memory pages of pruned tokens are
 * recycled for later decoding, and positions are reused): returns the replaced pages
 * to the free stack (ascending sequence, ascending logical page), installs the new
 * page-table rows and lengths, and moves every node boundary b of the flushed
 * sequences to rank[b], so that the task tree stays in current coordinates.
 */
int tim_plan_commit(tim_ctx *ctx, const tim_plan *plan, tim_stream stream);

/*
 * Paged grouped-query decode attention of one layer over each sequence's whole
 * working memory (Sec. 3.1: paged attention over the pruned cache): for query
 * head h and its KV head h/4, out = softmax(sm_scale * q K^T) V over tokens
 * 0..seq_len-1, bf16 inputs, fp32 accumulation.  q: device bf16
 * [max_batch][q_heads][128], rotated at position seq_len-1.  out: device
 * [max_batch][q_heads][128] in out_dtype.  max_seq_len: an upper bound on the
 * batch's lengths used only to size the launch (0 = assume full tables); longer
 * sequences are still handled in full.  Uses tim_state.attn_ws: a long sequence
 * is split over several blocks whose partial results pass through it, in fp32
 * when out_dtype is fp32 and as bf16 (normalised, with fp32 maximum and sum)
 * when it is bf16.
 */
int tim_decode_attn(tim_ctx *ctx, int32_t layer, const void *q, void *out, float sm_scale, int32_t out_dtype,
                    int32_t max_seq_len, tim_stream stream);

/*
 * Optional, once per decode step after the lengths are final (after tim_seq_advance and any
 * flush): lists, in tim_state.attn_ws, the blocks the step's attention launches need - only
 * the slots each sequence really uses, longest sequence first, in larger blocks while much
 * work is still to come and smaller ones at the end - so that all decode-attention calls up
 * to the next change of a length launch exactly that work in that order.  The
 * split-K decomposition of Sec. 3.1's paged attention is otherwise sized for the longest
 * sequence, and a batch of very unequal lengths (working memories before and after their
 * flush) spends a good part of a launch on blocks that find nothing to do.  max_seq_len as
 * in tim_decode_attn; the calls that follow use this call's bound and ignore their own.
 * When the bound's whole grid fits the chip at once, or the batch is one sequence, there is
 * nothing to reorder: the call then does nothing and the calls that follow run unscheduled;
 * so do batches of more than 4096 sequences (what the call's kernel holds in LDS).
 * The schedule lapses at the next tim_seq_advance, tim_seq_extend, tim_plan_commit,
 * tim_pool_reset or tim_bind.  A caller that changes tim_state.seq_len by other means must
 * call this again: a stale schedule is detected per block and reported as
 * TIM_ERR_INVALID_ARG in the status word (outputs are then undefined, accesses stay in
 * bounds).  Results are those of the unscheduled calls up to summation order.
 */
int tim_attn_schedule(tim_ctx *ctx, int32_t max_seq_len, tim_stream stream);

/*
 * tim_kv_append and tim_decode_attn of one layer in a single launch: the wave that reads a
 * sequence's last page takes the pending token's row from k_new / v_new (same layout as in
 * tim_kv_append), uses it, and stores it into the pool.  Results are those of the two calls.
 */
int tim_decode_attn_append(tim_ctx *ctx, int32_t layer, const void *q, const void *k_new, const void *v_new, void *out,
                           float sm_scale, int32_t out_dtype, int32_t max_seq_len, tim_stream stream);

/*
 * Attention half of the paper's own repositioning (Eq. 1, f_extend): after a flush is
 * committed, every survivor behind the first pruned token of a flushed sequence is
 * "extended", i.e. attends causally to the untouched prefix, the earlier extended tokens
 * and itself.  For flushed sequence e (row e of the plan) and j in [first_pruned, m):
 *   out[off_e + j - first_pruned][h] = softmax(sm_scale * q[..][h] . K[0..j]^T) V[0..j]
 * over the sequence's current cache, with off_e = TIM_HDR_EXT_OFF of row e.  q_ext: device
 * bf16 [TIM_TOT_EXT][q_heads][128], rotated at the new positions; out_ext: device, same
 * shape, out_dtype.  n_ext_total is the number of rows q_ext and out_ext hold; it must be at
 * least the plan's TIM_TOT_EXT (the caller reads that back to build the queries).  Rows
 * beyond TIM_TOT_EXT are left untouched; a smaller value writes nothing at all and sets
 * TIM_ERR_INVALID_ARG in the status word.  Weight-free: it does not recompute K/V, it is the attention the re-encoding
 * would run, so its cost can be set against tim_kv_compact's re-rotation.
 */
int tim_extend_attn(tim_ctx *ctx, int32_t layer, const tim_plan *plan, const void *q_ext, void *out_ext,
                    int32_t n_ext_total, float sm_scale, int32_t out_dtype, tim_stream stream);

/*
 * tim_decode_attn for callers that cannot allocate a workspace or may not call an allocating routine at
 * all: code being captured into a HIP graph, tight serving loops, harnesses that forbid allocation.
 * Same arguments, same result (up to summation order) as tim_decode_attn, but the partial results of split
 * sequences pass through a device array of TIM_NOALLOC_SCRATCH_BYTES that is part of the library's own
 * image (each GPU the library runs on holds one copy until the process ends) instead of
 * tim_state.attn_ws, which is not touched and may be NULL.  The call allocates and frees nothing, and
 * launches kernels only.  It never uses a schedule (tim_attn_schedule lives in attn_ws).
 * Limit: one slot's partials, max_batch * q_heads * 520 bytes, must fit the array, else
 * TIM_ERR_TOO_LARGE is returned and nothing is launched (32,263 (sequence, head) pairs: a batch of
 * 1,008 at 32 query heads).  Within the limit the launch uses as many slots per sequence as fit
 * (15 at batch 64 with 32 heads); longer sequences get larger blocks, never a wrong result.
 * All calls on one GPU share that GPU's array: calls that may overlap on one GPU (two streams, two
 * contexts, two threads) race on it and must be serialised by the caller.  Nothing in it needs
 * clearing between calls: every record a call reads, it has written first.
 */
#define TIM_NOALLOC_SCRATCH_BYTES (16 << 20)
int tim_decode_attn_noalloc(tim_ctx *ctx, int32_t layer, const void *q, void *out, float sm_scale, int32_t out_dtype,
                            int32_t max_seq_len, tim_stream stream);

/*
 * In-forward variant (Sec. 3.1 mentions it and rejects it as slower; Sec. 4.3 plots it as a
 * reference level below the baseline):
 * instead of moving anything, the tokens of the evicted lists are made invisible in
 * tim_state.keep_mask and tim_decode_attn_masked skips them inside attention: pages with no
 * visible token are not read, others are read in full and masked.  Positions, lengths,
 * page tables and node coordinates do not change, so positional slots are NOT reused: this
 * is the trade-off the paper's runtime avoids, kept here to measure it.  A context uses
 * either the flush calls or the mask calls, not both.  tim_pool_reset makes every token
 * visible.  The rule and the arguments are those of tim_prune_plan; `plan` only lends its
 * cover/new_pos scratch.
 */
int tim_prune_mask(tim_ctx *ctx, const int32_t *seq_ids, int32_t n_seqs, int32_t threshold, tim_plan *plan,
                   tim_stream stream);
int tim_decode_attn_masked(tim_ctx *ctx, int32_t layer, const void *q, void *out, float sm_scale, int32_t out_dtype,
                           int32_t max_seq_len, tim_stream stream);

/*
 * Page accounting (Sec. 1: pages of pruned tokens are recycled, none may leak).
 * out: device int32 [4] = (free pages; page-table entries that hold a page id, counted from
 * the tables themselves; pages the lengths call for, sum of ceil(seq_len / page_size);
 * 1 if some page id occurs twice among the free stack and the tables or lies outside the
 * pool, else 0).  A healthy context has out[0] + out[1] == num_pages, out[1] == out[2],
 * out[3] == 0.  The duplicate check runs only when scratch (device int32 [num_pages], any
 * contents) is given; with scratch == NULL out[3] is -1.
 */
int tim_pool_stats(tim_ctx *ctx, int32_t *out, int32_t *scratch, tim_stream stream);

/*
 * Benchmark aid: between tim_timing_begin and tim_timing_end the main kernel of every
 * tim_decode_attn call carries a pair of HIP events on its own dispatch (up to
 * max_launches calls; later calls run untimed).  tim_timing_end waits for them, writes
 * each launch's duration in milliseconds to ms_out (host, at least max_launches floats)
 * and the count to n_out (host), and releases the events.  Host objects only.
 */
int tim_timing_begin(tim_ctx *ctx, int32_t max_launches);
int tim_timing_end(tim_ctx *ctx, float *ms_out, int32_t *n_out);

/* Waits for the stream, returns the sticky device status and clears it. */
int tim_status(tim_ctx *ctx, tim_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* TIM_H */
