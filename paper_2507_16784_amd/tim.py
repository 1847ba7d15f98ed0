"""ctypes binding of libtim.so (the C ABI declared in include/tim.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory and the current stream.  Loading
fails loudly if the library has not been built; there is no fallback.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtim.so")

OK, ERR_INVALID_ARG, ERR_BAD_TREE, ERR_OOM_PAGES, ERR_HIP, ERR_SEQ_TOO_LONG, ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5, -6
NOALLOC_SCRATCH_BYTES = 16 << 20
MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, MARK_CLOSE = 1, 2, 3, 4
OUT_F32, OUT_BF16 = 0, 1
ATTN_VALU, ATTN_MFMA = 0, 1
PLAN_HDR, PLAN_TOTALS = 16, 8
(HDR_SEQ, HDR_N, HDR_N_KEPT, HDR_FIRST_PRUNED, HDR_KEEP_PAGES, HDR_NEED, HDR_PAGE_OFF, HDR_PUSH, HDR_PUSH_OFF,
 HDR_BAD, HDR_EXT, HDR_EXT_OFF, HDR_EXT_TILE_OFF) = range(13)
TOT_OK, TOT_NEED, TOT_PUSH, TOT_TOP_AFTER_POP, TOT_TOP_BEFORE, TOT_EXT, TOT_EXT_TILES = range(7)

EXPORTS = ["tim_attn_ws_bytes", "tim_ctx_create", "tim_ctx_destroy", "tim_bind", "tim_pool_reset", "tim_tree_mark",
           "tim_seq_advance", "tim_seq_extend", "tim_kv_write", "tim_kv_append", "tim_prune_plan", "tim_kv_compact", "tim_plan_commit",
           "tim_attn_schedule", "tim_decode_attn", "tim_decode_attn_append", "tim_decode_attn_masked", "tim_prune_mask", "tim_extend_attn", "tim_pool_stats", "tim_status", "tim_timing_begin", "tim_timing_end",
           "tim_ctx_get_tuning", "tim_ctx_set_tuning", "tim_decode_attn_noalloc"]


class tim_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("layers", "q_heads", "kv_heads", "head_dim", "page_size", "num_pages",
                                         "max_batch", "max_pages_per_seq", "max_nodes")] + [("rope_base", C.c_float),
                                                                                            ("rope_pairing", C.c_int32)]


class tim_state(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("k_pool", "v_pool", "page_table", "seq_len", "free_stack", "free_top",
                                          "status", "node_tok_begin", "node_sub_begin", "node_sub_end",
                                          "node_tok_end", "node_list_order", "n_nodes", "lists_done", "attn_ws")] + \
               [("attn_ws_bytes", C.c_int64), ("keep_mask", C.c_void_p)]


class tim_tuning(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("attn_impl", "chunks_per_block", "fill", "grade_big", "grade_small",
                                         "round_items", "block_waves", "short_list_chunks")]


_PLAN_PTRS = ("seq_ids", "cover", "rank", "kept_idx", "new_pos", "delta", "src_slot", "dst_slot", "new_table",
              "hdr", "totals")


class tim_plan(C.Structure):
    _fields_ = [("max_seqs", C.c_int32), ("n_seqs", C.c_int32)] + [(n, C.c_void_p) for n in _PLAN_PTRS]


def load_library(path: str = LIB_PATH) -> C.CDLL:
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it first (python -m paper_2507_16784_amd.build); "
                           "this package has no CPU fallback")
    lib = C.CDLL(path)
    p, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    sig = {
        "tim_attn_ws_bytes": (i64, [C.POINTER(tim_config)]),
        "tim_ctx_create": (C.c_int, [C.POINTER(p), C.POINTER(tim_config)]),
        "tim_ctx_destroy": (C.c_int, [p]),
        "tim_bind": (C.c_int, [p, C.POINTER(tim_state)]),
        "tim_pool_reset": (C.c_int, [p, p]),
        "tim_tree_mark": (C.c_int, [p, p, i32, p]),
        "tim_seq_advance": (C.c_int, [p, p]),
        "tim_seq_extend": (C.c_int, [p, p, p]),
        "tim_kv_write": (C.c_int, [p, i32, p, i32, p, p, p]),
        "tim_kv_append": (C.c_int, [p, i32, p, p, p]),
        "tim_prune_plan": (C.c_int, [p, p, i32, i32, C.POINTER(tim_plan), p]),
        "tim_kv_compact": (C.c_int, [p, C.POINTER(tim_plan), i32, i32, p]),
        "tim_plan_commit": (C.c_int, [p, C.POINTER(tim_plan), p]),
        "tim_attn_schedule": (C.c_int, [p, i32, p]),
        "tim_decode_attn": (C.c_int, [p, i32, p, p, f32, i32, i32, p]),
        "tim_decode_attn_noalloc": (C.c_int, [p, i32, p, p, f32, i32, i32, p]),
        "tim_decode_attn_append": (C.c_int, [p, i32, p, p, p, p, f32, i32, i32, p]),
        "tim_decode_attn_masked": (C.c_int, [p, i32, p, p, f32, i32, i32, p]),
        "tim_prune_mask": (C.c_int, [p, p, i32, i32, C.POINTER(tim_plan), p]),
        "tim_extend_attn": (C.c_int, [p, i32, C.POINTER(tim_plan), p, p, i32, f32, i32, p]),
        "tim_pool_stats": (C.c_int, [p, p, p, p]),
        "tim_ctx_get_tuning": (C.c_int, [p, C.POINTER(tim_tuning)]),
        "tim_ctx_set_tuning": (C.c_int, [p, C.POINTER(tim_tuning)]),
        "tim_status": (C.c_int, [p, p]),
        "tim_timing_begin": (C.c_int, [p, i32]),
        "tim_timing_end": (C.c_int, [p, C.POINTER(f32), C.POINTER(i32)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = load_library()
    return _lib


class TimError(RuntimeError):
    def __init__(self, code, where):
        super().__init__(f"{where} failed with tim_error {code}")
        self.code = code


def _check(code, where):
    if code != OK:
        raise TimError(code, where)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: torch.Tensor):
    return C.c_void_p(t.data_ptr())


class Plan:
    """Device scratch of one flush (tim_plan), allocated with torch."""

    def __init__(self, cfg: tim_config, max_seqs: int, device="cuda"):
        T = cfg.max_pages_per_seq * cfg.page_size
        i32 = dict(dtype=torch.int32, device=device)
        self.max_seqs = max_seqs
        self.T = T
        self.seq_ids = torch.zeros(max_seqs, **i32)
        self.cover = torch.zeros(max_seqs, T + 1, **i32)
        self.rank = torch.zeros(max_seqs, T + 1, **i32)
        self.kept_idx = torch.zeros(max_seqs, T, **i32)
        self.new_pos = torch.zeros(max_seqs, T, **i32)
        self.delta = torch.zeros(max_seqs, T, **i32)
        self.src_slot = torch.zeros(max_seqs, T, **i32)
        self.dst_slot = torch.zeros(max_seqs, T, **i32)
        self.new_table = torch.zeros(max_seqs, cfg.max_pages_per_seq, **i32)
        self.hdr = torch.zeros(max_seqs, PLAN_HDR, **i32)
        self.totals = torch.zeros(PLAN_TOTALS, **i32)
        self.c = tim_plan(max_seqs=max_seqs, n_seqs=0, **{n: getattr(self, n).data_ptr() for n in _PLAN_PTRS})


POOL_STAGGER_BYTES = 4096 + 256   # where the V pool starts relative to the K pool ...
POOL_STAGGER_PERIOD = 16384       # ... modulo this many bytes


def alloc_pools(shape, device="cuda", zero=False, stagger=True):
    """K and V pools of one context (bf16, `shape` = [layers, num_pages, kv_heads, page_size, 128]).

    The library takes any 16-byte-aligned pair.  This allocator starts the V pool one tile and one row (4096 +
    256 bytes, modulo 16 KiB) beyond the K pool: the K and V tile of a page - with page size 1 the K and V row of
    a token - which a wave of the attention kernel requests together, then fall on different memory channels
    (channels interleave every 256 bytes).  Measured on MI355X, attention over 16-32K-token working memories,
    same box: 16-token pages 6.64 TB/s against 6.59 with equal alignment (4, 8 or 12 KiB do the same, 2 KiB and
    16 KiB do not); page size 1 6.52 TB/s against 6.23 (256 bytes alone: 6.51, 512: 6.39, 1 KiB and more: 6.23)."""
    make = torch.zeros if zero else torch.empty
    n = 1
    for d in shape:
        n *= int(d)
    k = make(tuple(shape), dtype=torch.bfloat16, device=device)
    if not stagger:
        return k, make(tuple(shape), dtype=torch.bfloat16, device=device)
    buf = make(n + POOL_STAGGER_PERIOD // 2, dtype=torch.bfloat16, device=device)
    off = (k.data_ptr() + POOL_STAGGER_BYTES - buf.data_ptr()) % POOL_STAGGER_PERIOD
    assert off % 16 == 0
    return k, buf[off // 2: off // 2 + n].view(tuple(shape))


class Context:
    """One decoding context: owns the torch device buffers of tim_state and the tim_ctx handle."""

    def __init__(self, layers, q_heads, kv_heads, num_pages, max_batch, max_pages_per_seq, max_nodes,
                 head_dim=128, page_size=16, rope_base=1.0e6, device="cuda", pools=None, workspace=True,
                 rope_pairing=0):
        self.cfg = tim_config(layers, q_heads, kv_heads, head_dim, page_size, num_pages, max_batch,
                              max_pages_per_seq, max_nodes, rope_base, rope_pairing)
        self.handle = C.c_void_p()
        _check(lib().tim_ctx_create(C.byref(self.handle), C.byref(self.cfg)), "tim_ctx_create")
        i32 = dict(dtype=torch.int32, device=device)
        pool_shape = (layers, num_pages, kv_heads, page_size, head_dim)
        if pools is None:
            self.k_pool, self.v_pool = alloc_pools(pool_shape, device, zero=True)
        else:
            self.k_pool, self.v_pool = pools
            assert tuple(self.k_pool.shape) == pool_shape and tuple(self.v_pool.shape) == pool_shape
        self.page_table = torch.full((max_batch, max_pages_per_seq), -1, **i32)
        self.seq_len = torch.zeros(max_batch, **i32)
        self.free_stack = torch.zeros(num_pages, **i32)
        self.free_top = torch.zeros(1, **i32)
        self.status = torch.zeros(1, **i32)
        self.node_tok_begin = torch.full((max_batch, max_nodes), -1, **i32)
        self.node_sub_begin = torch.full((max_batch, max_nodes), -1, **i32)
        self.node_sub_end = torch.full((max_batch, max_nodes), -1, **i32)
        self.node_tok_end = torch.full((max_batch, max_nodes), -1, **i32)
        self.node_list_order = torch.full((max_batch, max_nodes), -1, **i32)
        self.n_nodes = torch.zeros(max_batch, **i32)
        self.lists_done = torch.zeros(max_batch, **i32)
        self.keep_mask = torch.full((max_batch, (max_pages_per_seq * page_size + 31) // 32), -1, **i32)  # all bits set
        ws_bytes = lib().tim_attn_ws_bytes(C.byref(self.cfg)) if workspace else 0
        self.attn_ws = torch.zeros(ws_bytes // 4, dtype=torch.float32, device=device) if workspace else None
        self.state = tim_state(
            **{n: getattr(self, n).data_ptr() for n in ("k_pool", "v_pool", "page_table", "seq_len", "free_stack",
                                                        "free_top", "status", "node_tok_begin", "node_sub_begin",
                                                        "node_sub_end", "node_tok_end", "node_list_order", "n_nodes",
                                                        "lists_done")},
            attn_ws=self.attn_ws.data_ptr() if workspace else None,
            attn_ws_bytes=ws_bytes, keep_mask=self.keep_mask.data_ptr())
        _check(lib().tim_bind(self.handle, C.byref(self.state)), "tim_bind")
        self.tim_pool_reset()

    def close(self):
        if self.handle:
            lib().tim_ctx_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the C ABI, same names ------------------------------------------------------
    def tim_pool_reset(self):
        _check(lib().tim_pool_reset(self.handle, _stream()), "tim_pool_reset")

    def tim_tree_mark(self, ops: torch.Tensor):
        """ops: int32 device tensor [n_ops, 4]."""
        assert ops.dtype == torch.int32 and ops.is_cuda and ops.is_contiguous()
        _check(lib().tim_tree_mark(self.handle, _ptr(ops), ops.shape[0], _stream()), "tim_tree_mark")

    def tim_seq_advance(self):
        _check(lib().tim_seq_advance(self.handle, _stream()), "tim_seq_advance")

    def tim_seq_extend(self, counts: torch.Tensor):
        assert counts.dtype == torch.int32 and counts.is_cuda and counts.is_contiguous()
        assert counts.shape[0] == self.cfg.max_batch
        _check(lib().tim_seq_extend(self.handle, _ptr(counts), _stream()), "tim_seq_extend")

    def tim_kv_write(self, layer: int, row_off: torch.Tensor, k_rows: torch.Tensor, v_rows: torch.Tensor):
        assert row_off.dtype == torch.int32 and row_off.is_cuda and row_off.shape[0] == self.cfg.max_batch + 1
        assert k_rows.dtype == torch.bfloat16 and v_rows.dtype == torch.bfloat16 and k_rows.is_cuda and v_rows.is_cuda
        assert k_rows.is_contiguous() and v_rows.is_contiguous() and k_rows.shape == v_rows.shape
        assert tuple(k_rows.shape[1:]) == (self.cfg.kv_heads, self.cfg.head_dim)
        _check(lib().tim_kv_write(self.handle, layer, _ptr(row_off), k_rows.shape[0], _ptr(k_rows), _ptr(v_rows),
                                  _stream()), "tim_kv_write")

    def tim_kv_append(self, layer: int, k_new: torch.Tensor, v_new: torch.Tensor):
        assert k_new.dtype == torch.bfloat16 and v_new.dtype == torch.bfloat16
        assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.is_cuda and v_new.is_cuda
        assert tuple(k_new.shape) == (self.cfg.max_batch, self.cfg.kv_heads, self.cfg.head_dim) == tuple(v_new.shape)
        _check(lib().tim_kv_append(self.handle, layer, _ptr(k_new), _ptr(v_new), _stream()), "tim_kv_append")

    def tim_prune_plan(self, seq_ids: torch.Tensor, threshold: int, plan: Plan):
        assert seq_ids.dtype == torch.int32 and seq_ids.is_cuda and seq_ids.is_contiguous()
        _check(lib().tim_prune_plan(self.handle, _ptr(seq_ids), seq_ids.shape[0], threshold, C.byref(plan.c),
                                    _stream()), "tim_prune_plan")

    def tim_kv_compact(self, plan: Plan, layer_begin: int, layer_end: int):
        _check(lib().tim_kv_compact(self.handle, C.byref(plan.c), layer_begin, layer_end, _stream()),
               "tim_kv_compact")

    def tim_plan_commit(self, plan: Plan):
        _check(lib().tim_plan_commit(self.handle, C.byref(plan.c), _stream()), "tim_plan_commit")

    def tim_attn_schedule(self, max_seq_len: int = 0):
        _check(lib().tim_attn_schedule(self.handle, max_seq_len, _stream()), "tim_attn_schedule")

    def tim_decode_attn(self, layer: int, q: torch.Tensor, out: torch.Tensor, sm_scale: float, max_seq_len: int = 0):
        assert q.dtype == torch.bfloat16 and q.is_cuda and q.is_contiguous()
        assert tuple(q.shape) == (self.cfg.max_batch, self.cfg.q_heads, self.cfg.head_dim) == tuple(out.shape)
        assert out.is_cuda and out.is_contiguous() and out.dtype in (torch.float32, torch.bfloat16)
        od = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
        _check(lib().tim_decode_attn(self.handle, layer, _ptr(q), _ptr(out), sm_scale, od, max_seq_len, _stream()),
               "tim_decode_attn")

    def tim_decode_attn_noalloc(self, layer: int, q: torch.Tensor, out: torch.Tensor, sm_scale: float, max_seq_len: int = 0):
        assert q.dtype == torch.bfloat16 and q.is_cuda and q.is_contiguous()
        assert tuple(q.shape) == (self.cfg.max_batch, self.cfg.q_heads, self.cfg.head_dim) == tuple(out.shape)
        assert out.is_cuda and out.is_contiguous() and out.dtype in (torch.float32, torch.bfloat16)
        od = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
        _check(lib().tim_decode_attn_noalloc(self.handle, layer, _ptr(q), _ptr(out), sm_scale, od, max_seq_len,
                                             _stream()), "tim_decode_attn_noalloc")

    def tim_decode_attn_append(self, layer: int, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                               out: torch.Tensor, sm_scale: float, max_seq_len: int = 0):
        assert q.dtype == torch.bfloat16 and q.is_cuda and q.is_contiguous()
        assert tuple(q.shape) == (self.cfg.max_batch, self.cfg.q_heads, self.cfg.head_dim) == tuple(out.shape)
        assert out.is_cuda and out.is_contiguous() and out.dtype in (torch.float32, torch.bfloat16)
        for t in (k_new, v_new):
            assert t.dtype == torch.bfloat16 and t.is_cuda and t.is_contiguous()
            assert tuple(t.shape) == (self.cfg.max_batch, self.cfg.kv_heads, self.cfg.head_dim)
        od = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
        _check(lib().tim_decode_attn_append(self.handle, layer, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), sm_scale,
                                            od, max_seq_len, _stream()), "tim_decode_attn_append")

    def tim_prune_mask(self, seq_ids: torch.Tensor, threshold: int, plan: Plan):
        assert seq_ids.dtype == torch.int32 and seq_ids.is_cuda and seq_ids.is_contiguous()
        _check(lib().tim_prune_mask(self.handle, _ptr(seq_ids), seq_ids.shape[0], threshold, C.byref(plan.c),
                                    _stream()), "tim_prune_mask")

    def tim_decode_attn_masked(self, layer: int, q: torch.Tensor, out: torch.Tensor, sm_scale: float,
                               max_seq_len: int = 0):
        assert q.dtype == torch.bfloat16 and q.is_cuda and q.is_contiguous()
        assert tuple(q.shape) == (self.cfg.max_batch, self.cfg.q_heads, self.cfg.head_dim) == tuple(out.shape)
        assert out.is_cuda and out.is_contiguous() and out.dtype in (torch.float32, torch.bfloat16)
        od = OUT_F32 if out.dtype == torch.float32 else OUT_BF16
        _check(lib().tim_decode_attn_masked(self.handle, layer, _ptr(q), _ptr(out), sm_scale, od, max_seq_len,
                                            _stream()), "tim_decode_attn_masked")

    def tim_extend_attn(self, layer: int, plan: Plan, q_ext: torch.Tensor, out_ext: torch.Tensor, sm_scale: float):
        assert q_ext.dtype == torch.bfloat16 and q_ext.is_cuda and q_ext.is_contiguous()
        assert q_ext.dim() == 3 and tuple(q_ext.shape[1:]) == (self.cfg.q_heads, self.cfg.head_dim)
        assert tuple(out_ext.shape) == tuple(q_ext.shape) and out_ext.is_cuda and out_ext.is_contiguous()
        assert out_ext.dtype in (torch.float32, torch.bfloat16)
        od = OUT_F32 if out_ext.dtype == torch.float32 else OUT_BF16
        _check(lib().tim_extend_attn(self.handle, layer, C.byref(plan.c), _ptr(q_ext), _ptr(out_ext),
                                     q_ext.shape[0], sm_scale, od, _stream()), "tim_extend_attn")

    def tim_pool_stats(self, check_duplicates: bool = True) -> torch.Tensor:
        """int32 [4]: free pages, page-table entries in use, pages the lengths call for, duplicate flag."""
        out = torch.empty(4, dtype=torch.int32, device=self.seq_len.device)
        scratch = torch.empty(self.cfg.num_pages, dtype=torch.int32, device=self.seq_len.device) if check_duplicates else None
        _check(lib().tim_pool_stats(self.handle, _ptr(out), _ptr(scratch) if check_duplicates else None, _stream()),
               "tim_pool_stats")
        return out

    def tim_ctx_get_tuning(self) -> tim_tuning:
        t = tim_tuning()
        _check(lib().tim_ctx_get_tuning(self.handle, C.byref(t)), "tim_ctx_get_tuning")
        return t

    def tim_ctx_set_tuning(self, **fields):
        """Reads the current tuning, replaces the named fields, installs the result."""
        t = self.tim_ctx_get_tuning()
        for k, v in fields.items():
            if k not in dict(tim_tuning._fields_):
                raise KeyError(k)
            setattr(t, k, v)
        _check(lib().tim_ctx_set_tuning(self.handle, C.byref(t)), "tim_ctx_set_tuning")

    def tim_status(self) -> int:
        return lib().tim_status(self.handle, _stream())

    def tim_timing_begin(self, max_launches: int):
        self._timing_cap = max_launches
        _check(lib().tim_timing_begin(self.handle, max_launches), "tim_timing_begin")

    def tim_timing_end(self):
        """Durations (ms) of the attention main kernel of each timed tim_decode_attn call."""
        buf = (C.c_float * self._timing_cap)()
        n = C.c_int32(0)
        _check(lib().tim_timing_end(self.handle, buf, C.byref(n)), "tim_timing_end")
        return list(buf[: n.value])
