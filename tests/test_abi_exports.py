"""The C-ABI library loads without a GPU and exports every function include/tim.h declares."""
import ctypes
import os
import re

from paper_2507_16784_amd import tim

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "tim.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(tim_[a-z_]+)\s*\(", src)))


def test_header_and_binding_agree():
    assert _declared() == sorted(tim.EXPORTS)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(tim.LIB_PATH):
        from paper_2507_16784_amd import build
        build.build()
    lib = ctypes.CDLL(tim.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name


def test_host_side_argument_checks_need_no_gpu():
    lib = tim.lib()
    h = ctypes.c_void_p()
    bad = tim.tim_config(1, 8, 2, 64, 16, 8, 1, 4, 4, 1.0e6)          # head_dim 64 is unsupported
    assert lib.tim_ctx_create(ctypes.byref(h), ctypes.byref(bad)) == tim.ERR_INVALID_ARG
    bad = tim.tim_config(1, 6, 2, 128, 16, 8, 1, 4, 4, 1.0e6)         # group size 3 is unsupported
    assert lib.tim_ctx_create(ctypes.byref(h), ctypes.byref(bad)) == tim.ERR_INVALID_ARG
    bad = tim.tim_config(1, 8, 2, 128, 16, 8, 1, 4, 4, 1.0e6, 2)       # neither rotary pairing
    assert lib.tim_ctx_create(ctypes.byref(h), ctypes.byref(bad)) == tim.ERR_INVALID_ARG
    ok = tim.tim_config(1, 8, 2, 128, 16, 8, 1, 4, 4, 1.0e6)
    assert lib.tim_ctx_create(ctypes.byref(h), ctypes.byref(ok)) == tim.OK
    # unbound context: every stream call is refused before anything is launched
    assert lib.tim_seq_advance(h, None) == tim.ERR_INVALID_ARG
    assert lib.tim_pool_reset(h, None) == tim.ERR_INVALID_ARG
    empty = tim.tim_state()
    assert lib.tim_bind(h, ctypes.byref(empty)) == tim.ERR_INVALID_ARG
    assert lib.tim_attn_schedule(h, 0, None) == tim.ERR_INVALID_ARG
    # partials [batch][q_heads][128 slots][128 + 2] fp32, then the schedule: 4 words, 4 per (sequence, slot), 1 per sequence
    assert lib.tim_attn_ws_bytes(ctypes.byref(ok)) == 1 * 8 * 128 * 130 * 4 + (4 + (4 * 128 + 1) * 1) * 4
    # launch-shape tuning is a host object: defaults, a round trip, and refused values
    t = tim.tim_tuning()
    assert lib.tim_ctx_get_tuning(h, ctypes.byref(t)) == tim.OK
    assert (t.attn_impl, t.chunks_per_block, t.fill, t.grade_big, t.grade_small, t.round_items, t.block_waves, t.short_list_chunks) == (tim.ATTN_MFMA, 6, 2, 32, 8, 0, 0, 0)
    t.chunks_per_block, t.round_items = 3, 4
    assert lib.tim_ctx_set_tuning(h, ctypes.byref(t)) == tim.OK
    t2 = tim.tim_tuning()
    assert lib.tim_ctx_get_tuning(h, ctypes.byref(t2)) == tim.OK and (t2.chunks_per_block, t2.round_items) == (3, 4)
    for field, bad_value in (("attn_impl", 2), ("chunks_per_block", 0), ("chunks_per_block", 65), ("fill", 0),
                             ("grade_small", 33), ("grade_small", -1), ("round_items", -1), ("block_waves", 5), ("short_list_chunks", -1)):
        t3 = tim.tim_tuning()
        lib.tim_ctx_get_tuning(h, ctypes.byref(t3))
        setattr(t3, field, bad_value)
        assert lib.tim_ctx_set_tuning(h, ctypes.byref(t3)) == tim.ERR_INVALID_ARG, field
    assert lib.tim_ctx_get_tuning(h, ctypes.byref(t3)) == tim.OK and t3.chunks_per_block == 3     # refused: unchanged
    # alignment is checked on the host: made-up addresses, nothing is launched and no GPU is touched
    st = tim.tim_state()
    for name, _ in tim.tim_state._fields_:
        if name != "attn_ws_bytes":
            setattr(st, name, 0x10000)
    st.attn_ws_bytes = lib.tim_attn_ws_bytes(ctypes.byref(ok))
    assert lib.tim_bind(h, ctypes.byref(st)) == tim.OK
    for name, off in (("k_pool", 8), ("v_pool", 2), ("attn_ws", 4), ("page_table", 2), ("seq_len", 1), ("keep_mask", 2)):
        st2 = tim.tim_state.from_buffer_copy(st)
        setattr(st2, name, 0x10000 + off)
        assert lib.tim_bind(h, ctypes.byref(st2)) == tim.ERR_INVALID_ARG, name
    vp = ctypes.c_void_p
    for q_addr, out_addr in ((0x20008, 0x30000), (0x20000, 0x30004)):
        assert lib.tim_decode_attn(h, 0, vp(q_addr), vp(out_addr), ctypes.c_float(1.0), 0, 0, None) == tim.ERR_INVALID_ARG
        assert lib.tim_decode_attn_noalloc(h, 0, vp(q_addr), vp(out_addr), ctypes.c_float(1.0), 0, 0, None) == tim.ERR_INVALID_ARG
    assert lib.tim_decode_attn_append(h, 0, vp(0x20000), vp(0x40002), vp(0x50000), vp(0x30000), ctypes.c_float(1.0), 0, 0,
                                      None) == tim.ERR_INVALID_ARG
    assert lib.tim_kv_append(h, 0, vp(0x40000), vp(0x50008), None) == tim.ERR_INVALID_ARG
    assert lib.tim_tree_mark(h, vp(0x60002), 1, None) == tim.ERR_INVALID_ARG
    assert lib.tim_seq_extend(h, vp(0x60001), None) == tim.ERR_INVALID_ARG
    assert lib.tim_ctx_destroy(h) == tim.OK


def test_bench_refuses_more_than_one_gpu_before_touching_any():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_pool_allocator_places_the_v_pool_one_tile_and_one_row_beyond_the_k_pools_alignment():
    shape = (2, 5, 2, 16, 128)
    for _ in range(3):                      # whatever base addresses the allocator hands out
        k, v = tim.alloc_pools(shape, device="cpu", zero=True)
        assert tuple(k.shape) == tuple(v.shape) == shape and k.is_contiguous() and v.is_contiguous()
        assert (v.data_ptr() - k.data_ptr()) % tim.POOL_STAGGER_PERIOD == tim.POOL_STAGGER_BYTES == 4096 + 256
        assert v.data_ptr() % 16 == 0 and k.data_ptr() % 16 == 0
        assert float(v.float().abs().sum()) == 0.0
    k, v = tim.alloc_pools(shape, device="cpu", stagger=False)
    assert tuple(v.shape) == shape
