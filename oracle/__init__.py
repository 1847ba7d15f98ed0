"""CPU oracle for the working-memory decoding path (TEST INFRASTRUCTURE ONLY).

A plain, slow, obviously-correct implementation of what the GPU library
computes: the rule-based subtask pruning (paper Sec. 2.1 "Subtask pruning",
Sec. 3.1), the resulting plan (kept tokens, contiguous new positions, page
remap), the deterministic page allocator, K/V compaction with RoPE
re-rotation (the weight-free reading of Eq. 1), and softmax attention over the
retained set.  Floating point runs in float64; K/V storage is bf16 with
round-to-nearest-even, as in the GPU pool.

Nothing in the product path may import this package: only tests/, the smoke
check and the benchmark's cpu_baseline leg do.  It shares no code with the
HIP kernels or their Python binding, and never imports them.

Parity pins (tests/test_oracle_*.py) cover every function here: the paper's
worked example of Sec. 3.1, the Fig. 3 caption scenario, brute force on tiny
trees, FIFO-vs-declarative agreement, the RoPE composition closed form,
prune-nothing == causal attention, page conservation, hand-worked allocator
examples, and - for the runtime's extend and masked attention wrappers - rows
of a library's dense causal attention per flushed sequence and a triple loop
over the visible tokens.  No function is "parity unpinned".
"""
