"""End-to-end oracle of one decoding context, mirroring the library's calls.

Order of one decode step (paper Sec. 3.1: pruning happens before decoding,
with the new token still pending):
    marks for the boundary  ->  [flush: prune_plan, kv_compact, commit]
    ->  advance (reserve the pending token's slot)  ->  per layer: append its
    K/V, attend over the whole retained working memory.

K/V live in a slot-major pool k[layer, slot, kv_head, dim] of bf16 bit
patterns, slot = page * page_size + offset; the page table maps logical page
-> physical page id.
"""
from dataclasses import dataclass

import numpy as np

from . import bf16
from .attention import attend, extend
from .pages import FreeStack
from .plan import Plan
from .prune_rule import PruningBuffer, kept_flags
from .rope import rotate

OK = 0
ERR_OOM_PAGES = -3
ERR_SEQ_TOO_LONG = -5
ERR_BAD_TREE = -2

MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, MARK_CLOSE = 1, 2, 3, 4


@dataclass
class Config:
    layers: int
    q_heads: int
    kv_heads: int
    head_dim: int
    page_size: int
    num_pages: int
    max_batch: int
    max_pages_per_seq: int
    max_nodes: int
    rope_base: float = 1.0e6
    rope_pairing: int = 0          # rope.HALF_SPLIT or rope.INTERLEAVED


class SeqPlan:
    """Plan of one sequence in one flush."""


class EventPlan:
    def __init__(self):
        self.ok = True
        self.seqs = []        # list of SeqPlan, ascending sequence id


class OracleRuntime:
    def __init__(self, cfg: Config, threshold: int):
        self.cfg = cfg
        c = cfg
        slots = c.num_pages * c.page_size
        self.k = np.zeros((c.layers, slots, c.kv_heads, c.head_dim), dtype=np.uint16)
        self.v = np.zeros_like(self.k)
        self.page_table = np.full((c.max_batch, c.max_pages_per_seq), -1, dtype=np.int32)
        self.seq_len = np.zeros(c.max_batch, dtype=np.int32)
        self.free = FreeStack(c.num_pages)
        self.status = OK
        shape = (c.max_batch, c.max_nodes)
        self.tok_begin = np.full(shape, -1, dtype=np.int32)
        self.sub_begin = np.full(shape, -1, dtype=np.int32)
        self.sub_end = np.full(shape, -1, dtype=np.int32)
        self.tok_end = np.full(shape, -1, dtype=np.int32)
        self.list_order = np.full(shape, -1, dtype=np.int32)
        self.n_nodes = np.zeros(c.max_batch, dtype=np.int32)
        self.lists_done = np.zeros(c.max_batch, dtype=np.int32)
        self.threshold = threshold
        self.buffers = [PruningBuffer(threshold) for _ in range(c.max_batch)]
        # in-forward variant only: visibility of every logical token (nothing is ever moved)
        self.visible = np.ones((c.max_batch, c.max_pages_per_seq * c.page_size), dtype=bool)

    # ---- helpers -------------------------------------------------------
    def _pages_of(self, n_tokens: int) -> int:
        ps = self.cfg.page_size
        return (n_tokens + ps - 1) // ps

    def slots_of(self, b: int, idx) -> np.ndarray:
        """Physical slots of logical token indices of sequence b."""
        ps = self.cfg.page_size
        idx = np.asarray(idx, dtype=np.int64)
        return self.page_table[b, idx // ps].astype(np.int64) * ps + idx % ps

    def gather_kv(self, layer: int, b: int):
        """Working memory of sequence b as (K, V) bf16 bits [T, Hkv, D]."""
        s = self.slots_of(b, np.arange(int(self.seq_len[b])))
        return self.k[layer, s], self.v[layer, s]

    # ---- structure tracking ---------------------------------------------
    def mark(self, ops) -> None:
        """Record structural marks (seq, code, node, boundary), in order.

        boundary = -1 means the sequence's current end (the mark sits right
        before the pending token); an explicit boundary serves preloading."""
        for b, code, node, at in ops:
            pos = int(self.seq_len[b]) if at < 0 else int(at)
            if code == MARK_OPEN:
                self.tok_begin[b, node] = pos
            elif code == MARK_SUB_BEGIN:
                self.sub_begin[b, node] = pos
            elif code == MARK_SUB_END:
                self.sub_end[b, node] = pos
                self.list_order[b, node] = self.lists_done[b]
                self.lists_done[b] += 1
                self.buffers[b].list_completed(node)
            elif code == MARK_CLOSE:
                self.tok_end[b, node] = pos
            else:
                raise ValueError("unknown mark")
            self.n_nodes[b] = max(int(self.n_nodes[b]), node + 1)

    # ---- one pending token per sequence ----------------------------------
    def advance(self) -> int:
        c = self.cfg
        need = [b for b in range(c.max_batch) if self.seq_len[b] % c.page_size == 0]
        if any(self.seq_len[b] // c.page_size >= c.max_pages_per_seq for b in need):
            self.status = self.status or ERR_SEQ_TOO_LONG
            return ERR_SEQ_TOO_LONG
        if len(need) > self.free.top:
            self.status = self.status or ERR_OOM_PAGES
            return ERR_OOM_PAGES
        for b in need:                                   # ascending id
            self.page_table[b, self.seq_len[b] // c.page_size] = self.free.pop()
        self.seq_len += 1
        return OK

    def extend_seq(self, counts) -> int:
        """Bulk form of advance(): a tool response enters the cache as a batch of new tokens
        (paper Sec. 2.1 "tooluse", Sec. 3.2).  Pages pop in ascending (sequence, page) order."""
        c = self.cfg
        if any(int(x) < 0 for x in counts):
            self.status = self.status or -1
            return -1
        have = [self._pages_of(int(n)) for n in self.seq_len]
        want = [self._pages_of(int(n) + int(x)) for n, x in zip(self.seq_len, counts)]
        if any(w > c.max_pages_per_seq for w in want):
            self.status = self.status or ERR_SEQ_TOO_LONG
            return ERR_SEQ_TOO_LONG
        if sum(w - h for w, h in zip(want, have)) > self.free.top:
            self.status = self.status or ERR_OOM_PAGES
            return ERR_OOM_PAGES
        for b in range(c.max_batch):
            for p in range(have[b], want[b]):
                self.page_table[b, p] = self.free.pop()
            self.seq_len[b] += int(counts[b])
        return OK

    def write_rows(self, layer: int, counts, k_rows: np.ndarray, v_rows: np.ndarray) -> None:
        """k_rows/v_rows: bf16 bits [sum(counts), Hkv, D], sequences ascending; they become the
        last counts[b] tokens of each sequence."""
        at = 0
        for b in range(self.cfg.max_batch):
            n, cb = int(self.seq_len[b]), int(counts[b])
            if cb:
                s = self.slots_of(b, np.arange(n - cb, n))
                self.k[layer, s] = k_rows[at : at + cb]
                self.v[layer, s] = v_rows[at : at + cb]
            at += cb

    def append(self, layer: int, k_new: np.ndarray, v_new: np.ndarray) -> None:
        """k_new/v_new: bf16 bits [B, Hkv, D]; K already carries its position."""
        for b in range(self.cfg.max_batch):
            s = int(self.slots_of(b, int(self.seq_len[b]) - 1))
            self.k[layer, s] = k_new[b]
            self.v[layer, s] = v_new[b]

    # ---- flush -----------------------------------------------------------
    def prune_plan(self, seq_ids) -> EventPlan:
        c = self.cfg
        ps = c.page_size
        ev = EventPlan()
        taken = []
        for b in sorted(seq_ids):
            n = int(self.seq_len[b])
            lists = self.buffers[b].take_pending()
            taken.append((b, lists))
            ranges = [(int(self.sub_begin[b, i]), int(self.sub_end[b, i])) for i in lists]
            sp = SeqPlan()
            sp.seq = b
            sp.n = n
            sp.plan = Plan(kept_flags(n, ranges))
            m, f = sp.plan.n_kept, sp.plan.first_pruned
            if ps == 1:
                # the paper's page size (Sec. 3.1): every token owns a page, so a survivor simply
                # keeps it; only the pruned tokens' pages go back, in ascending logical order
                sp.keep_pages = f
                sp.need = 0
                sp.old_pages = self.page_table[b, np.flatnonzero(sp.plan.new_pos < 0)].copy()
            else:
                # pages wholly before the first pruned token stay where they are;
                # if only a tail was pruned nothing moves and the boundary page stays too
                sp.keep_pages = self._pages_of(f) if m == f else f // ps
                sp.need = self._pages_of(m) - sp.keep_pages
                sp.old_pages = self.page_table[b, sp.keep_pages : self._pages_of(n)].copy()
            ev.seqs.append(sp)
        total = sum(sp.need for sp in ev.seqs)
        if total > self.free.top:
            ev.ok = False
            self.status = self.status or ERR_OOM_PAGES
            for b, lists in taken:                       # nothing happened
                self.buffers[b].pending = lists + self.buffers[b].pending
            return ev
        for sp in ev.seqs:
            b, pl = sp.seq, sp.plan
            m = pl.n_kept
            sp.new_table = self.page_table[b].copy()
            sp.new_table[sp.keep_pages :] = -1
            if ps == 1:
                sp.new_table[:m] = self.page_table[b, pl.kept_idx]        # same pages, closed up
            for p in range(sp.keep_pages, sp.keep_pages + sp.need):
                sp.new_table[p] = self.free.pop()
            moved = np.arange(sp.keep_pages * ps, m, dtype=np.int64)
            sp.moved_begin = sp.keep_pages * ps
            sp.src_slot = self.slots_of(b, pl.kept_idx[moved]).astype(np.int32)
            sp.dst_slot = (sp.new_table[moved // ps].astype(np.int64) * ps + moved % ps).astype(np.int32)
            sp.moved_delta = pl.delta[moved]
        return ev

    def kv_compact(self, ev: EventPlan, layer_begin: int, layer_end: int) -> None:
        if not ev.ok:
            return
        base = self.cfg.rope_base
        for sp in ev.seqs:
            if sp.src_slot.size == 0:
                continue
            for layer in range(layer_begin, layer_end):
                self.v[layer, sp.dst_slot] = self.v[layer, sp.src_slot]
                kb = self.k[layer, sp.src_slot]                     # [T, Hkv, D] bits
                kr = rotate(bf16.to_f64(kb), sp.moved_delta[:, None], base, self.cfg.rope_pairing)
                out = bf16.from_f64(kr)
                still = sp.moved_delta == 0                       # unmoved position: bit copy
                out[still] = kb[still]
                self.k[layer, sp.dst_slot] = out

    def commit(self, ev: EventPlan) -> None:
        if not ev.ok:
            return
        for sp in ev.seqs:                                # ascending id, ascending page
            for p in sp.old_pages:
                self.free.push(int(p))
        for sp in ev.seqs:
            b, pl = sp.seq, sp.plan
            self.page_table[b] = sp.new_table
            self.seq_len[b] = pl.n_kept
            for arr in (self.tok_begin, self.sub_begin, self.sub_end, self.tok_end):
                row = arr[b, : self.n_nodes[b]]                   # a view: boundaries of this sequence's nodes
                set_ = row >= 0                                   # -1 (not reached yet) stays -1
                row[set_] = pl.rank[row[set_]]                    # boundary t -> survivors before t

    # ---- attention ---------------------------------------------------------
    def decode_attn(self, layer: int, q: np.ndarray, scale: float) -> np.ndarray:
        """q: bf16 bits [B, Hq, D] -> float32 [B, Hq, D]."""
        c = self.cfg
        out = np.empty((c.max_batch, c.q_heads, c.head_dim), dtype=np.float32)
        for b in range(c.max_batch):
            kb, vb = self.gather_kv(layer, b)
            out[b] = attend(bf16.to_f64(q[b]), bf16.to_f64(kb), bf16.to_f64(vb), scale)
        return out

    # ---- in-forward variant: hide instead of move -------------------------------------------
    def prune_mask(self, seq_ids) -> None:
        """The lists that left the buffer become invisible; positions, pages and node
        coordinates stay as they are (Sec. 3.1's alternative that the paper's runtime avoids)."""
        for b in sorted(seq_ids):
            n = int(self.seq_len[b])
            for i in self.buffers[b].take_pending():
                sb, se = int(self.sub_begin[b, i]), int(self.sub_end[b, i])
                if sb < 0 or se < sb or se > n:
                    raise ValueError("bad range")
                self.visible[b, sb:se] = False

    def decode_attn_masked(self, layer: int, q: np.ndarray, scale: float) -> np.ndarray:
        c = self.cfg
        out = np.empty((c.max_batch, c.q_heads, c.head_dim), dtype=np.float32)
        for b in range(c.max_batch):
            kb, vb = self.gather_kv(layer, b)
            keep = self.visible[b, : int(self.seq_len[b])]
            out[b] = attend(bf16.to_f64(q[b]), bf16.to_f64(kb[keep]), bf16.to_f64(vb[keep]), scale)
        return out

    def extend_attn(self, layer: int, ev: EventPlan, q_ext: np.ndarray, scale: float) -> np.ndarray:
        """Attention half of Eq. 1 after `ev` was committed.  q_ext: bf16 bits [E_total, Hq, D],
        the extended tokens of the flushed sequences in ascending sequence order, each run
        covering new positions first_pruned .. m-1.  Returns float32 of the same shape."""
        out = np.zeros(q_ext.shape, dtype=np.float32)
        at = 0
        for sp in ev.seqs:
            f, m = sp.plan.first_pruned, sp.plan.n_kept
            e = max(m - f, 0)
            if e:
                kb, vb = self.gather_kv(layer, sp.seq)
                out[at : at + e] = extend(bf16.to_f64(q_ext[at : at + e]), bf16.to_f64(kb), bf16.to_f64(vb), f, scale)
            at += e
        return out

    # ---- accounting ----------------------------------------------------------
    def pages_in_use(self) -> int:
        return int(sum(self._pages_of(int(n)) for n in self.seq_len))
