"""Incremental maintenance of a flattened automaton (host side): the exported delta - patched walk
records and last eligible end positions, the overlay table of new and redirected transitions, the new
tokens - applied to a copy of the flattened arrays must answer every query as the oracle does on the
grown memory, and must agree with flattening the grown automaton from scratch."""
import numpy as np
import pytest

import paper_2512_18337_amd as A
from oracle import draft_oracle

M64 = (1 << 64) - 1


def _hash64(k):
    """The hash of csrc/sam_hash.h, restated."""
    k ^= k >> 33; k = (k * 0xff51afd7ed558ccd) & M64
    k ^= k >> 33; k = (k * 0xc4ceb9fe1a85ec53) & M64
    k ^= k >> 33
    return k


def _overlay_find(keys, dsts, s, c):
    mask = len(keys) - 1
    key = ((s << 32) | c) & M64
    j = _hash64(key) & mask
    for _ in range(len(keys)):
        if int(keys[j]) == key:
            return int(dsts[j])
        if int(keys[j]) == M64:
            return -1
        j = (j + 1) & mask
    return -1


class Live:
    """Host emulation of a maintained device copy: the arrays sam_draft_delta reads."""

    def __init__(self, sam, cap_tokens):
        f = A.sam_flatten([sam])
        self.sam, self.row_ptr, self.edge_tok, self.edge_dst = sam, f.row_ptr, f.edge_tok, f.edge_dst
        ns, nt = f.len.shape[0], f.corpus.shape[0]
        cap = 2 * cap_tokens + 2
        self.rec = np.full((cap, 4), -7, np.int32); self.rec[:ns] = f.state_rec.reshape(ns, 4)
        self.lastpos = np.full(cap, -7, np.int32); self.lastpos[:ns] = f.lastpos
        self.corpus = np.full(cap_tokens, -7, np.int32); self.corpus[:nt] = f.corpus
        self.nt, self.rows_end = nt, ns
        self.keys, self.dsts = A.overlay_table(2)

    def sync(self):
        n_ov = A.sam_delta_sizes(self.sam)[2]
        cap = 2
        while cap < 2 * n_ov:
            cap *= 2
        self.keys, self.dsts = A.overlay_table(cap)
        d = A.sam_delta_export(self.sam, self.keys, self.dsts)
        assert d.flat_states == self.rows_end
        self.rec[d.rec_idx] = d.rec_val
        self.lastpos[d.lastpos_idx] = d.lastpos_val
        self.corpus[self.nt:self.nt + d.new_tokens.shape[0]] = d.new_tokens
        self.nt += d.new_tokens.shape[0]
        return d

    def walk(self, q, k, sep, min_match=1):
        s, l = 0, 0
        for c in q:
            c = int(c)
            while True:
                r0, r1, lk, ll = (int(x) for x in self.rec[s])
                ll = -1 - ll if ll < 0 else ll                  # without the wide-state flag
                dst = -1
                if r0 == c:
                    dst = r1 if r1 >= 0 else -2 - r1
                elif r1 < -1:
                    dst = _overlay_find(self.keys, self.dsts, s, c)
                    if dst < 0 and s < self.rows_end:
                        a, b = self.row_ptr[s], self.row_ptr[s + 1]
                        j = a + np.searchsorted(self.edge_tok[a:b], c)
                        if j < b and self.edge_tok[j] == c:
                            dst = int(self.edge_dst[j])
                if dst >= 0:
                    s, l = dst, l + 1
                    break
                if s == 0:
                    l = 0
                    break
                s, l = lk, ll
        L, e = l, -1
        while s != 0:
            if self.lastpos[s] >= 0:
                e = int(self.lastpos[s]); break
            s, L = int(self.rec[s, 2]), int(self.rec[s, 3])
            L = -1 - L if L < 0 else L
        if e < 0 or L < min_match:
            return [], 0, -1
        d = []
        for j in range(k):
            i = e + 1 + j
            if i >= self.nt or self.corpus[i] == sep:
                break
            d.append(int(self.corpus[i]))
        return d, L, e


def test_no_delta_before_a_flatten_and_empty_delta_after():
    s = A.sam_build([1, 2, 3], 9)
    with pytest.raises(A.AgentSamError):
        A.sam_delta_sizes(s)
    A.sam_flatten([s])
    assert A.sam_delta_sizes(s) == (0, 0, 0, 0, 4)
    k, d = A.overlay_table(2)
    dl = A.sam_delta_export(s, k, d)
    assert dl.rec_idx.size == 0 and dl.new_tokens.size == 0 and (k == np.uint64(M64)).all()


def test_hand_example_tail_becomes_eligible():
    # memory 1 2 3: the window [2 3] only matches the tail; after 4 5 arrive the tail has a continuation
    s = A.sam_build([1, 2, 3], 9)
    live = Live(s, 16)
    assert live.walk([2, 3], 2, 9) == ([], 0, -1)
    A.sam_append(s, [4, 5])
    live.sync()
    assert live.walk([2, 3], 2, 9) == ([4, 5], 2, 2)
    assert live.walk([3, 4], 3, 9) == ([5], 2, 3)


@pytest.mark.parametrize("seed", range(6))
def test_maintained_copy_answers_like_the_oracle(seed):
    rng = np.random.default_rng(500 + seed)
    vocab = int(rng.integers(2, 6)) if seed < 4 else 150         # the larger one makes the root a wide state
    sep = vocab
    N0 = int(rng.integers(0, 120)) if seed < 4 else 900
    T = list(rng.integers(0, vocab, N0))
    sam = A.sam_build(T, sep)
    live = Live(sam, N0 + 400)
    for step in range(40):
        add = list(rng.integers(0, vocab, int(rng.integers(0, 10))))
        if add and rng.random() < 0.25:
            add[int(rng.integers(0, len(add)))] = sep
        if step % 7 == 3:
            add += [int(rng.integers(vocab + 1, vocab + 50))]      # a token never seen before: new root transition
        A.sam_append(sam, add)
        T += add
        if step % 3 == 2:
            continue                                             # several appends may go into one delta
        live.sync()
        Tn = np.asarray(T, np.int32)
        for _ in range(12):
            if len(T) > 4 and rng.random() < 0.7:                # a window cut from the memory, one token perturbed
                p = int(rng.integers(1, len(T))); ln = int(rng.integers(1, min(p, 14) + 1))
                q = [t for t in T[p - ln:p] if t != sep] or [0]
                if rng.random() < 0.4:
                    q[int(rng.integers(0, len(q)))] = int(rng.integers(0, vocab))
            else:
                q = list(rng.integers(0, vocab, int(rng.integers(1, 10))))
            k = int(rng.integers(0, 6)); mm = int(rng.integers(1, 3))
            d, nd, ml, me = draft_oracle(Tn, np.asarray(q, np.int32), k, sep, mm)
            assert live.walk(q, k, sep, mm) == (list(d[:nd]), ml, me), (step, q)
    # against flattening the grown automaton from scratch: same end positions, links, lengths and tokens
    live.sync()
    f = A.sam_flatten([sam])
    ns = f.len.shape[0]
    assert np.array_equal(live.lastpos[:ns], f.lastpos)
    unflag = lambda r: np.where(r[:, 3] < 0, -1 - r[:, 3], r[:, 3])
    assert np.array_equal(live.rec[:ns, 2], f.state_rec.reshape(ns, 4)[:, 2])
    assert np.array_equal(unflag(live.rec[:ns]), unflag(f.state_rec.reshape(ns, 4)))
    assert np.array_equal(live.corpus[:live.nt], f.corpus) and live.nt == len(T)
    # and the flatten has reset the log
    assert A.sam_delta_sizes(sam) == (0, 0, 0, 0, ns)


def test_export_argument_errors():
    s = A.sam_build([1, 2, 1, 2], 9)
    A.sam_flatten([s])
    A.sam_append(s, [3, 1, 2, 3])
    n_ov = A.sam_delta_sizes(s)[2]
    assert n_ov > 0
    k, d = A.overlay_table(2)                                     # too small: must stay at most half full
    with pytest.raises(A.AgentSamError):
        A.sam_delta_export(s, k, d)
    k = np.full(24, np.uint64(M64), np.uint64); d = np.full(24, -1, np.int32)      # not a power of two
    with pytest.raises(A.AgentSamError):
        A.sam_delta_export(s, k, d)
    k, d = A.overlay_table(64)
    A.sam_delta_export(s, k, d)                                   # a failed export loses nothing
    assert (k != np.uint64(M64)).sum() > 0
