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


def _overlay_insert(keys, dsts, new_keys, new_dsts):
    """What sam_apply_delta does with the exported transitions, on host arrays."""
    mask = len(keys) - 1
    for key, d in zip(new_keys, new_dsts):
        key = int(key)
        j = _hash64(key) & mask
        while int(keys[j]) != M64 and int(keys[j]) != key:
            j = (j + 1) & mask
        keys[j] = np.uint64(key)
        dsts[j] = d


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
        grow = 2 * n_ov > len(self.keys)
        if grow:                                              # a larger table: everything since the flatten goes in again
            cap = len(self.keys)
            while cap < 2 * n_ov:
                cap *= 2
            self.keys, self.dsts = A.overlay_table(cap)
        d = A.sam_delta_export(self.sam, overlay_all=grow)
        assert len(set(int(k) for k in d.ov_key)) == len(d.ov_key)      # every key once
        _overlay_insert(self.keys, self.dsts, d.ov_key, d.ov_dst)
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
    assert A.sam_delta_sizes(s) == (0, 0, 0, 0, 0, 4)
    dl = A.sam_delta_export(s)
    assert dl.rec_idx.size == 0 and dl.new_tokens.size == 0 and dl.ov_key.size == 0


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
    assert A.sam_delta_sizes(sam) == (0, 0, 0, 0, 0, ns)


def test_export_hands_out_new_transitions_once_and_all_on_request():
    s = A.sam_build([1, 2, 1, 2], 9)
    A.sam_flatten([s])
    A.sam_append(s, [3, 1, 2, 3])
    _, _, n_ov, n_new, _, _ = A.sam_delta_sizes(s)
    assert n_ov == n_new > 0
    d1 = A.sam_delta_export(s)
    assert 0 < d1.ov_key.size <= n_ov
    assert A.sam_delta_sizes(s)[2:4] == (n_ov, 0)              # the log stays, nothing new
    assert A.sam_delta_export(s).ov_key.size == 0
    A.sam_append(s, [1, 2, 3, 4])
    d2 = A.sam_delta_export(s)
    every = A.sam_delta_export(s, overlay_all=True)           # everything since the flatten, latest destination per key
    merged = dict(zip(d1.ov_key.tolist(), d1.ov_dst.tolist())); merged.update(zip(d2.ov_key.tolist(), d2.ov_dst.tolist()))
    assert dict(zip(every.ov_key.tolist(), every.ov_dst.tolist())) == merged
    # the policy: due once the log exceeds the stated fraction of the flattened transitions (6 here)
    assert A.sam_reflatten_due(s, 0.1) and not A.sam_reflatten_due(s, 100.0)
    A.sam_flatten([s])
    assert not A.sam_reflatten_due(s, 0.0)
    fresh = A.sam_build([1, 2], 9)
    assert A.sam_reflatten_due(fresh, 100.0)                  # never flattened


def test_periodic_memory_appends_cost_one_chain_walk_per_export_not_per_token():
    """A continuously repetitive 30k-token memory (the case Sec. 6's TTFT / TPOT table measures): the suffix-link
    chains are thousands of states long.  Appending with a maintained copy must stay within a small factor of
    appending without one, and the export must still give what a fresh flatten gives."""
    import time
    base = np.tile(np.array([5, 6, 7], np.int32), 10000)
    more = np.tile(np.array([5, 6, 7], np.int32), 3000)
    plain = A.sam_build(base, 9)
    t0 = time.perf_counter(); A.sam_append(plain, more); t_plain = time.perf_counter() - t0
    s = A.sam_build(base, 9)
    f0 = A.sam_flatten([s])
    lastpos = np.full(2 * (base.size + more.size) + 2, -1, np.int32); lastpos[:f0.lastpos.size] = f0.lastpos
    t0 = time.perf_counter()
    for i in range(0, more.size, 3):                          # a step commits a few tokens, then the delta is taken
        A.sam_append(s, more[i:i + 3])
        if i % 300 == 0:
            d = A.sam_delta_export(s)
            lastpos[d.lastpos_idx] = d.lastpos_val
    d = A.sam_delta_export(s)
    lastpos[d.lastpos_idx] = d.lastpos_val
    t_tracked = time.perf_counter() - t0
    f1 = A.sam_flatten([s])
    assert np.array_equal(lastpos[:f1.lastpos.size], f1.lastpos)
    print(f"9000 tokens appended to a period-3 memory of 30000: {t_plain * 1e3:.1f} ms plain, {t_tracked * 1e3:.1f} ms with "
          f"31 exports ({t_tracked / more.size * 1e6:.2f} us per token)")
    assert t_tracked < 0.3                                    # (one chain walk per token took 0.5 s here; this takes 0.05 s)


def test_export_argument_errors():
    s = A.sam_build([1, 2, 1, 2], 9)
    A.sam_flatten([s])
    A.sam_append(s, [3, 1, 2, 3])
    from paper_2512_18337_amd import binding
    import ctypes
    nw = ctypes.c_int64()
    # transitions to hand out but no arrays for them
    rc = binding.lib().sam_delta_export(s._h, 0, 0, None, None, None, None, 0, None, None, ctypes.byref(nw), None)
    assert rc == -1
    d = A.sam_delta_export(s)                                 # a failed export loses nothing
    assert d.ov_key.size > 0 and d.rec_idx.size > 0
