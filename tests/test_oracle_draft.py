"""Pins for the draft oracle: hand examples, an independent brute force, invariants, recall."""
import os

import numpy as np
import pytest

from oracle import draft_oracle, draft_oracle_batch
from paper_2512_18337_amd import workloads as W


def _parse(line):
    lhs, rhs = line.split("=>")
    T, q, k, sep, mm = [x.strip() for x in lhs.split("|")]
    ml, me, nd, dr = [x.strip() for x in rhs.split("|")]
    ints = lambda s: [int(x) for x in s.split()]
    return ints(T), ints(q), int(k), int(sep), int(mm), int(ml), int(me), int(nd), ints(dr)


def test_hand_examples(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "draft_hand_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        T, q, k, sep, mm, ml, me, nd, dr = _parse(line)
        d, n_d, m_l, m_e = draft_oracle(T, q, k, sep, mm)
        assert (m_l, m_e, n_d) == (ml, me, nd), line
        assert list(d[:n_d]) == dr and all(x == -1 for x in d[n_d:]), line
        n += 1
    assert n >= 10


def _second_brute_force(T, q, k, sep, min_match):
    """Independent restatement: try suffix lengths from long to short with list slicing."""
    T, q = list(T), list(q)
    N = len(T)
    for L in range(min(len(q), N), max(min_match, 1) - 1, -1):
        suf = q[len(q) - L:]
        ends = [e for e in range(L - 1, N) if T[e - L + 1:e + 1] == suf and e + 1 < N and T[e + 1] != sep]
        if ends:
            e = max(ends)
            cont = []
            for t in T[e + 1:e + 1 + k]:
                if t == sep:
                    break
                cont.append(t)
            return L, e, cont
    return 0, -1, []


@pytest.mark.parametrize("seed", range(6))
def test_against_second_brute_force(seed):
    rng = np.random.default_rng(seed)
    for _ in range(60):
        N = int(rng.integers(1, 120))
        vocab = int(rng.integers(1, 5))
        sep = vocab
        T = rng.integers(0, vocab, N)
        T[rng.random(N) < 0.1] = sep                     # sprinkle separators
        m = int(rng.integers(1, 12))
        q = rng.integers(0, vocab, m)
        k = int(rng.integers(0, 6))
        mm = int(rng.integers(1, 4))
        d, nd, ml, me = draft_oracle(T, q, k, sep, mm)
        L, e, cont = _second_brute_force(T, q, k, sep, mm)
        assert (ml, me, nd) == (L, e, len(cont))
        assert list(d[:nd]) == cont


def _small_cfg(i, **kw):
    return W.scaled(W.baseline_config(i), **kw)


@pytest.mark.parametrize("cfg", [
    W.baseline_config(0),
    _small_cfg(1, B=4, sam_session_len=4096),
    _small_cfg(2, B=8, sam_sessions=8, sam_session_len=1024),
    _small_cfg(3, B=8, sam_sessions=4, sam_session_len=2048),
], ids=lambda c: c.name)
def test_invariants_on_generated_workloads(cfg):
    nmem = cfg.B if cfg.sam_mode == "per_session" else 1
    mems = [W.token_memory(cfg, i) for i in range(nmem)]
    recent, rlen = W.recent_windows(cfg, mems)
    seen_match = 0
    for b in range(cfg.B):
        T = mems[b if nmem > 1 else 0]
        q = recent[b, cfg.m - rlen[b]:]
        d, nd, ml, me = draft_oracle(T, q, cfg.k, cfg.sep)
        assert 0 <= nd <= cfg.k and 0 <= ml <= len(q)
        if ml == 0:
            assert me == -1 and nd == 0
            # no single token of the window's end occurs at an eligible place
            ok = [e for e in range(len(T) - 1) if T[e] == q[-1] and T[e + 1] != cfg.sep]
            assert not ok
            continue
        seen_match += 1
        # the matched suffix really sits there, and the draft is what follows it
        assert np.array_equal(T[me - ml + 1:me + 1], q[len(q) - ml:])
        assert me + 1 < len(T) and T[me + 1] != cfg.sep and nd >= 1
        assert np.array_equal(d[:nd], T[me + 1:me + 1 + nd])
        assert not np.any(d[:nd] == cfg.sep) and np.all(d[nd:] == -1)
        if nd < cfg.k:
            assert me + 1 + nd == len(T) or T[me + 1 + nd] == cfg.sep
        # maximality: the next longer suffix has no eligible occurrence; recency: no later eligible one
        if ml < len(q):
            longer = q[len(q) - ml - 1:]
            hits = [e for e in range(ml, len(T) - 1)
                    if T[e + 1] != cfg.sep and np.array_equal(T[e - ml:e + 1], longer)]
            assert not hits
        later = [e for e in range(me + 1, len(T) - 1)
                 if T[e + 1] != cfg.sep and e - ml + 1 >= 0 and np.array_equal(T[e - ml + 1:e + 1], q[len(q) - ml:])]
        assert not later
    assert seen_match >= cfg.B // 2


def test_planted_copy_recall():
    """A window cut from inside the memory must be found at least as long as it was planted."""
    cfg = _small_cfg(2, B=1, sam_sessions=4, sam_session_len=2048)
    T = W.token_memory(cfg)
    rng = np.random.default_rng(5)
    for _ in range(40):
        L = int(rng.integers(1, 40))
        p = int(rng.integers(L, len(T) - 2))
        seg = T[p - L + 1:p + 1]
        if np.any(seg == cfg.sep) or T[p + 1] == cfg.sep:
            continue
        q = np.concatenate([[cfg.vocab - 1 - (int(T[p - L]) == cfg.vocab - 1)], seg]).astype(np.int32)
        d, nd, ml, me = draft_oracle(T, q, 4, cfg.sep)
        assert ml >= L and nd >= 1
        if ml == L:
            assert me >= p


def test_batch_form_equals_single_calls():
    cfg = W.baseline_config(0)
    mems = [W.token_memory(cfg, i) for i in range(cfg.B)]
    recent, rlen = W.recent_windows(cfg, mems)
    rlen = rlen.copy()
    rlen[1] = 5                                           # a shorter window
    T = np.concatenate(mems)
    begin = np.array([0, len(mems[0])])
    end = begin + np.array([len(m) for m in mems])
    D, ND, ML, ME = draft_oracle_batch(T, begin, end, recent, rlen, cfg.k, cfg.sep)
    for b in range(cfg.B):
        d, nd, ml, me = draft_oracle(mems[b], recent[b, cfg.m - rlen[b]:], cfg.k, cfg.sep)
        assert np.array_equal(D[b], d) and (ND[b], ML[b], ME[b]) == (nd, ml, me)


def test_empty_inputs():
    d, nd, ml, me = draft_oracle([], [1, 2], 3, sep=9)
    assert (nd, ml, me) == (0, 0, -1) and list(d) == [-1, -1, -1]
    d, nd, ml, me = draft_oracle([1, 2, 1, 2], [], 3, sep=9)
    assert (nd, ml, me) == (0, 0, -1)
    d, nd, ml, me = draft_oracle([1, 2, 1, 2], [1], 0, sep=9)
    assert (nd, ml, me) == (0, 1, 2) and len(d) == 0
