"""Host-side automaton builder: structure checks and a CPU walk of the flattened arrays against the oracle."""
import numpy as np
import pytest

import paper_2512_18337_amd as A
from oracle import draft_oracle
from paper_2512_18337_amd import workloads as W


def _distinct_substrings(T):
    T = list(T)
    return len({tuple(T[i:j]) for i in range(len(T)) for j in range(i + 1, len(T) + 1)})


def _walk(flat, ai, q, k, sep, min_match=1):
    """The lookup sam_draft performs, restated on the host arrays (test-only)."""
    root = int(flat.roots[ai])
    s, l = root, 0
    for c in q:
        while True:
            r0, r1 = flat.row_ptr[s], flat.row_ptr[s + 1]
            j = r0 + np.searchsorted(flat.edge_tok[r0:r1], c)
            if j < r1 and flat.edge_tok[j] == c:
                s, l = int(flat.edge_dst[j]), l + 1
                break
            if s == root:
                l = 0
                break
            s = int(flat.link[s]); l = int(flat.len[s])
    L, e = l, -1
    while s != root:
        if flat.lastpos[s] >= 0:
            e = int(flat.lastpos[s]); break
        s = int(flat.link[s]); L = int(flat.len[s])
    if e < 0 or L < min_match:
        return [], 0, -1
    d = []
    for j in range(k):
        i = e + 1 + j
        if i >= flat.corpus_end[ai] or flat.corpus[i] == sep:
            break
        d.append(int(flat.corpus[i]))
    return d, L, e - int(flat.corpus_begin[ai])


def test_repeated_token_chain():
    for n in (1, 2, 7, 50):
        s = A.sam_build([3] * n, sep_token=9)
        ns, ne, nt = A.sam_flat_sizes(s)
        assert (ns, ne, nt) == (n + 1, n, n)


@pytest.mark.parametrize("seed", range(5))
def test_size_bounds_and_substring_count(seed):
    rng = np.random.default_rng(seed)
    for _ in range(20):
        N = int(rng.integers(3, 60))
        T = rng.integers(0, int(rng.integers(1, 5)), N)
        s = A.sam_build(T, sep_token=99)
        ns, ne, nt = A.sam_flat_sizes(s)
        assert ns <= 2 * N - 1 + 1 and ne <= 3 * N - 4 + 1 and nt == N   # textbook bounds (root counted in ns)
        f = A.sam_flatten([s])
        assert f.len[0] == 0 and f.link[0] == -1
        # number of distinct substrings = sum over states of len[v] - len[link[v]]
        total = int(sum(f.len[v] - f.len[f.link[v]] for v in range(1, ns)))
        assert total == _distinct_substrings(T)
        # CSR rows sorted by token, transitions lengthen by at least one
        for v in range(ns):
            row = f.edge_tok[f.row_ptr[v]:f.row_ptr[v + 1]]
            assert np.all(np.diff(row) > 0)
            assert np.all(f.len[f.edge_dst[f.row_ptr[v]:f.row_ptr[v + 1]]] >= f.len[v] + 1)
        assert f.row_ptr[0] == 0 and f.row_ptr[ns] == ne and np.array_equal(f.corpus, T)
        # the 16-byte walk records restate the first transition, the link and the link's len
        rec = f.state_rec.reshape(ns, 4)
        for v in range(ns):
            r0, r1 = f.row_ptr[v], f.row_ptr[v + 1]
            if r1 == r0:
                assert rec[v, 0] == -1 and rec[v, 1] == -1
            else:
                assert rec[v, 0] == f.edge_tok[r0]
                assert rec[v, 1] == (f.edge_dst[r0] if r1 - r0 == 1 else -2 - f.edge_dst[r0])
            ll = 0 if f.link[v] < 0 else f.len[f.link[v]]
            assert rec[v, 2] == f.link[v] and rec[v, 3] == (ll if r1 - r0 <= 64 else -1 - ll)


@pytest.mark.parametrize("seed", range(4))
def test_walk_of_flat_arrays_matches_oracle_small(seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(40):
        N = int(rng.integers(1, 150))
        vocab = int(rng.integers(1, 5))
        sep = vocab
        T = rng.integers(0, vocab, N)
        T[rng.random(N) < 0.08] = sep
        f = A.sam_flatten([A.sam_build(T, sep)])
        for _ in range(10):
            q = rng.integers(0, vocab, int(rng.integers(1, 14)))
            k = int(rng.integers(0, 6)); mm = int(rng.integers(1, 3))
            d, nd, ml, me = draft_oracle(T, q, k, sep, mm)
            wd, wl, we = _walk(f, 0, q, k, sep, mm)
            assert (wl, we, wd) == (ml, me, list(d[:nd]))


def test_wide_table_holds_exactly_the_transitions_of_wide_states():
    from test_sam_delta import _hash64, M64
    rng = np.random.default_rng(11)
    T = np.concatenate([rng.integers(0, 400, 3000), np.tile([7, 8], 200)]).astype(np.int32)
    T[::2] = np.where(rng.random(T[::2].shape[0]) < 0.5, 7, T[::2])    # token 7 gets many different successors
    f = A.sam_flatten([A.sam_build(T, 999), A.sam_build(T[:500], 999)])
    tab = f.wide_table.reshape(-1, 4)
    slots = tab.shape[0]
    assert slots & (slots - 1) == 0
    found = {}
    for lo, hi, d, z in tab:
        if lo == -1 and hi == -1:
            continue
        found[(int(np.uint32(hi)), int(np.uint32(lo)))] = int(d)
    expect = {}
    ns = f.len.shape[0]
    rec = f.state_rec.reshape(ns, 4)
    for v in range(ns):
        r0, r1 = int(f.row_ptr[v]), int(f.row_ptr[v + 1])
        assert (rec[v, 3] < 0) == (r1 - r0 > 64)
        if r1 - r0 > 64:
            for j in range(r0, r1):
                expect[(v, int(f.edge_tok[j]))] = int(f.edge_dst[j])
    assert len(expect) > 300 and found == expect and 2 * len(found) <= slots
    assert int(f.roots[1]) in {v for v, _ in expect}                  # the second automaton's root, rebased
    for (v, c), d in list(expect.items())[::17]:                      # reachable by linear probing from the hash
        j = _hash64(((v << 32) | c) & M64) & (slots - 1)
        while not (np.uint32(tab[j, 1]) == v and np.uint32(tab[j, 0]) == c):
            assert not (tab[j, 0] == -1 and tab[j, 1] == -1)
            j = (j + 1) & (slots - 1)
        assert tab[j, 2] == d


def test_append_equals_build_and_updates_eligibility():
    rng = np.random.default_rng(7)
    T = rng.integers(0, 3, 200)
    a = A.sam_build(T, sep_token=3)
    b = A.sam_build(T[:77], sep_token=3)
    A.sam_append(b, T[77:150]); A.sam_append(b, T[150:]); A.sam_append(b, [])
    fa, fb = A.sam_flatten([a]), A.sam_flatten([b])
    for name in ("len", "link", "row_ptr", "edge_tok", "edge_dst", "lastpos", "corpus", "state_rec"):
        assert np.array_equal(getattr(fa, name), getattr(fb, name)), name
    # the old tail becomes a usable end position once a token follows it
    s = A.sam_build([1, 2, 3], sep_token=9)
    assert _walk(A.sam_flatten([s]), 0, [2, 3], 2, 9) == ([], 0, -1)
    A.sam_append(s, [4, 5])
    assert _walk(A.sam_flatten([s]), 0, [2, 3], 2, 9) == ([4, 5], 2, 2)


def test_packed_automata_and_generated_workload():
    cfg = W.baseline_config(0)
    mems = [W.token_memory(cfg, i) for i in range(cfg.B)]
    flat = A.sam_flatten([A.sam_build(m, cfg.sep) for m in mems])
    assert list(flat.corpus_begin) == [0, 2048] and list(flat.corpus_end) == [2048, 4096]
    assert flat.link[flat.roots[1]] == -1
    recent, rlen = W.recent_windows(cfg, mems)
    for b in range(cfg.B):
        q = recent[b, cfg.m - rlen[b]:]
        d, nd, ml, me = draft_oracle(mems[b], q, cfg.k, cfg.sep)
        assert _walk(flat, b, q, cfg.k, cfg.sep) == (list(d[:nd]), ml, me)


def test_shared_memory_workload_walk_matches_oracle():
    cfg = W.scaled(W.baseline_config(2), B=24, sam_sessions=8, sam_session_len=1024)
    T = W.token_memory(cfg)
    flat = A.sam_flatten([A.sam_build(T, cfg.sep)])
    recent, rlen = W.recent_windows(cfg, [T])
    lens = []
    for b in range(cfg.B):
        q = recent[b, cfg.m - rlen[b]:]
        d, nd, ml, me = draft_oracle(T, q, cfg.k, cfg.sep)
        assert _walk(flat, 0, q, cfg.k, cfg.sep) == (list(d[:nd]), ml, me)
        lens.append(ml)
    assert max(lens) >= 8 and min(lens) <= 2           # the windows exercise long and short matches


def test_error_codes():
    with pytest.raises(A.AgentSamError) as e:
        A.sam_build([1, -2, 3], sep_token=9)
    assert e.value.code == -7 and "negative" in str(e.value)
    s = A.sam_build([], sep_token=9)
    assert A.sam_flat_sizes(s) == (1, 0, 0)
    f = A.sam_flatten([s])
    assert list(f.row_ptr) == [0, 0] and f.lastpos[0] == -1
    assert A.strerror(0) == "ok" and A.strerror(-4).startswith("workspace")
    with pytest.raises(A.AgentSamError):                      # a tuning word with an undefined schedule
        A.spec_verify_attn_workspace(1, 5, 4, 1, 64, 64, 4, A.F32, tuning=3)


def test_build_rate_is_linear_and_above_the_papers_figure():
    """Sec. 5.4.3: construction is linear in the prompt; ~1 s for 128k tokens on the paper's host."""
    import time
    cfg = W.scaled(W.baseline_config(1), sam_session_len=131072)
    T = W.token_memory(cfg)
    t0 = time.perf_counter(); s = A.sam_build(T, cfg.sep); t1 = time.perf_counter() - t0
    ns, ne, nt = A.sam_flat_sizes(s)
    assert nt == 131072 and ns <= 2 * nt and ne <= 3 * nt
    assert t1 < 2.0
