"""GPU parity of the maintained automaton copy (sam_delta_export -> sam_apply_delta -> sam_draft_delta)
against the CPU oracle on the grown memory, bit-exact, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2512_18337_amd as A
from oracle import draft_oracle
from paper_2512_18337_amd import workloads as W
from _util import to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _sync(sams, fd, flat, mem_len):
    """Bring the device copy up to date: every automaton's delta is uploaded and applied with one launch, its new
    transitions going into the one device overlay table (kept on `fd` between calls; re-created larger, and
    refilled with everything since the flatten, when it would get more than half full)."""
    n_ov = sum(A.sam_delta_sizes(s)[2] for s in sams)
    table = getattr(fd, "overlay", None)
    grow = table is None or 2 * n_ov > table[0].numel()
    if grow:
        cap = 2
        while cap < 2 * n_ov:
            cap *= 2
        table = fd.overlay = A.overlay_table(cap, device=DEV)
    for i, s in enumerate(sams):
        d = A.sam_delta_export(s, int(flat.roots[i]), int(flat.corpus_begin[i]), overlay_all=grow)
        assert int(flat.roots[i]) + d.flat_states == int(flat.rows_end[i])
        A.sam_apply_delta(d, fd.state_rec, fd.lastpos, table[0], table[1])
        n = d.new_tokens.shape[0]
        if n:
            at = int(flat.corpus_begin[i]) + mem_len[i]
            fd.corpus[at:at + n] = torch.as_tensor(d.new_tokens, device=DEV)
            mem_len[i] += n
    return table


def _windows(rng, mems, owner, m, vocab):
    B = len(owner)
    recent = np.zeros((B, m), np.int32); rlen = np.zeros(B, np.int32)
    for b in range(B):
        T = mems[owner[b]]
        if len(T) > m + 2 and rng.random() < 0.85:
            p = int(rng.integers(m, len(T)))                 # may end inside the freshly appended tail
            w = np.array(T[p - m:p], np.int32)
            w[m - 1 - int(rng.integers(1, m))] = int(rng.integers(0, vocab))
        else:
            w = rng.integers(0, vocab, m).astype(np.int32)
        recent[b], rlen[b] = w, m if rng.random() < 0.9 else int(rng.integers(0, m))
    return recent, rlen


@pytest.mark.parametrize("wide", [True, False])      # long flattened rows through the hash table / searched
@pytest.mark.parametrize("shared", [True, False])
def test_maintained_copy_on_device_matches_oracle(shared, wide):
    cfg = W.scaled(W.baseline_config(2), B=24, sam_sessions=6, sam_session_len=1500, vocab=2000, m=32, k=8)
    rng = np.random.default_rng(77 + int(shared))
    if shared:
        mems = [list(W.token_memory(cfg))]
        owner = [0] * cfg.B
    else:
        one = W.scaled(cfg, sam_mode="per_session", sam_sessions=1, sam_session_len=2500)
        mems = [list(W.token_memory(one, i)) for i in range(3)]
        owner = [b % 3 for b in range(cfg.B)]
    sams = [A.sam_build(np.asarray(T, np.int32), cfg.sep) for T in mems]
    grow = 1200
    flat = A.sam_flatten(sams, grow_tokens=grow)
    fd = flat.to(DEV)
    mem_len = [len(T) for T in mems]
    for rnd in range(12):
        for i, T in enumerate(mems):
            add = []
            for _ in range(int(rng.integers(1, 5))):         # a few spans: copies of earlier text and fresh tokens
                if rng.random() < 0.6 and len(T) > 50:
                    p = int(rng.integers(0, len(T) - 20)); add += T[p:p + int(rng.integers(2, 20))]
                else:
                    add += [int(x) for x in rng.integers(0, cfg.vocab, int(rng.integers(1, 9)))]
            if rnd % 4 == 1:
                add.append(cfg.sep)                          # a session ends inside the appended text
            add = add[:grow // 12 - 1]
            A.sam_append(sams[i], np.asarray(add, np.int32))
            T += add
        keys, dsts = _sync(sams, fd, flat, mem_len)
        assert mem_len == [len(T) for T in mems]
        cend = np.array([int(flat.corpus_begin[owner[b]]) + mem_len[owner[b]] for b in range(cfg.B)], np.int32)
        root = np.array([flat.roots[owner[b]] for b in range(cfg.B)], np.int32)
        rows_end = np.array([flat.rows_end[owner[b]] for b in range(cfg.B)], np.int32)
        recent, rlen = _windows(rng, mems, owner, cfg.m, cfg.vocab)
        print(f"maintained copy round {rnd}: overlay capacity {keys.numel()}", flush=True)
        d, nd, ml, me = A.sam_draft_delta(fd, keys, dsts, rows_end, root, cend, recent, rlen, cfg.k, cfg.sep,
                                          use_wide_table=wide)
        torch.cuda.synchronize()
        d, nd, ml, me = to_np(d), to_np(nd), to_np(ml), to_np(me)
        for b in range(cfg.B):
            T = np.asarray(mems[owner[b]], np.int32)
            q = recent[b, cfg.m - rlen[b]:]
            od, ond, oml, ome = draft_oracle(T, q, cfg.k, cfg.sep, 1)
            got_end = int(me[b]) - int(flat.corpus_begin[owner[b]]) if me[b] >= 0 else -1
            assert (int(ml[b]), got_end, int(nd[b])) == (oml, ome, ond), (rnd, b)
            assert list(d[b, :ond]) == list(od[:ond]) and (d[b, ond:] == -1).all()
    # a fresh flatten of the grown automata, read by the plain kernel, gives the same answers
    flat2 = A.sam_flatten(sams)
    d2, nd2, ml2, me2 = A.sam_draft(flat2.to(DEV), [flat2.roots[o] for o in owner], [flat2.corpus_end[o] for o in owner],
                                    recent, rlen, cfg.k, cfg.sep)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(d2), d) and np.array_equal(to_np(ml2), ml) and np.array_equal(to_np(nd2), nd)


def test_update_on_a_second_stream_next_to_other_work():
    """The device copy is updated on a second stream while the first is busy: ordered by one event (the
    round's lookup has finished) and one stream wait (the next lookup sees the whole update)."""
    cfg = W.scaled(W.baseline_config(2), B=16, sam_sessions=4, sam_session_len=1200, vocab=1500, m=32, k=8)
    rng = np.random.default_rng(99)
    mems = [list(W.token_memory(cfg))]
    owner = [0] * cfg.B
    sams = [A.sam_build(np.asarray(T, np.int32), cfg.sep) for T in mems]
    flat = A.sam_flatten(sams, grow_tokens=2000)
    fd = flat.to(DEV)
    mem_len = [len(T) for T in mems]
    root = torch.as_tensor(np.array([flat.roots[0]] * cfg.B, np.int32), device=DEV)
    rows_end = torch.as_tensor(np.array([flat.rows_end[0]] * cfg.B, np.int32), device=DEV)
    keys, dsts = _sync(sams, fd, flat, mem_len)
    cend = torch.as_tensor(np.array([int(flat.corpus_begin[0]) + mem_len[0]] * cfg.B, np.int32), device=DEV)
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    busy_a = torch.randn(2048, 2048, device=DEV)
    pending = []
    for rnd in range(8):
        recent, rlen = _windows(rng, mems, owner, cfg.m, cfg.vocab)
        got = A.sam_draft_delta(fd, keys, dsts, rows_end, root, cend, torch.as_tensor(recent, device=DEV),
                                torch.as_tensor(rlen, device=DEV), cfg.k, cfg.sep)
        looked_up = torch.cuda.Event()
        looked_up.record(main)
        for _ in range(6):                                    # stands in for the attention of the step
            busy_a = torch.tanh(busy_a @ busy_a * 1e-3)
        pending.append((got, recent, rlen, [list(T) for T in mems]))
        add = []
        for _ in range(3):
            p = int(rng.integers(0, len(mems[0]) - 30)); add += mems[0][p:p + int(rng.integers(2, 25))]
        add += [int(x) for x in rng.integers(0, cfg.vocab, 3)]
        A.sam_append(sams[0], np.asarray(add, np.int32))
        mems[0] += add
        with torch.cuda.stream(side):
            side.wait_event(looked_up)
            keys, dsts = _sync(sams, fd, flat, mem_len)
            cend = torch.as_tensor(np.array([int(flat.corpus_begin[0]) + mem_len[0]] * cfg.B, np.int32), device=DEV)
        main.wait_stream(side)
    torch.cuda.synchronize()
    for (d, nd, ml, me), recent, rlen, snap in pending:       # every round's lookup saw exactly its own memory
        d, nd, ml, me = to_np(d), to_np(nd), to_np(ml), to_np(me)
        for b in range(cfg.B):
            od, ond, oml, ome = draft_oracle(np.asarray(snap[0], np.int32), recent[b, cfg.m - rlen[b]:], cfg.k, cfg.sep, 1)
            got_end = int(me[b]) - int(flat.corpus_begin[0]) if me[b] >= 0 else -1
            assert (int(ml[b]), got_end, int(nd[b])) == (oml, ome, ond)
            assert list(d[b, :ond]) == list(od[:ond])


def test_draft_delta_argument_errors():
    """Bad sizes and missing arrays are refused on the host; nothing is launched."""
    z = torch.zeros(8, dtype=torch.int32, device=DEV)
    L = A.binding.lib()
    p, n = A.binding._dp(z), A.binding._vp(0)

    def call(B=1, m=4, k=2, cap=8, ov=p, wide=n, wide_slots=0, arrays=p):
        return L.sam_draft_delta(arrays, arrays, arrays, arrays, arrays, arrays, ov, ov, cap, arrays, arrays, arrays,
                                 arrays, arrays, B, m, k, 1, 9, arrays, arrays, arrays, arrays, wide, wide_slots, n)

    assert call(cap=6) != 0                                   # overlay capacity not a power of two
    assert call(cap=0) != 0
    assert call(ov=n) != 0                                    # no overlay table
    assert call(wide=p, wide_slots=6) != 0                    # wide table size not a power of two
    assert call(wide=p, wide_slots=0) != 0
    assert call(m=65) != 0 and call(k=65) != 0 and call(B=-1) != 0
    assert call(arrays=n) != 0                                # missing automaton arrays
    assert call(B=0, arrays=n) == 0                           # an empty batch is a no-op
    torch.cuda.synchronize()


@pytest.mark.parametrize("i", [2, 3])
def test_maintained_copy_full_size(i):
    """The shared automata of workloads 2 and 3 at their full size (262 k / 2 M tokens, vocabularies of 32 k
    / 152 k, so the root's row is tens of thousands of transitions wide): three rounds of appended text,
    every session's lookup on the maintained copy against the oracle on the grown memory."""
    from _util import make_memories
    from oracle import draft_oracle_batch
    cfg = W.baseline_config(i)
    rng = np.random.default_rng(500 + i)
    mems = [list(m) for m in make_memories(cfg)]
    assert len(mems) == 1
    owner = [0] * cfg.B
    sams = [A.sam_build(np.asarray(mems[0], np.int32), cfg.sep)]
    grow = 4096
    flat = A.sam_flatten(sams, grow_tokens=grow)
    fd = flat.to(DEV)
    mem_len = [len(mems[0])]
    root = np.array([flat.roots[0]] * cfg.B, np.int32)
    rows_end = np.array([flat.rows_end[0]] * cfg.B, np.int32)
    for rnd in range(3):
        T = mems[0]
        add = []
        for _ in range(40):                                   # copies of earlier text and fresh tokens
            if rng.random() < 0.7:
                p = int(rng.integers(0, len(T) - 40)); add += T[p:p + int(rng.integers(2, 40))]
            else:
                add += [int(x) for x in rng.integers(0, cfg.vocab, int(rng.integers(1, 9)))]
        add = add[:grow // 3 - 2] + ([cfg.sep] if rnd == 1 else [])
        A.sam_append(sams[0], np.asarray(add, np.int32))
        T += add
        keys, dsts = _sync(sams, fd, flat, mem_len)
        cend = np.array([int(flat.corpus_begin[0]) + mem_len[0]] * cfg.B, np.int32)
        recent, rlen = _windows(rng, mems, owner, cfg.m, cfg.vocab)
        print(f"maintained copy, workload {i}, round {rnd}: overlay capacity {keys.numel()}", flush=True)
        d, nd, ml, me = A.sam_draft_delta(fd, keys, dsts, rows_end, root, cend, recent, rlen, cfg.k, cfg.sep)
        torch.cuda.synchronize()
        Tn = np.asarray(T, np.int32)
        od, ond, oml, ome = draft_oracle_batch(Tn, np.zeros(cfg.B, np.int64), np.full(cfg.B, len(Tn), np.int64),
                                               recent, rlen, cfg.k, cfg.sep)
        d, nd, ml, me = to_np(d), to_np(nd), to_np(ml), to_np(me)
        assert np.array_equal(nd, ond) and np.array_equal(ml, oml)
        assert np.array_equal(np.where(me >= 0, me - int(flat.corpus_begin[0]), -1), ome)
        for b in range(cfg.B):
            assert list(d[b, :ond[b]]) == list(od[b, :ond[b]]) and (d[b, ond[b]:] == -1).all()
        assert ml.max() > 8                                   # the windows really matched
