"""GPU parity of sam_draft_step (matched state carried from call to call) against the carried-match oracle,
bit-exact, through the C ABI: on a flattened automaton (with and without the wide-state table) and on a
maintained device copy whose memory grows between the calls."""
import numpy as np
import pytest
import torch

import paper_2512_18337_amd as A
from oracle import draft_step_oracle
from paper_2512_18337_amd import workloads as W
from _util import to_np
from test_gpu_sam_delta import _sync

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _next_tokens(rng, T, ctx, vocab, lo, hi):
    """What a session produces next: mostly text that continues a span of the memory, sometimes noise."""
    n = int(rng.integers(lo, hi + 1))
    out = []
    while len(out) < n:
        r = rng.random()
        if r < 0.75 and len(T) > 40:
            p = int(rng.integers(0, len(T) - 30)); out += [int(x) for x in T[p:p + int(rng.integers(3, 30))]]
        else:
            out += [int(x) for x in rng.integers(0, vocab, int(rng.integers(1, 4)))]
    return out[:n]


def _check_step(tag, mems, owner, ctxs, L_prev, n_new, got, cur_len, corpus_begin, k, sep):
    d, nd, ml, me = (to_np(x) for x in got)
    cl = to_np(cur_len)
    for b in range(len(owner)):
        T = np.asarray(mems[owner[b]], np.int32)
        L, od, ond, oml, ome = draft_step_oracle(T, np.asarray(ctxs[b], np.int32), L_prev[b], n_new[b], k, sep, 1)
        got_end = int(me[b]) - int(corpus_begin[owner[b]]) if me[b] >= 0 else -1
        assert int(cl[b]) == L, (tag, b, int(cl[b]), L)
        assert (int(ml[b]), got_end, int(nd[b])) == (oml, ome, ond), (tag, b)
        assert list(d[b, :ond]) == list(od[:ond]) and (d[b, ond:] == -1).all(), (tag, b)
        L_prev[b] = L
    return max(L_prev)


@pytest.mark.parametrize("wide", [True, False])
def test_carried_state_on_a_flattened_automaton(wide):
    cfg = W.scaled(W.baseline_config(2), B=20, sam_sessions=6, sam_session_len=1500, vocab=2000, m=32, k=8)
    rng = np.random.default_rng(31 + int(wide))
    mems = [list(W.token_memory(cfg))]
    # filter separators out of what sessions "say": a context never holds the separator
    owner = [0] * cfg.B
    sams = [A.sam_build(np.asarray(T, np.int32), cfg.sep) for T in mems]
    flat = A.sam_flatten(sams)
    fd = flat.to(DEV)
    root = np.array([flat.roots[o] for o in owner], np.int32)
    cend = np.array([flat.corpus_end[o] for o in owner], np.int32)
    cur_state = torch.full((cfg.B,), -1, dtype=torch.int32, device=DEV)
    cur_len = torch.zeros((cfg.B,), dtype=torch.int32, device=DEV)
    ctxs = [[] for _ in range(cfg.B)]
    L_prev = [0] * cfg.B
    sizes = [(100, 150), (0, 9), (1, 9), (1, 9), (0, 3), (60, 70), (1, 9), (1, 2)]   # first call: the prompt; one call > 64
    longest = 0
    for step, (lo, hi) in enumerate(sizes):
        new = [[t for t in _next_tokens(rng, mems[0], ctxs[b], cfg.vocab, lo, hi) if t != cfg.sep] for b in range(cfg.B)]
        if step == 3:
            new[0] = []                                       # a session with nothing new this call
        max_new = max(1, max(len(x) for x in new))
        tok = np.full((cfg.B, max_new), -7, np.int32)
        n_new = np.array([len(x) for x in new], np.int32)
        for b in range(cfg.B):
            tok[b, :len(new[b])] = new[b]
            ctxs[b] += new[b]
        print(f"draft step {step}: max_new {max_new} wide {wide}", flush=True)
        got = A.sam_draft_step(fd, root, cend, tok, n_new, cur_state, cur_len, cfg.k, cfg.sep, use_wide_table=wide)
        torch.cuda.synchronize()
        longest = max(longest, _check_step((wide, step), mems, owner, ctxs, L_prev, n_new, got, cur_len,
                                           flat.corpus_begin, cfg.k, cfg.sep))
    assert longest > 8                                        # the stream really carried long matches


@pytest.mark.parametrize("wide", [True, False])      # long flattened rows through the hash table / searched
def test_carried_state_on_a_growing_memory(wide):
    cfg = W.scaled(W.baseline_config(2), B=18, sam_sessions=1, sam_session_len=2500, vocab=1500, m=32, k=8,
                   sam_mode="per_session")
    rng = np.random.default_rng(303)
    mems = [list(W.token_memory(cfg, i)) for i in range(3)]
    owner = [b % 3 for b in range(cfg.B)]
    sams = [A.sam_build(np.asarray(T, np.int32), cfg.sep) for T in mems]
    grow = 1500
    flat = A.sam_flatten(sams, grow_tokens=grow)
    fd = flat.to(DEV)
    mem_len = [len(T) for T in mems]
    root = np.array([flat.roots[o] for o in owner], np.int32)
    rows_end = np.array([flat.rows_end[o] for o in owner], np.int32)
    cur_state = torch.full((cfg.B,), -1, dtype=torch.int32, device=DEV)
    cur_len = torch.zeros((cfg.B,), dtype=torch.int32, device=DEV)
    ctxs = [[] for _ in range(cfg.B)]
    L_prev = [0] * cfg.B
    for step in range(10):
        # the memories grow: mostly by what their own sessions said last (their contexts' tails), which is
        # what splits the very states the sessions stand in
        for i, T in enumerate(mems):
            add = []
            for b in range(cfg.B):
                if owner[b] == i and ctxs[b] and rng.random() < 0.6:
                    add += ctxs[b][-int(rng.integers(2, 12)):] + [int(rng.integers(0, cfg.vocab))]
            add += [int(x) for x in rng.integers(0, cfg.vocab, int(rng.integers(1, 6)))]
            if step % 4 == 2:
                add.append(cfg.sep)
            add = add[:grow // 10 - 1]
            A.sam_append(sams[i], np.asarray(add, np.int32))
            T += add
        keys, dsts = _sync(sams, fd, flat, mem_len)
        cend = np.array([int(flat.corpus_begin[owner[b]]) + mem_len[owner[b]] for b in range(cfg.B)], np.int32)
        lo, hi = ((40, 80) if step == 0 else (0, 9))
        new = [[t for t in _next_tokens(rng, mems[owner[b]], ctxs[b], cfg.vocab, lo, hi) if t != cfg.sep]
               for b in range(cfg.B)]
        max_new = max(1, max(len(x) for x in new))
        tok = np.full((cfg.B, max_new), -7, np.int32)
        n_new = np.array([len(x) for x in new], np.int32)
        for b in range(cfg.B):
            tok[b, :len(new[b])] = new[b]
            ctxs[b] += new[b]
        print(f"draft step on growing memory {step}: overlay capacity {keys.numel()}", flush=True)
        got = A.sam_draft_step(fd, root, cend, tok, n_new, cur_state, cur_len, cfg.k, cfg.sep,
                               overlay_key=keys, overlay_dst=dsts, rows_end=rows_end, use_wide_table=wide)
        torch.cuda.synchronize()
        _check_step(step, mems, owner, ctxs, L_prev, n_new, got, cur_len, flat.corpus_begin, cfg.k, cfg.sep)


def test_draft_step_argument_errors():
    z = torch.zeros(4, dtype=torch.int32, device=DEV)
    L = A.binding.lib()
    p = A.binding._dp
    n = A.binding._vp(0)

    def call(B=1, k=8, cur=p(z), arrays=p(z)):
        return L.sam_draft_step(arrays, arrays, arrays, arrays, arrays, arrays, n, n, 0, n, n, 0, arrays, arrays,
                                arrays, arrays, B, 1, k, 1, 9, cur, cur, arrays, arrays, arrays, arrays, n)

    assert call(k=65) != 0                                    # k out of range
    assert call(B=-1) != 0
    assert call(cur=n) != 0                                   # missing carried-state arrays
    assert call(B=0, cur=n, arrays=n) == 0                    # an empty batch is a no-op
    torch.cuda.synchronize()


def test_draft_step_edges_min_match_no_drafts_reset_and_empty_call():
    """min_match above the carried length suppresses the proposal but not the state; k = 0 keeps only the
    state; setting cur_len to 0 starts a session afresh; a call with no new tokens repeats the proposal."""
    cfg = W.scaled(W.baseline_config(2), B=6, sam_sessions=4, sam_session_len=800, vocab=500, m=32, k=5)
    rng = np.random.default_rng(8)
    T = list(W.token_memory(cfg))
    sams = [A.sam_build(np.asarray(T, np.int32), cfg.sep)]
    flat = A.sam_flatten(sams)
    fd = flat.to(DEV)
    root = np.full(cfg.B, flat.roots[0], np.int32)
    cend = np.full(cfg.B, flat.corpus_end[0], np.int32)
    cur_state = torch.full((cfg.B,), -1, dtype=torch.int32, device=DEV)
    cur_len = torch.zeros((cfg.B,), dtype=torch.int32, device=DEV)
    # every session consumes a span of the memory of a different length (1 .. 6 tokens, no separator inside)
    ctxs, tok = [], np.zeros((cfg.B, 8), np.int32)
    for b in range(cfg.B):
        while True:
            p = int(rng.integers(0, len(T) - 40))
            span = T[p:p + b + 1]
            if cfg.sep not in T[p:p + 20]:
                break
        ctxs.append(list(span)); tok[b, :b + 1] = span
    n_new = np.arange(1, cfg.B + 1, dtype=np.int32)
    min_match = 4
    d, nd, ml, me = (to_np(x) for x in A.sam_draft_step(fd, root, cend, tok, n_new, cur_state, cur_len, cfg.k, cfg.sep,
                                                         min_match=min_match))
    torch.cuda.synchronize()
    cl = to_np(cur_len)
    for b in range(cfg.B):
        L, od, ond, oml, ome = draft_step_oracle(np.asarray(T, np.int32), np.asarray(ctxs[b], np.int32), 0, b + 1, cfg.k,
                                                 cfg.sep, min_match)
        assert int(cl[b]) == L == b + 1                       # the whole span matches
        assert (int(nd[b]), int(ml[b]), int(me[b])) == (ond, oml, ome) and list(d[b, :ond]) == list(od[:ond])
        if b + 1 < min_match:
            assert nd[b] == 0 and ml[b] == 0 and me[b] == -1   # too short a match proposes nothing
    # no new tokens, no drafts asked for: the state stays, the outputs are those of k = 0
    zero = np.zeros(cfg.B, np.int32)
    before = (to_np(cur_state).copy(), to_np(cur_len).copy())
    d0, nd0, ml0, me0 = A.sam_draft_step(fd, root, cend, tok, zero, cur_state, cur_len, 0, cfg.sep)
    torch.cuda.synchronize()
    assert d0.shape == (cfg.B, 0) and (to_np(nd0) == 0).all()
    assert np.array_equal(to_np(cur_state), before[0]) and np.array_equal(to_np(cur_len), before[1])
    assert np.array_equal(to_np(ml0), np.arange(1, cfg.B + 1))    # min_match 1: every carried match counts
    # session 2 starts afresh: its next token is matched from the root
    cur_len[2] = 0
    one = np.zeros(cfg.B, np.int32); one[2] = 1
    tok2 = np.zeros((cfg.B, 1), np.int32); tok2[2, 0] = ctxs[2][0]
    A.sam_draft_step(fd, root, cend, tok2, one, cur_state, cur_len, cfg.k, cfg.sep)
    torch.cuda.synchronize()
    cl = to_np(cur_len)
    assert cl[2] == 1 and np.array_equal(np.delete(cl, 2), np.delete(before[1], 2))


@pytest.mark.parametrize("i", [2, 4])
def test_draft_step_full_size_memory(i):
    """The baseline workloads' full-size memories (workload 2: one 256k-token automaton for all sessions;
    workload 4: 1M tokens, long repeats): the window as the first call, then what a step commits."""
    from _util import draft_inputs, make_memories
    cfg = W.baseline_config(i)
    mems = make_memories(cfg)
    flat, root, cbeg, cend, recent, rlen = draft_inputs(cfg, mems)
    fd = flat.to(DEV)
    B = cfg.B
    sample = list(range(0, B, max(1, B // 12)))               # the oracle scans the whole memory per candidate length
    T = [np.asarray(mems[b if cfg.sam_mode == "per_session" else 0], np.int32) for b in range(B)]
    cur_state = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    cur_len = torch.zeros((B,), dtype=torch.int32, device=DEV)
    tok = np.zeros((B, cfg.m), np.int32)
    for b in range(B):
        tok[b, :rlen[b]] = recent[b, cfg.m - rlen[b]:]
    ctxs = [list(tok[b, :rlen[b]]) for b in range(B)]
    L_prev = [0] * B
    print(f"draft step full size {cfg.name}: first call", flush=True)
    got = A.sam_draft_step(fd, root, cend, tok, rlen, cur_state, cur_len, cfg.k, cfg.sep)
    torch.cuda.synchronize()
    # on an unchanging memory the carried match of the window is what the window lookup finds
    ref = A.sam_draft(fd, root, cend, recent, rlen, cfg.k, cfg.sep)
    torch.cuda.synchronize()
    for x, y in zip(got, ref):
        assert torch.equal(x, y)
    d, nd = to_np(got[0]), to_np(got[1])
    cl, ml, me = to_np(cur_len), to_np(got[2]), to_np(got[3])
    for b in sample:
        L, od, ond, oml, ome = draft_step_oracle(T[b], np.asarray(ctxs[b], np.int32), 0, len(ctxs[b]), cfg.k, cfg.sep, 1)
        assert (int(cl[b]), int(ml[b]), int(nd[b])) == (L, oml, ond), b
        assert (int(me[b]) - int(cbeg[b]) if me[b] >= 0 else -1) == ome and list(d[b, :ond]) == list(od[:ond])
        L_prev[b] = L
    # second call: the first drafts are accepted, then a token that breaks the match
    rng = np.random.default_rng(cfg.seed + 17)
    new = [[int(t) for t in d[b, :min(int(nd[b]), 3)]] + [int(rng.integers(0, cfg.vocab))] for b in range(B)]
    tok2 = np.zeros((B, 4), np.int32)
    n2 = np.array([len(x) for x in new], np.int32)
    for b in range(B):
        tok2[b, :len(new[b])] = new[b]
        ctxs[b] += new[b]
    print(f"draft step full size {cfg.name}: second call", flush=True)
    got = A.sam_draft_step(fd, root, cend, tok2, n2, cur_state, cur_len, cfg.k, cfg.sep)
    torch.cuda.synchronize()
    d, nd, ml, me = (to_np(x) for x in got)
    cl = to_np(cur_len)
    for b in sample:
        L, od, ond, oml, ome = draft_step_oracle(T[b], np.asarray(ctxs[b], np.int32), L_prev[b], int(n2[b]), cfg.k, cfg.sep, 1)
        assert (int(cl[b]), int(ml[b]), int(nd[b])) == (L, oml, ond), b
        assert (int(me[b]) - int(cbeg[b]) if me[b] >= 0 else -1) == ome and list(d[b, :ond]) == list(od[:ond])


def test_carried_state_across_a_flatten_on_the_child_thread():
    """The whole maintenance cycle: the memory grows through the builder's queue, the device copy follows by
    deltas, and when the log of transitions exceeds the stated fraction the automaton is flattened again ON THE
    CHILD THREAD into new arrays, which are uploaded and swapped in (with an empty overlay) between two steps.
    The (state, length) pairs the sessions carry stay valid across the swap: every step equals the oracle."""
    from paper_2512_18337_amd import binding
    import ctypes
    cfg = W.scaled(W.baseline_config(2), B=16, sam_sessions=4, sam_session_len=1500, vocab=1500, m=32, k=8)
    rng = np.random.default_rng(909)
    T = list(W.token_memory(cfg))
    bld = A.SamBuilder()
    bld.submit(1, np.asarray(T, np.int32), cfg.sep)
    bld.wait(1)
    sam, _ = bld.poll(1)
    grow = 4000
    flat = A.sam_flatten([sam], grow_tokens=grow)
    fd = flat.to(DEV)
    mems, owner, mem_len = [T], [0] * cfg.B, [len(T)]
    root = np.zeros(cfg.B, np.int32)
    cur_state = torch.full((cfg.B,), -1, dtype=torch.int32, device=DEV)
    cur_len = torch.zeros((cfg.B,), dtype=torch.int32, device=DEV)
    ctxs = [[] for _ in range(cfg.B)]
    L_prev = [0] * cfg.B
    swaps = 0
    for step in range(14):
        add = []
        for b in range(cfg.B):
            if ctxs[b] and rng.random() < 0.6:
                add += ctxs[b][-int(rng.integers(2, 12)):] + [int(rng.integers(0, cfg.vocab))]
        add += [int(x) for x in rng.integers(0, cfg.vocab, int(rng.integers(1, 6)))]
        if step % 5 == 3:
            add.append(cfg.sep)
        bld.submit(1, np.asarray(add, np.int32), cfg.sep)
        T += add
        bld.wait(1)
        sam, _ = bld.poll(1)
        if A.sam_reflatten_due(sam, 0.04):
            # flatten again off this thread, into arrays with room to grow, then swap the device copy
            ns, ne, nt = A.sam_flat_sizes(sam)
            fill = lambda n: np.full(n, -1, np.int32)
            cap_s, cap_t = ns + 2 * grow, nt + grow
            out = A.FlatSam(fill(cap_s), fill(cap_s), np.zeros(cap_s + 1, np.int32), fill(max(ne, 1)), fill(max(ne, 1)),
                            fill(cap_s), fill(cap_t), fill(4 * cap_s), np.zeros(1, np.int32), np.zeros(1, np.int32),
                            np.array([nt], np.int32), np.array([ns], np.int32))
            bld.flatten(1, out)
            bld.wait(1)
            assert bld.flatten_result(1) == 0
            sam, _ = bld.poll(1)
            out.row_ptr[ns:] = ne                             # states without a row yet
            slots = ctypes.c_int64()
            assert binding.lib().sam_wide_slots(sam._h, ctypes.byref(slots)) == 0
            out.wide_table = np.full(4 * slots.value, -1, np.int32)
            assert binding.lib().sam_wide_table(sam._h, 0, out.wide_table.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                                slots.value) == 0
            flat, fd = out, out.to(DEV)                       # the swap: new arrays, no overlay yet
            mem_len = [nt]
            swaps += 1
            assert A.sam_delta_sizes(sam)[:5] == (0, 0, 0, 0, 0)
        keys, dsts = _sync([sam], fd, flat, mem_len)
        rows_end = np.full(cfg.B, int(flat.rows_end[0]), np.int32)
        cend = np.full(cfg.B, mem_len[0], np.int32)
        lo, hi = ((40, 80) if step == 0 else (0, 9))
        new = [[t for t in _next_tokens(rng, T, ctxs[b], cfg.vocab, lo, hi) if t != cfg.sep] for b in range(cfg.B)]
        max_new = max(1, max(len(x) for x in new))
        tok = np.full((cfg.B, max_new), -7, np.int32)
        n_new = np.array([len(x) for x in new], np.int32)
        for b in range(cfg.B):
            tok[b, :len(new[b])] = new[b]
            ctxs[b] += new[b]
        print(f"draft step {step}: flattened again {swaps} times, overlay capacity {keys.numel()}", flush=True)
        got = A.sam_draft_step(fd, root, cend, tok, n_new, cur_state, cur_len, cfg.k, cfg.sep,
                               overlay_key=keys, overlay_dst=dsts, rows_end=rows_end)
        torch.cuda.synchronize()
        _check_step(step, mems, owner, ctxs, L_prev, n_new, got, cur_len, flat.corpus_begin, cfg.k, cfg.sep)
    assert swaps >= 2
    bld.close()
