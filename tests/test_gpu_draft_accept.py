"""GPU parity of sam_draft and spec_accept against the CPU oracle (bit-exact), through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2512_18337_amd as A
from paper_2512_18337_amd import workloads as W
from _util import draft_inputs, make_memories, oracle_drafts, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run_draft(cfg, min_match=1, recent_override=None):
    mems = make_memories(cfg)
    flat, root, cbeg, cend, recent, rlen = draft_inputs(cfg, mems)
    if recent_override is not None:
        recent, rlen = recent_override(recent, rlen)
    fd = flat.to(DEV)
    d, nd, ml, me = A.sam_draft(fd, root, cend, recent, rlen, cfg.k, cfg.sep, min_match)
    torch.cuda.synchronize()
    od, ond, oml, ome = oracle_drafts(cfg, mems, recent, rlen, min_match)
    me = to_np(me).astype(np.int64)
    me_rel = np.where(me >= 0, me - cbeg, -1)
    assert np.array_equal(to_np(ml), oml)
    assert np.array_equal(me_rel, ome)
    assert np.array_equal(to_np(nd), ond)
    assert np.array_equal(to_np(d), od)
    # the same without the table of wide states (their sorted rows are searched instead)
    d2, nd2, ml2, me2 = A.sam_draft(fd, root, cend, recent, rlen, cfg.k, cfg.sep, min_match, use_wide_table=False)
    torch.cuda.synchronize()
    assert torch.equal(d2, d) and torch.equal(nd2, nd) and torch.equal(ml2, ml) and np.array_equal(to_np(me2), me)
    return to_np(d), to_np(nd), to_np(ml)


@pytest.mark.parametrize("i", [0, 1, 2, 3, 4])
def test_sam_draft_full_size(i):
    """Every baseline workload at its full memory size: drafts, lengths and end positions bit-exact."""
    cfg = W.baseline_config(i)
    print(f"sam_draft parity {cfg.name}", flush=True)
    d, nd, ml = _run_draft(cfg)
    assert (nd > 0).sum() >= cfg.B // 2 and ml.max() >= min(8, cfg.m - 1)


def test_sam_draft_edge_cases():
    cfg = W.scaled(W.baseline_config(2), B=16, sam_sessions=8, sam_session_len=512)

    def override(recent, rlen):
        recent, rlen = recent.copy(), rlen.copy()
        rlen[0] = 0                                   # empty window -> no proposal
        rlen[1] = 1
        rlen[2] = 7
        recent[3] = cfg.vocab - 1 - np.arange(cfg.m) % 3  # ids that (almost surely) never occur
        return recent, rlen
    d, nd, ml = _run_draft(cfg, recent_override=override)
    assert nd[0] == 0 and ml[0] == 0
    _run_draft(cfg, min_match=5)
    _run_draft(W.scaled(cfg, k=0))
    _run_draft(W.scaled(cfg, k=64, m=64))
    _run_draft(W.scaled(cfg, m=1))
    # a memory with tiny vocabulary: wide repeats, long suffix-link chains, many clones
    _run_draft(W.scaled(cfg, vocab=3, zipf_s=0.0, sam_sessions=4, sam_session_len=700))
    # a root wider than 64 transitions per probe round is covered by the full-size cases (vocab 32000+)


@pytest.mark.parametrize("seed", range(12))
def test_sam_draft_seeded_random_memories(seed):
    """Memory shape, vocabulary, repetitiveness, window and draft lengths drawn from a seeded generator."""
    rng = np.random.default_rng(500 + seed)
    kw = dict(B=int(rng.choice([1, 3, 17, 40])), vocab=int(rng.choice([2, 5, 70, 3000, 60000])),
              zipf_s=float(rng.choice([0.0, 1.1])), copy_frac=float(rng.choice([0.0, 0.3, 0.8])),
              span=(int(rng.integers(2, 9)), int(rng.integers(9, 200))),
              sam_mode=str(rng.choice(["per_session", "shared"])), sam_sessions=int(rng.integers(1, 6)),
              sam_session_len=int(rng.choice([40, 700, 6000])), m=int(rng.choice([1, 7, 32, 64])),
              k=int(rng.choice([0, 1, 8, 33, 64])))
    print(f"sam_draft random memory {seed}: {kw}", flush=True)
    _run_draft(W.scaled(W.baseline_config(1), **kw), min_match=int(rng.choice([1, 1, 3])))


def test_sam_draft_empty_memory():
    s = A.sam_build([], sep_token=5)
    fd = A.sam_flatten([s]).to(DEV)
    recent = np.array([[1, 2, 3, 4]], dtype=np.int32)
    d, nd, ml, me = A.sam_draft(fd, [0], [0], recent, [4], 3, 5)
    torch.cuda.synchronize()
    assert to_np(nd)[0] == 0 and to_np(ml)[0] == 0 and to_np(me)[0] == -1 and list(to_np(d)[0]) == [-1, -1, -1]


def _accept_case(cfg, draft, n_draft):
    from oracle import accept_oracle
    logits = W.verify_logits(cfg, draft, n_draft, DEV)
    a, out, tgt = A.spec_accept(logits, torch.as_tensor(draft, device=DEV), torch.as_tensor(n_draft, device=DEV))
    torch.cuda.synchronize()
    oa, oout, otgt = accept_oracle(to_np(logits), draft, n_draft)
    assert np.array_equal(to_np(tgt), otgt)
    assert np.array_equal(to_np(a), oa)
    assert np.array_equal(to_np(out), oout)
    return oa


@pytest.mark.parametrize("i", [0, 1, 2, 3, 4])
def test_spec_accept_full_size(i):
    """Full logits shapes of every baseline workload; drafts come from the oracle's lookup."""
    cfg = W.baseline_config(i)
    print(f"spec_accept parity {cfg.name}", flush=True)
    mems = make_memories(cfg)
    recent, rlen = W.recent_windows(cfg, mems)
    od, ond, _, _ = oracle_drafts(cfg, mems, recent, rlen)
    oa = _accept_case(cfg, od, ond)
    assert np.all(oa <= ond) and (cfg.B < 16 or 0 < oa.sum())


def test_spec_accept_edge_cases():
    from oracle import accept_oracle
    rng = np.random.default_rng(3)
    # ties, NaN, -inf rows, odd vocab sizes (unaligned rows), bf16, k = 0
    for (B, k, V, dt) in [(3, 4, 1, torch.float32), (5, 2, 7, torch.float32), (4, 3, 1001, torch.bfloat16),
                          (2, 0, 333, torch.float32), (6, 5, 4099, torch.bfloat16), (3, 63, 130, torch.float32)]:
        lg = (torch.randn(B, k + 1, V) * 3).round().div(3).to(dt)     # coarse values -> exact ties
        if V > 6:
            lg[0, 0, 2] = float("nan"); lg[0, 0, 5] = float("inf"); lg[0, 0, 6] = float("inf")
            lg[B - 1, k] = float("-inf")
        lgd = lg.to(DEV)
        tg = np.argmax(np.nan_to_num(to_np(lg), nan=-np.inf), axis=2).astype(np.int32)
        draft = tg[:, :k].copy()
        if k:
            draft[0, rng.integers(0, k)] += 1
        nd = rng.integers(0, k + 1, B).astype(np.int32)
        a, out, tgt = A.spec_accept(lgd, torch.as_tensor(draft, device=DEV).reshape(B, k), torch.as_tensor(nd, device=DEV))
        torch.cuda.synchronize()
        oa, oout, otgt = accept_oracle(to_np(lg), draft, nd)
        assert np.array_equal(to_np(tgt), otgt) and np.array_equal(to_np(a), oa) and np.array_equal(to_np(out), oout)
    # a misaligned base pointer (row start not on a 16-byte boundary)
    base = torch.randn(2 * 3 * 515 + 1, device=DEV)
    lg = base[1:].view(2, 3, 515)
    draft = np.zeros((2, 2), np.int32); nd = np.array([2, 2], np.int32)
    a, out, tgt = A.spec_accept(lg, torch.as_tensor(draft, device=DEV), torch.as_tensor(nd, device=DEV))
    torch.cuda.synchronize()
    assert np.array_equal(to_np(tgt), accept_oracle(to_np(lg), draft, nd)[2])


def test_spec_accept_long_rows_special_values_and_calls_on_two_streams():
    """Few rows of a long vocabulary with the maximum occurring many times, as -0 and +0, rows that are half NaN,
    all NaN, all -inf, with several +inf; many calls back to back and on two streams, every one equal to the
    oracle; then a batch of 9000 short rows."""
    from oracle import accept_oracle
    rng = np.random.default_rng(11)
    B, k, V = 3, 2, 200003                                    # 9 rows x 800 KB (fp32): the maximum split
    lg = (torch.randn(B, k + 1, V) * 2).round().div(2)        # coarse values: the maximum occurs many times
    lg[0, 0] = torch.where(lg[0, 0] >= lg[0, 0].max(), torch.tensor(0.0), -lg[0, 0].abs())   # maximum 0 ...
    lg[0, 0, 150000] = -0.0; lg[0, 0, 70001] = 0.0            # ... as -0 and +0 in different segments
    lg[0, 1, ::2] = float("nan"); lg[0, 2] = float("-inf")    # half a row NaN; a row without a finite maximum
    lg[1, 0, 199999] = float("inf"); lg[1, 0, 31] = float("inf")
    lg[1, 1] = float("nan")
    for dt in (torch.float32, torch.bfloat16):
        lgd = lg.to(dt).to(DEV)
        ref = np.nan_to_num(to_np(lg.to(dt)), nan=-np.inf)
        tg = np.argmax(ref, axis=2).astype(np.int32)
        draft = tg[:, :k].copy(); draft[2, 1] += 1
        nd = np.array([2, 1, 2], np.int32)
        oa, oout, otgt = accept_oracle(to_np(lg.to(dt)), draft, nd)
        assert np.array_equal(otgt, tg) and otgt[0, 2] == 0 and otgt[1, 1] == 0
        dd, ndd = torch.as_tensor(draft, device=DEV), torch.as_tensor(nd, device=DEV)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        results = []
        for rep in range(40):
            results.append(A.spec_accept(lgd, dd, ndd))
            with torch.cuda.stream(side):
                results.append(A.spec_accept(lgd, dd, ndd))
        torch.cuda.synchronize()
        for a, out, tgt in results:
            assert np.array_equal(to_np(tgt), otgt) and np.array_equal(to_np(a), oa) and np.array_equal(to_np(out), oout)
    Bw, kw, Vw = 1500, 5, 257
    lgw = torch.randn(Bw, kw + 1, Vw, device=DEV)
    tgw = lgw.argmax(2).int()
    dw = tgw[:, :kw].contiguous(); ndw = torch.full((Bw,), kw, dtype=torch.int32, device=DEV)
    for rep in range(20):
        a, out, tgt = A.spec_accept(lgw, dw, ndw)
        assert torch.equal(tgt, tgw) and bool((a == kw).all())
