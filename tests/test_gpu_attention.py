"""GPU parity of spec_verify_attn against the fp64 oracle, through the C ABI.

Tolerances (max-abs): 1e-5 for fp32 storage, 2e-2 for bf16 storage with fp32 accumulation.
For bf16 the tests additionally hold the kernel to 3e-3, which is what rounding the
softmax weights to bf16 (relative 2^-9 per term) allows on N(0,1) values.
"""
import numpy as np
import pytest
import torch

import paper_2512_18337_amd as A
from paper_2512_18337_amd import workloads as W
from _util import oracle_attention_sample, to_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {"f32": 1e-5, "bf16": 2e-2}
TIGHT = {"f32": 1e-5, "bf16": 3e-3}


def _inputs(cfg):
    lay = W.kv_layout(cfg)
    q, kc, vc = W.kv_and_queries(cfg, lay, DEV)
    bt = torch.as_tensor(lay.block_table, device=DEV)
    seq = torch.as_tensor(lay.seq_lens, device=DEV)
    return lay, q, kc, vc, bt, seq


def _check(cfg, lay, q, kc, vc, out, pairs, dominated=False):
    scale = 1.0 / np.sqrt(cfg.D)
    ref = oracle_attention_sample(q, kc, vc, lay.block_table, lay.seq_lens, scale, pairs)
    o = to_np(out)
    worst = 0.0
    for (b, h), r in ref.items():
        worst = max(worst, float(np.max(np.abs(o[b, :, h] - r))))
    assert np.isfinite(o).all()
    assert worst <= TOL[cfg.dtype], worst
    # with only a few visible positions the 2^-9 rounding of single weights is not averaged out; a row
    # dominated by one or two keys shows the full half-ulp (2^-8) of its largest weight times |v|
    tight = TIGHT[cfg.dtype] if (cfg.dtype == "f32" or lay.seq_lens.min() >= 256) else 1e-2
    if dominated:
        tight = TOL[cfg.dtype]
    assert worst <= tight, worst
    return worst


def _all_pairs(cfg):
    return [(b, h) for b in range(cfg.B) for h in range(cfg.Hq)]


def test_cfg0_fp32_full():
    cfg = W.baseline_config(0)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D))
    torch.cuda.synchronize()
    _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg))


def test_fp32_ragged_multi_chunk_and_d128():
    cfg = W.scaled(W.baseline_config(0), B=3, Hq=4, Hkv=2, D=128, page=16, k=6, kv_mode="ragged",
                   kv_len=(7, 900), permute_pages=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D))
    torch.cuda.synchronize()
    _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg))


@pytest.mark.parametrize("k,D", [(0, 64), (31, 64), (31, 128)])
def test_fp32_fewest_and_most_query_rows(k, D):
    """fp32 storage: one query row (plain decoding) and the largest supported number, 32."""
    cfg = W.scaled(W.baseline_config(0), B=2, Hq=2, Hkv=1, D=D, page=16, k=k, kv_mode="ragged", kv_len=(k + 2, 700),
                   permute_pages=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D))
    torch.cuda.synchronize()
    _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg))


def test_fp32_more_than_32_query_rows_is_refused():
    cfg = W.scaled(W.baseline_config(0), B=1, Hq=1, Hkv=1, D=64, page=16, k=32, kv_mode="fixed", kv_len=(128, 128))
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    with pytest.raises(A.AgentSamError):
        A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D))


BF16_SMALL = [
    # several tiles per wavefront, ragged tails, every packed-row tile count, both head dims
    dict(B=3, Hq=8, Hkv=2, D=128, k=8, kv_mode="ragged", kv_len=(9, 3000), permute_pages=True),     # 36 rows
    dict(B=2, Hq=4, Hkv=4, D=128, k=3, kv_mode="ragged", kv_len=(4, 700), permute_pages=True),      # 4 rows
    dict(B=2, Hq=8, Hkv=4, D=128, k=8, kv_mode="fixed", kv_len=(1024, 1024)),                       # 18 rows
    dict(B=2, Hq=16, Hkv=2, D=128, k=16, kv_mode="ragged", kv_len=(17, 2500), permute_pages=True),  # 136 rows
    dict(B=2, Hq=10, Hkv=2, D=128, k=8, kv_mode="shared_prefix", kv_len=(40, 500), prefix_len=1024),  # 45 rows
    dict(B=2, Hq=8, Hkv=2, D=64, k=8, kv_mode="ragged", kv_len=(9, 2000), permute_pages=True, page=32),
    # head dim 64 with more than 48 packed rows: the wide kernel's ring of 8 slots, one 4 KB group per part
    dict(B=2, Hq=16, Hkv=2, D=64, k=8, kv_mode="ragged", kv_len=(33, 1800), permute_pages=True, page=32),   # 72 rows
    dict(B=2, Hq=16, Hkv=2, D=64, k=16, kv_mode="ragged", kv_len=(17, 2300), permute_pages=True),           # 136 rows
]


@pytest.mark.parametrize("case", range(len(BF16_SMALL)))
def test_bf16_small_all_heads(case):
    cfg = W.scaled(W.baseline_config(1), **BF16_SMALL[case])
    print(f"attn bf16 case {case}: {BF16_SMALL[case]}", flush=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D))
    torch.cuda.synchronize()
    _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg))


@pytest.mark.parametrize("case", range(len(BF16_SMALL)))
def test_bf16_small_balanced_schedule(case):
    """The balanced schedule on small inputs: shares of a few tiles, so every stream is spread over
    many workgroups and most segments start and end in the middle of a stream."""
    cfg = W.scaled(W.baseline_config(1), **BF16_SMALL[case])
    print(f"attn bf16 balanced case {case}: {BF16_SMALL[case]}", flush=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(schedule=2))
    torch.cuda.synchronize()
    _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg))


# (G, k): the packed-row counts at which the kernel variant changes (narrow: 16 / 32 / 48 rows; wide: 16 / 16+extra /
# 32 / 32+extra / 48 rows per wavefront) and the largest supported, 192
ROW_BOUNDARIES = [(4, 3), (17, 0), (8, 3), (11, 2), (8, 5),                                    # 16, 17, 32, 33, 48
                  (7, 6), (8, 7), (13, 4), (8, 9), (9, 8), (8, 15), (43, 2), (16, 8), (29, 4), (16, 11)]


@pytest.mark.parametrize("G,k", ROW_BOUNDARIES)
def test_bf16_row_count_boundaries(G, k):
    cfg = W.scaled(W.baseline_config(1), B=2, Hq=G, Hkv=1, D=128, k=k, kv_mode="ragged", kv_len=(k + 2, 1500),
                   permute_pages=True)
    print(f"attn bf16 rows {G * (k + 1)} (G={G}, k={k})", flush=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D))
    torch.cuda.synchronize()
    _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg))


@pytest.mark.parametrize("G,k,sched", [(4, 8, 0), (8, 16, 2), (8, 23, 1), (4, 8, 2)])
def test_bf16_results_repeat_bit_for_bit(G, k, sched):
    """The same call twenty times: every launch gives the same bits (no race in the tile rings, no
    order-dependent merge)."""
    cfg = W.scaled(W.baseline_config(1), B=24, Hq=2 * G, Hkv=2, D=128, k=k, kv_mode="ragged", kv_len=(k + 2, 6000),
                   permute_pages=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    first = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(schedule=sched)).clone()
    for _ in range(20):
        again = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(schedule=sched))
        assert torch.equal(again, first)
    torch.cuda.synchronize()


@pytest.mark.parametrize("seed", range(16))
def test_bf16_seeded_random_shapes(seed):
    """Shapes, lengths, page sizes and schedules drawn from a seeded generator: every output against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    D = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 5, 8, 12]))
    k = int(rng.integers(0, min(24, 192 // G - 1) + 1))
    B = int(rng.choice([1, 2, 5, 9, 33]))
    page = int(rng.choice([32, 64, 128]))
    lo = k + 1 + int(rng.integers(0, 40))
    hi = lo + int(rng.choice([0, 31, 200, 1500, 4000]))
    mode = str(rng.choice(["ragged", "fixed", "shared_prefix"]))
    kw = dict(B=B, Hq=G * Hkv, Hkv=Hkv, D=D, k=k, page=page, kv_mode=mode, kv_len=(lo, hi), permute_pages=bool(rng.integers(0, 2)))
    if mode == "shared_prefix":
        kw["prefix_len"] = page * int(rng.integers(1, 12))
    if mode == "fixed":
        kw["kv_len"] = (hi, hi)
    cfg = W.scaled(W.baseline_config(1), **kw)
    sched, casc = int(rng.integers(0, 3)), int(rng.choice([0, 1, 2]))
    print(f"attn random shape {seed}: {kw} schedule {sched} cascade {casc}", flush=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(schedule=sched, cascade=casc))
    torch.cuda.synchronize()
    pairs = _all_pairs(cfg)
    if len(pairs) > 60:
        pairs = [pairs[i] for i in rng.choice(len(pairs), 60, replace=False)]
    _check(cfg, lay, q, kc, vc, out, pairs, dominated=True)


ODD_PAGES = [
    dict(dtype="bf16", page=96, Hq=8, Hkv=2, D=128, k=8, B=3, kv_len=(9, 2500)),       # 36 rows, narrow kernel
    dict(dtype="bf16", page=160, Hq=16, Hkv=2, D=128, k=16, B=2, kv_len=(17, 2300)),   # 136 rows, wide kernel
    dict(dtype="bf16", page=96, Hq=16, Hkv=2, D=64, k=8, B=2, kv_len=(33, 1800)),      # 72 rows, head dim 64
    dict(dtype="f32", page=24, Hq=4, Hkv=2, D=64, k=6, B=3, kv_len=(7, 900)),
    dict(dtype="f32", page=7, Hq=2, Hkv=1, D=128, k=4, B=2, kv_len=(5, 300)),
]


@pytest.mark.parametrize("schedule", [1, 2])
@pytest.mark.parametrize("case", range(len(ODD_PAGES)))
def test_page_sizes_that_are_not_powers_of_two(case, schedule):
    """Positions are mapped to pages with a division instead of a shift (bf16: any multiple of the 32-position
    tile; fp32: any size)."""
    kw = dict(ODD_PAGES[case])
    base = W.baseline_config(0 if kw.pop("dtype") == "f32" else 1)
    cfg = W.scaled(base, kv_mode="ragged", permute_pages=True, **kw)
    print(f"attn odd page case {case} schedule {schedule}: {ODD_PAGES[case]}", flush=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(schedule=schedule))
    torch.cuda.synchronize()
    _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg))


def test_bf16_page_size_that_cuts_a_tile_is_refused():
    cfg = W.scaled(W.baseline_config(1), B=1, Hq=8, Hkv=2, D=128, k=8, page=48, kv_mode="fixed", kv_len=(480, 480))
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    with pytest.raises(Exception):
        A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D))
    torch.cuda.synchronize()


def test_bf16_more_than_192_rows_is_refused():
    cfg = W.scaled(W.baseline_config(1), B=1, Hq=8, Hkv=1, D=128, k=24, kv_mode="fixed", kv_len=(256, 256))
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    with pytest.raises(A.AgentSamError):
        A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D))


@pytest.mark.parametrize("k,Hq,B", [(8, 32, 70), (16, 64, 130)])
def test_bf16_many_short_sessions_balanced(k, Hq, B):
    """Enough (session, kv head) streams that the balanced schedule is chosen by itself, with streams
    much shorter than a share: most segments are whole streams, a workgroup walks several sessions."""
    cfg = W.scaled(W.baseline_config(1), B=B, Hq=Hq, Hkv=8, D=128, k=k, kv_mode="ragged", kv_len=(k + 1, 1500),
                   permute_pages=True)
    print(f"attn bf16 many sessions B={B} rows={(Hq // 8) * (k + 1)}", flush=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D))
    torch.cuda.synchronize()
    rng = np.random.default_rng(B)
    order = np.argsort(lay.seq_lens)
    bs = {int(order[0]), int(order[-1]), 0, B - 1} | {int(x) for x in rng.integers(0, B, 8)}
    pairs = [(b, int(h)) for b in sorted(bs) for h in rng.choice(Hq, 3, replace=False)]
    _check(cfg, lay, q, kc, vc, out, pairs)
    # every output element against the chunk-grid schedule
    ref = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(schedule=1))
    torch.cuda.synchronize()
    # (short sessions: single bf16-rounded weights are not averaged out, see _check)
    diff = float((out - ref).abs().max())
    assert diff < 4e-3, diff


def test_bf16_more_sessions_than_threads_balanced():
    """More sessions than a workgroup has threads: the scan over seq_lens takes several rounds, and most
    workgroups walk through dozens of whole streams."""
    cfg = W.scaled(W.baseline_config(1), B=700, Hq=4, Hkv=2, D=64, k=3, kv_mode="ragged", kv_len=(4, 300),
                   permute_pages=True, page=32)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    outs = {}
    for schedule in (2, 1):
        outs[schedule] = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(schedule=schedule))
        torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    pairs = [(int(b), int(h)) for b in list(rng.integers(0, cfg.B, 40)) + [0, 255, 256, 257, 511, 512, 699]
             for h in range(cfg.Hq)]
    _check(cfg, lay, q, kc, vc, outs[2], pairs)
    assert float((outs[2] - outs[1]).abs().max()) < 4e-3


CASCADE = [
    # B, Hq, Hkv, k, kv_mode, kv_len, prefix_len: groups of 4 / 5 / 2 sessions, a short last group, no sharing at all
    dict(B=6, Hq=10, Hkv=2, k=8, kv_mode="shared_prefix", kv_len=(40, 700), prefix_len=2048),     # 45 rows, groups 4 + 2
    dict(B=11, Hq=8, Hkv=2, k=8, kv_mode="shared_prefix", kv_len=(9, 300), prefix_len=1024),      # 36 rows, groups 5 + 5 + 1
    dict(B=5, Hq=16, Hkv=4, k=16, kv_mode="shared_prefix", kv_len=(17, 900), prefix_len=1536),    # 68 rows: too many for a shared-prefix run, plain run
    dict(B=7, Hq=8, Hkv=2, k=8, kv_mode="ragged", kv_len=(9, 2000), permute_pages=True),          # nothing shared
    dict(B=4, Hq=8, Hkv=2, k=8, kv_mode="shared_prefix", kv_len=(9, 60), prefix_len=64),          # one shared page
    dict(B=7, Hq=28, Hkv=4, k=8, kv_mode="shared_prefix", kv_len=(40, 1500), prefix_len=4096),    # 63 rows, groups of 3 (3 + 3 + 1)
    dict(B=9, Hq=4, Hkv=2, k=8, kv_mode="shared_prefix", kv_len=(9, 900), prefix_len=3072),       # 18 rows, groups of 9 + (none): 162 rows
    dict(B=40, Hq=12, Hkv=4, k=8, kv_mode="shared_prefix", kv_len=(30, 400), prefix_len=12288),   # 27 rows, groups of 7: shares of many tiles
]


@pytest.mark.parametrize("case", range(len(CASCADE)))
def test_bf16_shared_prefix_cascade(case):
    """The shared-prefix run: the common pages are processed once per group of sessions, each session's
    own part separately, and the two are merged.  Checked against the oracle on every output."""
    cfg = W.scaled(W.baseline_config(1), D=128, **CASCADE[case])
    print(f"attn cascade case {case}: {CASCADE[case]}", flush=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(cascade=2)).clone()
    for _ in range(5):                                    # and the same bits on every launch
        assert torch.equal(A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(cascade=2)), out)
    torch.cuda.synchronize()
    _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg))


def test_bf16_cascade_partial_sharing_and_short_session():
    """Sharing that stops early for one session (its third page differs), and a session shorter than the
    others' common prefix: the shared prefix is the minimum over the batch and the result is unchanged."""
    cfg = W.scaled(W.baseline_config(1), B=5, Hq=10, Hkv=2, D=128, k=8, kv_mode="shared_prefix", kv_len=(100, 600),
                   prefix_len=1024)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    scale = 1.0 / np.sqrt(cfg.D)
    ref = A.spec_verify_attn(q, kc, vc, bt, seq, scale)                   # plain run
    for variant in ("third page differs", "short session"):
        bt2, seq2, kc2, vc2 = bt.clone(), seq.clone(), kc, vc
        if variant == "third page differs":
            # session 3 gets a private copy of its third page: same contents, another page id
            kc2 = torch.cat([kc, kc[bt[3, 2]][None]]); vc2 = torch.cat([vc, vc[bt[3, 2]][None]])
            bt2[3, 2] = kc.shape[0]
        else:
            seq2[1] = 200                                                  # ends inside the others' prefix
        out = A.spec_verify_attn(q, kc2, vc2, bt2, seq2, scale, tuning=A.attn_tuning(cascade=2))
        torch.cuda.synchronize()
        plain = A.spec_verify_attn(q, kc2, vc2, bt2, seq2, scale)
        torch.cuda.synchronize()
        diff = float((out - plain).abs().max())
        print(f"  {variant}: cascade vs plain {diff:.2e}", flush=True)
        assert diff < 4e-3                                   # (the split decides what each weight is rounded against)
        if variant == "third page differs":
            assert float((out - ref).abs().max()) < 4e-3


def test_bf16_minimum_and_boundary_lengths():
    """seq_len == R (every row sees only the new positions), lengths around tile / page / chunk edges."""
    base = W.scaled(W.baseline_config(1), B=1, Hq=8, Hkv=2, D=128, k=8)
    for S in (9, 33, 129, 389):                              # the same through the balanced schedule
        cfg = W.scaled(base, kv_len=(S, S), seed=2000 + S)
        lay, q, kc, vc, bt, seq = _inputs(cfg)
        out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(schedule=2))
        torch.cuda.synchronize()
        _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg))
    for S in (9, 10, 31, 32, 33, 64, 65, 127, 128, 129, 130, 136, 137, 255, 257, 384 + 5):
        cfg = W.scaled(base, kv_len=(S, S), seed=1000 + S)
        lay, q, kc, vc, bt, seq = _inputs(cfg)
        out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(kv_chunk=128))
        torch.cuda.synchronize()
        _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg))


@pytest.mark.parametrize("schedule", [1, 2])
@pytest.mark.parametrize("k,Hq", [(8, 8), (16, 16)])
def test_scores_far_above_the_first_tile(k, Hq, schedule):
    """Late keys whose scores exceed everything seen before by hundreds of log2 units (a fixed softmax
    reference would overflow): both the 36-row and the 136-row kernels must still match the oracle."""
    cfg = W.scaled(W.baseline_config(1), B=2, Hq=Hq, Hkv=2, D=128, k=k, kv_mode="ragged", kv_len=(700, 2100),
                   permute_pages=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    kc = kc * 0.05                                              # quiet keys ...
    for b in range(cfg.B):
        S = int(lay.seq_lens[b])
        for pos, row, h in ((S // 2, 0, 0), (S // 2 + 37, cfg.R - 1, Hq - 1), (S - cfg.R - 3, 1, Hq // 2)):
            page, slot = int(lay.block_table[b, pos // cfg.page]), pos % cfg.page
            kc[page, h // cfg.G, slot] = (q[b, row, h].float() * 16.0).to(kc.dtype)   # ... and a few loud ones
    kc = kc.contiguous()
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(schedule=schedule))
    torch.cuda.synchronize()
    _check(cfg, lay, q, kc, vc, out, _all_pairs(cfg), dominated=True)


def test_split_and_page_permutation_invariance():
    cfg = W.scaled(W.baseline_config(1), B=2, Hq=8, Hkv=2, D=128, k=8, kv_mode="ragged", kv_len=(1500, 4000))
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    scale = 1.0 / np.sqrt(cfg.D)
    outs = []
    for chunk in (0, 128, 512, 1024, 4096):
        outs.append(to_np(A.spec_verify_attn(q, kc, vc, bt, seq, scale, tuning=A.attn_tuning(kv_chunk=chunk))))
    for o in outs[1:]:
        # the split changes the running maximum each weight is rounded to bf16 against, and the
        # fp32 summation order; both stay far inside the parity tolerance
        diff = float(np.max(np.abs(o - outs[0])))
        assert diff < 1e-3, diff
    # move the pages around physically (same logical content): results must not change at all
    perm = torch.randperm(lay.num_pages, device=DEV)
    inv = torch.empty_like(perm); inv[perm] = torch.arange(lay.num_pages, device=DEV)
    kc2, vc2 = kc[perm].contiguous(), vc[perm].contiguous()
    bt2 = torch.where(bt >= 0, inv[bt.clamp(min=0).long()].int(), bt)
    o2 = to_np(A.spec_verify_attn(q, kc2, vc2, bt2, seq, scale))
    assert bool(np.array_equal(o2, outs[0]))


def test_bad_page_id_reads_zeros_and_bf16_output():
    cfg = W.scaled(W.baseline_config(1), B=2, Hq=8, Hkv=2, D=128, k=8, kv_len=(640, 640))
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    scale = 1.0 / np.sqrt(cfg.D)
    bt_bad = bt.clone(); bt_bad[0, 3] = lay.num_pages + 7; bt_bad[1, 2] = -5
    out = A.spec_verify_attn(q, kc, vc, bt_bad, seq, scale)
    # the same thing with real pages of zeros
    kc2 = torch.cat([kc, torch.zeros_like(kc[:1])]); vc2 = torch.cat([vc, torch.zeros_like(vc[:1])])
    bt_z = bt.clone(); bt_z[0, 3] = lay.num_pages; bt_z[1, 2] = lay.num_pages
    ref = A.spec_verify_attn(q, kc2, vc2, bt_z, seq, scale)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)
    ob = A.spec_verify_attn(q, kc, vc, bt, seq, scale, out_dtype=torch.bfloat16)
    of = A.spec_verify_attn(q, kc, vc, bt, seq, scale)
    torch.cuda.synchronize()
    assert ob.dtype == torch.bfloat16 and torch.equal(ob, of.to(torch.bfloat16))


def test_error_returns_on_device_arguments():
    cfg = W.scaled(W.baseline_config(1), B=1, Hq=8, Hkv=2, D=128, k=8, kv_len=(20000, 20000))
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    tiny = torch.empty(4, device=DEV)
    from paper_2512_18337_amd import binding
    rc = binding.lib().spec_verify_attn(q.data_ptr(), kc.data_ptr(), vc.data_ptr(), bt.data_ptr(), bt.shape[1],
                                        seq.data_ptr(), 1, 9, 8, 2, 128, 64, lay.num_pages, 0.1, 1, 0,
                                        q.data_ptr(), tiny.data_ptr(), 16, 0, None)
    assert rc == -4


def _one_head_per_kv_group(cfg, rng):
    """Every session x one query head of every kv head (seeded choice within the group)."""
    return [(b, g * cfg.G + int(rng.integers(0, cfg.G))) for b in range(cfg.B) for g in range(cfg.Hkv)]


@pytest.mark.parametrize("i", [1, 2, 3, 4])
def test_full_size_every_session_and_kv_head(i):
    """Baseline shapes in the launch configuration the benchmark times.  The oracle checks EVERY session and,
    for each of its kv heads, one query head of the group (every row of it): each (session, kv head)
    stream, every workgroup's share of it and every merge is covered."""
    cfg = W.baseline_config(i)
    print(f"attn full-size {cfg.name}", flush=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D))
    torch.cuda.synchronize()
    rng = np.random.default_rng(cfg.seed)
    pairs = _one_head_per_kv_group(cfg, rng)
    worst = _check(cfg, lay, q, kc, vc, out, pairs)
    print(f"  max-abs error {worst:.3e} on {len(pairs)} (session, head) pairs", flush=True)
    assert torch.isfinite(out).all()
    # the other schedule (chunk grid <-> balanced shares) must give the same output everywhere: the
    # split only changes the reference each weight is rounded against and the summation order
    auto_balanced = cfg.B * cfg.Hkv >= 2 * 256 * (2 if cfg.G * cfg.R > 48 else 1)
    other = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), tuning=A.attn_tuning(schedule=1 if auto_balanced else 2))
    torch.cuda.synchronize()
    diff = float((out - other).abs().max())
    print(f"  schedules differ by {diff:.3e}", flush=True)
    assert diff < 1e-3


SCALE_CASES = [
    # one per kernel family, with a softmax scale that is NOT 1/sqrt(D): a scale folded wrongly with the head
    # dimension or with log2(e) shows here and nowhere else
    dict(base=0, kw=dict(B=2, Hq=4, Hkv=2, D=128, page=16, k=6, kv_mode="ragged", kv_len=(7, 900)), tuning={}),            # fp32 kernel
    dict(base=1, kw=dict(B=3, Hq=8, Hkv=2, D=128, k=8, kv_mode="ragged", kv_len=(9, 3000)), tuning=dict(schedule=1)),      # narrow, chunk grid + merge
    dict(base=1, kw=dict(B=3, Hq=8, Hkv=2, D=64, k=8, kv_mode="ragged", kv_len=(9, 3000), page=32), tuning=dict(schedule=2)),  # narrow, balanced, head dim 64
    dict(base=1, kw=dict(B=2, Hq=16, Hkv=2, D=128, k=16, kv_mode="ragged", kv_len=(17, 2500)), tuning=dict(schedule=2)),   # wide, 136 rows
    dict(base=1, kw=dict(B=6, Hq=10, Hkv=2, D=128, k=8, kv_mode="shared_prefix", kv_len=(40, 700), prefix_len=2048),
         tuning=dict(cascade=2)),                                                                                        # shared-prefix run
]


@pytest.mark.parametrize("scale", [0.3, 0.02])
@pytest.mark.parametrize("case", range(len(SCALE_CASES)))
def test_softmax_scale_other_than_inverse_sqrt_d(case, scale):
    c = SCALE_CASES[case]
    cfg = W.scaled(W.baseline_config(c["base"]), permute_pages=True, **c["kw"])
    print(f"attn scale {scale} case {case}: {c['kw']}", flush=True)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, scale, tuning=A.attn_tuning(**c["tuning"]))
    torch.cuda.synchronize()
    ref = oracle_attention_sample(q, kc, vc, lay.block_table, lay.seq_lens, scale, _all_pairs(cfg))
    o = to_np(out)
    worst = max(float(np.max(np.abs(o[b, :, h] - r))) for (b, h), r in ref.items())
    # scale 0.3 makes rows that one or two keys dominate (full half-ulp of the largest weight): the stated tolerance
    assert worst <= TOL[cfg.dtype], worst
    # the result must really depend on the scale (a kernel that ignored it would pass one of the two values at most)
    other = oracle_attention_sample(q, kc, vc, lay.block_table, lay.seq_lens, 1.0 / np.sqrt(cfg.D), _all_pairs(cfg)[:1])
    (b, h), r = next(iter(other.items()))
    assert float(np.max(np.abs(o[b, :, h] - r))) > 5 * max(worst, 1e-4)


@pytest.mark.parametrize("case", [1, 3, 4])
def test_bf16_output_against_the_oracle(case):
    """out_dtype = bf16 compared with the fp64 oracle directly (not with the kernel's own fp32 output)."""
    c = SCALE_CASES[case]
    cfg = W.scaled(W.baseline_config(c["base"]), permute_pages=True, **c["kw"])
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    out = A.spec_verify_attn(q, kc, vc, bt, seq, 1.0 / np.sqrt(cfg.D), out_dtype=torch.bfloat16,
                             tuning=A.attn_tuning(**c["tuning"]))
    torch.cuda.synchronize()
    assert out.dtype == torch.bfloat16
    ref = oracle_attention_sample(q, kc, vc, lay.block_table, lay.seq_lens, 1.0 / np.sqrt(cfg.D), _all_pairs(cfg))
    o = to_np(out)
    worst = max(float(np.max(np.abs(o[b, :, h] - r))) for (b, h), r in ref.items())
    big = max(float(np.max(np.abs(r))) for r in ref.values())
    print(f"  bf16 output: max-abs error {worst:.3e}, largest |out| {big:.2f}", flush=True)
    assert worst <= TOL["bf16"]
    assert worst <= 1e-2 + big * 2.0 ** -8                   # the kernel's own error + half an ulp of the output


SHORT_CASES = [
    (0, dict(B=5, Hq=4, Hkv=2, D=64, page=16, k=6), {}),                                   # fp32 kernel
    (1, dict(B=5, Hq=8, Hkv=2, D=128, k=8), dict(schedule=1)),                             # narrow, chunk grid
    (1, dict(B=5, Hq=8, Hkv=2, D=128, k=8), dict(schedule=2)),                             # narrow, balanced
    (1, dict(B=5, Hq=16, Hkv=2, D=128, k=16), dict(schedule=1)),                           # wide, chunk grid
    (1, dict(B=5, Hq=16, Hkv=2, D=128, k=16), dict(schedule=2)),                           # wide, balanced
    (1, dict(B=5, Hq=8, Hkv=2, D=128, k=8), dict(cascade=2)),                              # cascade run (nothing shared)
]


@pytest.mark.parametrize("case", range(len(SHORT_CASES)))
def test_sessions_shorter_than_the_query_rows(case):
    """seq_lens[b] < R: row i sits at position seq_lens[b] - R + i; a row at a negative position sees nothing
    and its output is defined as zeros, the other rows attend positions 0 .. seq_lens[b] - R + i as always.
    An empty session gives all zeros.  Nothing is NaN and the full-length sessions are unaffected."""
    base, kw, tun = SHORT_CASES[case]
    cfg = W.scaled(W.baseline_config(base), kv_mode="ragged", kv_len=(600, 900), permute_pages=True, **kw)
    lay, q, kc, vc, bt, seq = _inputs(cfg)
    R = cfg.R
    lens = lay.seq_lens.copy()
    lens[0], lens[2], lens[4] = 0, 1, R - 1
    seq2 = torch.as_tensor(lens, device=DEV)
    scale = 1.0 / np.sqrt(cfg.D)
    out = A.spec_verify_attn(q, kc, vc, bt, seq2, scale, tuning=A.attn_tuning(**tun))
    full = A.spec_verify_attn(q, kc, vc, bt, seq, scale, tuning=A.attn_tuning(**tun))
    torch.cuda.synchronize()
    o = to_np(out)
    assert np.isfinite(o).all()
    from oracle import attention_oracle_head
    G, P = cfg.G, cfg.page
    for b in (0, 2, 4):
        S = int(lens[b])
        assert not o[b, :R - S].any()                        # rows in front of position 0: zeros
        for h in range(cfg.Hq):
            if S == 0:
                continue
            pages = torch.as_tensor(lay.block_table[b, :(S + P - 1) // P].astype(np.int64), device=DEV)
            K = to_np(kc[pages, h // G]).reshape(-1, cfg.D)[:S]
            V = to_np(vc[pages, h // G]).reshape(-1, cfg.D)[:S]
            # the S visible rows are an ordinary problem with S query rows over S positions
            ref = attention_oracle_head(to_np(q[b, R - S:, h]), K, V, scale)
            assert float(np.max(np.abs(o[b, R - S:, h] - ref))) <= TOL[cfg.dtype]
    for b in (1, 3):
        # (other sessions' lengths move the balanced schedule's cut points, which changes what each weight is rounded against)
        assert float((out[b] - full[b]).abs().max()) < 4e-3
