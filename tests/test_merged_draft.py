"""Several automata per session (MergeSAM with weights): the oracle's choice rule against hand cases, and
the device entry point against the oracle."""
import numpy as np
import pytest

import paper_2512_18337_amd as A
from oracle import draft_oracle, merged_draft_oracle


def test_oracle_choice_rule_by_hand():
    own = [1, 2, 3, 4, 5, 1, 2, 3]            # window [1 2 3]: match 3 ending at 2 -> draft 4 5 1
    other = [9, 2, 3, 7, 7]                   # match 2 ([2 3]) -> draft 7 7
    q = [1, 2, 3]
    d, nd, ml, me, src = merged_draft_oracle([own, other], [1.0, 1.0], q, 3, 99)
    assert (list(d[:nd]), ml, src) == ([4, 5, 1], 3, 0)
    # a weight of 2 on the other memory turns 2 * 2 = 4 > 1 * 3
    d, nd, ml, me, src = merged_draft_oracle([own, other], [1.0, 2.0], q, 3, 99)
    assert (list(d[:nd]), ml, src) == ([7, 7], 2, 1)
    # equal scores (1.5 * 2 == 1 * 3): the longer match wins
    assert merged_draft_oracle([own, other], [1.0, 1.5], q, 3, 99)[4] == 0
    # a memory that matches but has nothing to propose, or a weight of zero, is skipped
    assert merged_draft_oracle([[1, 2, 3], other], [5.0, 1.0], q, 3, 99)[4] == 1
    assert merged_draft_oracle([own, other], [0.0, 1.0], q, 3, 99)[4] == 1
    assert merged_draft_oracle([[8, 8], [6]], [1.0, 1.0], q, 3, 99)[2:] == (0, -1, -1)
    # one memory: the plain lookup
    d1 = draft_oracle(np.array(own, np.int32), np.array(q, np.int32), 3, 99, 1)
    dm = merged_draft_oracle([own], [0.3], q, 3, 99)
    assert list(dm[0]) == list(d1[0]) and dm[1:4] == d1[1:4]


@pytest.mark.gpu
def test_device_matches_oracle():
    import torch
    from paper_2512_18337_amd import workloads as W
    DEV = "cuda:0"
    cfg = W.scaled(W.baseline_config(1), sam_session_len=3000, vocab=500, m=24, k=6)
    rng = np.random.default_rng(8)
    mems = [list(W.token_memory(cfg, i)) for i in range(5)]
    flat = A.sam_flatten([A.sam_build(np.asarray(T, np.int32), cfg.sep) for T in mems])
    fd = flat.to(DEV)
    B, M = 40, 3
    which = np.stack([rng.choice(5, M, replace=False) for _ in range(B)])        # the session's own + two "retrieved"
    weight = rng.choice([0.0, 0.25, 0.5, 1.0, 1.0, 2.0], (B, M)).astype(np.float32)
    recent = np.zeros((B, cfg.m), np.int32); rlen = np.full(B, cfg.m, np.int32)
    for b in range(B):
        T = mems[which[b, rng.integers(0, M)]]
        p = int(rng.integers(cfg.m, len(T)))
        w = np.array(T[p - cfg.m:p], np.int32); w[w == cfg.sep] = 0
        w[cfg.m - 1 - int(rng.integers(1, cfg.m))] = int(rng.integers(0, cfg.vocab))
        recent[b] = w
        if b % 7 == 0:
            rlen[b] = int(rng.integers(0, cfg.m))
    root = flat.roots[which]; cend = flat.corpus_end[which]
    d, nd, ml, me, src = A.sam_draft_merged(fd, root, cend, weight, recent, rlen, cfg.k, cfg.sep)
    torch.cuda.synchronize()
    d, nd, ml, me, src = (x.cpu().numpy() for x in (d, nd, ml, me, src))
    for b in range(B):
        q = recent[b, cfg.m - rlen[b]:]
        od, ond, oml, ome, osrc = merged_draft_oracle([mems[j] for j in which[b]], weight[b], q, cfg.k, cfg.sep)
        assert (int(nd[b]), int(ml[b]), int(src[b])) == (ond, oml, osrc), b
        assert list(d[b, :ond]) == list(od[:ond]) and (d[b, ond:] == -1).all()
        if osrc >= 0:
            assert int(me[b]) - int(flat.corpus_begin[which[b, osrc]]) == ome
        else:
            assert me[b] == -1
    assert (src >= 0).sum() > B // 2 and len(set(src.tolist())) >= 3
    # workspace too small is refused
    from paper_2512_18337_amd import binding
    tiny = torch.empty(4, dtype=torch.int32, device=DEV)
    rc = binding.lib().sam_draft_merged(*[binding._dp(x) for x in (fd.row_ptr, fd.edge_tok, fd.edge_dst, fd.lastpos, fd.corpus,
                                                                    fd.state_rec, tiny, tiny, tiny)], M,
                                        binding._dp(tiny), binding._dp(tiny), B, cfg.m, cfg.k, 1, cfg.sep,
                                        *[binding._dp(tiny)] * 5, binding._dp(tiny), 16, None, 0, None)
    assert rc == -4
