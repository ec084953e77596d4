"""AgentSched pick (Alg. 3) and the adaptive speculation switch (Alg. 4 step 4): the oracle against what
the formulas fix, and the library against the oracle."""
import math

import numpy as np
import pytest

import paper_2512_18337_amd as A
from oracle import adaptive_k_oracle, agentsched_oracle

P = dict(lambda_max=4.0, k=6.0, eps=1e-6, a=1.0, b=0.5, c=0.1, tokens_per_block=16)


def _oracle(free, hit, need, ptok, wait, **p):
    return agentsched_oracle(free, hit, need, ptok, wait, p["lambda_max"], p["k"], p["eps"], p["a"], p["b"], p["c"],
                             p["tokens_per_block"])


def test_oracle_closed_forms():
    # demand equal to the effective capacity: z = 1 (up to eps), the logistic sits at its midpoint
    lam, _, _ = _oracle(100, [10, 10], [40, 40], [640, 640], [0, 0], **P)
    assert abs(lam - P["lambda_max"] / 2) < 1e-5
    # no pressure: lambda -> 0, the mix is pure shortest-job-first on prompt length; with a = c = 0 the
    # shortest prompt wins whatever the cache state
    p = dict(P, a=0.0, c=0.0, k=60.0)
    lam, sc, picked = _oracle(10**6, [500, 0, 0], [1, 200, 100], [4000, 320, 1600], [5, 0, 9], **p)
    assert lam < 1e-12 and picked == 1
    assert sc[1] == pytest.approx(-p["b"] * 320 / 16) and sc[0] == pytest.approx(-p["b"] * 4000 / 16)
    # full pressure: lambda -> lambda_max, the demand term uses the NEW blocks only, so the long request
    # whose blocks are cached beats the short uncached one
    lam, sc, picked = _oracle(260, [250, 0], [2, 30], [4032, 480], [0, 0], **dict(P, k=60.0))   # U = 10, D = 32
    assert abs(lam - P["lambda_max"]) < 1e-9 and picked == 0
    assert sc[0] == pytest.approx(250 - (0.5 + lam) * 2) and sc[1] == pytest.approx(-(0.5 + lam) * 30)
    # waiting is rewarded linearly; an infeasible request is passed over; nothing feasible -> -1
    _, sc, _ = _oracle(100, [0, 0], [5, 5], [80, 80], [0, 7], **P)
    assert sc[1] - sc[0] == pytest.approx(P["c"] * 7)
    assert _oracle(10, [0, 0], [50, 4], [800, 64], [1000, 0], **P)[2] == 1
    assert _oracle(3, [0, 0], [50, 4], [800, 64], [0, 0], **P)[2] == -1
    assert _oracle(3, [], [], [], [], **P)[2] == -1
    # ties go to the earlier request
    assert _oracle(100, [1, 1], [5, 5], [80, 80], [2, 2], **P)[2] == 0


def test_oracle_logistic_is_monotone_and_bounded():
    lams = [_oracle(100, [0], [d], [16 * d], [0], **P)[0] for d in (0, 10, 50, 100, 200, 10**6)]
    assert all(x < y for x, y in zip(lams, lams[1:5])) and 0 < lams[0] and lams[-1] <= P["lambda_max"]
    assert lams[0] == pytest.approx(P["lambda_max"] / (1 + math.exp(P["k"])))


@pytest.mark.parametrize("seed", range(5))
def test_library_matches_oracle(seed):
    rng = np.random.default_rng(seed)
    for _ in range(60):
        n = int(rng.integers(0, 40))
        hit = rng.integers(0, 300, n); need = rng.integers(0, 300, n)
        ptok = (hit + need) * 16 + rng.integers(0, 16, n)
        wait = rng.random(n) * 50
        free = int(rng.integers(0, 3000))
        p = dict(lambda_max=float(rng.uniform(0.5, 8)), k=float(rng.uniform(0.5, 20)), eps=1e-6,
                 a=float(rng.uniform(0, 2)), b=float(rng.uniform(0, 2)), c=float(rng.uniform(0, 1)),
                 tokens_per_block=int(rng.choice([16, 32, 128])))
        lam, sc, picked = A.agentsched_pick(free, hit, need, ptok, wait, **p)
        olam, osc, opicked = _oracle(free, list(hit), list(need), list(ptok), list(wait), **p)
        assert lam == pytest.approx(olam, rel=1e-12, abs=1e-300)
        assert np.allclose(sc, osc, rtol=1e-12, atol=1e-9) and picked == opicked


def test_adaptive_switch():
    assert adaptive_k_oracle(8, 30000, 4, 16, 65536) == 4
    for batch, ctx in [(8, 30000), (16, 65536), (17, 100), (1, 65537), (0, 0), (64, 10**6)]:
        assert A.spec_adaptive_k(batch, ctx, 4, 16, 65536) == adaptive_k_oracle(batch, ctx, 4, 16, 65536)
    assert A.spec_adaptive_k(17, 100, 4, 16, 65536) == 0 and A.spec_adaptive_k(16, 65536, 4, 16, 65536) == 4
    with pytest.raises(A.AgentSamError):
        A.spec_adaptive_k(-1, 0, 4, 16, 65536)


def test_argument_errors():
    with pytest.raises(A.AgentSamError):
        A.agentsched_pick(10, [1], [1], [16], [0.0], **dict(P, lambda_max=0.0))
    with pytest.raises(A.AgentSamError):
        A.agentsched_pick(10, [-1], [1], [16], [0.0], **P)
