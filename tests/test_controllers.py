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


# ------------------------------------------------------------------------------------------ speculation depth
from oracle import choose_k_oracle, expected_committed_oracle, switch_frontier_oracle   # noqa: E402


def _enumerated_committed(k, p):
    """Every accept / reject outcome of the k drafts written out: 2^k outcomes, each with its probability and the
    tokens it commits (accepted prefix up to the first rejection, plus one)."""
    total = 0.0
    for mask in range(1 << k):
        prob, prefix, running = 1.0, 0, True
        for j in range(k):
            ok = (mask >> j) & 1
            prob *= p if ok else (1.0 - p)
            if running and ok:
                prefix += 1
            else:
                running = False
        total += prob * (prefix + 1)
    return total


def test_expected_committed_tokens_oracle_pins():
    for p in (0.0, 0.17, 0.6, 0.65, 0.99, 1.0):
        for k in range(0, 11):
            e = expected_committed_oracle(k, p)
            assert e == pytest.approx(_enumerated_committed(k, p), rel=1e-12)                 # brute force over outcomes
            if p < 1.0:
                assert e == pytest.approx((1 - p ** (k + 1)) / (1 - p), rel=1e-12)            # geometric series
            assert 1.0 <= e <= k + 1 + 1e-12
    assert expected_committed_oracle(8, 1.0) == 9.0 and expected_committed_oracle(8, 0.0) == 1.0
    # the workload list's own figures: E[accepted drafts] = sum p^j
    assert expected_committed_oracle(8, 0.6) - 1 == pytest.approx(1.475, abs=1e-3)
    assert expected_committed_oracle(8, 0.7) - 1 == pytest.approx(2.199, abs=1e-3)
    assert expected_committed_oracle(4, 0.7) - 1 == pytest.approx(1.773, abs=1e-3)


def test_choose_k_oracle_pins():
    ks = list(range(0, 9))
    # constant cost: every extra draft is free, the deepest wins; p = 0: nothing is ever accepted, k = 0 wins
    assert choose_k_oracle(ks, [1.0] * 9, 0.5)[0] == 8
    assert choose_k_oracle(ks, [1.0 + 0.01 * k for k in ks], 0.0) == (0, 1.0)
    # p = 1 and cost a + b(1+k): (1+k)/(a + b(1+k)) grows with k whenever a > 0
    assert choose_k_oracle(ks, [2.0 + 0.5 * (1 + k) for k in ks], 1.0)[0] == 8
    # cost proportional to the rows and p < 1: (1 + p + ..)/(1+k) falls with k, so no speculation
    assert choose_k_oracle(ks, [0.3 * (1 + k) for k in ks], 0.9)[0] == 0
    # the break-even rule: depth k beats no speculation iff p + .. + p^k > cost(k)/cost(0) - 1
    for p in (0.04, 0.06, 0.3):
        t = [1.0, 1.055]                                      # cost of 8 drafts: 5.5 % over a plain step
        pays = sum(p ** j for j in range(1, 9)) > t[1] / t[0] - 1
        assert (choose_k_oracle([0, 8], t, p)[0] == 8) == pays
    # the other layers: free below the floor, per row above it -> the depth stops where the rows reach the floor
    k, gain = choose_k_oracle(ks, [1.0] * 9, 0.8, batch=4, other_floor=2.0, other_per_row=0.1)   # floor reached at 20 rows = k 4
    assert k == 4 and gain == pytest.approx(expected_committed_oracle(4, 0.8) * 3.0 / 3.0)
    # gain is relative to k = 0
    k, gain = choose_k_oracle([0, 4], [2.0, 2.5], 0.5)
    assert k == 4 and gain == pytest.approx(expected_committed_oracle(4, 0.5) / 2.5 * 2.0)


def test_switch_frontier_oracle_pins():
    # a surface on which verification costs nothing at short contexts and k-proportionally more at long ones:
    # t(B, S, k) = S/1000 * (1 + k * S / 64000); with p = 0.5 (sum p^j < 1) speculation stops paying beyond a context
    batches, contexts, ks = [1, 8, 64], [1000, 8000, 32000, 128000], [0, 2, 4]
    t = [[[S / 1000 * (1 + k * S / 64000) for k in ks] for S in contexts] for _ in batches]
    kstar, cthr, bthr = switch_frontier_oracle(batches, contexts, ks, t, 0.5)
    for i in range(3):
        for j, S in enumerate(contexts):
            pays = any(sum(0.5 ** m for m in range(1, k + 1)) > (1 + k * S / 64000) - 1 for k in ks[1:])
            assert (kstar[i][j] > 0) == pays
    assert cthr == [8000, 8000, 8000] and bthr == [64, 64, -1, -1]
    # row-proportional other layers switch speculation off beyond a batch size
    t1 = [[[1.0 for _ in ks] for _ in contexts] for _ in batches]
    kstar, cthr, bthr = switch_frontier_oracle(batches, contexts, ks, t1, 0.5, other_floor=1.0, other_per_row=0.05)
    assert [row[0] for row in kstar] == [4, 2, 0]             # 1 + k <= 20 rows / batch stay under the floor
    assert bthr == [8] * 4 and cthr == [128000, 128000, -1]


@pytest.mark.parametrize("seed", range(4))
def test_speculation_controller_matches_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(50):
        nk = int(rng.integers(1, 9))
        ks = [0] + sorted(rng.choice(np.arange(1, 33), nk - 1, replace=False).tolist())
        t = (rng.uniform(0.5, 2.0) * (1 + np.asarray(ks) * rng.uniform(0, 0.1))).tolist()
        p = float(rng.choice([0.0, 1.0, rng.uniform(0, 1)]))
        batch = int(rng.integers(1, 200))
        floor_, per_row = float(rng.choice([0.0, rng.uniform(0, 3)])), float(rng.choice([0.0, rng.uniform(0, 0.02)]))
        k1, g1 = A.spec_choose_k(ks, t, p, per_row, batch, floor_)
        k0, g0 = choose_k_oracle(ks, t, p, batch, floor_, per_row)
        assert k1 == k0 and g1 == pytest.approx(g0, rel=1e-12)
    batches = sorted(rng.choice(np.arange(1, 300), 4, replace=False).tolist())
    contexts = sorted(rng.choice(np.arange(1, 200000), 5, replace=False).tolist())
    ks = [0, 1, 3, 8, 16]
    t = rng.uniform(0.5, 1.0, (4, 5, 1)) * (1 + np.asarray(ks)[None, None, :] * rng.uniform(0, 0.3, (4, 5, 1)))
    for p in (0.2, 0.6, 0.95):
        got = A.spec_switch_frontier(batches, contexts, ks, t, p, 0.7, 0.002)
        want = switch_frontier_oracle(batches, contexts, ks, t.tolist(), p, 0.7, 0.002)
        assert got[0].tolist() == want[0] and got[1].tolist() == want[1] and got[2].tolist() == want[2]
        # the thresholds feed the switch: inside both, speculation stays on
        for i, b in enumerate(batches):
            for j, s in enumerate(contexts):
                if s <= got[1][i] and b <= got[2][j]:
                    assert got[0][i, j] > 0


def test_speculation_controller_argument_errors():
    with pytest.raises(A.AgentSamError):
        A.spec_choose_k([1, 2], [1.0, 1.0], 0.5)              # the table must start at k = 0
    with pytest.raises(A.AgentSamError):
        A.spec_choose_k([0, 2, 2], [1.0, 1.0, 1.0], 0.5)
    with pytest.raises(A.AgentSamError):
        A.spec_choose_k([0, 2], [1.0, 0.0], 0.5)
    with pytest.raises(A.AgentSamError):
        A.spec_choose_k([0, 2], [1.0, 1.0], 1.5)
