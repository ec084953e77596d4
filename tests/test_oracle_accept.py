"""Pins for the accept oracle: numpy.argmax, greedy decoding, closed-form expectation, edge cases."""
import numpy as np
import pytest
import torch

from oracle import accept_oracle
from paper_2512_18337_amd import workloads as W


def test_argmax_is_first_maximum_like_numpy():
    rng = np.random.default_rng(0)
    logits = rng.integers(-3, 4, size=(5, 4, 50)).astype(np.float32)    # many exact ties
    a, out, tgt = accept_oracle(logits, np.zeros((5, 3), np.int32), np.zeros(5, np.int32))
    assert np.array_equal(tgt, np.argmax(logits, axis=2))
    assert np.all(a == 0) and np.array_equal(out[:, 0], tgt[:, 0]) and np.all(out[:, 1:] == -1)


def test_greedy_decoding_equivalence_and_bounds():
    """Committed tokens equal what token-by-token greedy decoding over the same rows emits."""
    rng = np.random.default_rng(1)
    B, k, V = 40, 6, 30
    logits = rng.normal(size=(B, k + 1, V)).astype(np.float32)
    tgt_np = np.argmax(logits, axis=2)
    draft = tgt_np[:, :k].astype(np.int32).copy()
    n_draft = rng.integers(0, k + 1, B).astype(np.int32)
    for b in range(B):                                    # break the draft at a random place
        j = rng.integers(0, k + 1)
        if j < k:
            draft[b, j] = (draft[b, j] + 1) % V
    a, out, tgt = accept_oracle(logits, draft, n_draft)
    for b in range(B):
        emitted = []
        for i in range(k + 1):                            # row i is valid only while drafts 0..i-1 were right
            emitted.append(int(tgt_np[b, i]))
            if i >= n_draft[b] or draft[b, i] != tgt_np[b, i]:
                break
        assert 0 <= a[b] <= n_draft[b] <= k
        assert list(out[b, :a[b] + 1]) == emitted and np.all(out[b, a[b] + 1:] == -1)


def test_all_or_none_injected():
    cfg = W.scaled(W.baseline_config(0), B=16, match_prob=(1.0, 1.0))
    rng = np.random.default_rng(2)
    draft = rng.integers(0, cfg.vocab, (cfg.B, cfg.k)).astype(np.int32)
    n_draft = rng.integers(0, cfg.k + 1, cfg.B).astype(np.int32)
    lg = W.verify_logits(cfg, draft, n_draft, "cpu").numpy()
    a, out, tgt = accept_oracle(lg, draft, n_draft)
    assert np.array_equal(a, n_draft)
    cfg0 = W.scaled(cfg, match_prob=(0.0, 0.0))
    lg = W.verify_logits(cfg0, draft, n_draft, "cpu").numpy()
    a, out, tgt = accept_oracle(lg, draft, n_draft)
    assert a.sum() <= 1                                   # a chance hit has probability 1/V per row


def test_expected_accept_length_closed_form():
    """With injection probability p per draft, E[a] = sum_{j=1..k} p^j (this is the synthetic OTE - 1)."""
    cfg = W.scaled(W.baseline_config(0), B=3000, vocab=64, k=4, match_prob=(0.7, 0.7))
    rng = np.random.default_rng(3)
    draft = rng.integers(0, cfg.vocab, (cfg.B, cfg.k)).astype(np.int32)
    n_draft = np.full(cfg.B, cfg.k, dtype=np.int32)
    lg = W.verify_logits(cfg, draft, n_draft, "cpu").numpy()
    a, _, _ = accept_oracle(lg, draft, n_draft)
    p = 0.7 + 0.3 / 64                                    # an uninjected row still hits with probability 1/V
    expect = sum(p ** j for j in range(1, cfg.k + 1))
    assert abs(a.mean() - expect) < 0.08


def test_nan_and_inf_rows():
    lg = np.zeros((1, 3, 6), dtype=np.float32)
    lg[0, 0] = [np.nan, 1.0, np.nan, 1.0, 0.5, np.nan]    # NaN never wins; first of the two 1.0
    lg[0, 1] = -np.inf                                    # nothing finite: index 0
    lg[0, 2] = [-np.inf, -np.inf, 3.0, np.inf, np.inf, 0] # +inf is a legitimate maximum; first one
    a, out, tgt = accept_oracle(lg, np.array([[1, 0]], np.int32), np.array([2], np.int32))
    assert list(tgt[0]) == [1, 0, 3] and a[0] == 2 and list(out[0]) == [1, 0, 3]


def test_bf16_ties_use_stored_values():
    torch.manual_seed(0)
    lg = (torch.randn(4, 3, 5000) * 4).round().div(4).to(torch.bfloat16)   # coarse values: the maximum is tied
    f = lg.float().numpy()
    a, out, tgt = accept_oracle(f, np.zeros((4, 2), np.int32), np.zeros(4, np.int32))
    assert np.array_equal(tgt, np.argmax(f, axis=2))
    ties = (f == f.max(axis=2, keepdims=True)).sum(axis=2)
    assert (ties > 1).any()


def test_k_zero_is_plain_decoding():
    lg = np.array([[[0.1, 0.9, 0.3]]], dtype=np.float32)
    a, out, tgt = accept_oracle(lg, np.zeros((1, 0), np.int32), np.array([0], np.int32))
    assert a[0] == 0 and out.tolist() == [[1]] and tgt.tolist() == [[1]]
