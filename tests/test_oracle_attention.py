"""Pins for the fp64 attention oracle: closed forms, invariants, and torch's SDPA on a contiguous cache."""
import numpy as np
import pytest
import torch

from oracle import attention_oracle, attention_oracle_head


def _paged(K, V, P, rng, permute=True):
    """Scatter contiguous K,V [B,S,Hkv,D] into a paged cache [num_pages,Hkv,P,D]."""
    B, S, Hkv, D = K.shape
    npg = (S + P - 1) // P
    total = B * npg + 3                                  # a few unused pages
    order = rng.permutation(total) if permute else np.arange(total)
    kc = rng.normal(size=(total, Hkv, P, D)) * 50.0       # junk in unused slots must not matter
    vc = rng.normal(size=(total, Hkv, P, D)) * 50.0
    bt = np.full((B, npg + 2), -1, dtype=np.int32)
    for b in range(B):
        for p in range(npg):
            pg = order[b * npg + p]
            bt[b, p] = pg
            n = min(P, S - p * P)
            kc[pg, :, :n] = K[b, p * P:p * P + n].transpose(1, 0, 2)
            vc[pg, :, :n] = V[b, p * P:p * P + n].transpose(1, 0, 2)
    return kc, vc, bt


def test_single_position_returns_v():
    rng = np.random.default_rng(0)
    q = rng.normal(size=(1, 7)); K = rng.normal(size=(1, 7)); V = rng.normal(size=(1, 7))
    assert np.allclose(attention_oracle_head(q, K, V, 0.3), V, rtol=0, atol=1e-15)


def test_two_position_closed_form():
    # scores 0 and ln 3 -> weights 1/4 and 3/4
    q = np.array([[1.0]]); K = np.array([[0.0], [np.log(3.0)]]); V = np.array([[8.0], [4.0]])
    out = attention_oracle_head(q, K, V, 1.0)
    assert abs(out[0, 0] - (0.25 * 8 + 0.75 * 4)) < 1e-14
    # scale enters the exponent: scale 2 -> weights 1/10 and 9/10
    out = attention_oracle_head(q, K, V, 2.0)
    assert abs(out[0, 0] - (0.1 * 8 + 0.9 * 4)) < 1e-14


def test_equal_keys_give_prefix_means():
    rng = np.random.default_rng(1)
    S, R, D = 37, 5, 6
    K = np.tile(rng.normal(size=(1, D)), (S, 1)); V = rng.normal(size=(S, D)); q = rng.normal(size=(R, D))
    out = attention_oracle_head(q, K, V, 0.7)
    for i in range(R):
        assert np.allclose(out[i], V[: S - R + i + 1].mean(axis=0), atol=1e-13)


def test_convexity_and_causality():
    rng = np.random.default_rng(2)
    S, R, D = 50, 4, 8
    q = rng.normal(size=(R, D)); K = rng.normal(size=(S, D)); V = rng.normal(size=(S, D))
    out = attention_oracle_head(q, K, V, 1 / np.sqrt(D))
    for i in range(R):
        vis = V[: S - R + i + 1]
        assert np.all(out[i] <= vis.max(axis=0) + 1e-12) and np.all(out[i] >= vis.min(axis=0) - 1e-12)
    for i in range(R):
        p = S - R + i
        K2, V2 = K.copy(), V.copy()
        K2[p + 1:] += 3.0; V2[p + 1:] -= 5.0             # the future of row i
        out2 = attention_oracle_head(q, K2, V2, 1 / np.sqrt(D))
        assert np.array_equal(out2[i], out[i])
        V3 = V.copy(); V3[p] += 1.0                      # row i's own position is visible
        out3 = attention_oracle_head(q, K, V3, 1 / np.sqrt(D))
        assert np.max(np.abs(out3[i] - out[i])) > 1e-6
        if i > 0:
            assert np.array_equal(out3[i - 1], out[i - 1])


def test_large_scores_do_not_overflow():
    q = np.array([[1000.0, 0.0]]); K = np.array([[1.0, 0.0], [2.0, 0.0], [-5.0, 1.0]]); V = np.eye(3)[:, :2] + 1.0
    out = attention_oracle_head(q, K, V, 1.0)
    assert np.all(np.isfinite(out)) and np.allclose(out[0], V[1], atol=1e-12)


@pytest.mark.parametrize("B,R,Hq,Hkv,D,S,P", [(2, 5, 4, 1, 64, 100, 16), (3, 3, 6, 2, 32, 77, 8), (1, 9, 8, 8, 16, 40, 64)])
def test_matches_torch_sdpa_float64(B, R, Hq, Hkv, D, S, P):
    """Library special case: contiguous cache + explicit boolean mask through torch SDPA in float64;
    the paged, permuted layout must give the same numbers; query head h reads kv head h // (Hq/Hkv)."""
    rng = np.random.default_rng(B * 100 + R)
    q = rng.normal(size=(B, R, Hq, D)); K = rng.normal(size=(B, S, Hkv, D)); V = rng.normal(size=(B, S, Hkv, D))
    scale = 1.0 / np.sqrt(D)
    kc, vc, bt = _paged(K, V, P, rng)
    out = attention_oracle(q, kc, vc, bt, np.full(B, S, dtype=np.int32), scale)
    G = Hq // Hkv
    tq = torch.from_numpy(q).permute(0, 2, 1, 3)                                        # [B,Hq,R,D]
    tk = torch.from_numpy(K).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)            # [B,Hq,S,D]
    tv = torch.from_numpy(V).permute(0, 2, 1, 3).repeat_interleave(G, dim=1)
    mask = torch.arange(S)[None, :] <= (S - R + torch.arange(R))[:, None]               # [R,S]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    ref = ref.permute(0, 2, 1, 3).numpy()
    assert out.shape == ref.shape and np.max(np.abs(out - ref)) < 1e-12


def test_ragged_lengths_and_sampled_heads():
    rng = np.random.default_rng(7)
    B, R, Hq, Hkv, D, P = 3, 4, 4, 2, 8, 8
    lens = [4, 19, 33]
    S = max(lens)
    q = rng.normal(size=(B, R, Hq, D)); K = rng.normal(size=(B, S, Hkv, D)); V = rng.normal(size=(B, S, Hkv, D))
    kc, vc, bt = _paged(K, V, P, rng)
    out = attention_oracle(q, kc, vc, bt, np.array(lens, dtype=np.int32), 0.5)
    for b in range(B):
        for h in range(Hq):
            ref = attention_oracle_head(q[b, :, h], K[b, :lens[b], h // 2], V[b, :lens[b], h // 2], 0.5)
            assert np.array_equal(out[b, :, h], ref)
    part = attention_oracle(q, kc, vc, bt, np.array(lens, dtype=np.int32), 0.5, heads=[(1, 3)])
    assert np.array_equal(part[1, :, 3], out[1, :, 3]) and np.isnan(part[0]).all()
    with pytest.raises(ValueError):
        attention_oracle(q, kc, vc, bt, np.array([3, 19, 33], dtype=np.int32), 0.5)


def test_group_heads_with_equal_queries_agree():
    rng = np.random.default_rng(9)
    q = rng.normal(size=(1, 3, 4, 8)); q[:, :, 1] = q[:, :, 0]
    K = rng.normal(size=(1, 20, 2, 8)); V = rng.normal(size=(1, 20, 2, 8))
    kc, vc, bt = _paged(K, V, 4, rng)
    out = attention_oracle(q, kc, vc, bt, np.array([20], dtype=np.int32), 0.4)
    assert np.array_equal(out[0, :, 0], out[0, :, 1])
    assert not np.allclose(out[0, :, 1], out[0, :, 2])    # heads 2,3 read the other kv head
