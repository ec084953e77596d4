"""fp64 verification attention (test infrastructure; see the package docstring).

The paper only says the main model validates the base token and the k drafts in
one pass (Alg. 4, "Validate with main LLM").  The attention of that pass is the
textbook definition, written out here in float64:

    for session b, query row i (0 = base token, 1..k = drafts), query head h:
        position of the row     p_i = S_b - R + i          (R = 1 + k; S_b counts the R new positions)
        kv head                 g   = h // (Hq // Hkv)
        s_j = scale * sum_d q[b,i,h,d] * K_b[j,g,d]        for j = 0 .. p_i   (causal)
        w_j = exp(s_j - max_j s_j)
        out[b,i,h,:] = sum_j w_j * V_b[j,g,:] / sum_j w_j

KV position j of session b lives in page block_table[b, j // P], slot j % P of
caches laid out [num_pages, Hkv, P, D].  Inputs are converted to float64 exactly
(bf16 and fp32 values are representable), so the oracle reads the same stored
values as the device.
"""
from __future__ import annotations

import numpy as np


def attention_oracle_head(q_rows: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """q_rows[R,D], K[S,D], V[S,D] -> out[R,D]; row i attends positions 0 .. S-R+i."""
    q_rows = np.asarray(q_rows, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    R, D = q_rows.shape
    S = K.shape[0]
    if S < R:
        raise ValueError("sequence shorter than the number of query rows")
    out = np.zeros((R, D), dtype=np.float64)
    for i in range(R):
        p = S - R + i
        s = scale * (K[: p + 1] @ q_rows[i])
        w = np.exp(s - s.max())
        out[i] = (w @ V[: p + 1]) / w.sum()
    return out


def gather_kv(cache: np.ndarray, block_table_row: np.ndarray, S: int, g: int) -> np.ndarray:
    """The S positions of one session and kv head, in sequence order: [S, D]."""
    P = cache.shape[2]
    npages = (S + P - 1) // P
    pages = np.asarray(block_table_row[:npages], dtype=np.int64)
    return cache[pages, g].reshape(npages * P, cache.shape[3])[:S]


def attention_oracle(q, k_cache, v_cache, block_table, seq_lens, scale: float,
                     heads=None) -> np.ndarray:
    """q[B,R,Hq,D]; caches [num_pages,Hkv,P,D]; block_table[B,max_pages]; seq_lens[B] -> out[B,R,Hq,D] (f64).

    `heads` optionally restricts the computation to some (b, h) pairs (the rest of
    `out` is NaN) so full-size workloads can be checked on a sample."""
    q = np.asarray(q)
    B, R, Hq, D = q.shape
    Hkv = k_cache.shape[1]
    G = Hq // Hkv
    out = np.full((B, R, Hq, D), np.nan, dtype=np.float64)
    pairs = heads if heads is not None else [(b, h) for b in range(B) for h in range(Hq)]
    for (b, h) in pairs:
        S = int(seq_lens[b])
        g = h // G
        K = gather_kv(k_cache, block_table[b], S, g)
        V = gather_kv(v_cache, block_table[b], S, g)
        out[b, :, h, :] = attention_oracle_head(q[b, :, h, :], K, V, scale)
    return out
