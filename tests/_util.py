"""Helpers shared by the GPU parity tests (inputs from the seeded generators, oracle calls)."""
import numpy as np
import torch

import paper_2512_18337_amd as A
from paper_2512_18337_amd import workloads as W


def make_memories(cfg):
    n = cfg.B if cfg.sam_mode == "per_session" else 1
    return [W.token_memory(cfg, i) for i in range(n)]


def draft_inputs(cfg, mems):
    """Flattened automata on the device plus per-session root / corpus range and the windows."""
    flat = A.sam_flatten([A.sam_build(m, cfg.sep) for m in mems])
    recent, rlen = W.recent_windows(cfg, mems)
    idx = np.arange(cfg.B) if cfg.sam_mode == "per_session" else np.zeros(cfg.B, dtype=np.int64)
    return flat, flat.roots[idx], flat.corpus_begin[idx], flat.corpus_end[idx], recent, rlen


def oracle_drafts(cfg, mems, recent, rlen, min_match=1):
    from oracle import draft_oracle_batch
    T = np.concatenate(mems)
    if cfg.sam_mode == "per_session":
        sizes = np.array([len(m) for m in mems], dtype=np.int64)
        begin = np.concatenate([[0], np.cumsum(sizes)[:-1]])
        end = begin + sizes
    else:
        begin = np.zeros(cfg.B, dtype=np.int64)
        end = np.full(cfg.B, len(T), dtype=np.int64)
    return draft_oracle_batch(T, begin, end, recent, rlen, cfg.k, cfg.sep, min_match)


def to_np(t):
    t = t.detach().cpu()                                      # bf16 crosses the bus as 2 bytes per value
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.numpy()


def oracle_attention_sample(q, kc, vc, bt, seq, scale, pairs):
    """fp64 oracle on the (b, h) pairs; copies only the pages those sessions use."""
    from oracle import attention_oracle_head
    out = {}
    G = q.shape[2] // kc.shape[1]
    P = kc.shape[2]
    for (b, h) in pairs:
        S = int(seq[b])
        npg = (S + P - 1) // P
        pages = torch.as_tensor(bt[b, :npg].astype(np.int64), device=kc.device)
        K = to_np(kc[pages, h // G]).reshape(npg * P, -1)[:S]
        V = to_np(vc[pages, h // G]).reshape(npg * P, -1)[:S]
        out[(b, h)] = attention_oracle_head(to_np(q[b, :, h]), K, V, scale)
    return out
