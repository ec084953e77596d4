"""ctypes wrapper around draft_oracle.c (test infrastructure; see the package docstring)."""
from __future__ import annotations

import ctypes
from typing import Tuple

import numpy as np

from ._clib import build_oracle_lib, load as _load, ptr as _p  # noqa: F401


def draft_oracle(T, q, k: int, sep: int, min_match: int = 1) -> Tuple[np.ndarray, int, int, int]:
    """One window against one memory.  Returns (draft[k] (-1 padded), n_draft, match_len, match_end)."""
    lib = _load()
    T = np.ascontiguousarray(T, dtype=np.int32)
    q = np.ascontiguousarray(q, dtype=np.int32)
    draft = np.full(max(k, 1), -1, dtype=np.int32)
    nd = ctypes.c_int32(0)
    ml = ctypes.c_int32(0)
    me = ctypes.c_int64(0)
    lib.draft_oracle(_p(T, ctypes.c_int32), T.shape[0], sep, _p(q, ctypes.c_int32), q.shape[0], k, min_match,
                     _p(draft, ctypes.c_int32), ctypes.byref(nd), ctypes.byref(ml), ctypes.byref(me))
    return draft[:k], nd.value, ml.value, me.value


def draft_oracle_batch(T, mem_begin, mem_end, recent, recent_len, k: int, sep: int, min_match: int = 1):
    """Batch form.  `T` is one int32 array holding every memory; session b searches
    T[mem_begin[b]:mem_end[b]] with the last recent_len[b] tokens of recent[b].
    Returns draft[B,k], n_draft[B], match_len[B], match_end[B] (relative to mem_begin[b])."""
    lib = _load()
    T = np.ascontiguousarray(T, dtype=np.int32)
    mb = np.ascontiguousarray(mem_begin, dtype=np.int64)
    me = np.ascontiguousarray(mem_end, dtype=np.int64)
    recent = np.ascontiguousarray(recent, dtype=np.int32)
    rl = np.ascontiguousarray(recent_len, dtype=np.int32)
    B, m = recent.shape
    draft = np.full((B, max(k, 1)), -1, dtype=np.int32)
    nd = np.zeros(B, dtype=np.int32)
    ml = np.zeros(B, dtype=np.int32)
    mend = np.zeros(B, dtype=np.int64)
    lib.draft_oracle_batch(_p(T, ctypes.c_int32), _p(mb, ctypes.c_int64), _p(me, ctypes.c_int64), sep,
                           _p(recent, ctypes.c_int32), _p(rl, ctypes.c_int32), B, m, k, min_match,
                           _p(draft, ctypes.c_int32), _p(nd, ctypes.c_int32), _p(ml, ctypes.c_int32),
                           _p(mend, ctypes.c_int64))
    return draft[:, :k], nd, ml, mend


def merged_draft_oracle(memories, weights, q, k, sep, min_match=1):
    """Several memories queried with one window (Alg. 4: MergeSAM with weights).  PARITY UNPINNED as to the
    rule: the paper prints no merge rule.  The reading checked here: every memory proposes as draft_oracle does, and the proposal with the
    largest weight * match_len is taken among memories with a positive weight that propose at least one
    token (equal scores: the longer match, then the earlier memory).  Scores are compared in float32, the
    precision the weights are given in.  Returns (draft, n_draft, match_len, match_end, source)."""
    import numpy as np
    best = None
    for j, (T, w) in enumerate(zip(memories, weights)):
        d, nd, ml, me = draft_oracle(np.asarray(T, np.int32), np.asarray(q, np.int32), k, sep, min_match)
        w = np.float32(w)
        if nd <= 0 or not (w > 0):
            continue
        score = np.float32(w * np.float32(ml))
        if best is None or score > best[0] or (score == best[0] and ml > best[3]):
            best = (score, d, nd, ml, me, j)
    if best is None:
        return np.full(k, -1, np.int32), 0, 0, -1, -1
    return best[1], best[2], best[3], best[4], best[5]


def _occurs(T: np.ndarray, pat: np.ndarray) -> bool:
    """Does pat occur in T as a contiguous run?  Plain scan."""
    n, m = T.shape[0], pat.shape[0]
    if m == 0:
        return True
    if m > n:
        return False
    cand = np.flatnonzero(T[: n - m + 1] == pat[0])
    for j in range(1, m):
        if cand.size == 0:
            return False
        cand = cand[T[cand + j] == pat[j]]
    return cand.size > 0


def carried_match_len_oracle(T, ctx, L_prev: int, n_new: int) -> int:
    """Length of the match carried from call to call (Alg. 4, the decoding loop: the decoder follows
    transitions from the current verified suffix).  ctx = every token of the session so far, the last n_new
    of them not yet consumed; L_prev = the carried length before them; T = the memory as it is NOW.
    For each new token t_n, in order:
        L_n = max { l+1 : 0 <= l <= L_(n-1), ctx[n-l .. n] occurs in T },  0 if t_n does not occur in T.
    (A match is extended by one token or cut from the left; a longer one is never looked for.)"""
    T = np.ascontiguousarray(T, dtype=np.int32)
    ctx = np.ascontiguousarray(ctx, dtype=np.int32)
    L = int(L_prev)
    for n in range(ctx.shape[0] - n_new, ctx.shape[0]):
        new_L = 0
        for l in range(min(L, n), -1, -1):
            if _occurs(T, ctx[n - l: n + 1]):
                new_L = l + 1
                break
        L = new_L
    return L


def draft_step_oracle(T, ctx, L_prev: int, n_new: int, k: int, sep: int, min_match: int = 1):
    """One call of the stateful lookup: the carried length after the new tokens, then the proposal that
    draft_oracle makes for a window of exactly that many tokens.
    Returns (L, draft[k], n_draft, match_len, match_end)."""
    L = carried_match_len_oracle(T, ctx, L_prev, n_new)
    ctx = np.ascontiguousarray(ctx, dtype=np.int32)
    if L == 0:
        return 0, np.full(k, -1, np.int32), 0, 0, -1
    d, nd, ml, me = draft_oracle(T, ctx[ctx.shape[0] - L:], k, sep, min_match)
    return L, d, nd, ml, me
