"""ctypes wrapper around accept_oracle.c (test infrastructure; see the package docstring)."""
from __future__ import annotations

import ctypes

import numpy as np

from ._clib import load as _load, ptr as _p


def accept_oracle(logits, draft, n_draft):
    """logits[B,R,V] float32 (bf16 widened exactly by the caller), draft[B,k], n_draft[B]
    -> accept_len[B], out_tokens[B,R], tgt[B,R]   with R = 1 + k."""
    lib = _load()
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    B, R, V = logits.shape
    k = R - 1
    draft = np.ascontiguousarray(draft, dtype=np.int32).reshape(B, k)
    n_draft = np.ascontiguousarray(n_draft, dtype=np.int32)
    accept_len = np.zeros(B, dtype=np.int32)
    out_tokens = np.full((B, R), -1, dtype=np.int32)
    tgt = np.zeros((B, R), dtype=np.int32)
    dptr = _p(draft, ctypes.c_int32) if k > 0 else ctypes.POINTER(ctypes.c_int32)()
    lib.accept_oracle(_p(logits, ctypes.c_float), dptr, _p(n_draft, ctypes.c_int32), B, k, V,
                      _p(accept_len, ctypes.c_int32), _p(out_tokens, ctypes.c_int32), _p(tgt, ctypes.c_int32))
    return accept_len, out_tokens, tgt
