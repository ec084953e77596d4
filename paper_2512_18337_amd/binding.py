"""ctypes binding of libagentsam.so: argument marshalling only.

Every function has the name and the meaning of the C entry point it calls (see
include/agentsam.h).  torch is used for device memory and the current stream; no
step of the path is computed here.  If the library has not been built this module
raises on first use: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libagentsam.so")
_lib = None

F32, BF16 = 0, 1
_i32p = ctypes.POINTER(ctypes.c_int32)
_vp = ctypes.c_void_p

EXPORTS = ["agentsam_strerror", "sam_build", "sam_append", "sam_flat_sizes",
           "sam_flatten", "sam_wide_slots", "sam_wide_table", "sam_free", "sam_builder_create", "sam_builder_submit", "sam_builder_poll",
           "sam_builder_wait", "sam_builder_release", "sam_builder_destroy", "sam_builder_flatten", "sam_builder_flatten_result",
           "sam_delta_sizes", "sam_delta_export", "sam_apply_delta", "sam_reflatten_due",
           "sam_draft", "sam_draft_delta", "sam_draft_step", "sam_draft_merged", "spec_verify_attn_workspace", "spec_verify_attn", "spec_verify_attn_static", "spec_accept",
           "spec_adaptive_k", "spec_choose_k", "spec_switch_frontier", "agentsched_pick"]


class AgentSamError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2512_18337_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        L.agentsam_strerror.restype = ctypes.c_char_p
        L.agentsam_strerror.argtypes = [ctypes.c_int]
        L.sam_build.argtypes = [_i32p, ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(_vp)]
        L.sam_append.argtypes = [_vp, _i32p, ctypes.c_int64]
        L.sam_flat_sizes.argtypes = [_vp] + [ctypes.POINTER(ctypes.c_int64)] * 3
        L.sam_flatten.argtypes = [_vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32] + [_i32p] * 8
        L.sam_free.argtypes = [_vp]
        L.sam_free.restype = None
        L.sam_draft.argtypes = [_vp] * 12 + [ctypes.c_int32] * 5 + [_vp] * 4 + [_vp, ctypes.c_int64, _vp]
        L.sam_draft_merged.argtypes = ([_vp] * 9 + [ctypes.c_int32] + [_vp] * 2 + [ctypes.c_int32] * 5 + [_vp] * 5 +
                                       [_vp, ctypes.c_size_t, _vp, ctypes.c_int64, _vp])
        L.sam_wide_slots.argtypes = [_vp, ctypes.POINTER(ctypes.c_int64)]
        L.sam_wide_table.argtypes = [_vp, ctypes.c_int32, _i32p, ctypes.c_int64]
        L.sam_delta_sizes.argtypes = [_vp] + [ctypes.POINTER(ctypes.c_int64)] * 6
        L.sam_reflatten_due.argtypes = [_vp, ctypes.c_double, ctypes.POINTER(ctypes.c_int32)]
        L.sam_builder_flatten.argtypes = [_vp, ctypes.c_int64] + [ctypes.c_int32] * 3 + [_vp] * 8 + [ctypes.c_int64] * 3
        L.sam_builder_flatten_result.argtypes = [_vp, ctypes.c_int64]
        L.spec_adaptive_k.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
                                      ctypes.POINTER(ctypes.c_int32)]
        L.spec_choose_k.argtypes = [_vp, _vp, ctypes.c_int32, ctypes.c_double, ctypes.c_int32, ctypes.c_double,
                                    ctypes.c_double, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)]
        L.spec_switch_frontier.argtypes = [_vp, ctypes.c_int32, _vp, ctypes.c_int32, _vp, ctypes.c_int32, _vp,
                                           ctypes.c_double, ctypes.c_double, ctypes.c_double, _vp, _vp, _vp]
        L.agentsched_pick.argtypes = ([ctypes.c_int64, _vp, _vp, _vp, _vp, ctypes.c_int64] + [ctypes.c_double] * 6 +
                                      [ctypes.c_int32, ctypes.POINTER(ctypes.c_double), _vp,
                                       ctypes.POINTER(ctypes.c_int64)])
        L.sam_builder_create.argtypes = [ctypes.POINTER(_vp)]
        L.sam_builder_submit.argtypes = [_vp, ctypes.c_int64, _i32p, ctypes.c_int64, ctypes.c_int32]
        L.sam_builder_poll.argtypes = [_vp, ctypes.c_int64, ctypes.POINTER(_vp), ctypes.POINTER(ctypes.c_int64)]
        L.sam_builder_wait.argtypes = [_vp, ctypes.c_int64]
        L.sam_builder_release.argtypes = [_vp, ctypes.c_int64]
        L.sam_builder_destroy.argtypes = [_vp]
        L.sam_builder_destroy.restype = None
        L.sam_delta_export.argtypes = ([_vp, ctypes.c_int32, ctypes.c_int32] + [_vp] * 4 + [ctypes.c_int32, _vp, _vp,
                                       ctypes.POINTER(ctypes.c_int64), _vp])
        L.sam_apply_delta.argtypes = ([_vp, _vp, ctypes.c_int64, _vp, _vp, ctypes.c_int64, _vp, _vp, ctypes.c_int64] +
                                      [_vp, _vp, _vp, _vp, ctypes.c_int64, _vp])
        L.sam_draft_delta.argtypes = ([_vp] * 8 + [ctypes.c_int64] + [_vp] * 5 + [ctypes.c_int32] * 5 +
                                      [_vp] * 4 + [_vp, ctypes.c_int64, _vp])
        L.sam_draft_step.argtypes = ([_vp] * 8 + [ctypes.c_int64, _vp, _vp, ctypes.c_int64] + [_vp] * 4 +
                                     [ctypes.c_int32] * 5 + [_vp] * 6 + [_vp])
        L.spec_verify_attn_workspace.argtypes = [ctypes.c_int32] * 8 + [ctypes.c_uint64, ctypes.POINTER(ctypes.c_size_t)]
        L.spec_verify_attn.argtypes = ([_vp, _vp, _vp, _vp, ctypes.c_int32, _vp] + [ctypes.c_int32] * 6 +
                                       [ctypes.c_int64, ctypes.c_float, ctypes.c_int32, ctypes.c_int32,
                                        _vp, _vp, ctypes.c_size_t, ctypes.c_uint64, _vp])
        L.spec_verify_attn_static.argtypes = ([_vp, _vp, _vp, _vp, ctypes.c_int32, _vp] + [ctypes.c_int32] * 6 +
                                              [ctypes.c_int64, ctypes.c_float, ctypes.c_int32, ctypes.c_int32,
                                               _vp, ctypes.c_uint64, _vp])
        L.spec_accept.argtypes = [_vp, ctypes.c_int32, _vp, _vp, ctypes.c_int32, ctypes.c_int32,
                                  ctypes.c_int64, _vp, _vp, _vp, _vp]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().agentsam_strerror(code).decode()


def _check(rc: int, where: str):
    if rc != 0:
        raise AgentSamError(rc, where)


def attn_tuning(schedule: int = 0, cascade: int = 0, kv_chunk: int = 0) -> int:
    """The per-call tuning word of spec_verify_attn (AGENTSAM_ATTN_* in the header): schedule 0 auto / 1 chunk
    grid / 2 balanced; cascade 0 auto / 1 off / 2 on; kv_chunk 0 auto or KV positions per workgroup."""
    if kv_chunk % 128:
        raise ValueError("kv_chunk must be a multiple of 128")
    return int(schedule) | (int(cascade) << 2) | ((int(kv_chunk) // 128) << 8)


# ----------------------------------------------------------------------------- host automaton
def _np_i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _npp(a: np.ndarray):
    return a.ctypes.data_as(_i32p)


class Sam:
    """Owner of one sam_t handle."""

    def __init__(self, handle: int, owned: bool = True):
        self._h = _vp(handle)
        self._owned = owned            # False: the handle belongs to a SamBuilder

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h is not None and h.value and _lib is not None and getattr(self, "_owned", True):
            _lib.sam_free(h)


class SamBuilder:
    """Asynchronous construction: one child thread, a waiting queue, the automata of the submitted requests."""

    def __init__(self):
        h = _vp()
        _check(lib().sam_builder_create(ctypes.byref(h)), "sam_builder_create")
        self._h = h

    def submit(self, request_id: int, tokens, sep_token: int) -> None:
        t = _np_i32(tokens)
        _check(lib().sam_builder_submit(self._h, int(request_id), _npp(t), t.shape[0], int(sep_token)),
               "sam_builder_submit")

    def poll(self, request_id: int):
        """(Sam or None, tokens not yet in the automaton).  None: not available yet, decode without drafts."""
        out, pending = _vp(), ctypes.c_int64()
        _check(lib().sam_builder_poll(self._h, int(request_id), ctypes.byref(out), ctypes.byref(pending)),
               "sam_builder_poll")
        return (Sam(out.value, owned=False) if out.value else None), pending.value

    def flatten(self, request_id: int, out: "FlatSam") -> None:
        """Queue a sam_flatten of the request's automaton into the host arrays of `out` (one automaton at state,
        edge and corpus base 0; the arrays' sizes are the capacities).  Keep `out` alive and untouched until
        poll() hands the automaton out again; flatten_result() then tells whether it fitted."""
        pp = lambda a: _vp(a.ctypes.data)
        _check(lib().sam_builder_flatten(self._h, int(request_id), 0, 0, 0, pp(out.len), pp(out.link), pp(out.row_ptr),
                                         pp(out.edge_tok), pp(out.edge_dst), pp(out.lastpos), pp(out.corpus),
                                         pp(out.state_rec), out.len.shape[0], out.edge_tok.shape[0], out.corpus.shape[0]),
               "sam_builder_flatten")

    def flatten_result(self, request_id: int) -> int:
        return lib().sam_builder_flatten_result(self._h, int(request_id))

    def wait(self, request_id: int) -> None:
        _check(lib().sam_builder_wait(self._h, int(request_id)), "sam_builder_wait")

    def release(self, request_id: int) -> None:
        _check(lib().sam_builder_release(self._h, int(request_id)), "sam_builder_release")

    def close(self) -> None:
        h, self._h = getattr(self, "_h", None), None
        if h is not None and h.value and _lib is not None:
            _lib.sam_builder_destroy(h)

    __del__ = close


def sam_build(tokens, sep_token: int) -> Sam:
    t = _np_i32(tokens)
    h = _vp()
    _check(lib().sam_build(_npp(t), t.shape[0], int(sep_token), ctypes.byref(h)), "sam_build")
    return Sam(h.value)


def sam_append(s: Sam, tokens) -> None:
    t = _np_i32(tokens)
    _check(lib().sam_append(s._h, _npp(t), t.shape[0]), "sam_append")


def sam_flat_sizes(s: Sam):
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(lib().sam_flat_sizes(s._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)), "sam_flat_sizes")
    return a.value, b.value, c.value


@dataclass
class FlatSam:
    """The flattened arrays of one or several automata packed back to back (host numpy or device torch)."""
    len: object
    link: object
    row_ptr: object
    edge_tok: object
    edge_dst: object
    lastpos: object
    corpus: object
    state_rec: object          # [4*ns] walk records (see sam_flatten in the header)
    roots: np.ndarray          # [n_automata] root state id of each automaton
    corpus_begin: np.ndarray   # [n_automata]
    corpus_end: np.ndarray     # [n_automata] exclusive
    rows_end: np.ndarray = None  # [n_automata] end of the state ids that have a transition row (root + states flattened)
    wide_table: object = None    # [4*slots] transitions of the very wide states (see sam_wide_table in the header)

    def to(self, device):
        import torch
        cv = lambda a: torch.as_tensor(a, dtype=torch.int32).to(device)
        # zero-length arrays still need a valid (non-null) device pointer
        pad = lambda a: a if a.shape[0] > 0 else np.zeros(1, dtype=np.int32)
        return FlatSam(cv(self.len), cv(self.link), cv(self.row_ptr), cv(pad(self.edge_tok)),
                       cv(pad(self.edge_dst)), cv(self.lastpos), cv(pad(self.corpus)), cv(self.state_rec),
                       self.roots, self.corpus_begin, self.corpus_end, self.rows_end, cv(self.wide_table))


def sam_flatten(sams: Sequence[Sam], grow_tokens: int = 0) -> FlatSam:
    """sam_flatten of each automaton into one packed set of host arrays.

    With grow_tokens > 0 every automaton gets room for that many more tokens (and two states per
    token) behind its slice, so that the copy can be maintained with sam_delta_export / sam_apply_delta;
    the unused entries hold -1."""
    sizes = [sam_flat_sizes(s) for s in sams]
    g = int(grow_tokens)
    scap = [a + (2 * g if g else 0) for a, _, _ in sizes]
    ccap = [c + g for _, _, c in sizes]
    ns, ne, nt = sum(scap), sum(x[1] for x in sizes), sum(ccap)
    fill = lambda n: np.full(n, -1, np.int32)
    out = FlatSam(fill(ns), fill(ns), np.zeros(ns + 1, np.int32), np.zeros(ne, np.int32), np.zeros(ne, np.int32),
                  fill(ns), fill(nt), fill(4 * ns), np.zeros(len(sams), np.int32),
                  np.zeros(len(sams), np.int32), np.zeros(len(sams), np.int32), np.zeros(len(sams), np.int32))
    sb = eb = cb = 0
    for i, (s, (a, b, c)) in enumerate(zip(sams, sizes)):
        _check(lib().sam_flatten(s._h, sb, eb, cb, _npp(out.len[sb:]), _npp(out.link[sb:]),
                                 _npp(out.row_ptr[sb:]), _npp(out.edge_tok[eb:]) if b else None,
                                 _npp(out.edge_dst[eb:]) if b else None, _npp(out.lastpos[sb:]),
                                 _npp(out.corpus[cb:]) if c else None, _npp(out.state_rec[4 * sb:])), "sam_flatten")
        out.roots[i], out.corpus_begin[i], out.corpus_end[i], out.rows_end[i] = sb, cb, cb + c, sb + a
        out.row_ptr[sb + a:sb + scap[i] + 1] = eb + b          # states without a row (not read; kept consistent)
        sb, eb, cb = sb + scap[i], eb + b, cb + ccap[i]
    need = []
    for s in sams:
        v = ctypes.c_int64()
        _check(lib().sam_wide_slots(s._h, ctypes.byref(v)), "sam_wide_slots")
        need.append(v.value)
    slots = 2
    while slots < sum(need):
        slots *= 2
    out.wide_table = np.full(4 * slots, -1, np.int32)
    for i, s in enumerate(sams):
        _check(lib().sam_wide_table(s._h, int(out.roots[i]), _npp(out.wide_table), slots), "sam_wide_table")
    return out


@dataclass
class SamDelta:
    """What sam_delta_export wrote (host numpy arrays), see the header."""
    rec_idx: np.ndarray
    rec_val: np.ndarray        # [n_rec, 4]
    lastpos_idx: np.ndarray
    lastpos_val: np.ndarray
    ov_key: np.ndarray         # uint64, every key once
    ov_dst: np.ndarray
    new_tokens: np.ndarray
    n_overlay: int             # transitions in the log since the last sam_flatten
    flat_states: int


def sam_delta_sizes(s: Sam):
    v = [ctypes.c_int64() for _ in range(6)]
    _check(lib().sam_delta_sizes(s._h, *[ctypes.byref(x) for x in v]), "sam_delta_sizes")
    return tuple(x.value for x in v)      # n_rec, n_lastpos, n_overlay, n_overlay_new, n_new_tokens, flat_states


def sam_reflatten_due(s: Sam, max_overlay_fraction: float) -> bool:
    due = ctypes.c_int32()
    _check(lib().sam_reflatten_due(s._h, float(max_overlay_fraction), ctypes.byref(due)), "sam_reflatten_due")
    return bool(due.value)


def overlay_table(cap: int, device=None):
    """An empty overlay table: keys ~0, capacity a power of two.  Host numpy arrays (uint64, int32), or with
    `device` a pair of device tensors (int64 bit pattern of the keys, int32)."""
    assert cap >= 2 and cap & (cap - 1) == 0
    if device is None:
        return np.full(cap, np.uint64(0xFFFFFFFFFFFFFFFF), dtype=np.uint64), np.full(cap, -1, dtype=np.int32)
    import torch
    return (torch.full((cap,), -1, dtype=torch.int64, device=device),
            torch.full((cap,), -1, dtype=torch.int32, device=device))


def sam_delta_export(s: Sam, state_base: int = 0, corpus_base: int = 0, overlay_all: bool = False) -> SamDelta:
    n_rec, n_lp, n_ov, n_ov_new, n_tok, flat_states = sam_delta_sizes(s)
    n_list = n_ov if overlay_all else n_ov_new
    d = SamDelta(np.zeros(n_rec, np.int32), np.zeros((n_rec, 4), np.int32), np.zeros(n_lp, np.int32),
                 np.zeros(n_lp, np.int32), np.zeros(n_list, np.uint64), np.zeros(n_list, np.int32),
                 np.zeros(n_tok, np.int32), n_ov, flat_states)
    ptr = lambda a: _vp(a.ctypes.data) if a.size else _vp(0)
    nw = ctypes.c_int64()
    _check(lib().sam_delta_export(s._h, int(state_base), int(corpus_base), ptr(d.rec_idx), ptr(d.rec_val),
                                  ptr(d.lastpos_idx), ptr(d.lastpos_val), 1 if overlay_all else 0, ptr(d.ov_key),
                                  ptr(d.ov_dst), ctypes.byref(nw), ptr(d.new_tokens)), "sam_delta_export")
    d.ov_key, d.ov_dst = d.ov_key[:nw.value], d.ov_dst[:nw.value]
    return d


# ----------------------------------------------------------------------------- device entry points
def _stream_ptr():
    import torch
    return _vp(torch.cuda.current_stream().cuda_stream)


def _dp(t) -> _vp:
    return _vp(t.data_ptr()) if t is not None else _vp(0)


def _dev_i32(a, device):
    import torch
    if isinstance(a, torch.Tensor):
        assert a.dtype == torch.int32 and a.is_contiguous() and a.is_cuda
        return a
    return torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32)).to(device)


def sam_draft(flat: FlatSam, root, corpus_end, recent, recent_len, k: int, sep_token: int, min_match: int = 1,
              use_wide_table: bool = True):
    """Returns device tensors draft[B,k], n_draft[B], match_len[B], match_end[B]."""
    import torch
    dev = flat.len.device
    root, corpus_end = _dev_i32(root, dev), _dev_i32(corpus_end, dev)
    recent, recent_len = _dev_i32(recent, dev), _dev_i32(recent_len, dev)
    B, m = recent.shape
    draft = torch.empty((B, k), dtype=torch.int32, device=dev)
    n_draft = torch.empty((B,), dtype=torch.int32, device=dev)
    match_len = torch.empty((B,), dtype=torch.int32, device=dev)
    match_end = torch.empty((B,), dtype=torch.int32, device=dev)
    rc = lib().sam_draft(_dp(flat.len), _dp(flat.link), _dp(flat.row_ptr), _dp(flat.edge_tok), _dp(flat.edge_dst),
                         _dp(flat.lastpos), _dp(flat.corpus), _dp(flat.state_rec), _dp(root), _dp(corpus_end), _dp(recent),
                         _dp(recent_len), B, m, k, min_match, sep_token,
                         _dp(draft) if k > 0 else _vp(0), _dp(n_draft), _dp(match_len), _dp(match_end),
                         _dp(flat.wide_table) if use_wide_table else _vp(0),
                         flat.wide_table.numel() // 4 if use_wide_table else 0, _stream_ptr())
    _check(rc, "sam_draft")
    return draft, n_draft, match_len, match_end


def sam_draft_merged(flat: FlatSam, root, corpus_end, weight, recent, recent_len, k: int, sep_token: int,
                     min_match: int = 1):
    """root, corpus_end, weight: [B, M].  Returns draft[B,k], n_draft[B], match_len[B], match_end[B], source[B]."""
    import torch
    dev = flat.state_rec.device
    root, corpus_end = _dev_i32(root, dev), _dev_i32(corpus_end, dev)
    recent, recent_len = _dev_i32(recent, dev), _dev_i32(recent_len, dev)
    weight = torch.as_tensor(np.ascontiguousarray(weight, dtype=np.float32)).to(dev)
    B, m = recent.shape
    M = root.shape[1]
    assert root.shape == (B, M) and corpus_end.shape == (B, M) and weight.shape == (B, M)
    out = [torch.empty((B, k), dtype=torch.int32, device=dev)] + [torch.empty((B,), dtype=torch.int32, device=dev)
                                                                  for _ in range(4)]
    ws = torch.empty(max(1, B * M * (k + 3)), dtype=torch.int32, device=dev)
    rc = lib().sam_draft_merged(_dp(flat.row_ptr), _dp(flat.edge_tok), _dp(flat.edge_dst), _dp(flat.lastpos),
                                _dp(flat.corpus), _dp(flat.state_rec), _dp(root), _dp(corpus_end), _dp(weight), M,
                                _dp(recent), _dp(recent_len), B, m, k, min_match, sep_token,
                                _dp(out[0]) if k > 0 else _vp(0), _dp(out[1]), _dp(out[2]), _dp(out[3]), _dp(out[4]),
                                _dp(ws), ws.numel() * 4, _dp(flat.wide_table), flat.wide_table.numel() // 4,
                                _stream_ptr())
    _check(rc, "sam_draft_merged")
    return tuple(out)


def sam_apply_delta(delta: SamDelta, state_rec, lastpos, overlay_key=None, overlay_dst=None) -> None:
    """Scatter an exported delta into the device arrays state_rec [4*cap] and lastpos [cap] and insert its
    transitions into the device overlay table (overlay_key int64/uint64 bit patterns, overlay_dst int32).
    The delta's arrays may be host numpy arrays (uploaded here) or device tensors."""
    import torch
    dev = state_rec.device
    ri, rv = _dev_i32(delta.rec_idx, dev), _dev_i32(delta.rec_val.reshape(-1), dev)
    li, lv = _dev_i32(delta.lastpos_idx, dev), _dev_i32(delta.lastpos_val, dev)
    ok = delta.ov_key
    if not isinstance(ok, torch.Tensor):
        ok = torch.as_tensor(np.ascontiguousarray(ok).view(np.int64)).to(dev)
    od = _dev_i32(delta.ov_dst, dev)
    if ok.numel() and overlay_key is None:
        raise ValueError("the delta has transitions: pass the device overlay table")
    z = lambda t: _dp(t) if t is not None and t.numel() else _vp(0)
    # (the staging tensors are allocated, written and read on the current stream, and the caching allocator
    # hands their memory out again in stream order, so nothing has to be awaited here)
    _check(lib().sam_apply_delta(z(ri), z(rv), ri.numel(), z(li), z(lv), li.numel(), z(ok), z(od), ok.numel(),
                                 _dp(state_rec), _dp(lastpos), z(overlay_key), z(overlay_dst),
                                 overlay_key.numel() if overlay_key is not None else 0, _stream_ptr()), "sam_apply_delta")


def sam_draft_delta(flat: FlatSam, overlay_key, overlay_dst, rows_end, root, corpus_end, recent, recent_len, k: int,
                    sep_token: int, min_match: int = 1, use_wide_table: bool = True):
    """sam_draft on a maintained device copy; overlay_key is a device int64/uint64 tensor, overlay_dst int32.
    flat.wide_table (written when the automaton was flattened) serves the long flattened rows."""
    import torch
    dev = flat.state_rec.device
    root, corpus_end, rows_end = _dev_i32(root, dev), _dev_i32(corpus_end, dev), _dev_i32(rows_end, dev)
    recent, recent_len = _dev_i32(recent, dev), _dev_i32(recent_len, dev)
    B, m = recent.shape
    wt = flat.wide_table if use_wide_table else None
    draft = torch.empty((B, k), dtype=torch.int32, device=dev)
    n_draft = torch.empty((B,), dtype=torch.int32, device=dev)
    match_len = torch.empty((B,), dtype=torch.int32, device=dev)
    match_end = torch.empty((B,), dtype=torch.int32, device=dev)
    rc = lib().sam_draft_delta(_dp(flat.row_ptr), _dp(flat.edge_tok), _dp(flat.edge_dst), _dp(flat.lastpos),
                               _dp(flat.corpus), _dp(flat.state_rec), _dp(overlay_key), _dp(overlay_dst),
                               overlay_key.numel(), _dp(rows_end), _dp(root), _dp(corpus_end), _dp(recent),
                               _dp(recent_len), B, m, k, min_match, sep_token,
                               _dp(draft) if k > 0 else _vp(0), _dp(n_draft), _dp(match_len), _dp(match_end),
                               _dp(wt) if wt is not None else _vp(0), (wt.numel() // 4) if wt is not None else 0,
                               _stream_ptr())
    _check(rc, "sam_draft_delta")
    return draft, n_draft, match_len, match_end


def sam_draft_step(flat: FlatSam, root, corpus_end, new_tok, n_new, cur_state, cur_len, k: int, sep_token: int,
                   min_match: int = 1, overlay_key=None, overlay_dst=None, rows_end=None, use_wide_table: bool = True):
    """sam_draft with the matched state carried from call to call.  cur_state / cur_len are device int32
    tensors updated in place (start a session with cur_len = 0).  With overlay_key / overlay_dst /
    rows_end the arrays are a maintained device copy (as for sam_draft_delta)."""
    import torch
    dev = flat.state_rec.device
    root, corpus_end = _dev_i32(root, dev), _dev_i32(corpus_end, dev)
    new_tok, n_new = _dev_i32(new_tok, dev), _dev_i32(n_new, dev)
    B, max_new = new_tok.shape
    for t in (cur_state, cur_len):
        if t.dtype != torch.int32 or t.device != dev or not t.is_contiguous() or t.numel() != B:
            raise ValueError("cur_state / cur_len must be contiguous int32 device tensors of B elements")
    maintained = overlay_key is not None
    if maintained:
        rows_end = _dev_i32(rows_end, dev)
    wt = flat.wide_table if use_wide_table else None
    draft = torch.empty((B, k), dtype=torch.int32, device=dev)
    n_draft = torch.empty((B,), dtype=torch.int32, device=dev)
    match_len = torch.empty((B,), dtype=torch.int32, device=dev)
    match_end = torch.empty((B,), dtype=torch.int32, device=dev)
    rc = lib().sam_draft_step(_dp(flat.row_ptr), _dp(flat.edge_tok), _dp(flat.edge_dst), _dp(flat.lastpos),
                              _dp(flat.corpus), _dp(flat.state_rec),
                              _dp(overlay_key) if maintained else _vp(0), _dp(overlay_dst) if maintained else _vp(0),
                              overlay_key.numel() if maintained else 0, _dp(rows_end) if maintained else _vp(0),
                              _dp(wt) if wt is not None else _vp(0), (wt.numel() // 4) if wt is not None else 0,
                              _dp(root), _dp(corpus_end), _dp(new_tok) if max_new > 0 else _vp(0), _dp(n_new), B, max_new,
                              k, min_match, sep_token, _dp(cur_state), _dp(cur_len),
                              _dp(draft) if k > 0 else _vp(0), _dp(n_draft), _dp(match_len), _dp(match_end),
                              _stream_ptr())
    _check(rc, "sam_draft_step")
    return draft, n_draft, match_len, match_end


def spec_adaptive_k(batch: int, context_len: int, k: int, batch_threshold: int, context_threshold: int) -> int:
    out = ctypes.c_int32()
    _check(lib().spec_adaptive_k(int(batch), int(context_len), int(k), int(batch_threshold), int(context_threshold),
                                 ctypes.byref(out)), "spec_adaptive_k")
    return out.value


def spec_choose_k(k_values, t_step, p_accept: float, other_per_row: float = 0.0, batch: int = 1,
                  other_floor: float = 0.0):
    """Returns (k*, committed tokens per unit of cost relative to k = 0)."""
    kv = np.ascontiguousarray(k_values, dtype=np.int32)
    ts = np.ascontiguousarray(t_step, dtype=np.float64)
    assert kv.shape == ts.shape and kv.ndim == 1
    ks, gain = ctypes.c_int32(), ctypes.c_double()
    _check(lib().spec_choose_k(_vp(kv.ctypes.data), _vp(ts.ctypes.data), kv.shape[0], float(p_accept), int(batch),
                               float(other_floor), float(other_per_row), ctypes.byref(ks), ctypes.byref(gain)),
           "spec_choose_k")
    return ks.value, gain.value


def spec_switch_frontier(batches, contexts, k_values, t_step, p_accept: float, other_floor: float = 0.0,
                         other_per_row: float = 0.0):
    """t_step[nb][nc][nk].  Returns (k_star[nb][nc], context_threshold[nb], batch_threshold[nc])."""
    bs = np.ascontiguousarray(batches, dtype=np.int32)
    cs = np.ascontiguousarray(contexts, dtype=np.int64)
    kv = np.ascontiguousarray(k_values, dtype=np.int32)
    ts = np.ascontiguousarray(t_step, dtype=np.float64)
    assert ts.shape == (bs.shape[0], cs.shape[0], kv.shape[0])
    kstar = np.zeros((bs.shape[0], cs.shape[0]), np.int32)
    cthr = np.zeros(bs.shape[0], np.int64)
    bthr = np.zeros(cs.shape[0], np.int32)
    ptr = lambda x: _vp(x.ctypes.data)
    _check(lib().spec_switch_frontier(ptr(bs), bs.shape[0], ptr(cs), cs.shape[0], ptr(kv), kv.shape[0], ptr(ts),
                                      float(p_accept), float(other_floor), float(other_per_row), ptr(kstar), ptr(cthr),
                                      ptr(bthr)), "spec_switch_frontier")
    return kstar, cthr, bthr


def agentsched_pick(free_blocks: int, hit, need, prompt_tok, wait, *, lambda_max: float, k: float, eps: float,
                    a: float, b: float, c: float, tokens_per_block: int):
    """Returns (lambda, scores[n], picked index or -1)."""
    hit, need, prompt_tok = (np.ascontiguousarray(x, dtype=np.int64) for x in (hit, need, prompt_tok))
    wait = np.ascontiguousarray(wait, dtype=np.float64)
    n = hit.shape[0]
    score = np.zeros(n, np.float64)
    lam, picked = ctypes.c_double(), ctypes.c_int64()
    ptr = lambda x: _vp(x.ctypes.data) if x.size else _vp(0)
    _check(lib().agentsched_pick(int(free_blocks), ptr(hit), ptr(need), ptr(prompt_tok), ptr(wait), n,
                                 float(lambda_max), float(k), float(eps), float(a), float(b), float(c),
                                 int(tokens_per_block), ctypes.byref(lam), ptr(score), ctypes.byref(picked)),
           "agentsched_pick")
    return lam.value, score, picked.value


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def spec_verify_attn_workspace(B, R, Hq, Hkv, D, page_size, max_pages, dtype_code, tuning: int = 0) -> int:
    n = ctypes.c_size_t()
    _check(lib().spec_verify_attn_workspace(B, R, Hq, Hkv, D, page_size, max_pages, dtype_code, int(tuning),
                                            ctypes.byref(n)), "spec_verify_attn_workspace")
    return n.value


def spec_verify_attn(q, k_cache, v_cache, block_table, seq_lens, scale: float, out=None, workspace=None,
                     out_dtype=None, tuning: int = 0):
    """q[B,R,Hq,D]; caches [num_pages,Hkv,P,D]; block_table[B,max_pages] int32; seq_lens[B] int32 (device).
    tuning: see attn_tuning()."""
    import torch
    B, R, Hq, D = q.shape
    num_pages, Hkv, P, D2 = k_cache.shape
    assert D2 == D and v_cache.shape == k_cache.shape and k_cache.dtype == q.dtype == v_cache.dtype
    assert q.is_contiguous() and k_cache.is_contiguous() and v_cache.is_contiguous()
    assert block_table.dtype == torch.int32 and block_table.is_contiguous() and seq_lens.dtype == torch.int32
    max_pages = block_table.shape[1]
    code = _dtype_code(q)
    if out is None:
        out = torch.empty((B, R, Hq, D), dtype=out_dtype or torch.float32, device=q.device)
    need = spec_verify_attn_workspace(B, R, Hq, Hkv, D, P, max_pages, code, tuning)
    if workspace is None or workspace.numel() * workspace.element_size() < need:
        workspace = torch.empty((max(need, 16) + 3) // 4, dtype=torch.float32, device=q.device)
    rc = lib().spec_verify_attn(_dp(q), _dp(k_cache), _dp(v_cache), _dp(block_table), max_pages, _dp(seq_lens),
                                B, R, Hq, Hkv, D, P, num_pages, float(scale), code, _dtype_code(out),
                                _dp(out), _dp(workspace), workspace.numel() * workspace.element_size(),
                                int(tuning), _stream_ptr())
    _check(rc, "spec_verify_attn")
    return out


STATIC_WORKSPACE_BYTES = 32 << 20


def spec_verify_attn_static(q, k_cache, v_cache, block_table, seq_lens, scale: float, out, tuning: int = 0):
    """spec_verify_attn with the library's static workspace; `out` is the caller's (this call allocates nothing)."""
    import torch
    B, R, Hq, D = q.shape
    num_pages, Hkv, P, D2 = k_cache.shape
    assert D2 == D and v_cache.shape == k_cache.shape and k_cache.dtype == q.dtype == v_cache.dtype
    assert q.is_contiguous() and k_cache.is_contiguous() and v_cache.is_contiguous() and out.is_contiguous()
    assert block_table.dtype == torch.int32 and block_table.is_contiguous() and seq_lens.dtype == torch.int32
    assert tuple(out.shape) == (B, R, Hq, D)
    rc = lib().spec_verify_attn_static(_dp(q), _dp(k_cache), _dp(v_cache), _dp(block_table), block_table.shape[1],
                                       _dp(seq_lens), B, R, Hq, Hkv, D, P, num_pages, float(scale), _dtype_code(q),
                                       _dtype_code(out), _dp(out), int(tuning), _stream_ptr())
    _check(rc, "spec_verify_attn_static")
    return out


def spec_accept(logits, draft, n_draft):
    """logits[B,1+k,V] (f32|bf16), draft[B,k] int32, n_draft[B] int32 -> accept_len[B], out_tokens[B,1+k], tgt[B,1+k]."""
    import torch
    B, R, V = logits.shape
    k = R - 1
    assert logits.is_contiguous() and draft.dtype == torch.int32 and n_draft.dtype == torch.int32
    dev = logits.device
    accept_len = torch.empty((B,), dtype=torch.int32, device=dev)
    out_tokens = torch.empty((B, R), dtype=torch.int32, device=dev)
    tgt = torch.empty((B, R), dtype=torch.int32, device=dev)
    rc = lib().spec_accept(_dp(logits), _dtype_code(logits), _dp(draft) if k > 0 else _vp(0), _dp(n_draft),
                           B, k, V, _dp(accept_len), _dp(out_tokens), _dp(tgt), _stream_ptr())
    _check(rc, "spec_accept")
    return accept_len, out_tokens, tgt
