"""Seeded synthetic inputs for one AgentSAM speculative step.

This module only *draws inputs* (token memories, recent-token windows, paged
KV caches, query rows, verification logits).  It contains none of the method's
arithmetic: no suffix matching, no attention, no argmax/accept logic.  It is
the one module shared by the HIP path's tests/bench and by the CPU oracle's
tests; neither of those two imports the other.

The workloads stand in for the agent trajectories the paper evaluates on
(Sec. "Evaluation on AgentSAM"): token memories are Zipf-distributed base text
with copied spans (agent contexts revisit retrieved content, Sec. 5.4.1), and
the verification logits are random with the draft token planted as the row
maximum with a given probability, so accept lengths are truncated-geometric.

Token-side data comes from a counter-based splitmix64 generator implemented
here with numpy integer ops, so it is identical on every machine.  Bulk float
tensors (K/V pages, queries, logits) come from a seeded torch generator on the
device they are needed on.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import List, Optional, Tuple

import numpy as np

SEED_BASE = 18337

# sub-stream ids under one config seed
_SUB_TOKENS, _SUB_WINDOWS, _SUB_KV, _SUB_LOGITS, _SUB_PAGES = range(5)


# --------------------------------------------------------------------------- PRNG
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _splitmix64(z: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = z + _GOLD
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


class Stream:
    """Counter-based uniform generator: value i is splitmix64(key + i*gold)."""

    def __init__(self, seed: int, sub: int):
        key = np.array([(seed * 16 + sub) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64)
        self._key = _splitmix64(_splitmix64(key))[0]
        self._ctr = 0

    def u64(self, n: int) -> np.ndarray:
        idx = np.arange(self._ctr, self._ctr + n, dtype=np.uint64)
        self._ctr += n
        with np.errstate(over="ignore"):
            return _splitmix64(self._key + idx * _GOLD)

    def uniform(self, n: int) -> np.ndarray:
        """float64 in [0, 1) with 53 random bits."""
        return (self.u64(n) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))

    def randint(self, lo: int, hi: int, n: int) -> np.ndarray:
        """int64 uniform in [lo, hi] inclusive."""
        span = hi - lo + 1
        return lo + np.minimum((self.uniform(n) * span).astype(np.int64), span - 1)

    def one_uniform(self) -> float:
        return float(self.uniform(1)[0])

    def one_int(self, lo: int, hi: int) -> int:
        return int(self.randint(lo, hi, 1)[0])


# --------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class Config:
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    page: int
    k: int
    dtype: str                      # "f32" | "bf16"  (Q/K/V storage type)
    kv_mode: str                    # "fixed" | "ragged" | "shared_prefix"
    kv_len: Tuple[int, int]         # fixed: (S, S); ragged: U[lo, hi]; shared_prefix: private suffix U[lo, hi]
    prefix_len: int                 # shared_prefix only
    permute_pages: bool
    sam_mode: str                   # "per_session" (one automaton per session) | "shared"
    sam_sessions: int               # number of SEP-terminated segments in one automaton's memory
    sam_session_len: int            # tokens per segment, SEP included
    vocab: int
    zipf_s: float                   # 0 => uniform base tokens
    copy_frac: float                # covered fraction of the memory that is copied spans
    span: Tuple[int, int]
    cross_session: bool             # copy sources come from a different (earlier) segment
    m: int                          # recent-token window length
    logits_dtype: str               # "f32" | "bf16"
    match_prob: Tuple[float, float]  # injection probability at draft 0 and at draft k-1 (linear between)
    seed: int

    @property
    def R(self) -> int:
        return 1 + self.k

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def sep(self) -> int:
        return self.vocab            # separator id lies outside the vocabulary


def baseline_config(i: int) -> Config:
    """The five workloads of the build's baseline list, by index."""
    s = SEED_BASE + i
    if i == 0:
        return Config("cfg0-tiny-fp32", 2, 4, 1, 64, 64, 4, "f32", "fixed", (256, 256), 0, False,
                      "per_session", 1, 2048, 1024, 0.0, 0.3, (8, 32), False, 16, "f32", (0.7, 0.7), s)
    if i == 1:
        return Config("cfg1-b16-8k", 16, 32, 8, 128, 64, 8, "bf16", "fixed", (8192, 8192), 0, False,
                      "per_session", 1, 65536, 32000, 1.1, 0.3, (8, 64), False, 64, "f32", (0.7, 0.7), s)
    if i == 2:
        return Config("cfg2-b64-32k", 64, 32, 8, 128, 64, 8, "bf16", "fixed", (32768, 32768), 0, False,
                      "shared", 64, 4096, 32000, 1.1, 0.4, (16, 128), True, 64, "f32", (0.6, 0.6), s)
    if i == 3:
        return Config("cfg3-ragged-b128", 128, 64, 8, 128, 64, 16, "bf16", "ragged", (1024, 65536), 0, True,
                      "shared", 128, 16384, 151936, 1.05, 0.35, (8, 256), False, 64, "bf16", (0.8, 0.3), s)
    if i == 4:
        return Config("cfg4-shared-prefix", 32, 40, 8, 128, 64, 8, "bf16", "shared_prefix", (4096, 16384),
                      98304, False, "shared", 32, 32768, 151936, 1.05, 0.5, (64, 512), False, 64, "f32",
                      (0.65, 0.65), s)
    raise ValueError(f"no baseline config {i}")


def scaled(cfg: Config, **kw) -> Config:
    """A copy of `cfg` with some fields overridden (used for oracle-sized parity cases)."""
    return dataclasses.replace(cfg, **kw)


# --------------------------------------------------------------------------- token memories
def _zipf_cdf(vocab: int, s: float) -> Optional[np.ndarray]:
    if s <= 0.0:
        return None
    w = 1.0 / np.power(np.arange(1, vocab + 1, dtype=np.float64), s)
    c = np.cumsum(w)
    return c / c[-1]


def _base_tokens(st: Stream, n: int, vocab: int, cdf: Optional[np.ndarray]) -> np.ndarray:
    u = st.uniform(n)
    if cdf is None:
        return np.minimum((u * vocab).astype(np.int64), vocab - 1).astype(np.int32)
    return np.minimum(np.searchsorted(cdf, u, side="right"), vocab - 1).astype(np.int32)


def token_memory(cfg: Config, which: int = 0) -> np.ndarray:
    """One automaton's token memory: `sam_sessions` segments, each ending in SEP.

    Base tokens are Zipf(s) ranks (id = rank-1) or uniform.  Walking left to
    right, outside a span a copied span starts with the probability that makes
    the covered fraction `copy_frac`; its length is U[span] and its source a
    uniform earlier offset (in an earlier segment when `cross_session`).
    `which` selects the automaton when there is one per session.
    """
    st = Stream(cfg.seed, _SUB_TOKENS)
    st._ctr = which * (1 << 40)      # disjoint counter ranges per automaton
    seg, nseg = cfg.sam_session_len, cfg.sam_sessions
    n = seg * nseg
    cdf = _zipf_cdf(cfg.vocab, cfg.zipf_s)
    T = _base_tokens(st, n, cfg.vocab, cdf)
    a, b = cfg.span
    mean_len = 0.5 * (a + b)
    f = cfg.copy_frac
    q = f / (mean_len * (1.0 - f) + f) if f > 0 else 0.0
    if q > 0:
        est = int(n / (mean_len + 1.0 / q) * 1.5) + 64
        gaps = np.floor(np.log1p(-st.uniform(est)) / np.log1p(-q)).astype(np.int64)
        lens = st.randint(a, b, est)
        usrc = st.uniform(est)
        useg = st.uniform(est)
        pos = 0
        for i in range(est):
            pos += int(gaps[i])
            L = int(lens[i])
            if pos + L > n:
                break
            s_idx = pos // seg
            # a span stays inside its segment and never overwrites the segment's SEP slot
            L = min(L, (s_idx + 1) * seg - 1 - pos)
            if L >= 1:
                if cfg.cross_session and s_idx > 0:
                    src_seg = min(int(useg[i] * s_idx), s_idx - 1)
                    lo, hi = src_seg * seg, (src_seg + 1) * seg - 1 - L
                else:
                    lo, hi = 0, pos - L
                if hi >= lo:
                    src = lo + min(int(usrc[i] * (hi - lo + 1)), hi - lo)
                    T[pos:pos + L] = T[src:src + L]
                pos += L
    # SEP-terminate every segment (done last, so no copy ever carries a SEP)
    T[seg - 1::seg] = cfg.sep
    return T


def recent_windows(cfg: Config, memories: List[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """`recent[B, m]` (right-aligned, -1 padded on the left) and `recent_len[B]`.

    With probability 0.85 the window is cut from the session's automaton memory
    ending at a random position whose successor exists and is not SEP, and the
    token at distance U[1, m) from the window's end is replaced by a random id
    (so match lengths spread over 1..m-1); otherwise it is m random ids.
    """
    st = Stream(cfg.seed, _SUB_WINDOWS)
    B, m = cfg.B, cfg.m
    recent = np.full((B, m), -1, dtype=np.int32)
    rlen = np.full((B,), m, dtype=np.int32)
    for b in range(B):
        T = memories[b if cfg.sam_mode == "per_session" else 0]
        n = T.shape[0]
        if st.one_uniform() < 0.85 and n > m + 1:
            w = None
            for _ in range(64):
                p = st.one_int(m - 1, n - 2)
                cand = T[p - m + 1:p + 1]
                if T[p + 1] != cfg.sep and not np.any(cand == cfg.sep):
                    w = cand.copy()
                    break
            if w is None:
                w = st.randint(0, cfg.vocab - 1, m).astype(np.int32)
            elif m >= 2:
                d = st.one_int(1, m - 1)
                w[m - 1 - d] = st.one_int(0, cfg.vocab - 1)
        else:
            w = st.randint(0, cfg.vocab - 1, m).astype(np.int32)
        recent[b] = w
    return recent, rlen


# --------------------------------------------------------------------------- paged KV layout
@dataclass
class KVLayout:
    seq_lens: np.ndarray        # [B] int32, counts the R new positions too
    block_table: np.ndarray     # [B, max_pages] int32, -1 where unused
    num_pages: int


def kv_layout(cfg: Config) -> KVLayout:
    st = Stream(cfg.seed, _SUB_PAGES)
    B, P = cfg.B, cfg.page
    if cfg.kv_mode == "fixed":
        seq = np.full(B, cfg.kv_len[0], dtype=np.int64)
        shared_pages = 0
    elif cfg.kv_mode == "ragged":
        seq = st.randint(cfg.kv_len[0], cfg.kv_len[1], B)
        shared_pages = 0
    elif cfg.kv_mode == "shared_prefix":
        assert cfg.prefix_len % P == 0
        seq = cfg.prefix_len + st.randint(cfg.kv_len[0], cfg.kv_len[1], B)
        shared_pages = cfg.prefix_len // P
    else:
        raise ValueError(cfg.kv_mode)
    npages = (seq + P - 1) // P
    private = npages - shared_pages
    total = shared_pages + int(private.sum())
    if cfg.permute_pages:
        order = np.argsort(st.u64(total), kind="stable").astype(np.int64)
    else:
        order = np.arange(total, dtype=np.int64)
    max_pages = int(npages.max())
    bt = np.full((B, max_pages), -1, dtype=np.int32)
    nxt = shared_pages
    for b in range(B):
        bt[b, :shared_pages] = order[:shared_pages]
        bt[b, shared_pages:npages[b]] = order[nxt:nxt + private[b]]
        nxt += int(private[b])
    return KVLayout(seq.astype(np.int32), bt, total)


def torch_dtype(name: str):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def kv_and_queries(cfg: Config, layout: KVLayout, device: str):
    """q[B,R,Hq,D], k_cache, v_cache[num_pages,Hkv,P,D] ~ N(0,1) in cfg.dtype, drawn page-block-wise."""
    import torch
    dt = torch_dtype(cfg.dtype)
    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed * 16 + _SUB_KV)
    q = torch.randn((cfg.B, cfg.R, cfg.Hq, cfg.D), generator=g, device=device, dtype=torch.float32).to(dt)
    shape = (layout.num_pages, cfg.Hkv, cfg.page, cfg.D)
    kc = torch.empty(shape, device=device, dtype=dt)
    vc = torch.empty(shape, device=device, dtype=dt)
    step = max(1, (1 << 26) // (cfg.Hkv * cfg.page * cfg.D))      # ~256 MB of fp32 per draw
    for p0 in range(0, layout.num_pages, step):
        p1 = min(layout.num_pages, p0 + step)
        kc[p0:p1] = torch.randn((p1 - p0,) + shape[1:], generator=g, device=device, dtype=torch.float32).to(dt)
        vc[p0:p1] = torch.randn((p1 - p0,) + shape[1:], generator=g, device=device, dtype=torch.float32).to(dt)
    return q, kc, vc


def verify_logits(cfg: Config, draft: np.ndarray, n_draft: np.ndarray, device: str):
    """logits[B,R,V] ~ N(0,1); for row j < n_draft[b], with probability p_j the
    entry of the draft token is raised to (row maximum + 1)."""
    import torch
    st = Stream(cfg.seed, _SUB_LOGITS)
    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed * 16 + _SUB_LOGITS)
    B, R, V, k = cfg.B, cfg.R, cfg.vocab, cfg.k
    dt = torch_dtype(cfg.logits_dtype)
    logits = torch.empty((B, R, V), device=device, dtype=dt)
    for b in range(B):
        logits[b] = torch.randn((R, V), generator=g, device=device, dtype=torch.float32).to(dt)
    u = st.uniform(B * k).reshape(B, k)
    p0, p1 = cfg.match_prob
    pj = np.array([p0 + (p1 - p0) * (j / max(1, k - 1)) for j in range(k)])
    bs, js = np.nonzero((u < pj[None, :]) & (np.arange(k)[None, :] < n_draft[:, None]))
    if bs.size:
        tb = torch.as_tensor(bs, device=device)
        tj = torch.as_tensor(js, device=device)
        tt = torch.as_tensor(draft[bs, js].astype(np.int64), device=device)
        rowmax = logits[tb, tj].float().max(dim=1).values
        logits[tb, tj, tt] = (rowmax + 1.0).to(dt)
    return logits
