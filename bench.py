#!/usr/bin/env python3
"""Benchmark of one AgentSAM speculative step on one MI355X.

A step = sam_draft + spec_verify_attn + spec_accept back to back on one stream over one batch
of synthetic sessions (inputs resident in HBM before the timed region).  The default workload
is the configuration the headline metric is quoted on: B=64 sessions, 32k-token KV per session,
k=8 drafts (baseline workload 2).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--seed S] [--no-cpu-baseline]
                    [--no-targets] [--ksweep] [--maintain STEPS] ...

Beside the headline step the default run also times spec_verify_attn alone on workloads 3 and 4
(`detail.targets`), the two other configurations the bandwidth target is stated for.
"""
from __future__ import annotations

import argparse
import ctypes
import hashlib
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = 2500.0        # MI355X published dense bf16 matrix rate
ATTN_SOURCE = os.path.join(ROOT, "paper_2512_18337_amd", "csrc", "spec_verify_attn.hip")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")
# An idle GPU takes some 15 ms of work to reach its clocks (the first ten launches of the headline workload run 9 %
# slower than the ones after them): a warm-up lasts at least this long, however few steps were asked for.
MIN_WARMUP_S = 0.03
SEED_GEMM = 18337                # operands of the library-GEMM yardstick


def warm_up(fn, min_calls=3):
    """Calls fn (which queues GPU work) at least min_calls times and for at least MIN_WARMUP_S of GPU time."""
    import torch
    t_w, n = time.perf_counter(), 0
    while n < min_calls or time.perf_counter() - t_w < MIN_WARMUP_S:
        fn()
        n += 1
        if n >= min_calls:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    return n


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=2, help="baseline workload index (default: the headline one)")
    ap.add_argument("--seed", type=int, default=None, help="seed of the synthetic inputs (default: the workload's own)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-targets", action="store_true", help="skip the attention-only timings of workloads 3 and 4")
    ap.add_argument("--attn-only", action="store_true", help="time only spec_verify_attn (for profiling)")
    ap.add_argument("--kv-chunk", type=int, default=0)
    ap.add_argument("--schedule", type=int, default=0, help="attention schedule: 0 auto, 1 chunk grid, 2 balanced")
    ap.add_argument("--cascade", type=int, default=0, help="shared-prefix run: 0 auto, 1 off, 2 on")
    ap.add_argument("--ksweep", action="store_true",
                    help="also time spec_verify_attn for k = 0..16 drafts on this workload's batch and context lengths and "
                         "derive the speculation controller's choice from that table (detail.ksweep)")
    ap.add_argument("--maintain", type=int, default=0, metavar="STEPS",
                    help="also time STEPS rounds of incremental automaton maintenance (append, delta export, "
                         "device update, sam_draft_delta); reported under detail.sam_maintenance")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy (5 times): a kernel of known HBM traffic "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters with")
    ap.add_argument("--cold", action="store_true",
                    help="write a 512 MiB scratch buffer before every step (outside the timed events), so that nothing of "
                         "the previous step is left in the caches; ms_per_step is then the sum of the kernels' event times")
    ap.add_argument("--zero-inputs", action="store_true",
                    help="experiments only, with --attn-only: K, V and Q all zero - the same instruction stream without "
                         "data toggling in the matrix pipes, which shows what the GPU's power limit costs a workload")
    ap.add_argument("--set", action="append", default=[], metavar="FIELD=VALUE",
                    help="override a workload field (experiments only), e.g. --set permute_pages=False")
    return ap.parse_args()


# ------------------------------------------------------------------------------------- CPU oracle timing
def host_threads() -> int:
    """Host cores this process may use (a one-GPU machine gives 16 whatever the machine has)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(n, 16))


def cpu_baseline(cfg, mems, recent, rlen, q, kc, vc, lay, logits, draft_h, nd_h, budget_s=18.0):
    """The CPU oracle as it stands, timed on this machine's host cores on a bounded sample of the step: once with
    its sessions / (session, head) pairs farmed out to one thread per core (the numerical library held to one
    thread each), once on a single thread."""
    import torch
    from threadpoolctl import threadpool_limits
    from oracle import accept_oracle, attention_oracle_head, draft_oracle
    from oracle.attention import gather_kv
    nthr = host_threads()
    P = cfg.page
    scale = 1.0 / np.sqrt(cfg.D)
    if cfg.sam_mode == "per_session":
        mem_of = lambda b: mems[b]
    else:
        mem_of = lambda b: mems[0]
    lg = logits.float().cpu().numpy()
    total_pos = int(lay.seq_lens.astype(np.int64).sum()) * cfg.Hq

    def draft_one(b):
        draft_oracle(mem_of(b), recent[b, cfg.m - rlen[b]:], cfg.k, cfg.sep)

    def accept_one(b):
        accept_oracle(lg[b:b + 1], draft_h[b:b + 1], nd_h[b:b + 1])

    def attn_pair(job):
        qh, Kp, Vp, S = job
        ident = np.arange(Kp.shape[0])
        attention_oracle_head(qh, gather_kv(Kp, ident, S, 0), gather_kv(Vp, ident, S, 0), scale)

    def stage_session(b, heads):
        """Host copies of what the oracle reads for some query heads of session b (not timed: the oracle's input)."""
        S = int(lay.seq_lens[b]); npg = (S + P - 1) // P
        pages = torch.as_tensor(lay.block_table[b, :npg].astype(np.int64), device=kc.device)
        jobs, kv = [], {}
        for h in heads:
            g = h // cfg.G
            if g not in kv:
                kv[g] = (kc[pages, g].cpu().float().numpy()[:, None], vc[pages, g].cpu().float().numpy()[:, None])
            jobs.append((q[b, :, h].float().cpu().numpy(), kv[g][0], kv[g][1], S))
        return jobs

    def run(workers, budget):
        """(t_draft, t_accept, t_attn extrapolated to the whole batch, pairs done, t_attn measured)"""
        with threadpool_limits(limits=1), ThreadPoolExecutor(max_workers=workers) as pool:
            t0 = time.perf_counter(); list(pool.map(draft_one, range(cfg.B))); t_draft = time.perf_counter() - t0
            t0 = time.perf_counter(); list(pool.map(accept_one, range(cfg.B))); t_accept = time.perf_counter() - t0
            rng = np.random.default_rng(cfg.seed)
            done, pos_done, t_attn = 0, 0, 0.0
            for b in rng.permutation(cfg.B):                  # whole sessions, in a seeded order, until the budget is spent
                if t_attn >= budget:
                    break
                heads = list(range(cfg.Hq)) if workers > 1 else [int(h) for h in rng.choice(cfg.Hq, 4, replace=False)]
                jobs = stage_session(int(b), heads)
                t0 = time.perf_counter(); list(pool.map(attn_pair, jobs)); t_attn += time.perf_counter() - t0
                done += len(jobs); pos_done += int(lay.seq_lens[b]) * len(jobs)
        return t_draft, t_accept, t_attn * total_pos / max(1, pos_done), done, t_attn

    cpu0, wall0 = time.process_time(), time.perf_counter()
    td, ta, tattn_full, done, tattn = run(nthr, budget_s)
    cpu1, wall1 = time.process_time(), time.perf_counter()
    td1, ta1, tattn_full1, done1, tattn1 = run(1, budget_s / 4)
    model = ""
    try:
        with open("/proc/cpuinfo") as f:
            model = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), "")
    except OSError:
        pass
    return {
        "value": cfg.B * cfg.k / (td + tattn_full + ta), "unit": "tokens/s", "cores": nthr, "kind": "oracle",
        "sample": (f"{nthr} worker threads, one per host core, the numerical library held to one thread each: draft oracle "
                   f"on all {cfg.B} sessions ({td:.3f} s) + accept oracle on all {cfg.B * cfg.R} rows ({ta:.3f} s) + fp64 "
                   f"attention oracle on {done} (session, head) pairs of {cfg.B * cfg.Hq}, whole sessions in a seeded order "
                   f"({tattn:.1f} s, extrapolated linearly by KV positions to {tattn_full:.1f} s)"),
        "cpu_time_over_wall_time": (cpu1 - cpu0) / max(1e-9, wall1 - wall0),
        "host_cpus": os.cpu_count(), "cpu_model": model,
        "single_thread": {"value": cfg.B * cfg.k / (td1 + tattn_full1 + ta1), "unit": "tokens/s", "cores": 1,
                          "sample": (f"the same on one thread: draft {td1:.3f} s, accept {ta1:.3f} s, attention oracle on "
                                     f"{done1} pairs ({tattn1:.1f} s, extrapolated to {tattn_full1:.1f} s)")},
    }


# ------------------------------------------------------------------------------------- roofline
def attention_work(cfg, lay):
    """Algorithmic bytes (every session's whole K/V once per kv head), the bytes of the distinct pages, and the matrix work."""
    kv_elem = 2 if cfg.dtype == "bf16" else 4
    positions = float(lay.seq_lens.astype(np.int64).sum())
    alg_bytes = positions * cfg.Hkv * 2 * cfg.D * kv_elem
    used_pages = np.unique(lay.block_table[lay.block_table >= 0]).size
    unique_bytes = float(used_pages) * cfg.page * cfg.Hkv * 2 * cfg.D * kv_elem
    flops = 4.0 * cfg.D * cfg.G * cfg.R * positions * cfg.Hkv
    return alg_bytes, unique_bytes, flops


def measured_traffic(workload: str):
    """HBM bytes per spec_verify_attn call from the rocprofv3 counter runs recorded in profiles/traffic.json, or None
    when the kernel source has changed since they were taken (the record names the source it was measured on)."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f).get(workload)
        with open(ATTN_SOURCE, "rb") as f:
            sha = hashlib.sha256(f.read()).hexdigest()
    except (OSError, ValueError):
        return None
    if not rec or rec.get("kernel_source_sha256") != sha:
        return None
    return float(rec["hbm_bytes_per_call"])


def attention_roofline(cfg, lay, t_attn_ms, stream_gbs=None, paged_gbs=None):
    """What bounds spec_verify_attn on this workload and how close the launch came.  Pages that several sessions
    list are needed from HBM once, so the memory bound counts the DISTINCT pages; the bound of the workload is the
    larger of that and the matrix work at the dense bf16 rate, and `frac` = bound / measured time."""
    alg_bytes, unique_bytes, flops = attention_work(cfg, lay)
    unique_bytes = min(unique_bytes, alg_bytes)              # (whole pages: the unused end of a last page is not read)
    t = t_attn_ms * 1e-3
    t_hbm = unique_bytes / (HBM_PEAK_GBS * 1e9)
    t_mfma = flops / (MFMA_PEAK_TFLOPS * 1e12) if cfg.dtype == "bf16" else 0.0
    r = {"kernel": "spec_verify_attn", "launch_ms": t_attn_ms, "traffic": measured_traffic(cfg.name),
         "algorithmic_bytes": alg_bytes, "unique_bytes": unique_bytes, "matrix_flops": flops,
         "hbm_bound_ms": t_hbm * 1e3, "mfma_bound_ms": t_mfma * 1e3,
         "logical_GBs": alg_bytes / t / 1e9, "unique_GBs": unique_bytes / t / 1e9,
         "mfma_TFLOPs": flops / t / 1e12, "mfma_frac_of_2500": flops / t / (MFMA_PEAK_TFLOPS * 1e12)}
    if t_hbm >= t_mfma:
        r.update({"bound": "hbm", "achieved": unique_bytes / t / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"})
    else:
        r.update({"bound": "mfma", "achieved": flops / t / 1e12, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s"})
    r["frac"] = r["achieved"] / r["peak"]
    if stream_gbs:
        r["stream_read_GBs"] = stream_gbs
        r["frac_of_stream_read"] = unique_bytes / t / 1e9 / stream_gbs
    if paged_gbs:                                            # the same loads through the block table, nothing else
        r["paged_read_GBs"] = paged_gbs
        r["frac_of_paged_read"] = unique_bytes / t / 1e9 / paged_gbs
    return r


# ------------------------------------------------------------------------------------- inputs and timing
class AttnInputs:
    def __init__(self, A, W, cfg, dev, tuning):
        import torch
        self.cfg, self.tuning = cfg, tuning
        self.lay = W.kv_layout(cfg)
        self.q, self.kc, self.vc = W.kv_and_queries(cfg, self.lay, dev)
        self.bt = torch.as_tensor(self.lay.block_table, device=dev)
        self.seq = torch.as_tensor(self.lay.seq_lens, device=dev)
        self.scale = 1.0 / float(np.sqrt(cfg.D))
        self.ws_bytes = A.spec_verify_attn_workspace(cfg.B, cfg.R, cfg.Hq, cfg.Hkv, cfg.D, cfg.page, self.bt.shape[1],
                                                     A.BF16 if cfg.dtype == "bf16" else A.F32, tuning)
        self.ws = torch.empty(max(self.ws_bytes, 16) // 4 + 1, dtype=torch.float32, device=dev)
        self.out = torch.empty((cfg.B, cfg.R, cfg.Hq, cfg.D), dtype=torch.float32, device=dev)
        self.A = A

    def attn(self):
        self.A.spec_verify_attn(self.q, self.kc, self.vc, self.bt, self.seq, self.scale, out=self.out, workspace=self.ws,
                                tuning=self.tuning)

    def time_attn(self, launches, warmup=10):
        """Mean HIP-event time of one spec_verify_attn call (all its launches), in ms, on the launch stream.
        (An idle GPU takes some 15 ms of work to reach its clocks: the first ten launches of the headline
        workload run 9 % slower than the ones after them, so the warm-up is that long.)"""
        import torch
        warm_up(self.attn, warmup)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(launches)]
        for e0, e1 in evs:
            e0.record(); self.attn(); e1.record()
        torch.cuda.synchronize()
        return float(np.mean([e0.elapsed_time(e1) for e0, e1 in evs]))


def stream_read_rate(dev):
    """The rate this device delivers to a kernel that only streams (4 GiB, 5 launches), GB/s."""
    import torch
    from paper_2512_18337_amd.build import BENCH_LIB
    probe_lib = ctypes.CDLL(BENCH_LIB)                       # the benchmark's own helper, not the product library
    probe_lib.bench_stream_read_probe.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    buf = torch.ones(1 << 30, dtype=torch.float32, device=dev)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)

    def probe():
        rc = probe_lib.bench_stream_read_probe(buf.data_ptr(), buf.numel() * 4, sink.data_ptr(),
                                               torch.cuda.current_stream().cuda_stream)
        assert rc == 0, rc

    probe()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        probe()
    e1.record()
    torch.cuda.synchronize()
    return buf.numel() * 4 * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9


def paged_read_rate(inp, dev):
    """The rate at which a kernel that makes the narrow attention kernel's loads through the block table and nothing
    else reads this workload's K and V (sessions of one length, bf16 only), GB/s; None for other workloads."""
    import torch
    from paper_2512_18337_amd.build import BENCH_LIB
    cfg, lay = inp.cfg, inp.lay
    if cfg.dtype != "bf16" or int(lay.seq_lens.min()) != int(lay.seq_lens.max()) or cfg.page % 32 != 0:
        return None
    tiles = int(lay.seq_lens.min()) // 32
    if tiles < 1:
        return None
    probe_lib = ctypes.CDLL(BENCH_LIB)
    probe_lib.bench_paged_read_probe.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                                 ctypes.c_longlong, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                 ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    sink = torch.zeros(4, dtype=torch.float32, device=dev)

    def probe():
        rc = probe_lib.bench_paged_read_probe(inp.kc.data_ptr(), inp.vc.data_ptr(), inp.bt.data_ptr(), inp.bt.shape[1],
                                              int(lay.num_pages), cfg.B, cfg.Hkv, cfg.page, cfg.D, tiles,
                                              sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert rc == 0, rc

    for _ in range(3):
        probe()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        probe()
    e1.record()
    torch.cuda.synchronize()
    nbytes = 2.0 * cfg.B * cfg.Hkv * tiles * 32 * cfg.D * 2
    return nbytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9


def library_gemm_rate(dev, n=8192, launches=20):
    """A yardstick for the matrix-bound workload, as the streaming probe is one for the HBM-bound ones: what the
    vendor library's plain bf16 GEMM (torch.matmul, n x n x n, N(0,1) operands) sustains on this GPU, in TFLOP/s.
    Not part of the path: nothing in the library calls it."""
    import torch
    g = torch.Generator(device=dev)
    g.manual_seed(SEED_GEMM)
    a = torch.randn(n, n, device=dev, dtype=torch.bfloat16, generator=g)
    b = torch.randn(n, n, device=dev, dtype=torch.bfloat16, generator=g)
    c = torch.empty(n, n, device=dev, dtype=torch.bfloat16)
    warm_up(lambda: torch.matmul(a, b, out=c), 10)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(launches):
        torch.matmul(a, b, out=c)
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * n ** 3 * launches / (e0.elapsed_time(e1) * 1e-3) / 1e12


def measure_targets(A, W, dev, stream_gbs, seed):
    """spec_verify_attn alone (10 launches) on the two other workloads the bandwidth target names."""
    import torch
    out = {}
    gemm_tflops = library_gemm_rate(dev)
    for i in (3, 4):
        cfg = W.baseline_config(i)
        if seed is not None:
            cfg = W.scaled(cfg, seed=seed + i)
        inp = AttnInputs(A, W, cfg, dev, 0)
        t = inp.time_attn(10)
        out[cfg.name] = attention_roofline(cfg, inp.lay, t, stream_gbs)
        out[cfg.name]["library_gemm_bf16_TFLOPs"] = gemm_tflops
        out[cfg.name]["mfma_frac_of_library_gemm"] = out[cfg.name]["mfma_TFLOPs"] / gemm_tflops
        del inp
        torch.cuda.empty_cache()
    return out


def measure_ksweep(A, W, cfg, dev, p_accept):
    """t_attn(k) for k = 0..16 on this workload's batch and context lengths, and what the controller makes of it."""
    import torch
    ks, ts = list(range(0, 17)), []
    for k in ks:
        c = W.scaled(cfg, k=k, name=f"{cfg.name}+k{k}")
        inp = AttnInputs(A, W, c, dev, 0)
        ts.append(inp.time_attn(8) * 1e-3)
        del inp
        torch.cuda.empty_cache()
    res = {"k": ks, "t_attn_ms": [t * 1e3 for t in ts], "accept_probability": p_accept}
    # the layers outside this path cost something per verified row: nothing (the attention layer alone), then 1 % and
    # 10 % of a plain decoding step of this layer per row
    for name, per_row in (("attention_only", 0.0), ("rows_cost_1pct_of_step_each", 0.01 * ts[0]),
                          ("rows_cost_10pct_of_step_each", 0.10 * ts[0])):
        kstar, gain = A.spec_choose_k(ks, ts, p_accept, per_row)
        res[name] = {"per_row_cost_ms": per_row * 1e3, "k_star": kstar, "tokens_per_time_vs_k0": gain}
    return res


def measure_maintenance(A, W, cfg, mems, recent_d, rlen_d, idx, steps, dev, rest=None):
    """Incremental maintenance of the device automaton: every round appends 2 tokens per session (about
    what a verified step commits) to the memories, exports the delta (only what is new since the last
    export), and one launch scatters it into the device copy and inserts its transitions into the device
    overlay table; the lookup then runs on the maintained copy.  Host times are wall clock, device times
    HIP events."""
    import dataclasses
    import torch
    rng = np.random.default_rng(cfg.seed)
    mems = [list(m) for m in mems]
    sams = [A.sam_build(np.asarray(m, np.int32), cfg.sep) for m in mems]
    per_mem = 2 * cfg.B // len(mems)
    t0 = time.perf_counter()
    flat = A.sam_flatten(sams, grow_tokens=per_mem * (4 * steps + 1))
    t_flatten = time.perf_counter() - t0
    fd = flat.to(dev)
    mem_len = [len(m) for m in mems]
    root_d = torch.as_tensor(flat.roots[idx], device=dev)
    rows_end_d = torch.as_tensor(flat.rows_end[idx], device=dev)
    # the overlay table lives on the device for the whole run: room for every transition the run can log
    cap = 1 << 12
    while cap < 2 * 8 * per_mem * len(mems) * (4 * steps + 1):
        cap *= 2
    keys_d, dsts_d = A.overlay_table(cap, device=dev)

    def up(a):                                                # pinned staging: the copy is a DMA on the current stream
        return torch.from_numpy(np.ascontiguousarray(a)).pin_memory().to(dev, non_blocking=True)

    def host_part():
        for i, T in enumerate(mems):
            p = int(rng.integers(0, max(1, len(T) - per_mem)))
            add = [x for x in T[p:p + per_mem] if x != cfg.sep] or [0]      # text seen before: matches, clones
            A.sam_append(sams[i], np.asarray(add, np.int32))
            T += add
        deltas = [A.sam_delta_export(s, int(flat.roots[i]), int(flat.corpus_begin[i])) for i, s in enumerate(sams)]
        assert 2 * sum(d.n_overlay for d in deltas) <= cap
        return deltas

    def device_part(deltas):
        for i, d in enumerate(deltas):
            dd = dataclasses.replace(d, rec_idx=up(d.rec_idx), rec_val=up(d.rec_val), lastpos_idx=up(d.lastpos_idx),
                                     lastpos_val=up(d.lastpos_val), ov_key=up(d.ov_key.view(np.int64)), ov_dst=up(d.ov_dst))
            A.sam_apply_delta(dd, fd.state_rec, fd.lastpos, keys_d, dsts_d)
            n = d.new_tokens.shape[0]
            at = int(flat.corpus_begin[i]) + mem_len[i]
            fd.corpus[at:at + n] = up(d.new_tokens)
            mem_len[i] += n
        return up((flat.corpus_begin + np.asarray(mem_len))[idx].astype(np.int32))

    t_host, t_dev, t_draft, n_ov, n_ov_round = [], [], [], 0, []
    for _ in range(steps):
        th = time.perf_counter()
        deltas = host_part()
        t_host.append(time.perf_counter() - th)
        n_ov = sum(d.n_overlay for d in deltas); n_ov_round.append(sum(d.ov_key.size for d in deltas))
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        e0.record()
        cend_d = device_part(deltas)
        e1.record()
        A.sam_draft_delta(fd, keys_d, dsts_d, rows_end_d, root_d, cend_d, recent_d, rlen_d, cfg.k, cfg.sep)
        e2.record()
        torch.cuda.synchronize()
        t_dev.append(e0.elapsed_time(e1)); t_draft.append(e1.elapsed_time(e2))
    res_rounds = {}
    if rest is not None:
        # Whole rounds, wall clock: (a) one thing after the other; (b) the step is launched first, the host
        # appends and exports while the GPU runs it, and the device copy is updated on a second stream as soon
        # as the step's lookup has finished, next to the attention (Sec. 5.4.2: maintenance off the decoding path).
        main, side = torch.cuda.current_stream(), torch.cuda.Stream()
        # third mode: as "overlapped", with the lookup carrying its matched state (three tokens consumed per call)
        new_tok_d = recent_d[:, -3:].contiguous()
        n_new_d = torch.full((recent_d.shape[0],), 3, dtype=torch.int32, device=dev)
        cur_state = torch.full((recent_d.shape[0],), -1, dtype=torch.int32, device=dev)
        cur_len = torch.zeros((recent_d.shape[0],), dtype=torch.int32, device=dev)
        # the bare step on the same maintained copy, nothing appended: what a round is compared with
        def bare_step():
            d, nd, _, _ = A.sam_draft_delta(fd, keys_d, dsts_d, rows_end_d, root_d, cend_d, recent_d, rlen_d, cfg.k, cfg.sep)
            rest(d, nd)
        warm_up(bare_step)
        tr0 = time.perf_counter()
        for _ in range(steps):
            d, nd, _, _ = A.sam_draft_delta(fd, keys_d, dsts_d, rows_end_d, root_d, cend_d, recent_d, rlen_d, cfg.k, cfg.sep)
            rest(d, nd)
        torch.cuda.synchronize()
        res_rounds["step_ms_without_maintenance"] = (time.perf_counter() - tr0) / steps * 1e3
        for mode in ("sequential", "overlapped", "overlapped_carried_state"):
            torch.cuda.synchronize()
            tr0 = time.perf_counter()
            for _ in range(steps):
                if mode == "sequential":
                    cend_d = device_part(host_part())
                    d, nd, _, _ = A.sam_draft_delta(fd, keys_d, dsts_d, rows_end_d, root_d, cend_d, recent_d, rlen_d,
                                                    cfg.k, cfg.sep)
                    rest(d, nd)
                    torch.cuda.synchronize()
                else:
                    if mode == "overlapped":
                        d, nd, _, _ = A.sam_draft_delta(fd, keys_d, dsts_d, rows_end_d, root_d, cend_d, recent_d,
                                                        rlen_d, cfg.k, cfg.sep)
                    else:
                        d, nd, _, _ = A.sam_draft_step(fd, root_d, cend_d, new_tok_d, n_new_d, cur_state, cur_len,
                                                       cfg.k, cfg.sep, overlay_key=keys_d, overlay_dst=dsts_d,
                                                       rows_end=rows_end_d)
                    looked_up = torch.cuda.Event()
                    looked_up.record(main)
                    rest(d, nd)                               # attention + accept, queued behind the lookup
                    hp = host_part()                          # the GPU is busy with the step meanwhile
                    with torch.cuda.stream(side):
                        side.wait_event(looked_up)            # the lookup must not see a half-updated copy
                        cend_d = device_part(hp)
                    main.wait_stream(side)                    # the next lookup sees the whole update
            torch.cuda.synchronize()
            res_rounds["round_ms_" + mode] = (time.perf_counter() - tr0) / steps * 1e3
    return {"rounds": steps, "tokens_appended_per_round": per_mem * len(mems), **res_rounds,
            "host_append_and_export_us": float(np.median(t_host)) * 1e6,
            "device_update_us_incl_uploads": float(np.median(t_dev)) * 1e3,
            "t_draft_delta_us": float(np.median(t_draft)) * 1e3,
            "overlay_transitions_per_round": float(np.median(n_ov_round)),
            "overlay_transitions_at_end": int(n_ov), "overlay_capacity": cap, "full_flatten_ms": t_flatten * 1e3}


def measure_periodic_append(A):
    """Maintenance on a continuously repetitive memory (the prompt of the paper's TTFT / TPOT table): 30k and 128k
    tokens of period 3, then 3 tokens appended and one delta exported per round, 300 rounds."""
    out = {}
    for name, n in (("30k", 30000), ("128k", 131072)):
        base = np.tile(np.array([5, 6, 7], np.int32), n // 3 + 1)[:n]
        s = A.sam_build(base, 9)
        A.sam_flatten([s])
        t0 = time.perf_counter()
        n_lp = 0
        for r in range(300):
            A.sam_append(s, np.array([5, 6, 7], np.int32) if n % 3 == 0 else np.roll(np.array([5, 6, 7], np.int32), -(n % 3)))
            n_lp += A.sam_delta_export(s).lastpos_idx.size
        dt = time.perf_counter() - t0
        out[name] = {"round_us_append3_and_export": dt / 300 * 1e6, "lastpos_updates_per_round": n_lp / 300}
    return out


def measure_build(A, cfg):
    """Host cost of making a prompt's automaton available (Sec. 5.4.2, asynchronous construction): building
    and flattening 30k- and 128k-token prompts on the calling thread, against what the calling thread pays
    when the child thread builds (the submit call)."""
    out = {}
    rng = np.random.default_rng(cfg.seed)
    for name, n in (("30k", 30000), ("128k", 131072)):
        # a repetitive prompt: spans of an 8k-token base text repeated with small edits
        base = rng.integers(0, cfg.vocab, 8192).astype(np.int32)
        toks = np.concatenate([base[int(rng.integers(0, 4096)):][:int(rng.integers(256, 2048))] for _ in range(n // 256)])[:n]
        toks = np.ascontiguousarray(np.where(rng.random(toks.shape[0]) < 0.02, rng.integers(0, cfg.vocab, toks.shape[0]), toks),
                                    dtype=np.int32)
        t0 = time.perf_counter(); sm = A.sam_build(toks, cfg.sep); t1 = time.perf_counter()
        A.sam_flatten([sm]); t2 = time.perf_counter()
        bld = A.SamBuilder()
        t3 = time.perf_counter(); bld.submit(1, toks, cfg.sep); t4 = time.perf_counter()
        bld.wait(1); t5 = time.perf_counter()
        bld.close()
        out[name] = {"tokens": int(toks.shape[0]), "build_ms": (t1 - t0) * 1e3, "flatten_ms": (t2 - t1) * 1e3,
                     "async_submit_ms": (t4 - t3) * 1e3, "async_ready_ms": (t5 - t3) * 1e3}
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); multi-GPU sharding is design-only.",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2512_18337_amd as A
    from paper_2512_18337_amd import workloads as W

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "bytes_read": src.numel() * 4, "bytes_written": dst.numel() * 4,
                          "launches": 5}))
        return
    cfg = W.baseline_config(args.config)
    if args.seed is not None:
        cfg = W.scaled(cfg, seed=args.seed)
    if args.set:
        import ast
        cfg = W.scaled(cfg, name=cfg.name + "+" + ",".join(args.set),
                       **{kv.split("=")[0]: ast.literal_eval(kv.split("=", 1)[1]) for kv in args.set})
    tuning = A.attn_tuning(schedule=args.schedule, cascade=args.cascade, kv_chunk=args.kv_chunk)

    # ---- inputs (all resident in HBM before timing)
    nmem = cfg.B if cfg.sam_mode == "per_session" else 1
    mems = [W.token_memory(cfg, i) for i in range(nmem)]
    t0 = time.perf_counter()
    sams = [A.sam_build(m, cfg.sep) for m in mems]
    t_build = time.perf_counter() - t0
    flat = A.sam_flatten(sams)
    fd = flat.to(dev)
    idx = np.arange(cfg.B) if nmem > 1 else np.zeros(cfg.B, dtype=np.int64)
    recent, rlen = W.recent_windows(cfg, mems)
    root_d = torch.as_tensor(flat.roots[idx], device=dev)
    cend_d = torch.as_tensor(flat.corpus_end[idx], device=dev)
    recent_d = torch.as_tensor(recent, device=dev)
    rlen_d = torch.as_tensor(rlen, device=dev)
    inp = AttnInputs(A, W, cfg, dev, tuning)
    lay, q, kc, vc = inp.lay, inp.q, inp.kc, inp.vc
    if args.zero_inputs:
        if not args.attn_only:
            sys.exit("--zero-inputs is an experiment on spec_verify_attn alone: add --attn-only")
        q.zero_(); kc.zero_(); vc.zero_()

    # the logits stand in for the LM head: built once from the library's own drafts
    draft, n_draft, _, _ = A.sam_draft(fd, root_d, cend_d, recent_d, rlen_d, cfg.k, cfg.sep)
    torch.cuda.synchronize()
    draft_h, nd_h = draft.cpu().numpy(), n_draft.cpu().numpy()
    logits = W.verify_logits(cfg, draft_h, nd_h, dev)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    flush = torch.zeros(128 << 20, dtype=torch.float32, device=dev) if args.cold else None

    def step(events=None):
        if flush is not None:
            flush.add_(1.0)
        if not args.attn_only:
            if events: events[0].record()
            d, nd, ml, me = A.sam_draft(fd, root_d, cend_d, recent_d, rlen_d, cfg.k, cfg.sep)
        if events: events[1].record()
        inp.attn()
        if events: events[2].record()
        if not args.attn_only:
            res = A.spec_accept(logits, d, nd)
            if events: events[3].record()
            return res
        return None

    n_warm = warm_up(step, args.warmup) if args.warmup > 0 else 0
    evs = [[ev() for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        res = step(evs[i])
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t0
    ms_step = t_total / args.steps * 1e3
    if args.cold:                                             # the flush kernel is not part of the step
        first, last = (1, 2) if args.attn_only else (0, 3)
        ms_step = float(np.mean([e[first].elapsed_time(e[last]) for e in evs]))

    t_attn = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))             # ms, whole call
    if args.attn_only:
        t_draft = t_accept = 0.0
        accept_len = np.zeros(cfg.B, dtype=np.int32)
    else:
        t_draft = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
        t_accept = float(np.mean([e[2].elapsed_time(e[3]) for e in evs]))
        accept_len = res[0].cpu().numpy()

    stream_gbs = stream_read_rate(dev)
    result = {
        "metric": "verified tokens/s/GPU (B=64, 32k ctx, k=8); verify-attn HBM GB/s % of peak",
        "value": cfg.B * cfg.k / (ms_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": n_warm, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "head_dim": cfg.D,
                   "kv_len": [int(lay.seq_lens.min()), int(lay.seq_lens.max())], "page": cfg.page, "k": cfg.k,
                   "sam_tokens": int(sum(len(m) for m in mems)), "vocab": cfg.vocab, "seed": cfg.seed,
                   "step": "sam_draft + spec_verify_attn + spec_accept", "attn_only": bool(args.attn_only), "zero_inputs": bool(args.zero_inputs),
                   "cold_caches": bool(args.cold)},
        "roofline": attention_roofline(cfg, lay, t_attn, stream_gbs, paged_read_rate(inp, dev)),
        "detail": {"t_draft_us": t_draft * 1e3, "t_attn_us": t_attn * 1e3, "t_accept_us": t_accept * 1e3,
                   "sessions_per_s_sam_draft": (cfg.B / (t_draft * 1e-3)) if t_draft else None,
                   # the walk makes at least one dependent 16-byte record load per window token
                   "sam_draft_dependent_loads_per_s": (float(np.asarray(rlen).sum()) / (t_draft * 1e-3)) if t_draft else None,
                   "accepted_tokens_per_s": float((accept_len + 1).sum()) / (ms_step * 1e-3),
                   "synthetic_OTE": float((accept_len + 1).mean()),
                   "synthetic_SHR": (float(accept_len[nd_h > 0].sum()) / float(max(1, cfg.k) * max(1, (nd_h > 0).sum()))),
                   "accept_hbm_GBs": (logits.numel() * logits.element_size() / (t_accept * 1e-3) / 1e9)
                   if t_accept else None,
                   "sam_build_tokens_per_s": sum(len(m) for m in mems) / t_build,
                   "attn_workspace_bytes": inp.ws_bytes},
    }
    if not args.attn_only:
        # the stateful lookup: the window once (the prompt), then calls that consume only what a step commits
        tok0 = np.zeros_like(recent)
        for b in range(cfg.B):
            tok0[b, :rlen[b]] = recent[b, cfg.m - rlen[b]:]
        cur_state = torch.full((cfg.B,), -1, dtype=torch.int32, device=dev)
        cur_len = torch.zeros((cfg.B,), dtype=torch.int32, device=dev)
        A.sam_draft_step(fd, root_d, cend_d, tok0, rlen, cur_state, cur_len, cfg.k, cfg.sep)
        n_commit = 3                                          # about the accepted drafts + the bonus token
        tok1 = np.where(draft_h[:, :n_commit] >= 0, draft_h[:, :n_commit], 1).astype(np.int32)
        tok1_d = torch.as_tensor(np.ascontiguousarray(tok1), device=dev)
        nn_d = torch.full((cfg.B,), n_commit, dtype=torch.int32, device=dev)
        for _ in range(3):
            A.sam_draft_step(fd, root_d, cend_d, tok1_d, nn_d, cur_state, cur_len, cfg.k, cfg.sep)
        se0, se1 = ev(), ev()
        inp.attn()                                            # the host queues the calls behind it
        se0.record()
        for _ in range(20):
            A.sam_draft_step(fd, root_d, cend_d, tok1_d, nn_d, cur_state, cur_len, cfg.k, cfg.sep)
        se1.record()
        torch.cuda.synchronize()
        result["detail"]["t_draft_step_us"] = se0.elapsed_time(se1) / 20 * 1e3
        result["detail"]["draft_step_tokens_per_call"] = n_commit
        # the whole step with the stateful lookup in place of the window lookup (not the headline: the hot
        # path is defined with the stateless one)
        def step_stateful():
            d, nd, _, _ = A.sam_draft_step(fd, root_d, cend_d, tok1_d, nn_d, cur_state, cur_len, cfg.k, cfg.sep)
            inp.attn()
            return A.spec_accept(logits, d, nd)
        warm_up(step_stateful)
        t0s = time.perf_counter()
        for _ in range(args.steps):
            step_stateful()
        torch.cuda.synchronize()
        result["detail"]["ms_per_step_with_draft_step"] = (time.perf_counter() - t0s) / args.steps * 1e3
    if not args.cold:
        # the same step recorded once into a HIP graph and replayed (no host work between its kernels)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        warm_up(graph.replay)
        tg0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        result["detail"]["ms_per_step_graph"] = (time.perf_counter() - tg0) / args.steps * 1e3
    if not args.attn_only:
        result["detail"]["sam_prompt_build"] = measure_build(A, cfg)
        result["detail"]["sam_periodic_memory_maintenance"] = measure_periodic_append(A)
    if args.maintain > 0:
        def rest(d, nd):
            inp.attn()
            A.spec_accept(logits, d, nd)
        result["detail"]["sam_maintenance"] = measure_maintenance(A, W, cfg, mems, recent_d, rlen_d, idx,
                                                                  args.maintain, dev, rest)
    if args.ksweep:
        p_acc = float(np.mean(cfg.match_prob))
        result["detail"]["ksweep"] = measure_ksweep(A, W, cfg, dev, p_acc)
    if not args.no_cpu_baseline and not args.attn_only:
        result["cpu_baseline"] = cpu_baseline(cfg, mems, recent, rlen, q, kc, vc, lay, logits, draft_h, nd_h)
    else:
        result["cpu_baseline"] = None
    if not args.no_targets and not args.attn_only and args.config == 2 and not args.set:
        result["detail"]["targets"] = measure_targets(A, W, dev, stream_gbs, args.seed)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
