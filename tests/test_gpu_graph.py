"""The whole step recorded once into a HIP graph and replayed: the library only launches kernels on the
caller's stream (no allocation, no memset, no synchronisation), so a captured step must reproduce the eager
results on every replay, also with other work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import paper_2512_18337_amd as A
from paper_2512_18337_amd import workloads as W
from _util import draft_inputs, make_memories

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("shape", [
    dict(B=8, Hq=8, Hkv=2, k=8, kv_len=(64, 5000), kv_mode="ragged", permute_pages=True),       # narrow kernel, chunk grid + merge
    dict(B=40, Hq=16, Hkv=2, k=16, kv_len=(40, 3000), kv_mode="ragged", permute_pages=True),    # wide kernel, balanced
    dict(B=6, Hq=10, Hkv=2, k=8, kv_len=(40, 700), kv_mode="shared_prefix", prefix_len=2048, cascade=2),   # shared-prefix run
])
def test_captured_step_replays_like_the_eager_step(shape):
    shape = dict(shape)
    cascade = shape.pop("cascade", 0)
    cfg = W.scaled(W.baseline_config(1), D=128, sam_session_len=4096, vocab=4000, **shape)
    _captured_step_case(cfg, A.attn_tuning(cascade=cascade))


def _captured_step_case(cfg, tuning=0):
    mems = make_memories(cfg)
    flat, root, cbeg, cend, recent, rlen = draft_inputs(cfg, mems)
    fd = flat.to(DEV)
    dev_i32 = lambda a: torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32), device=DEV)
    root_d, cend_d, recent_d, rlen_d = dev_i32(root), dev_i32(cend), dev_i32(recent), dev_i32(rlen)
    lay = W.kv_layout(cfg)
    q, kc, vc = W.kv_and_queries(cfg, lay, DEV)
    bt, seq = dev_i32(lay.block_table), dev_i32(lay.seq_lens)
    scale = 1.0 / float(np.sqrt(cfg.D))
    need = A.spec_verify_attn_workspace(cfg.B, cfg.R, cfg.Hq, cfg.Hkv, cfg.D, cfg.page, bt.shape[1], A.BF16, tuning)
    ws = torch.empty(max(need, 16) // 4 + 1, dtype=torch.float32, device=DEV)
    out = torch.empty((cfg.B, cfg.R, cfg.Hq, cfg.D), dtype=torch.float32, device=DEV)
    d0, nd0, _, _ = A.sam_draft(fd, root_d, cend_d, recent_d, rlen_d, cfg.k, cfg.sep)
    torch.cuda.synchronize()
    logits = W.verify_logits(cfg, d0.cpu().numpy(), nd0.cpu().numpy(), DEV)

    def step():
        d, nd, ml, me = A.sam_draft(fd, root_d, cend_d, recent_d, rlen_d, cfg.k, cfg.sep)
        A.spec_verify_attn(q, kc, vc, bt, seq, scale, out=out, workspace=ws, tuning=tuning)
        a, toks, tgt = A.spec_accept(logits, d, nd)
        return d, nd, ml, me, a, toks, tgt

    eager = [t.clone() for t in step()] + [out.clone()]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                             # warm-up on the capture stream, as torch asks
        step()
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        captured = step()
    for rep in range(4):
        out.fill_(float("nan"))                               # eager work between the replays
        for t in captured:
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip(list(captured) + [out], eager):
            assert torch.equal(got, want), rep
