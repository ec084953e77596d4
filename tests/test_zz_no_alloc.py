"""spec_verify_attn_static (the entry point that allocates nothing: its workspace is a static device array
inside the library) against spec_verify_attn on the same inputs, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2512_18337_amd as A
from paper_2512_18337_amd import binding, workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(cfg):
    lay = W.kv_layout(cfg)
    q, kc, vc = W.kv_and_queries(cfg, lay, DEV)
    return lay, q, kc, vc, torch.as_tensor(lay.block_table, device=DEV), torch.as_tensor(lay.seq_lens, device=DEV)


# (first call, second call with a smaller input): the second runs on whatever the first left in the array
PAIRS = [
    # balanced schedule (512 streams), then fewer and shorter sessions through the chunk grid + merge kernel
    (dict(B=70, Hq=32, Hkv=8, D=128, k=8, kv_mode="ragged", kv_len=(9, 1500)), dict(schedule=2),
     dict(B=5, Hq=8, Hkv=2, D=128, k=8, kv_mode="ragged", kv_len=(9, 1200)), dict(kv_chunk=256)),
    # wide kernel, balanced; then a shared-prefix run that keeps page counts, prefix sums and records there
    (dict(B=40, Hq=8, Hkv=2, D=128, k=12, kv_mode="ragged", kv_len=(40, 3000)), dict(schedule=2),
     dict(B=6, Hq=10, Hkv=2, D=128, k=8, kv_mode="shared_prefix", kv_len=(40, 700), prefix_len=2048), dict(cascade=2)),
    # fp32 storage, several chunks per session; then a smaller fp32 batch
    (dict(base=0, B=3, Hq=4, Hkv=2, D=128, page=16, k=6, kv_mode="ragged", kv_len=(300, 900)), {},
     dict(base=0, B=2, Hq=2, Hkv=1, D=64, page=16, k=4, kv_mode="ragged", kv_len=(5, 600)), {}),
]


@pytest.mark.parametrize("case", range(len(PAIRS)))
def test_static_workspace_entry_point_matches_the_workspace_one(case):
    kw1, tun1, kw2, tun2 = PAIRS[case]
    results = []
    for kw, tun in ((kw1, tun1), (kw2, tun2)):                # two calls in a row, the second one smaller
        kw = dict(kw)
        cfg = W.scaled(W.baseline_config(kw.pop("base", 1)), permute_pages=True, **kw)
        lay, q, kc, vc, bt, seq = _inputs(cfg)
        scale = 1.0 / float(np.sqrt(cfg.D))
        tuning = A.attn_tuning(**tun)
        need = A.spec_verify_attn_workspace(cfg.B, cfg.R, cfg.Hq, cfg.Hkv, cfg.D, cfg.page, bt.shape[1],
                                            binding._dtype_code(q), tuning)
        assert 0 < need <= binding.STATIC_WORKSPACE_BYTES
        out = torch.full((cfg.B, cfg.R, cfg.Hq, cfg.D), float("nan"), dtype=torch.float32, device=DEV)
        print(f"static workspace case {case}: {kw} tuning {tun} needs {need} bytes", flush=True)
        A.spec_verify_attn_static(q, kc, vc, bt, seq, scale, out, tuning=tuning)
        results.append((out, (q, kc, vc, bt, seq, scale, tuning)))
    torch.cuda.synchronize()
    for out, (q, kc, vc, bt, seq, scale, tuning) in results:
        ref = A.spec_verify_attn(q, kc, vc, bt, seq, scale, tuning=tuning)     # workspace from torch
        torch.cuda.synchronize()
        # same kernels, same schedule, same arithmetic: the same bits (inside the 1e-5 / 2e-2 bars by a wide margin)
        assert torch.equal(out, ref)


def test_static_workspace_rejects_what_does_not_fit():
    """The ragged 128-session batch of 136 packed rows needs 72 MB of records: refused with the workspace
    error before anything is launched, and the array is untouched."""
    L = binding.lib()
    tiny = torch.zeros(64, dtype=torch.int32, device=DEV)
    need = A.spec_verify_attn_workspace(128, 17, 64, 8, 128, 64, 1024, A.BF16)
    assert need > binding.STATIC_WORKSPACE_BYTES
    p = tiny.data_ptr()
    rc = L.spec_verify_attn_static(p, p, p, p, 1024, p, 128, 17, 64, 8, 128, 64, 100000, 0.1, A.BF16, A.F32, p, 0, None)
    assert rc == -4
