"""The C-ABI library loads and exports every symbol the header declares (no GPU compute here)."""
import ctypes
import os
import re

import paper_2512_18337_amd as A
from paper_2512_18337_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    txt = open(os.path.join(ROOT, "include", "agentsam.h")).read()
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*\s*|int\s+|void\s+)(\w+)\s*\(", txt, flags=re.M)
    return sorted(set(names))


def test_header_symbols_are_exported():
    names = _declared()
    assert set(names) == set(binding.EXPORTS), names
    L = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert getattr(L, n) is not None


def test_argument_errors_without_a_gpu():
    L = binding.lib()
    n = ctypes.c_size_t()
    # D unsupported, Hq % Hkv != 0, bf16 page size not a multiple of 32, too many packed rows
    assert L.spec_verify_attn_workspace(1, 5, 4, 1, 96, 64, 4, binding.F32, 0, ctypes.byref(n)) == -3
    assert L.spec_verify_attn_workspace(1, 5, 5, 2, 64, 64, 4, binding.F32, 0, ctypes.byref(n)) == -2
    assert L.spec_verify_attn_workspace(1, 5, 4, 1, 64, 16, 4, binding.BF16, 0, ctypes.byref(n)) == -3
    assert L.spec_verify_attn_workspace(1, 33, 8, 1, 128, 64, 4, binding.BF16, 0, ctypes.byref(n)) == -3
    assert L.spec_verify_attn_workspace(1, 5, 4, 1, 64, 64, 4, binding.F32, 0, None) == -1
    assert L.spec_verify_attn_workspace(64, 9, 32, 8, 128, 64, 512, binding.BF16, 0, ctypes.byref(n)) == 0
    # 512 streams on 256 resident workgroups: balanced schedule, prefix sums + two records per workgroup
    assert n.value == 512 + 2 * 256 * 36 * 130 * 4
    assert L.spec_verify_attn_workspace(64, 9, 32, 8, 128, 64, 512, binding.BF16, A.attn_tuning(schedule=1),
                                        ctypes.byref(n)) == 0
    assert n.value == 64 * 8 * 4 * 36 * 130 * 4          # chunk grid: 32768 / 8192 = 4 chunks of 36 packed rows
    # undefined field values of the tuning word
    assert L.spec_verify_attn_workspace(64, 9, 32, 8, 128, 64, 512, binding.BF16, 3, ctypes.byref(n)) == -2
    assert L.spec_verify_attn_workspace(64, 9, 32, 8, 128, 64, 512, binding.BF16, 3 << 2, ctypes.byref(n)) == -2
    assert L.spec_verify_attn_workspace(64, 9, 32, 8, 128, 64, 512, binding.BF16, 1 << 40, ctypes.byref(n)) == -2
    # entry points reject bad sizes before touching the device
    assert L.sam_draft(*([None] * 12), 4, 65, 4, 1, 0, *([None] * 5), 0, None) == -2
    assert L.sam_draft(*([None] * 12), 4, 16, 4, 1, 0, *([None] * 5), 0, None) == -1
    assert L.sam_draft(*([None] * 12), 0, 16, 4, 1, 0, *([None] * 5), 0, None) == 0
    assert L.spec_accept(None, 0, None, None, 4, 65, 100, None, None, None, None) == -2
    assert L.spec_accept(None, 7, None, None, 4, 4, 100, None, None, None, None) == -3
    assert L.spec_accept(None, 0, None, None, 4, 4, 100, None, None, None, None) == -1
    assert L.spec_verify_attn(None, None, None, None, 4, None, 2, 5, 4, 1, 64, 64, 8, 0.125, 0, 0,
                              None, None, 0, 0, None) == -1
    assert L.spec_verify_attn(None, None, None, None, 4, None, 2, 5, 4, 1, 64, 64, 8, -1.0, 0, 0,
                              None, None, 0, 0, None) == -2
