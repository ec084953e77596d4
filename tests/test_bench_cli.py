"""Host-side checks of bench.py's command line (no GPU): more than one GPU is refused with a message."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_bench_helper_library_exports_its_probes_and_checks_arguments():
    """libagentsam_bench.so (measurement aids, not the product ABI): both probes are there, and bad arguments are
    turned down before anything is launched."""
    import ctypes
    from paper_2512_18337_amd.build import BENCH_LIB
    lib = ctypes.CDLL(BENCH_LIB)
    assert hasattr(lib, "bench_stream_read_probe") and hasattr(lib, "bench_paged_read_probe")
    lib.bench_stream_read_probe.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    lib.bench_paged_read_probe.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong,
                                           ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_void_p, ctypes.c_void_p]
    assert lib.bench_stream_read_probe(None, 1 << 30, None, None) == -1
    assert lib.bench_paged_read_probe(None, None, None, 8, 8, 1, 1, 64, 128, 4, None, None) == -1
    fake = ctypes.c_void_p(256)                              # never dereferenced: the shape is refused first
    assert lib.bench_stream_read_probe(fake, 1024, fake, None) == -2            # fewer than 16 MiB
    for P, D, tiles, max_pages in ((48, 128, 4, 8), (64, 96, 4, 8), (64, 128, 0, 8), (64, 128, 100, 8)):
        assert lib.bench_paged_read_probe(fake, fake, fake, max_pages, 8, 1, 1, P, D, tiles, fake, None) == -2
