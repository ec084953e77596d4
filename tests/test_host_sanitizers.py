"""The host side of the library (automaton, delta export, asynchronous builder, controllers) compiled with
g++ under AddressSanitizer + UndefinedBehaviorSanitizer and under ThreadSanitizer and driven by
tests/host_sanitize.cpp on the CPU (no GPU code is involved; GPU sanitizers are not available)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_18337_amd", "csrc")
SOURCES = [os.path.join(ROOT, "tests", "host_sanitize.cpp")] + [os.path.join(CSRC, f) for f in
                                                               ("sam_host.cpp", "sam_builder.cpp", "controllers.cpp")]


@pytest.mark.parametrize("name,flags", [("asan_ubsan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]),
                                        ("tsan", ["-fsanitize=thread"])])
def test_host_code_is_clean_under_sanitizers(tmp_path, name, flags):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / name)
    cmd = [gxx, "-std=c++17", "-O1", "-g", *flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, *SOURCES, "-pthread",
           "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    if built.returncode != 0 and "sanitize" in built.stderr and "cannot find" in built.stderr:
        pytest.skip("sanitizer runtime not installed")
    assert built.returncode == 0, built.stderr[-2000:]
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=1", ASAN_OPTIONS="detect_leaks=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok"), (run.stdout[-1000:], run.stderr[-3000:])
