"""The host side of the C ABI under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Every source of the library is compiled once more with the host pass instrumented (the device pass is
not: `-Xarch_host`), linked with tests/host_abi_sanitized.cpp and run here.  The driver walks through
what happens before any GPU call: descriptor checks, the argument validation of every entry point, the
launch plan of stage 4 over sweeps of shapes and knobs, the chunk reordering on random inputs.  Any
finding of a sanitizer aborts the driver; any unexpected status makes it return 1.
"""
import glob
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
HOST_SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined"]
COMMON = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Wno-unused-command-line-argument",
          "-Wno-option-ignored", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2603_05353_amd", "csrc")]


def _run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, **kw)


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc in this environment")
def test_host_abi_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    sources = sorted(glob.glob(os.path.join(ROOT, "paper_2603_05353_amd", "csrc", "*.hip")))
    sources.append(os.path.join(ROOT, "tests", "host_abi_sanitized.cpp"))
    objects = [str(tmp_path / (os.path.splitext(os.path.basename(s))[0] + ".o")) for s in sources]

    def compile_one(pair):
        src, obj = pair
        return src, _run([HIPCC] + COMMON + HOST_SAN + ["-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=8) as pool:
        for src, r in pool.map(compile_one, zip(sources, objects)):
            assert r.returncode == 0, f"{src}:\n{r.stderr[-3000:]}"
    exe = str(tmp_path / "host_abi_sanitized")
    r = _run([HIPCC, "-fsanitize=address", "-fsanitize=undefined"] + objects + ["-o", exe])
    assert r.returncode == 0, r.stderr[-3000:]
    # the runtime is really in there
    syms = _run(["nm", exe]).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:halt_on_error=1:abort_on_error=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = _run([exe], env=env, timeout=300)
    assert r.returncode == 0, f"stdout:\n{r.stdout[-3000:]}\nstderr:\n{r.stderr[-3000:]}"
    assert "host ABI under the sanitizers: ok" in r.stdout
    assert "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
