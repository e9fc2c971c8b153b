"""Host layer of the library under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU.

Every source file is compiled for the host only (no device code, a few seconds), linked with stand-ins for
the HIP runtime (tests/host_sanitize/hip_stubs.cpp) and with a checker (tests/host_sanitize/driver.cpp) that
walks the size queries, the exact-integer bucket tables, the kernel-path query and every error path that the
entry points take before any device work.  Passes when the checker's own expectations hold and neither
sanitizer reports anything."""
import glob
import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2203_17189_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "host_sanitize")
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
       "-Xarch_host", "-fno-sanitize-recover=undefined"]
COMMON = ["--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17", "-Wno-unused-command-line-argument"]


def _run(cmd, **kw):
    r = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert r.returncode == 0, (" ".join(cmd), r.stdout[-2000:], r.stderr[-4000:])
    return r


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_host_layer_under_asan_and_ubsan(tmp_path):
    sources = sorted(glob.glob(os.path.join(CSRC, "*.hip"))) + [os.path.join(HERE, "driver.cpp"),
                                                                 os.path.join(HERE, "hip_stubs.cpp")]

    def compile_one(src):
        obj = str(tmp_path / (os.path.basename(src).rsplit(".", 1)[0] + ".o"))
        lang = ["-x", "hip"] if src.endswith(".cpp") and "driver" in src else []
        _run(["hipcc", *COMMON, *SAN, *lang, "-c", src, "-o", obj])
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, sources))
    # host-only objects still name their (absent) device code objects: give those names something to point at
    undefined = _run(["nm", "-u", *objs]).stdout
    fat = sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", undefined)))
    stub = tmp_path / "fatbin_names.c"
    stub.write_text("".join(f"const char {name}[16] = {{0}};\n" for name in fat))
    stub_o = str(tmp_path / "fatbin_names.o")
    _run(["gcc", "-c", str(stub), "-o", stub_o])
    clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    exe = str(tmp_path / "host_check")
    _run([clangxx if os.path.exists(clangxx) else "clang++", "-fsanitize=address", "-fsanitize=undefined", *objs, stub_o,
          "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-6000:])
    assert "OK: 0 failure(s)" in r.stdout, r.stdout[-3000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-6000:]
