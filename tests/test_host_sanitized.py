"""libsig's host logic under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, nothing is launched).

The planner, the plan checks, the footprint query and the gradient's segment rule are index and size arithmetic that
decides LDS sizes and grid shapes.  Every translation unit of the library is compiled for the host only (hipcc
--cuda-host-only, a few seconds) with both sanitizers, the device code objects they would embed are replaced by empty
bundles, and tests/host_sweep.cpp drives the host-only entry points over some ten thousand seeded shapes and
twenty thousand arbitrary plans.  The run fails on any sanitizer report and on any broken invariant (the planner's own
plan refused by the plan check, LDS above the library's limit, a grid beyond 2^31 - 1, ...).
"""
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2501_08455_amd import build as lib_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLANGXX = "/opt/rocm/lib/llvm/bin/clang++"


def test_host_logic_runs_clean_under_sanitizers(tmp_path):
    if not os.path.exists(CLANGXX):
        pytest.skip("no ROCm clang++ here")
    flags = ["--cuda-host-only", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-omit-frame-pointer",
             "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-Wno-unused-command-line-argument",
             "-I" + os.path.join(ROOT, "include"), "-I" + lib_build.CSRC]

    def compile_one(src):
        obj = str(tmp_path / (os.path.splitext(src)[0] + ".o"))
        res = subprocess.run([lib_build._hipcc()] + flags + ["-c", os.path.join(lib_build.CSRC, src), "-o", obj],
                             capture_output=True, text=True)
        return obj, res

    with ThreadPoolExecutor(max_workers=8) as pool:
        results = list(pool.map(compile_one, lib_build.SOURCES))
    for obj, res in results:
        if res.returncode != 0 and "sanitize" in res.stderr and "unsupported" in res.stderr:
            pytest.skip("this toolchain has no host sanitizer runtime")
        assert res.returncode == 0, res.stderr[-3000:]
    objs = [obj for obj, _ in results]
    # the host objects refer to the device code objects that a full build embeds: empty offload bundles stand in
    undefined = subprocess.run(["nm", "-u"] + objs, capture_output=True, text=True).stdout
    stubs = sorted(set(re.findall(r"__hip_fatbin_[0-9a-f]+", undefined)))
    stub_c = tmp_path / "fatbin_stubs.c"
    stub_c.write_text("".join('__attribute__((aligned(4096))) const char %s[32] = "__CLANG_OFFLOAD_BUNDLE__";\n' % s
                              for s in stubs))
    exe = str(tmp_path / "host_sweep")
    link = subprocess.run([CLANGXX, "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-g",
                           "-I" + os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "host_sweep.cpp"),
                           "-x", "c", str(stub_c), "-x", "none"] + objs +
                          ["-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe],
                          capture_output=True, text=True)
    assert link.returncode == 0, link.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    ran = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert ran.returncode == 0, (ran.stdout[-4000:] + ran.stderr[-4000:])
    assert "host sweep ok" in ran.stdout
