"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer, without
a GPU: every source is compiled for the host only and linked with a stand-in for the HIP
runtime (tests/host_sanitizer/host_harness.cpp), which records kernel launches instead of
performing them.  The harness drives every entry point over the benchmark's shapes, ragged
and extreme shapes and the documented refusals, and checks status codes, workspace layout
and launch geometry; the sanitizers watch the host logic meanwhile (device pointers are
addresses in a PROT_NONE mapping)."""
import os
import shutil
import subprocess

import pytest

from paper_2604_16855_amd import build as B

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"),
                    reason="hipcc not found")
def test_host_code_under_sanitizers(tmp_path):
    hipcc = B.hipcc()
    flags = ["--offload-arch=gfx950", "--cuda-host-only", "-O1", "-g", "-std=c++17", "-fno-omit-frame-pointer",
             "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unknown-warning-option",
             "-I", os.path.join(B.ROOT, "include"), "-I", B.CSRC]
    objs = []
    jobs = []
    for src in B.SOURCES:
        obj = str(tmp_path / src.replace(".hip", ".o"))
        jobs.append(subprocess.Popen([hipcc, *flags, "-c", os.path.join(B.CSRC, src), "-o", obj],
                                     stderr=subprocess.PIPE, text=True))
        objs.append(obj)
    hobj = str(tmp_path / "host_harness.o")
    jobs.append(subprocess.Popen([hipcc, *flags, "-x", "hip", "-c",
                                  os.path.join(HERE, "host_sanitizer", "host_harness.cpp"), "-o", hobj],
                                 stderr=subprocess.PIPE, text=True))
    for j in jobs:
        err = j.communicate()[1]
        assert j.returncode == 0, err
    exe = str(tmp_path / "host_harness")
    # the device images the host objects refer to do not exist in a host-only build; the
    # stand-in runtime never looks at them
    linker = next((c for c in (os.path.join(os.path.dirname(hipcc), "amdclang++"),
                               "/opt/rocm/lib/llvm/bin/clang++", "/opt/rocm/llvm/bin/clang++",
                               shutil.which("clang++")) if c and os.path.exists(c)), None)
    if linker is None:
        pytest.skip("no clang++ of the ROCm toolchain to link the host-only objects with")
    r = subprocess.run([linker, "-fsanitize=address,undefined", *objs, hobj, "-o", exe,
                        "-Wl,--unresolved-symbols=ignore-all"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-6000:]
    assert "0 failures" in r.stdout
