"""The library's host layer (argument validation, workspace plans, the parameter blob) built for the CPU with
AddressSanitizer and UndefinedBehaviorSanitizer and driven by tests/sanitizer/abi_check.cpp: no sanitizer report, every
status as documented, and no call reaches a kernel launcher under a host-only context."""
import concurrent.futures
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2402_05628_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "sanitizer")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# host passes only are instrumented: each -fsanitize= option directly follows an -Xarch_host
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
       "-Xarch_host", "-fno-omit-frame-pointer"]
FLAGS = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes", "-Wno-unused-value", "-ffp-contract=off",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]
HOST_LAYER = ["rq_api.hip", "block.hip", "params_blob.hip"]


def _compile(src, obj, hip):
    cmd = [HIPCC, *FLAGS, *SAN, "-c", src, "-o", obj] if hip else \
          [HIPCC, "-x", "hip", *FLAGS, *SAN, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    return obj


@pytest.fixture(scope="module")
def checker(tmp_path_factory):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not found")
    out = tmp_path_factory.mktemp("abi_sanitizer")
    jobs = [(os.path.join(CSRC, f), str(out / (f + ".o")), True) for f in HOST_LAYER]
    jobs += [(os.path.join(HERE, f), str(out / (f + ".o")), False) for f in ("launch_stubs.cpp", "abi_check.cpp")]
    with concurrent.futures.ThreadPoolExecutor(max_workers=5) as ex:
        objs = list(ex.map(lambda j: _compile(*j), jobs))
    exe = str(out / "abi_check")
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-o", exe, *objs],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    return exe


def test_host_layer_is_clean_under_asan_and_ubsan(checker):
    env = dict(os.environ)
    # the sanitizer runtime is linked into the program; whatever else the loader brings in first is none of its business.
    # Leak checking is off: the HIP runtime the program links against keeps its own process-lifetime allocations.
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    r = subprocess.run([checker], capture_output=True, text=True, env=env, timeout=600)
    tail = (r.stdout + r.stderr)[-4000:]
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    assert r.returncode == 0, tail
    assert "OK: 0 failed expectations, 0 launches" in r.stdout, tail
