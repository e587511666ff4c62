"""Sanitizer leg (CPU only): the oracle's pins and the host-side argument validation of the C-ABI
library are run once more against builds with AddressSanitizer and UndefinedBehaviorSanitizer
(host code only; nothing here touches a GPU).  Each build is loaded by a child interpreter that
has the matching sanitizer runtime preloaded, and the child runs the ordinary test files."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def _child_env(runtime, extra):
    env = dict(os.environ)
    env.update(extra)
    env["LD_PRELOAD"] = " ".join(x for x in (runtime, os.environ.get("LD_PRELOAD", "")) if x)
    # Python itself is not instrumented: its arenas would all be reported as leaks
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    return env


def _run_pytest(files, env):
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu", *files]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    assert " passed" in r.stdout, tail


def test_oracle_pins_under_sanitizers(tmp_path):
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc has no AddressSanitizer runtime here")
    lib = str(tmp_path / "libvq_oracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                           "-fno-fast-math", "-fno-omit-frame-pointer", *SAN, "-o", lib,
                           os.path.join(ROOT, "oracle", "vq_oracle.c"), "-lm"])
    _run_pytest(["tests/test_oracle_pins.py", "tests/test_oracle_producer_pins.py"],
                _child_env(runtime, {"VQ_ORACLE_LIB": lib}))


def test_host_validation_under_sanitizers(tmp_path):
    from paper_2406_02540_amd import build as hb
    hipcc = hb.hipcc()
    probe = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    runtime = os.path.realpath(probe.stdout.strip()) if probe.returncode == 0 else ""
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("hipcc's clang has no AddressSanitizer runtime here")
    # the front end (validation, workspace arithmetic, status strings) with host sanitizers; the kernels' objects
    # as the ordinary build leaves them
    others = [os.path.join(hb.CSRC, s.replace(".hip", ".o")) for s in hb.SOURCES if s != "vq_api.hip"]
    if not all(os.path.exists(o) for o in others):
        hb.build(verbose=False)
    host_san = [f for flag in SAN + ["-fno-omit-frame-pointer"] for f in ("-Xarch_host", flag)]
    flags = [f for f in hb.HIPCC_FLAGS if f != "-O3"]
    obj = str(tmp_path / "vq_api_san.o")
    subprocess.check_call([hipcc, *flags, "-O1", "-g", *host_san, "-I", os.path.join(ROOT, "include"), "-I", hb.CSRC,
                           "-c", os.path.join(hb.CSRC, "vq_api.hip"), "-o", obj], stderr=subprocess.DEVNULL)
    lib = str(tmp_path / "libvidiq_san.so")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *host_san, "-shared-libsan", obj, *others,
                           "-o", lib], stderr=subprocess.DEVNULL)
    _run_pytest(["tests/test_host_api.py"], _child_env(runtime, {"VQ_LIBVIDIQ_PATH": lib}))
