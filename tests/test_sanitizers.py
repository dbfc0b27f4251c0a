"""CPU builds under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU needed): the oracle's C loops on small ragged
shapes with exact-size heap buffers, and the host-only logic of libpbkd's runtime (descriptor validation, workspace
layout, FLOP counts, scheduler, early argument checks) linked against the already built kernel objects."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)


def _clean(out):
    bad = [l for l in out.splitlines() if "AddressSanitizer" in l or "runtime error" in l or "LeakSanitizer" in l]
    return not bad, bad


def test_oracle_c_loops_under_asan_ubsan(tmp_path):
    if not shutil.which("gcc"):
        pytest.skip("no gcc")
    exe = str(tmp_path / "ref_driver")
    build = _run(["gcc", "-O1", "-g", "-fopenmp", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                  "-fno-omit-frame-pointer", "-o", exe, os.path.join(SAN, "ref_driver.c"), os.path.join(ROOT, "oracle", "pbkd_ref.c"), "-lm"])
    assert build.returncode == 0, build.stdout
    run = _run([exe], env=dict(ENV, OMP_NUM_THREADS="3"), timeout=120)
    ok, bad = _clean(run.stdout)
    assert run.returncode == 0 and ok and run.stdout.strip().endswith("ok"), run.stdout[-3000:]


def test_runtime_host_logic_under_asan_ubsan(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    from paper_2012_03096_amd import build as pbuild
    csrc = pbuild.CSRC
    objs = [os.path.join(csrc, s.replace(".hip", ".o")) for s in pbuild.SOURCES if s != "pbkd_runtime.hip"]
    if not all(os.path.exists(o) for o in objs):
        pbuild.build()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
    rt = str(tmp_path / "pbkd_runtime_san.o")
    build = _run([hipcc, *pbuild.FLAGS, "-g", *san, "-c", os.path.join(csrc, "pbkd_runtime.hip"), "-o", rt])
    assert build.returncode == 0, build.stdout[-3000:]
    drv = str(tmp_path / "host_driver.o")
    build = _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", *san, "-x", "hip", "-c", os.path.join(SAN, "host_driver.cpp"), "-o", drv])
    assert build.returncode == 0, build.stdout[-3000:]
    exe = str(tmp_path / "host_driver")
    link = _run([hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-o", exe, drv, rt, *objs])
    assert link.returncode == 0, link.stdout[-3000:]
    run = _run([exe], env=ENV, timeout=120)
    ok, bad = _clean(run.stdout)
    assert run.returncode == 0 and ok and run.stdout.strip().endswith("ok"), run.stdout[-3000:]
