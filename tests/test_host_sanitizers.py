"""The library's host side under AddressSanitizer and UndefinedBehaviorSanitizer: every source is
compiled with the sanitizers on the host pass only (device code as in the product build), linked
with a plain-C program that drives every entry point down its argument checks, and run.  No GPU
is touched; the GPU side cannot be run under a sanitizer here."""
import os
import shutil
import subprocess

import pytest

from paper_2410_00161_amd import build as KB

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OUT = os.path.join(ROOT, "_build", "san")


def test_host_code_is_clean_under_asan_and_ubsan():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    os.makedirs(OUT, exist_ok=True)
    # host pass only: every sanitizer flag rides behind its own -Xarch_host (the GPU side cannot run sanitized here)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    flags = [f for f in KB.HIPCC_FLAGS if f != "-O3"] + ["-O1"]
    procs, objs = [], []
    for src in KB.SOURCES:
        obj = os.path.join(OUT, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *flags, *KB.EXTRA_FLAGS.get(src, []), *san, "-c", os.path.join(KB.CSRC, src), "-o", obj]
        procs.append(subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True))
    for p in procs:
        out, _ = p.communicate()
        assert p.returncode == 0, out[-3000:]
    cobj = os.path.join(OUT, "host_check.o")
    ccmd = [hipcc, "-x", "c", "-std=c11", "-O1", *san, "-I", os.path.join(ROOT, "include"), "-c", os.path.join(ROOT, "tests", "host", "host_check.c"), "-o", cobj]
    r = subprocess.run(ccmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    exe = os.path.join(OUT, "host_check")
    lcmd = [hipcc, "--offload-arch=gfx950", *san, "-o", exe, cobj, *objs]
    r = subprocess.run(lcmd, capture_output=True, text=True)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"   # the HIP runtime keeps its own allocations
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "host checks passed" in r.stdout, (r.stdout + r.stderr)[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
