"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host-side code, run on the CPU:
the float64 oracle (all entry points, ragged shapes, masks) and the library's argument validation
(the host pass of csrc/attn_api.hip; device code is not instrumented)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]


def _run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, **kw)


def _clean(stderr):
    bad = ("AddressSanitizer", "runtime error", "LeakSanitizer")
    return not any(b in stderr for b in bad)


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    r = _run(["gcc", "-O1", "-g", "-std=c99", "-fopenmp", *SAN, "-o", exe,
              os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
              os.path.join(ROOT, "oracle", "attn_oracle.c"), "-lm"])
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0")
    env.pop("LD_PRELOAD", None)
    r = _run([exe], env=env)
    assert r.returncode == 0 and _clean(r.stderr), r.stderr[-2000:]
    assert r.stdout.startswith("checksum")


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_host_validation_under_asan_ubsan(tmp_path):
    from paper_2410_09397_amd import build as hip_build
    hip_build.build()  # the other translation units, uninstrumented
    csrc = os.path.join(ROOT, "paper_2410_09397_amd", "csrc")
    obj = str(tmp_path / "attn_api_san.o")
    host_san = [a for f in SAN for a in ("-Xarch_host", f)]
    r = _run(["hipcc", *[f for f in hip_build.FLAGS if f != "-fvisibility=hidden"], *host_san, "-g", "-c",
              os.path.join(csrc, "attn_api.hip"), "-o", obj])
    assert r.returncode == 0, r.stderr[-2000:]
    others = [os.path.join(hip_build.OBJ, s.replace(".hip", ".o")) for s in hip_build.SOURCES if s != "attn_api.hip"]
    drv = str(tmp_path / "host_api_driver.o")
    r = _run(["g++", "-O1", "-g", "-std=c++17", *SAN, "-c", os.path.join(ROOT, "tests", "sanitize", "host_api_driver.cpp"),
              "-o", drv])
    assert r.returncode == 0, r.stderr[-2000:]
    exe = str(tmp_path / "host_api_san")
    r = _run(["hipcc", "--offload-arch=gfx950", "--hip-link", "-fsanitize=address", "-fsanitize=undefined",
              "-fno-gpu-sanitize", "-g", "-o", exe, drv, obj, *others])
    assert r.returncode == 0, r.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:protect_shadow_gap=0")
    env.pop("LD_PRELOAD", None)
    r = _run([exe], env=env)
    assert r.returncode == 0 and _clean(r.stderr), (r.stdout[-2000:], r.stderr[-2000:])
    assert "0 failed" in r.stdout
