"""Host sanitizers (CPU only).

1. The C oracle is compiled with AddressSanitizer + UndefinedBehaviorSanitizer together with
   tests/sanitize_oracle_driver.c, which calls every oracle routine on small seeded inputs (ragged
   sizes, a zero row, the extreme fp16 magnitudes, an empty batch, a rejected +inf).  The run must end
   without a report, and its result hashes must equal those of the ordinary build of the oracle on the
   same inputs.
2. The host side of the C ABI (argument checks, the launch planner with its int64 -> int narrowing)
   is compiled with UndefinedBehaviorSanitizer in trap mode, linked with the already built kernels,
   and the host-only ABI tests run against that library in a child process: undefined behaviour on
   any path they reach kills the child.
"""
import os
import shutil
import subprocess
import sys

import numpy as np
import pytest

from oracle import fp6_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _fnv(a: np.ndarray) -> str:
    h = 1469598103934665603
    for byte in np.ascontiguousarray(a).view(np.uint8).ravel().tolist():
        h = ((h ^ byte) * 1099511628211) & 0xFFFFFFFFFFFFFFFF
    return "%016x" % h


class _Lcg:
    def __init__(self, seed):
        self.x = seed

    def finite16(self) -> int:
        self.x = (self.x * 6364136223846793005 + 1442695040888963407) & 0xFFFFFFFFFFFFFFFF
        p = self.x >> 48
        if (p >> 10) & 31 == 31:
            p &= ~0x4000 & 0xFFFF
        return p


def _expected_hashes():
    N, K, M, BLOCK = 7, 192, 3, 64
    g = _Lcg(231208583)
    W = np.array([g.finite16() for _ in range(N * K)], dtype=np.uint16).reshape(N, K)
    X = np.array([g.finite16() & 0xBFFF for _ in range(M * K)], dtype=np.uint16).reshape(M, K)
    W[2] = [0x8000 if k & 1 else 0 for k in range(K)]
    W[3, :4] = [0x7BFF, 0xFBFF, 0x0001, 0x8001]
    W[4] = [k % 3 for k in range(K)]
    out = {}
    codes, scales = O.quantize(W)
    out["q6.codes"], out["q6.scales"] = _fnv(codes), _fnv(scales)
    hi, lo = O.split42(codes)
    assert np.array_equal(O.join42(hi, lo), codes)
    out["q6.hi"] = _fnv(hi)
    out["q6.what"] = _fnv(O.dequantize(codes, scales))
    out["q6.y"] = _fnv(O.linear(X, codes, scales))
    out["q6.ybf16"] = _fnv(O.linear_bf16(X, codes, scales))
    codes, scales = O.quantize_fgq(W, BLOCK)
    out["fgq.codes"], out["fgq.scales"] = _fnv(codes), _fnv(scales)
    out["fgq.what"] = _fnv(O.dequantize_fgq(codes, scales, BLOCK))
    out["fgq.y"] = _fnv(O.linear_fgq(X, codes, scales, BLOCK))
    codes, scales = O.quantize5(W)
    out["q5.codes"], out["q5.scales"] = _fnv(codes), _fnv(scales)
    out["q5.lo"] = _fnv(O.split41(codes)[1])
    out["q5.what"] = _fnv(O.dequantize5(codes, scales))
    out["q5.y"] = _fnv(O.linear5(X, codes, scales))
    return out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-o", exe, os.path.join(ROOT, "tests", "sanitize_oracle_driver.c"),
           os.path.join(ROOT, "oracle", "fp6_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr
    got = dict(line.split() for line in r.stdout.splitlines() if " " in line)
    assert r.stdout.strip().endswith("done")
    for name, h in _expected_hashes().items():
        assert got[name] == h, name


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")
def test_host_abi_is_clean_under_ubsan(tmp_path):
    from paper_2312_08583_amd import build as hip_build
    objs = [os.path.join(hip_build.OBJ, os.path.splitext(s)[0] + ".o") for s in hip_build.SOURCES if s != "fp6_abi.hip"]
    if not all(os.path.exists(o) for o in objs):
        hip_build.build()
    abi_obj = str(tmp_path / "fp6_abi_ubsan.o")
    lib = str(tmp_path / "libfp6_linear_ubsan.so")
    host_san = ["-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined"]
    subprocess.run(["hipcc", *hip_build.FLAGS, *host_san, "-c", os.path.join(hip_build.CSRC, "fp6_abi.hip"), "-o", abi_obj],
                   check=True, capture_output=True)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, abi_obj, *objs], check=True,
                   capture_output=True)
    env = dict(os.environ, FP6_LINEAR_LIB=lib)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_abi_host.py")], env=env, cwd=ROOT, capture_output=True,
                       text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
