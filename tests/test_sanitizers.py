"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the oracle, and the
host side of the library (host-only entry points, argument validation, schedule arithmetic). Each
is built with -fsanitize=address,undefined together with a small C driver (tests/c/) and run; a
report from either sanitizer makes the run fail, and the values the drivers print are compared
with what the ordinary builds return."""
import shutil
import subprocess
from pathlib import Path

import numpy as np
import pytest

import oracle
from paper_2512_23966_amd import _build
from paper_2512_23966_amd import binding as B

ROOT = Path(__file__).resolve().parents[1]
SAN_ENV = {"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0:exitcode=23", "UBSAN_OPTIONS": "halt_on_error=1:exitcode=24",
           "PATH": "/usr/bin:/bin"}
INT64_MAX = (1 << 63) - 1


def _run(exe):
    res = subprocess.run([str(exe)], capture_output=True, text=True, env=SAN_ENV)
    assert res.returncode == 0, f"sanitizer run failed ({res.returncode}):\n{res.stderr[-3000:]}"
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-3000:]
    return {line.split()[0]: line.split()[1:] for line in res.stdout.splitlines()}


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = tmp_path / "sanitize_oracle"
    subprocess.run([gcc, "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    str(ROOT / "oracle" / "ssa_oracle.c"), str(ROOT / "tests" / "c" / "sanitize_oracle.c"),
                    "-o", str(exe), "-lm", "-lpthread"], check=True)
    got = _run(exe)
    # the same inputs through the ordinary build: the driver's generator, re-run here
    state = [12345]

    def rnd():
        x = state[0]
        x ^= (x << 13) & 0xFFFFFFFF; x ^= x >> 17; x ^= (x << 5) & 0xFFFFFFFF
        state[0] = x
        return np.float32((x % 65 - 32) / 16.0)
    Bn, Hq, Hkv, S, DQK, DV = 2, 4, 2, 37, 12, 8
    import torch
    q = torch.tensor([rnd() for _ in range(Bn * S * Hq * DQK)], dtype=torch.float32).view(Bn, S, Hq, DQK)
    k = torch.tensor([rnd() for _ in range(Bn * S * Hkv * DQK)], dtype=torch.float32).view(Bn, S, Hkv, DQK)
    dout = torch.tensor([rnd() for _ in range(Bn * S * Hq * DV)], dtype=torch.float32).view(Bn, S, Hq, DV)
    rb, rh, ri = (x.ravel().astype(np.int64) for x in np.meshgrid(np.arange(Bn), np.arange(Hq), np.arange(S), indexing="ij"))
    q_rows = q[rb, ri, rh].contiguous()
    out, lse, w = oracle.ssa_rows(q_rows, k, ("alias", DV), rb, rh, ri, Hq=Hq, n_sink=3, window=5, scale=0.25, want_weights=True)
    assert got["rows"][0] == "0"
    np.testing.assert_allclose([float(x) for x in got["rows"][1:]], [out.sum(), lse.sum(), w.sum()], rtol=1e-9)
    out, lse = oracle.ssa_rows(q_rows, k, ("alias", DV), rb, rh, ri, Hq=Hq, n_sink=1, window=2, scale=0.25, block=4)
    np.testing.assert_allclose([float(x) for x in got["rows_blocks"][1:]], [out.sum(), lse.sum()], rtol=1e-9)
    assert got["pairs"] == [str(oracle.count_pairs(S, 3, 5))] * 2 + [str(S * (S + 1) // 2)]
    assert got["pairs_blocks"] == [str(oracle.count_pairs_blocks(S, 1, 2, 4))] * 2 + [str(S * (S + 1) // 2)]
    dq, dk, dv = oracle.ssa_backward(q, k, ("alias", DV), dout, n_sink=3, window=5, scale=0.25)
    np.testing.assert_allclose([float(x) for x in got["backward"][1:]], [dq.sum(), dk.sum(), dv.sum()], rtol=1e-8, atol=1e-9)
    np.testing.assert_allclose([float(x) for x in got["backward_rows"][1:]], [dq.sum(), dk.sum(), dv.sum()], rtol=1e-8, atol=1e-9)
    assert got["bad"] == ["-1", "-1", "-1"]


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    hipcc, clang = shutil.which("hipcc"), shutil.which("amdclang")
    if hipcc is None or clang is None:
        pytest.skip("no hipcc / amdclang")
    lib = tmp_path / "libloza_ssa_san.so"
    # every -fsanitize= directly after -Xarch_host: the device pass is not instrumented
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = [f for f in _build.HIPCC_FLAGS if f != "-O3"] + ["-O1", "-g"]
    # The C ABI, the validation and the schedule arithmetic live in one source; only that one is built
    # instrumented. The kernel launchers it calls (never reached by the driver: every launching call it
    # makes is rejected first) resolve against the ordinary build of the library, which is linked behind
    # the instrumented one, so that the instrumented definitions of the entry points are the ones used.
    res = subprocess.run([hipcc, *flags, *san, str(_build.CSRC / "ssa_api.hip"), "-o", str(lib)], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    exe = tmp_path / "sanitize_host"
    lib_dir = Path(B.LIB_PATH).parent
    # (the driver is built by the same clang as the library's host code: one sanitizer runtime for both)
    subprocess.run([clang, "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-I", str(ROOT / "include"),
                    str(ROOT / "tests" / "c" / "sanitize_host.c"), "-o", str(exe), "-L", str(tmp_path), "-lloza_ssa_san",
                    "-L", str(lib_dir), "-lloza_ssa", f"-Wl,-rpath,{tmp_path}", f"-Wl,-rpath,{lib_dir}",
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    got = _run(exe)
    # the same sweep through the ordinary build
    big = [0, 1, 127, 128, 8192, 2147483518, 2147483519, INT64_MAX - 1, INT64_MAX]
    L = B.lib()
    import ctypes
    i64 = ctypes.c_int64
    acc = 0
    nb = len(big)
    for x in range(nb):
        for y in range(nb):
            for z in range(nb):
                a, b, c = i64(-1), i64(-1), i64(-1)
                rc = L.loza_ssa_live_ranges(big[x], big[y], big[z], ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
                acc += rc + ((a.value % 1000) + (b.value % 1000) + (c.value % 1000) if rc == 0 else 0)
                rc = L.loza_ssa_live_ranges_blocks(big[x], big[y], big[z], big[(x + y) % nb], ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
                acc += rc + ((a.value % 1000) + (b.value % 1000) + (c.value % 1000) if rc == 0 else 0)
                c_mod = lambda v: int(np.fmod(v, 1000))  # C's % truncates towards zero
                acc += c_mod(L.loza_ssa_live_pairs(min(big[x], 3000000), big[y], big[z]))
                acc += c_mod(L.loza_ssa_live_pairs_blocks(min(big[x], 100000), big[y], big[z], big[(x + z) % nb]))
                acc += L.loza_ssa_decode_num_splits(64, 64, 1, big[x], big[y], big[z])
                acc += L.loza_ssa_decode_workspace_bytes(3, 16, 2, big[x], 512, big[y], big[z]) % 1000
                acc += L.loza_ssa_backward_workspace_bytes(1, 64, 1, big[x], 576, 512, big[y], big[z], 1) % 1000
                acc += L.loza_ssa_backward_workspace_bytes_blocks(2, 8, 2, big[x], 128, 128, big[y], big[z], big[(y + z) % nb], 0) % 1000
    assert got["edges"] == [str(acc)]
    assert got["calibration_ws"] == [str(B.loza_ssa_calibration_workspace_bytes(1, 64, 4096, 512)), "0"]
    assert got["alpha_grad_ws"][0] == str(B.loza_ssa_calibration_alpha_grad_workspace_bytes(4096))
    assert got["rejected"] == ["-1", "-2", "-2", "-3", "-6", "-4", "-4"]
    assert " ".join(got["status"]) == B.loza_status_str(-6)
