"""The boundary as a C program sees it: tests/c_abi/consumer.c (plain C99, compiled here with
gcc against include/attnpack.h and the built library; no C++, Python or torch in its process).
Without a GPU it checks the host-only entry points and the argument validation; on the GPU it
runs a decode call on inputs this test writes to a file and the test compares what the program
wrote back with the fp64 oracle."""
import math
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle
from paper_2603_23914_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2603_23914_amd")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
MAGIC = 0x41504B31
DT = {"f32": 0, "f16": 1, "bf16": 2}


@pytest.fixture(scope="module")
def consumer(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("c_abi") / "consumer")
    cmd = ["gcc", "-std=c99", "-Wall", "-Werror", "-O1", "-D__HIP_PLATFORM_AMD__",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROCM, "include"),
           os.path.join(ROOT, "tests", "c_abi", "consumer.c"), "-o", exe,
           "-L" + PKG, "-lattnpack", "-L" + os.path.join(ROCM, "lib"), "-lamdhip64",
           "-Wl,-rpath," + PKG, "-Wl,-rpath," + os.path.join(ROCM, "lib")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return exe


def test_c_consumer_host_checks(consumer):
    res = subprocess.run([consumer, "host"], capture_output=True, text=True, timeout=60)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "host checks passed" in res.stdout


def run_consumer(consumer, tmp_path, dtype, B, H, Hkv, d, r, T0, step, shared, seed):
    steps = 1 if step else 0
    T = T0 + steps
    case = wl.decode_case(dtype, B, Hkv, d, r, T0, steps=steps, seed=seed, append=step, shared_basis=shared)
    P = lambda x: oracle.promote(x, dtype)
    q = wl.store(wl.rng_for(seed, 7).standard_normal((B, H, d)), dtype)
    scale = 1.0 / math.sqrt(d)
    arrays = [q]
    if step:
        kn, vn = wl.step_new_token(case, 0, P(case.Bk), P(case.Bv))
        arrays += [kn, vn]
    arrays += [case.Ck, case.Cv, case.Bk, case.Bv]
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        f.write(struct.pack("<11i", MAGIC, B, H, Hkv, d, T, case.T_cap, r, DT[dtype], int(step), int(shared)))
        f.write(struct.pack("<f", scale))
        for a in arrays:
            f.write(np.ascontiguousarray(a).tobytes())
    print(f"C consumer {dtype} B={B} H={H}/{Hkv} d={d} r={r} T={T} step={step}", flush=True)
    res = subprocess.run([consumer, "run", fin, fout], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    raw = open(fout, "rb").read()
    n = B * H * d
    out = np.frombuffer(raw, np.float32, n).reshape(B, H, d).astype(np.float64)
    lse = np.frombuffer(raw, np.float32, B * H, offset=4 * n).reshape(B, H).astype(np.float64)
    Ck, Cv = case.Ck.copy(), case.Cv.copy()
    if step:
        store_dt = Ck.dtype
        rows = np.frombuffer(raw, store_dt, 2 * B * r, offset=4 * n + 4 * B * H).reshape(2, B, r)
        Ck[:, T - 1], Cv[:, T - 1] = rows[0], rows[1]
        c_ref = oracle.compact(P(kn)[0][None], P(case.Bk) if shared else P(case.Bk)[0])[0]
        tol = {"bf16": 2.0 ** -7, "f16": 2.0 ** -10, "f32": 1e-5}[dtype]
        assert np.abs(P(Ck)[0, T - 1] - c_ref).max() <= tol * np.abs(c_ref).max() + 1e-6
    ref = oracle.decode_attn_batched(P(q), P(Ck), P(Cv), P(case.Bk), P(case.Bv), T, absorbed=True,
                                     kv_heads=None if Hkv == H else Hkv)
    tol = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}[dtype]
    assert np.isfinite(out).all()
    assert np.abs(out - ref).max() <= tol * np.abs(ref).max()
    _, ref_lse = oracle.decode_attn(P(q)[0], P(Ck)[0, :T], P(Cv)[0, :T], P(case.Bk) if shared else P(case.Bk)[0],
                                    P(case.Bv) if shared else P(case.Bv)[0], return_lse=True,
                                    kv_heads=None if Hkv == H else Hkv)
    assert np.abs(lse[0] - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,B,H,Hkv,d,r,T0,step,shared", [
    ("bf16", 2, 40, 40, 128, 640, 150, True, False),
    ("f16", 3, 32, 8, 128, 256, 333, False, True),
    ("f32", 1, 4, 4, 32, 16, 64, False, False),
])
def test_c_consumer_decode(consumer, tmp_path, dtype, B, H, Hkv, d, r, T0, step, shared):
    run_consumer(consumer, tmp_path, dtype, B, H, Hkv, d, r, T0, step, shared, seed=101)
