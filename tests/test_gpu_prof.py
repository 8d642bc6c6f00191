"""GPU: the kernel timer of the library (ap_prof_enable / ap_prof_read) counts one launch per decode
call, reports a time that lies inside the wall time of those calls, and leaves results unchanged."""
import math
import time

import numpy as np
import pytest
import torch

from paper_2603_23914_amd import workloads as wl
from gpu_util import to_dev, workspace

pytestmark = pytest.mark.gpu


def test_kernel_timer_counts_launches_and_stays_inside_wall_time():
    from paper_2603_23914_amd import binding as ap
    dtype, B, H, d, r, T = "bf16", 8, 16, 64, 256, 1500
    case = wl.decode_case(dtype, B, H, d, r, T, steps=0, seed=71, append=False)
    q = wl.step_query(case, 0)
    dq, dCk, dCv, dBk, dBv = (to_dev(x, dtype) for x in (q, case.Ck, case.Cv, case.Bk, case.Bv))
    out0 = torch.empty((B, H, d), dtype=torch.float32, device="cuda")
    out1 = torch.empty_like(out0)
    ws = workspace(ap.ap_decode_workspace_bytes(B, H, d, T, r, ap.AP_BF16))
    scale = 1.0 / math.sqrt(d)
    ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out0, ws, T=T, sm_scale=scale)     # untimed, also warms up
    torch.cuda.synchronize()
    print("timed launches", flush=True)
    ap.ap_prof_enable(True)
    t0 = time.perf_counter()
    for _ in range(5):
        ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out1, ws, T=T, sm_scale=scale)
    ms, n = ap.ap_prof_read()                                                   # waits for the last launch
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ap.ap_prof_enable(False)
    assert n == 5
    assert 0.0 < ms < wall_ms
    assert ms / n < 1.0                     # a few MB of coefficients: microseconds, not milliseconds
    assert torch.equal(out0, out1)
    ap.ap_prof_enable(3)                    # every third launch: 7 launches -> the 1st, 4th and 7th
    for _ in range(7):
        ap.ap_decode_attn(dq, dCk, dCv, dBk, dBv, out1, ws, T=T, sm_scale=scale)
    ms3, n3 = ap.ap_prof_read()
    each = ap.ap_prof_read_launches()
    ap.ap_prof_enable(False)
    assert n3 == 3 and 0.0 < ms3 / n3 < 1.0
    assert len(each) == 3 and all(0.0 < u < 1000.0 for u in each)
    assert abs(sum(each) - ms3 * 1e3) <= 1e-3 * ms3 * 1e3 + 0.01
    ap.ap_prof_enable(True)                 # enabling clears the records
    ms, n = ap.ap_prof_read()
    ap.ap_prof_enable(False)
    assert n == 0 and ms == 0.0


def test_stream_read_probe_reads_every_byte():
    """The yardstick kernel XORs what it reads: flipping one word anywhere in the buffer flips the
    same bits of exactly one of its outputs."""
    from paper_2603_23914_amd import binding as ap
    gran = ap.ap_probe_read_granule()
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    buf = torch.randint(-2 ** 31, 2 ** 31 - 1, (gran // 4,), generator=g, dtype=torch.int32, device="cuda")
    s0 = torch.zeros(8192, dtype=torch.int32, device="cuda")
    s1 = torch.zeros_like(s0)
    ap.ap_probe_read(buf, gran, s0)
    for pos in (0, gran // 8 + 5, gran // 4 - 1):
        buf[pos] ^= 0x5A5A
        ap.ap_probe_read(buf, gran, s1)
        torch.cuda.synchronize()
        diff = (s0 ^ s1).cpu().numpy()
        assert (diff != 0).sum() == 1 and int(diff[diff != 0][0]) == 0x5A5A
        buf[pos] ^= 0x5A5A
    ref = np.bitwise_xor.reduce(buf.cpu().numpy().view(np.uint32))
    assert np.bitwise_xor.reduce(s0.cpu().numpy().view(np.uint32)) == ref
    with pytest.raises(RuntimeError):
        ap.ap_probe_read(buf, gran - 16, s1)
    s2 = torch.zeros_like(s0)
    ap.ap_probe_read_stream(buf, gran, s2)                  # the non-temporal variant reads the same bytes
    torch.cuda.synchronize()
    assert torch.equal(s0, s2)
