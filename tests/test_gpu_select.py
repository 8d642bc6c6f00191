"""GPU parity: attention-aware rank groups (ap_select_ranks) against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_23914_amd import workloads as wl
from gpu_util import workspace

pytestmark = pytest.mark.gpu


def run_select(mass, group_rank, cum_num, den):
    from paper_2603_23914_amd import binding as ap
    B, T = mass.shape
    F = len(group_rank)
    dm = torch.from_numpy(np.ascontiguousarray(mass, dtype=np.float32)).cuda()
    rank = torch.full((B, T), -1, dtype=torch.int32, device="cuda")
    off = torch.full((B, F + 1), -1, dtype=torch.int32, device="cuda")
    idx = torch.full((B, T), -1, dtype=torch.int32, device="cuda")
    ws = workspace(ap.ap_select_workspace_bytes(B, T, F))
    ap.ap_select_ranks(dm, group_rank, cum_num, den, rank, off, idx, ws)
    torch.cuda.synchronize()
    return rank.cpu().numpy(), off.cpu().numpy(), idx.cpu().numpy()


def check(mass, group_rank, cum_num, den, what):
    print(f"select {what}: B={mass.shape[0]} T={mass.shape[1]} F={len(group_rank)}", flush=True)
    rank, off, idx = run_select(mass, group_rank, cum_num, den)
    for b in range(mass.shape[0]):
        r_ref, o_ref, i_ref = oracle.select_ranks(mass[b], group_rank, cum_num, den)
        assert (off[b] == o_ref).all(), f"{what}: bucket_off differs (b={b})"
        assert (rank[b] == r_ref).all(), f"{what}: ranks differ (b={b}) at {np.flatnonzero(rank[b] != r_ref)[:8]}"
        assert (idx[b] == i_ref).all(), f"{what}: bucket_idx differs (b={b})"


QUART = ((512, 256, 128, 64), (1, 2, 3, 4), 4)


@pytest.mark.parametrize("T", [1, 5, 63, 64, 1000, 1024, 1025, 4288, 32768])
def test_select_random_mass(T):
    rng = wl.rng_for(21, T)
    mass = rng.random((3, T)).astype(np.float32)
    check(mass, *QUART, "uniform random")


def test_select_config4_mass_all_epochs():
    T = 32768
    for epoch in range(5):
        mass = wl.config4_mass(T, 0, epoch)[None, :]
        check(mass, wl.C4_GROUP_RANK, wl.C4_CUM_NUM, wl.C4_DEN, f"config 4 epoch {epoch}")


def test_select_ties():
    rng = wl.rng_for(22)
    T = 3000
    coarse = (np.floor(rng.random((2, T)) * 16) / 16).astype(np.float32)      # 16 distinct values
    check(coarse, *QUART, "mass in multiples of 1/16")
    check(np.full((2, T), 0.25, np.float32), *QUART, "all equal")
    z = np.zeros((1, T), np.float32)
    z[0, ::3] = -0.0                                                         # -0 and +0 compare equal
    z[0, 7] = 1.0
    check(z, *QUART, "zeros of both signs")
    two = np.where(rng.random((1, T)) < 0.5, np.float32(1e-30), np.float32(3e38)).astype(np.float32)
    check(two, *QUART, "two extreme values")


def test_select_group_shapes():
    rng = wl.rng_for(23)
    mass = rng.standard_exponential((2, 777)).astype(np.float32)
    check(mass, (640,), (1,), 1, "F=1")
    check(mass, (640, 64), (1, 10), 10, "paper-style F=2, 10% at full rank")
    check(mass, (512, 256, 128), (0, 5, 5), 5, "empty first and last group")
    check(mass, (512, 512, 448, 384, 320, 256, 128, 64), (1, 2, 3, 5, 8, 13, 21, 34), 34, "F=8 uneven")
    check(mass[:, :3], (512, 256, 128, 64), (1, 2, 3, 4), 4, "fewer tokens than groups")
