"""A seeded sweep of random shapes through the whole-model calls (projection of one and of k gradients, the entry
point that allocates nothing, expansion + update with g~ stored) for every storage type, each against the oracle
on the stored matrix.  The shapes are drawn around the tile, block and column-slot boundaries of the kernels
(D = 1, 2047, 2048, 2049, ...; n = 1, 24, 25, 26, 32, 33, 97, 100, 101, 128) and at random in between."""
import numpy as np
import pytest
import torch

from oracle import twa_oracle as orc
from paper_2205_13104_amd import binding as twa
from tests.gpu_common import REL_L2_TOL, rel_l2, to_oracle

pytestmark = pytest.mark.gpu

D_EDGES = [1, 2, 31, 127, 128, 129, 1023, 2047, 2048, 2049, 4097, 65537, 300_001]
N_EDGES = [1, 2, 3, 4, 5, 24, 25, 26, 32, 33, 64, 97, 100, 101, 127, 128]


def coefficient_bars(dense, G, ref):
    """Per-coefficient bar for a sum that may cancel to almost nothing (n = 1, or D of a few elements): 1e-5 of the
    rms coefficient, plus 8 standard deviations of the rounding model of an fp32 running sum -- 2^-24 sqrt(m/6) times
    the root of the sum of the squared terms, with m <= 1024 terms per running sum."""
    B = np.sqrt(np.einsum("jd,cd->cj", dense ** 2, G ** 2))
    return 1e-5 * np.sqrt(np.mean(ref ** 2)) + 8 * 2.0 ** -24 * np.sqrt(1024 / 6) * B


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_shapes_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    for case in range(10):
        D = int(rng.choice(D_EDGES + [int(rng.integers(1, 1_200_000))]))
        n = min(int(rng.choice(N_EDGES)), max(1, D))
        k = int(rng.integers(2, 9))
        ld = (D + 2047) // 2048 * 2048
        P32 = torch.zeros((n, ld))
        P32[:, :D] = torch.from_numpy(rng.normal(size=(n, D)).astype(np.float32)) / max(D, 1) ** 0.5
        P32 = P32.cuda()
        ldg = (D + 3) // 4 * 4
        G = torch.zeros((k, ldg))
        G[:, :D] = torch.from_numpy(rng.normal(size=(k, D)).astype(np.float32) * 1e-2)
        G = G.cuda()
        w0 = torch.from_numpy(rng.normal(size=D).astype(np.float32) * 0.05).cuda()
        G_h = G[:, :D].cpu().numpy().astype(np.float64)
        for dt in (twa.F32, twa.BF16, twa.I8, twa.I4):
            print(f"random shape: seed {seed} case {case} D {D} n {n} k {k} dtype {dt}", flush=True)
            pm = twa.wrap_f32(P32, D) if dt == twa.F32 else twa.quantize(P32, D, dt)
            po = to_oracle(pm)
            ref = orc.project(po, G_h)                                     # (k, n)
            bars = coefficient_bars(po.dense(), G_h, ref)
            ws = twa.Workspace(twa.project_workspace_bytes(n, k))
            g0 = G[0, :D].contiguous()
            s1 = twa.project(pm, g0, ws=ws)
            Sk = twa.project(pm, G, ws=ws)
            s_na = torch.full((n,), float("nan"), device="cuda")
            twa.project_noalloc(pm, g0, s_na)
            w = w0.clone()
            gt = torch.full((D,), float("nan"), device="cuda")
            twa.expand_update(pm, s1, w, 0.1, g_tilde=gt)
            torch.cuda.synchronize()
            assert torch.equal(s_na, s1)
            assert np.all(np.abs(s1.cpu().numpy() - ref[0]) <= bars[0]), (D, n, dt)
            assert np.all(np.abs(Sk.cpu().numpy() - ref) <= bars), (D, n, k, dt)
            if n > 1 and D >= 2048:
                assert rel_l2(Sk.cpu().numpy(), ref) <= REL_L2_TOL
            wo = w0.cpu().numpy().astype(np.float64)
            gto = orc.expand_update(po, s1.cpu().numpy().astype(np.float64), wo, float(np.float32(0.1)), want_gt=True)
            assert rel_l2(gt.cpu().numpy(), gto) <= REL_L2_TOL and rel_l2(w.cpu().numpy(), wo) <= REL_L2_TOL
