"""The entry point that allocates nothing (twa_project_noalloc) against twa_project, through the C ABI:
same kernels and reduction order, so the coefficients must be bit-equal, and within the parity bar of the
fp64 oracle.  Two calls in a row share the library's fixed device array; the second is smaller and must
not see what the first left there."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import twa_oracle as orc
from paper_2205_13104_amd import binding as twa
from tests.gpu_common import REL_L2_TOL, random_basis_like, rel_l2, store_as, to_oracle

pytestmark = pytest.mark.gpu


def _call_noalloc(pm, g, s):
    """Straight through the C ABI (no binding helper)."""
    lib = twa.lib()
    st = pm.c_struct()
    k, ldg = (1, 0) if g.dim() == 1 else (int(g.shape[0]), int(g.shape[1]))
    return lib.twa_project_noalloc(C.byref(st), C.c_void_p(g.data_ptr()), k, ldg, C.c_void_p(s.data_ptr()),
                                   C.c_void_p(torch.cuda.current_stream().cuda_stream))


@pytest.mark.parametrize("dtype", [twa.I8, twa.F32, twa.I4, twa.BF16], ids=["i8", "f32", "i4", "bf16"])
def test_two_calls_in_a_row_second_smaller(dtype):
    cases = [(1_300_021, 100, 1), (70_001, 37, 1)]           # (D, n, k): the second call is the smaller one
    mats = []
    for D, n, k in cases:
        ldm = 2048 if dtype in (twa.I8, twa.I4) else 128
        P32 = random_basis_like(D, n, seed=D % 1000, ld=(D + ldm - 1) // ldm * ldm)
        pm = store_as(P32, D, dtype)
        gen = torch.Generator(device="cpu").manual_seed(D)
        g = (torch.randn(D, generator=gen) * 1e-2).cuda()
        ws = twa.Workspace(twa.project_workspace_bytes(n, k))
        mats.append((pm, g, ws, torch.empty(n, device="cuda"), torch.full((n,), float("nan"), device="cuda")))
    torch.cuda.synchronize()
    for pm, g, ws, s_ref, s_new in mats:                      # the existing entry point
        twa.project(pm, g, s_ref, ws)
    for pm, g, ws, s_ref, s_new in mats:                      # the new one, back to back on the stream
        print("twa_project_noalloc", "dtype", dtype, "D", pm.D, "n", pm.n, flush=True)
        assert _call_noalloc(pm, g, s_new) == twa.OK
    torch.cuda.synchronize()
    for pm, g, ws, s_ref, s_new in mats:
        assert torch.equal(s_ref, s_new)
        so = orc.project(to_oracle(pm), g.cpu().numpy().astype(np.float64))
        assert rel_l2(s_new.cpu().numpy(), so) <= REL_L2_TOL


def test_batched_and_limit():
    D, n, k = 200_003, 20, 8
    P32 = random_basis_like(D, n, seed=5)
    pm = store_as(P32, D, twa.BF16)
    gen = torch.Generator(device="cpu").manual_seed(9)
    ldg = (D + 3) // 4 * 4
    G = torch.zeros((k, ldg))
    G[:, :D] = torch.randn((k, D), generator=gen) * 1e-2
    G = G.cuda()
    S_ref = twa.project(pm, G)
    S_new = torch.full((k, n), float("nan"), device="cuda")
    assert _call_noalloc(pm, G, S_new) == twa.OK
    # a smaller single-gradient call right behind it
    s_ref = twa.project(pm, G[3, :D].contiguous())
    s_new = torch.full((n,), float("nan"), device="cuda")
    assert _call_noalloc(pm, G[3, :D].contiguous(), s_new) == twa.OK
    torch.cuda.synchronize()
    assert torch.equal(S_ref, S_new) and torch.equal(s_ref, s_new)
    So = orc.project(to_oracle(pm), G[:, :D].cpu().numpy().astype(np.float64))
    assert rel_l2(S_new.cpu().numpy(), So) <= REL_L2_TOL
    # beyond the fixed array: n * k = 800 > 512 is refused on the host, nothing runs
    P100 = store_as(random_basis_like(50_000, 100, seed=6), 50_000, twa.F32)
    G100 = torch.zeros((8, 50_000), device="cuda")
    S100 = torch.zeros((8, 100), device="cuda")
    assert _call_noalloc(P100, G100, S100) == twa.ERR_LIMIT
    assert "fixed device array" in twa.strerror(twa.ERR_LIMIT)
