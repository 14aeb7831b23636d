"""twa_build_basis_async: the basis construction that never synchronises (Cholesky factor, triangular inverse and
the product of the two passes' factors on the device).  Its P and R must be the host path's, bit for bit -- so every
invariant checked for twa_build_basis holds for it -- and a whole set-up (basis, stored matrix, steps) can be
captured into a HIP graph."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import twa_oracle as orc
from paper_2205_13104_amd import binding as twa
from paper_2205_13104_amd import synth
from tests.gpu_common import ORTHO_TOL, REL_L2_TOL, rel_l2, to_oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,D,n", [("tiny", 200_003, 10), ("cifar_resnet18", 60_017, 100), ("large", 30_011, 128),
                                      ("vit_b16_finetune", 100_003, 20), ("tiny", 5_000, 1), ("cifar_resnet18", 33_333, 17)])
def test_async_path_equals_the_host_path_bit_for_bit(name, D, n):
    wl = synth.WORKLOADS[name]
    W = synth.checkpoints(wl, seed=2, device="cuda", D=D, n=n)
    P_host, R_host = twa.build_basis(W, D)
    R_dev = torch.full((n, n), float("nan"), dtype=torch.float64, device="cuda")
    print("twa_build_basis_async", name, D, n, flush=True)
    P_dev, _, status = twa.build_basis_async(W, D, R=R_dev)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    assert torch.equal(R_dev.cpu(), R_host)
    assert torch.equal(P_dev, P_host)
    Ph = P_dev[:, :D].cpu().numpy().astype(np.float64)
    assert np.max(np.abs(Ph @ Ph.T - np.eye(n))) <= ORTHO_TOL
    # the oracle's Householder factor of the same checkpoints
    _, Ro = orc.build_basis(W[:, :D].cpu().numpy().astype(np.float64))
    assert np.max(np.abs(R_dev.cpu().numpy() - Ro)) <= 1e-5 * np.max(np.abs(Ro))
    # in place, without R
    W2 = W.clone()
    P2, _, st2 = twa.build_basis_async(W2, D, out=W2)
    torch.cuda.synchronize()
    assert P2.data_ptr() == W2.data_ptr() and torch.equal(P2, P_host) and int(st2.item()) == 0


def test_dependent_checkpoints_are_reported_through_the_status_word():
    D, n = 40_000, 6
    W = synth.trajectory(D, n, 0.9, 0.5, seed=3, device="cuda")
    W[4] = 0.5 * W[1] - 2.0 * W[3]
    with pytest.raises(twa.TwaError) as e:
        twa.build_basis(W, D)
    assert e.value.code == twa.ERR_RANK
    R = torch.zeros((n, n), dtype=torch.float64, device="cuda")
    P, _, status = twa.build_basis_async(W, D, R=R)
    torch.cuda.synchronize()
    assert int(status.item()) == 4 + 1                       # 1 + the index of the dependent checkpoint
    assert torch.isnan(P[:, :D]).all() and torch.isnan(R[torch.triu(torch.ones(n, n, dtype=torch.bool))]).all()
    # the status word is the library's to reset: a good matrix afterwards reports 0 through the same word
    Wg = synth.trajectory(D, n, 0.9, 0.5, seed=3, device="cuda")
    twa.build_basis_async(Wg, D, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0


def test_factor_of_a_panel_pass_on_the_device():
    """twa_gram_factor_async in the panel calls: same R^-1 as twa_gram_factor, nothing synchronises in between."""
    D, n, panel = 150_001, 33, 65_536
    W = synth.trajectory(D, n, 0.97, 0.3, seed=4, device="cuda", ld=(D + 2047) // 2048 * 2048)
    st_a, st_b = twa.BasisState(n), twa.BasisState(n)
    for k, r0 in enumerate(range(0, D, panel)):
        rows = min(panel, D - r0)
        twa.gram_accumulate(W[:, r0:], rows, st_a, first=k == 0)
        twa.gram_accumulate(W[:, r0:], rows, st_b, first=k == 0)
    R_host = torch.zeros((n, n), dtype=torch.float64)
    twa.gram_factor(st_a, R_host)
    R_dev = torch.zeros((n, n), dtype=torch.float64, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    rc = twa.lib().twa_gram_factor_async(st_b.gram.ptr, n, st_b.rinv.ptr, R_dev.data_ptr(), status.data_ptr(),
                                         C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == twa.OK
    torch.cuda.synchronize()
    assert int(status.item()) == 0 and torch.equal(R_dev.cpu(), R_host)
    assert torch.equal(st_a.rinv.buf, st_b.rinv.buf)


def test_basis_storage_and_steps_captured_in_one_graph():
    """Set-up and steps in ONE graph: checkpoints -> orthonormal basis (no synchronisation) -> int8 storage ->
    three projected steps.  Every replay must give the bits of the eager sequence, with eager work in between."""
    wl = synth.WORKLOADS["cifar_resnet18"]
    D, n = 150_001, 40
    W0 = synth.checkpoints(wl, seed=7, device="cuda", D=D, n=n, ld=(D + 2047) // 2048 * 2048)
    gs = [synth.gradient(D, 1e-2, seed=7, step=i, device="cuda") for i in range(3)]
    w0 = W0[:, :D].mean(dim=0).contiguous()
    W = W0.clone()
    P = torch.empty_like(W)
    pm = twa.alloc_pmat(twa.I8, D, n)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    wsb = twa.Workspace(twa.build_basis_workspace_bytes(n))
    wsp = twa.Workspace(twa.project_workspace_bytes(n))
    s = torch.empty(n, device="cuda")

    def everything(w):
        twa.build_basis_async(W, D, out=P, status=status, ws=wsb)
        twa.quantize(P, D, twa.I8, out=pm)
        for g in gs:
            twa.project(pm, g, s, wsp)
            twa.expand_update(pm, s, w, wl.lr)

    w_eager = w0.clone()
    everything(w_eager)
    torch.cuda.synchronize()
    codes_eager = pm.data.clone()
    # against the oracle, once: the stored matrix is the oracle's quantisation of P, the steps are within the bar
    o = orc.quantize_i8(P.cpu().numpy(), D=D, ld=pm.ld)
    assert np.array_equal(codes_eager.cpu().numpy(), o.data)
    po = to_oracle(pm)
    wo = w0.cpu().numpy().astype(np.float64)
    for g in gs:
        orc.expand_update(po, orc.project(po, g.cpu().numpy().astype(np.float64)), wo, float(np.float32(wl.lr)))
    assert rel_l2(w_eager.cpu().numpy(), wo) <= REL_L2_TOL
    w_graph = w0.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        everything(w_graph)                                  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        everything(w_graph)
    for rep in range(4):
        w_graph.copy_(w0)
        pm.data.zero_()
        P.zero_()
        status.fill_(9)
        graph.replay()
        torch.cuda.synchronize()
        assert int(status.item()) == 0 and torch.equal(pm.data, codes_eager) and torch.equal(w_graph, w_eager), rep
        twa.project(pm, gs[rep % 3], s, wsp)                 # eager work of the program's own between the replays
        torch.cuda.synchronize()


def test_async_argument_errors():
    L = twa.lib()
    wsb = twa.build_basis_workspace_bytes(4)
    assert L.twa_build_basis_async(0x6000, 1000, 4, 1024, 0x7000, 1024, None, None, 0x8000, wsb, None) == twa.ERR_NULL
    assert L.twa_build_basis_async(0x6000, 3, 4, 128, 0x7000, 128, None, 0x9000, 0x8000, wsb, None) == twa.ERR_SHAPE
    assert L.twa_build_basis_async(0x6000, 1000, 4, 1024, 0x7000, 1024, None, 0x9002, 0x8000, wsb, None) == twa.ERR_ALIGN
    assert L.twa_build_basis_async(0x6000, 1000, 4, 1024, 0x7000, 1024, None, 0x9000, 0x8000, 8, None) == twa.ERR_WORKSPACE
    assert L.twa_gram_factor_async(None, 4, 0x7000, None, 0x9000, None) == twa.ERR_NULL
    assert L.twa_gram_factor_async(0x6000, 4, 0x7000, None, None, None) == twa.ERR_NULL
    assert L.twa_gram_factor_async(0x6000, 129, 0x7000, None, 0x9000, None) == twa.ERR_SHAPE
