"""Parity of the HIP library (through its C ABI) against the fp64 CPU oracle, element by element, on
seeded synthetic inputs.  Bars: integer codes, scales and 16-bit conversions bit-exact; s, g~, w
within a relative L2 error of 1e-5 of the oracle evaluated on the SAME stored P; max|P^T P - I| <= 1e-5
after basis construction.  Sizes span several tiles of every kernel plus a ragged tail."""
import math

import numpy as np
import pytest
import torch

from oracle import twa_oracle as orc
from paper_2205_13104_amd import binding as twa
from paper_2205_13104_amd import synth
from tests.gpu_common import ORTHO_TOL, REL_L2_TOL, random_basis_like, rel_l2, store_as, to_oracle

pytestmark = pytest.mark.gpu

DTYPES = [twa.F32, twa.BF16, twa.I8, twa.I4]
NAMES = {twa.F32: "f32", twa.BF16: "bf16", twa.I8: "i8", twa.I4: "i4"}


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------------------------------------ quantize
@pytest.mark.parametrize("D,n,block", [(128 * 9 + 40, 3, 128), (70001, 5, 128), (4096, 2, 32), (5000, 4, 64),
                                       (100000, 7, 256), (17, 1, 128)])
def test_quantize_i8_bit_exact(D, n, block):
    say("quantize_i8", D, n, block)
    P = random_basis_like(D, n, seed=D + n)
    P[0, 128:256] = 0.0 if D > 256 else P[0, 128:256]          # an all-zero block
    pm = twa.quantize(P, D, twa.I8, block=block)
    torch.cuda.synchronize()
    assert pm.ld % 2048 == 0 and pm.ld - D < 2048
    ref = orc.quantize_i8(P.cpu().numpy(), D=D, block=block, ld=pm.ld)
    assert np.array_equal(pm.scales_by_vector().cpu().numpy().view(np.uint32), ref.scales.view(np.uint32))
    assert np.array_equal(pm.data.cpu().numpy(), ref.data)


@pytest.mark.parametrize("mag", [1.0, 3e-5, 250.0])
def test_quantize_i8_bit_exact_near_ties(mag):
    # values placed on and next to rounding ties of the recipe
    D, n = 128 * 64, 2
    g = torch.Generator().manual_seed(5)
    base = torch.rand((n, D), generator=g) * 2 - 1
    amax = base.abs().amax()
    k = torch.randint(-126, 127, (n, D), generator=g).float() + 0.5
    P = (k * (amax / 127.0)).float()
    P[:, ::3] = base[:, ::3]
    P[:, 0] = amax
    P = (P * mag).contiguous().cuda()
    pm = twa.quantize(P, D, twa.I8)
    ref = orc.quantize_i8(P.cpu().numpy(), ld=pm.ld)
    assert np.array_equal(pm.scales_by_vector().cpu().numpy().view(np.uint32), ref.scales.view(np.uint32))
    assert np.array_equal(pm.data.cpu().numpy(), ref.data)


@pytest.mark.parametrize("D,n,block", [(64 * 9 + 21, 3, 64), (70001, 5, 64), (4096, 2, 32), (100000, 3, 256),
                                       (33, 1, 64)])
def test_quantize_i4_bit_exact(D, n, block):
    say("quantize_i4", D, n, block)
    P = random_basis_like(D, n, seed=D + 3 * n)
    if D > 256:
        P[0, 128:256] = 0.0
    Pn = P.cpu().numpy()
    gs = orc.gscale_i4(Pn, D)
    pm = twa.quantize(P, D, twa.I4, block=block)              # gscale chosen by the library
    ref = orc.quantize_i4(Pn, D=D, block=block, ld=pm.ld, gscale=gs)
    assert pm.gscale == gs
    assert np.array_equal(pm.scales_by_vector().view(torch.int16).cpu().numpy().view(np.uint16), ref.scales)
    assert np.array_equal(pm.data.cpu().numpy(), ref.data)
    # caller-supplied power of two: no synchronisation inside, same rules
    pm2 = twa.quantize(P, D, twa.I4, block=block, gscale=gs * 4)
    ref2 = orc.quantize_i4(Pn, D=D, block=block, ld=pm.ld, gscale=gs * 4)
    assert np.array_equal(pm2.scales_by_vector().view(torch.int16).cpu().numpy().view(np.uint16), ref2.scales)
    assert np.array_equal(pm2.data.cpu().numpy(), ref2.data)


def test_quantize_bf16_and_f32_bit_exact():
    D, n = 70001, 3
    P = random_basis_like(D, n, seed=9)
    P[1, :6] = torch.tensor([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e38])
    ref = orc.to_bf16(P.cpu().numpy(), D=D, ld=P.shape[1])
    pm = twa.quantize(P, D, twa.BF16)
    assert np.array_equal(pm.data.view(torch.int16).cpu().numpy().view(np.uint16), ref.data)
    pf = twa.quantize(P, D, twa.F32)
    assert torch.equal(pf.data[:, :D], P[:, :D]) and not pf.data[:, D:].any()


# ------------------------------------------------------------------------------------------------ project
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("D,n", [(300017, 100), (65536, 10), (1000, 1), (40000, 128), (123457, 37), (9, 3)])
def test_project_matches_oracle(dtype, D, n):
    say("project", NAMES[dtype], D, n)
    P32 = random_basis_like(D, n, seed=11 + n)
    pm = store_as(P32, D, dtype)
    g = synth.gradient(D, 1e-2, seed=1, device="cuda")
    s = twa.project(pm, g)
    ref = orc.project(to_oracle(pm), g.cpu().numpy().astype(np.float64))
    err = rel_l2(s.cpu().numpy(), ref)
    say("  rel_l2", err)
    assert err <= REL_L2_TOL
    # deterministic reduction order: a second call returns identical bits
    s2 = twa.project(pm, g)
    assert torch.equal(s, s2)


def test_project_ignores_padding_garbage():
    D, n = 5000, 6
    P32 = random_basis_like(D, n, seed=3)
    P32[:, D:] = float("nan")
    pm = twa.wrap_f32(P32, D)
    g = synth.gradient(D, 1e-2, seed=2, device="cuda")
    s = twa.project(pm, g)
    ref = orc.project(to_oracle(pm), g.cpu().numpy().astype(np.float64))
    assert rel_l2(s.cpu().numpy(), ref) <= REL_L2_TOL


@pytest.mark.parametrize("dtype,n,k", [(twa.BF16, 20, 8), (twa.F32, 10, 3), (twa.I8, 32, 8), (twa.I4, 12, 2),
                                       (twa.BF16, 40, 4), (twa.I8, 100, 8), (twa.F32, 128, 3), (twa.BF16, 33, 8),
                                       (twa.I8, 65, 2), (twa.F32, 97, 8), (twa.I4, 100, 3), (twa.I4, 100, 8), (twa.I4, 128, 4),
                                       (twa.I4, 61, 5), (twa.I4, 3, 2)])
def test_project_batched_matches_oracle(dtype, n, k):
    D = 150001
    say("project_batched", NAMES[dtype], D, n, k)
    P32 = random_basis_like(D, n, seed=21 + n)
    pm = store_as(P32, D, dtype)
    G = synth.gradient(D, 1e-2, seed=4, device="cuda", k=k, ldg=D + 3 + (4 - (D + 3) % 4) % 4)
    S = twa.project(pm, G)
    ref = orc.project(to_oracle(pm), G.cpu().numpy().astype(np.float64))
    assert S.shape == (k, n)
    err = rel_l2(S.cpu().numpy(), ref)
    say("  rel_l2", err)
    assert err <= REL_L2_TOL
    # each gradient alone gives the same row
    s0 = twa.project(pm, G[0, :D].contiguous())
    assert rel_l2(S[0].cpu().numpy(), s0.cpu().numpy()) <= 1e-6


# ------------------------------------------------------------------------------------------------ expand_update
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("D,n", [(300017, 100), (65536, 10), (1000, 1), (40000, 128), (123457, 37), (9, 3)])
def test_expand_update_matches_oracle(dtype, D, n):
    say("expand_update", NAMES[dtype], D, n)
    P32 = random_basis_like(D, n, seed=31 + n)
    pm = store_as(P32, D, dtype)
    gen = torch.Generator().manual_seed(7)
    s = (torch.randn(n, generator=gen) * 1e-2).cuda()
    w0 = (torch.randn(D, generator=gen) * 0.05).cuda()
    lr = 0.1
    w = w0.clone()
    gt = torch.empty(D, device="cuda")
    twa.expand_update(pm, s, w, lr, gt)
    wo = w0.cpu().numpy().astype(np.float64)
    gto = orc.expand_update(to_oracle(pm), s.cpu().numpy().astype(np.float64), wo, lr, want_gt=True)
    e_gt, e_w = rel_l2(gt.cpu().numpy(), gto), rel_l2(w.cpu().numpy(), wo)
    say("  rel_l2 g~", e_gt, "w", e_w)
    assert e_gt <= REL_L2_TOL and e_w <= REL_L2_TOL
    # the update itself is one fused multiply-add per element: from the same fp32 w and the library's
    # own g~ the new weight is the exactly computed w - lr*g~ rounded once (1 ulp allowed for the
    # double rounding of this check)
    lr32 = float(np.float32(lr))
    exact = w0.cpu().numpy().astype(np.float64) - lr32 * gt.cpu().numpy().astype(np.float64)
    ulp = np.spacing(np.abs(exact).astype(np.float32)).astype(np.float64)
    assert np.all(np.abs(w.cpu().numpy().astype(np.float64) - exact) <= ulp)
    # without the optional output the weights come out identical
    w2 = w0.clone()
    twa.expand_update(pm, s, w2, lr, None)
    assert torch.equal(w, w2)


def test_expand_update_does_not_touch_memory_past_D():
    D, n = 1000 * 4 + 3, 5                     # D % 4 != 0: the last 128-bit store straddles the end
    P32 = random_basis_like(D, n, seed=2)
    pm = twa.wrap_f32(P32, D)
    buf = torch.full((D + 61,), 7.0, device="cuda")
    gbuf = torch.full((D + 61,), 9.0, device="cuda")
    s = torch.ones(n, device="cuda")
    twa.expand_update(pm, s, buf, 1.0, gbuf)
    assert torch.all(buf[D:] == 7.0) and torch.all(gbuf[D:] == 9.0)
    assert not torch.any(buf[:D] == 7.0)


# ------------------------------------------------------------------------------------------------ chained steps
@pytest.mark.parametrize("dtype", [twa.F32, twa.I8])
def test_chained_steps_tiny_config(dtype):
    # the small benchmark configuration at reduced D: trajectory checkpoints, basis on the GPU, T steps
    wl = synth.WORKLOADS["tiny"]
    D, n, T = 50021, wl.n, 20
    W = synth.checkpoints(wl, seed=0, device="cuda", D=D)
    P, _ = twa.build_basis(W, D)
    pm = store_as(P, D, dtype)
    po = to_oracle(pm)
    w = W[:, :D].mean(dim=0).contiguous()
    wo = w.cpu().numpy().astype(np.float64)
    w_start = wo.copy()
    ws = twa.Workspace(twa.project_workspace_bytes(n))
    s = torch.empty(n, device="cuda")
    for t in range(T):
        g = synth.gradient(D, wl.sigma_g, seed=0, step=t, device="cuda")
        twa.project(pm, g, s, ws)
        twa.expand_update(pm, s, w, wl.lr)
        so = orc.project(po, g.cpu().numpy().astype(np.float64))
        assert rel_l2(s.cpu().numpy(), so) <= REL_L2_TOL
        orc.expand_update(po, so, wo, wl.lr)
    assert rel_l2(w.cpu().numpy(), wo) <= REL_L2_TOL
    # displacement w_T - w_0: limited by the fp32 rounding of every in-place store, reported only
    say("  displacement rel_l2", rel_l2(w.cpu().numpy().astype(np.float64) - w_start, wo - w_start))


# ------------------------------------------------------------------------------------------------ build_basis
def _basis_checks(W, P, R, D, n):
    Wh = W[:, :D].cpu().numpy().astype(np.float64)
    Ph = P[:, :D].cpu().numpy().astype(np.float64)
    ortho = np.max(np.abs(Ph @ Ph.T - np.eye(n)))
    say("  max|PtP-I|", ortho)
    assert ortho <= ORTHO_TOL
    Rh = R.numpy()
    assert np.all(np.diag(Rh) > 0) and np.max(np.abs(np.tril(Rh, -1))) == 0.0
    resid = np.linalg.norm(Wh - Rh.T @ Ph) / np.linalg.norm(Wh)
    say("  |W-PR|/|W|", resid)
    assert resid <= 1e-5
    # R agrees with P^T W and the first vector is the first checkpoint normalised
    Rchk = Ph @ Wh.T
    assert np.max(np.abs(np.tril(Rchk, -1))) <= 1e-4 * np.max(np.abs(Rchk))
    assert rel_l2(Ph[0], Wh[0] / np.linalg.norm(Wh[0])) <= 1e-5
    return Wh, Ph


@pytest.mark.parametrize("name,D,n", [("tiny", 200003, 10), ("cifar_resnet18", 60017, 100), ("large", 30011, 128),
                                      ("vit_b16_finetune", 90001, 20), ("tiny", 64, 5)])
def test_build_basis_invariants(name, D, n):
    say("build_basis", name, D, n)
    wl = synth.WORKLOADS[name]
    W = synth.checkpoints(wl, seed=1, device="cuda", D=D, n=n)
    P, R = twa.build_basis(W, D)
    Wh, Ph = _basis_checks(W, P, R, D, n)
    assert not P[:, D:].any()
    # span(P) = span(W): each checkpoint is reproduced by its projection on P, and the oracle's basis
    # (Householder, fp64) spans the same space: its vectors are reproduced by P as well
    assert np.linalg.norm(Wh - (Wh @ Ph.T) @ Ph) <= 1e-5 * np.linalg.norm(Wh)
    Po, Ro = orc.build_basis(Wh)
    assert np.max(np.abs(Po - (Po @ Ph.T) @ Ph)) <= 2e-3          # conditioning-limited (kappa * eps32), reported
    say("  max|P_oracle - proj|", np.max(np.abs(Po - (Po @ Ph.T) @ Ph)), " |R-R_oracle|/|R|",
        np.linalg.norm(R.numpy() - Ro) / np.linalg.norm(Ro))
    assert np.linalg.norm(R.numpy() - Ro) <= 1e-5 * np.linalg.norm(Ro)


@pytest.mark.parametrize("n", [16, 17, 33, 48, 49, 64, 65, 81, 96, 97, 112, 113])
def test_build_basis_every_count_of_column_blocks(n):
    # the Gram and apply kernels are compiled per number of 16-column blocks, and the waves' shares of the
    # blocks differ with it: every count from 1 to 8, at a full last block and at a last block of one column;
    # D leaves a ragged last tile of rows and gives several workgroups several tiles each
    D = 70001
    say("build_basis, column blocks", (n + 15) // 16, "n", n)
    W = synth.checkpoints(synth.WORKLOADS["cifar_resnet18"], seed=3, device="cuda", D=D, n=n)
    P, R = twa.build_basis(W, D)
    Wh, Ph = _basis_checks(W, P, R, D, n)
    assert not P[:, D:].any()
    assert np.linalg.norm(Wh - (Wh @ Ph.T) @ Ph) <= 1e-5 * np.linalg.norm(Wh)
    _, Ro = orc.build_basis(Wh)
    assert np.linalg.norm(R.numpy() - Ro) <= 1e-5 * np.linalg.norm(Ro)


def test_build_basis_in_place_and_n1():
    D = 40001
    wl = synth.WORKLOADS["tiny"]
    W = synth.checkpoints(wl, seed=2, device="cuda", D=D, n=10)
    P_ref, R_ref = twa.build_basis(W, D)
    W2 = W.clone()
    P2, R2 = twa.build_basis(W2, D, out=W2)
    assert P2.data_ptr() == W2.data_ptr()
    assert torch.equal(P2, P_ref) and torch.equal(R2, R_ref)
    # n = 1 closed form
    w1 = W[:1].contiguous()
    P1, R1 = twa.build_basis(w1, D)
    nrm = float(np.linalg.norm(w1[0, :D].cpu().numpy().astype(np.float64)))
    assert abs(R1[0, 0].item() - nrm) <= 1e-6 * nrm
    assert rel_l2(P1[0, :D].cpu().numpy(), w1[0, :D].cpu().numpy().astype(np.float64) / nrm) <= 1e-6


@pytest.mark.parametrize("name,D,n,panel", [("tiny", 200003, 10, 65536), ("cifar_resnet18", 60017, 100, 4096),
                                            ("large", 300_011, 128, 100_000), ("tiny", 64, 5, 16)])
def test_build_basis_from_panels_of_rows(name, D, n, panel):
    """CholeskyQR2 with the rows arriving in panels (the largest configuration streams its checkpoints that way):
    the same invariants, the same R as the fp64 oracle, and a basis that agrees with the one-shot call to the
    rounding of a Gram matrix summed in another order."""
    say("build_basis panels", name, D, n, panel)
    wl = synth.WORKLOADS[name]
    W = synth.checkpoints(wl, seed=1, device="cuda", D=D, n=n)
    P, R = twa.build_basis_panels(W, D, panel)
    Wh, Ph = _basis_checks(W, P, R, D, n)
    assert not P[:, D:].any()
    Po, Ro = orc.build_basis(Wh)
    assert np.linalg.norm(R.numpy() - Ro) <= 1e-5 * np.linalg.norm(Ro)
    P1, R1 = twa.build_basis(W, D)
    assert np.linalg.norm(R.numpy() - R1.numpy()) <= 1e-6 * np.linalg.norm(R1.numpy())
    # in place, panel by panel
    W2 = W.clone()
    P2, R2 = twa.build_basis_panels(W2, D, panel, out=W2)
    assert P2.data_ptr() == W2.data_ptr() and torch.equal(P2[:, :D], P[:, :D]) and torch.equal(R2, R)
    # a dependent checkpoint is reported by the factorisation
    W3 = W.clone()
    if n >= 5:
        W3[4] = 0.25 * W3[1] - 3.0 * W3[2]
        with pytest.raises(twa.TwaError) as ei:
            twa.build_basis_panels(W3, D, panel)
        assert ei.value.code == twa.ERR_RANK and "checkpoint 4" in str(ei.value)


@pytest.mark.parametrize("n", [10, 100, 128])
def test_gram_of_an_orthonormal_matrix_in_fp32_products(n):
    """The second pass's Gram matrix (TWA_GRAM_ORTHONORMAL_INPUT: fp32 products per 64-row tile, tiles summed in
    fp64) against the fp64 one and against numpy, on a basis the library has just built; and the flag word is
    checked."""
    import ctypes as C
    D = 300_011
    W = synth.checkpoints(synth.WORKLOADS["cifar_resnet18"], seed=5, device="cuda", D=D, n=n)
    P, _ = twa.build_basis(W, D)
    L = twa.lib()
    gb, rb, wb = C.c_size_t(), C.c_size_t(), C.c_size_t()
    assert L.twa_basis_state_bytes(n, C.byref(gb), C.byref(rb), C.byref(wb)) == twa.OK
    NP = (n + 15) // 16 * 16
    assert gb.value == NP * NP * 8
    ws = twa.Workspace(wb.value)
    grams = []
    for flags in (0, twa.GRAM_ORTHONORMAL_INPUT):
        g = torch.full((NP, NP), float("nan"), dtype=torch.float64, device="cuda")
        st = torch.cuda.current_stream().cuda_stream
        assert L.twa_gram_accumulate(P.data_ptr(), D, n, P.shape[1], g.data_ptr(), flags, ws.ptr, ws.nbytes, st) == twa.OK
        torch.cuda.synchronize()
        grams.append(np.triu(g.cpu().numpy()[:n, :n]))
    Ph = P[:, :D].cpu().numpy().astype(np.float64)
    ref = np.triu(Ph @ Ph.T)
    say("gram fp64 vs numpy", np.max(np.abs(grams[0] - ref)), " fp32 products vs numpy", np.max(np.abs(grams[1] - ref)))
    assert np.max(np.abs(grams[0] - ref)) <= 1e-12
    assert np.max(np.abs(grams[1] - ref)) <= 2e-8           # fp32 products of numbers ~ D^-1/2, summed in fp64
    # adding: twice the matrix
    g2 = torch.from_numpy(np.zeros((NP, NP))).cuda()
    for k in range(2):
        flags = twa.GRAM_ORTHONORMAL_INPUT | (twa.GRAM_ADD if k else 0)
        assert L.twa_gram_accumulate(P.data_ptr(), D, n, P.shape[1], g2.data_ptr(), flags, ws.ptr, ws.nbytes,
                                     torch.cuda.current_stream().cuda_stream) == twa.OK
    torch.cuda.synchronize()
    assert np.max(np.abs(np.triu(g2.cpu().numpy()[:n, :n]) - 2.0 * grams[1])) <= 1e-15


def test_build_basis_rank_deficient():
    D, n = 5000, 6
    W = random_basis_like(D, n, seed=8)
    W[4] = 0.25 * W[1] - 3.0 * W[2]
    with pytest.raises(twa.TwaError) as ei:
        twa.build_basis(W, D)
    assert ei.value.code == twa.ERR_RANK and "checkpoint 4" in str(ei.value)


def test_projector_identities_on_gpu_basis():
    wl = synth.WORKLOADS["tiny"]
    D, n = 100003, 10
    W = synth.checkpoints(wl, seed=3, device="cuda", D=D)
    P, _ = twa.build_basis(W, D)
    pm = twa.wrap_f32(P, D)
    g = synth.gradient(D, 1e-2, seed=5, device="cuda")
    s = twa.project(pm, g)
    z = torch.zeros(D, device="cuda")
    gt = torch.empty(D, device="cuda")
    twa.expand_update(pm, s, z, 1.0, gt)
    assert abs(gt.norm().item() - s.norm().item()) <= 1e-5 * s.norm().item()
    assert s.norm().item() <= g.norm().item()
    # idempotence: projecting g~ again returns g~
    s2 = twa.project(pm, gt)
    assert rel_l2(s2.cpu().numpy(), s.cpu().numpy()) <= 1e-5
    # a checkpoint lies in the span: it is reproduced
    v = W[3, :D].contiguous()
    sv = twa.project(pm, v)
    out = torch.empty(D, device="cuda")
    twa.expand_update(pm, sv, torch.zeros(D, device="cuda"), 1.0, out)
    assert rel_l2(out.cpu().numpy(), v.cpu().numpy()) <= 1e-5
    # block identity of the distributed scheme (column partition of P)
    acc = torch.zeros(D, device="cuda")
    for part in (range(0, 5), range(5, 10)):
        Pi = twa.wrap_f32(P[list(part)].contiguous(), D)
        si = twa.project(Pi, g)
        gi = torch.empty(D, device="cuda")
        twa.expand_update(Pi, si, torch.zeros(D, device="cuda"), 1.0, gi)
        acc += gi
    assert rel_l2(acc.cpu().numpy(), gt.cpu().numpy()) <= 1e-5


# ------------------------------------------------------------------------------------------------ HIP graph
def test_step_captured_in_a_graph_replays_bit_for_bit():
    """The step calls neither allocate nor synchronise, so a caller may capture them in a HIP graph.  Every
    replay (with eager work and synchronisations of the program's own in between) must reproduce the eager
    result bit for bit."""
    D, n = 1_500_007, 100
    pm = store_as(random_basis_like(D, n, seed=31), D, twa.I8)
    gs = [synth.gradient(D, 1e-2, seed=31, step=i, device="cuda") for i in range(3)]
    plan = twa.LayerPlan(synth.layer_offsets(synth.random_layer_sizes(D, 20, seed=3)), D)
    s = torch.empty(n, device="cuda")
    S = torch.empty((plan.L, n), device="cuda")
    ws = twa.Workspace(max(twa.project_workspace_bytes(n), twa.project_layers_workspace_bytes(n, plan.L)))
    w0 = synth.gradient(D, 0.05, seed=32, device="cuda")

    def steps(w):
        for g in gs:
            twa.project(pm, g, s, ws)
            twa.expand_update(pm, s, w, 0.1)
            twa.project_layers(pm, g, plan, S, ws)
            twa.expand_update_layers(pm, S, plan, w, 0.05)

    w_eager = w0.clone()
    steps(w_eager)
    torch.cuda.synchronize()
    w_graph = w0.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        steps(w_graph)                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        steps(w_graph)
    for rep in range(4):
        w_graph.copy_(w0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(w_graph, w_eager), rep
        # eager work of the program's own between the replays
        twa.project(pm, gs[rep % 3], s, ws)
        torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------------ several launches
@pytest.mark.parametrize("D", [33_000_001, 61_000_001], ids=["two", "three"])
@pytest.mark.parametrize("dtype", [twa.F32, twa.BF16, twa.I8, twa.I4], ids=["f32", "bf16", "i8", "i4"])
def test_expand_in_several_launches(dtype, D):
    """A vector so long that a wave cannot keep the sums of all its tiles on chip is expanded by several
    launches, one run of tiles each (runs that do not divide evenly; two and three launches) -- same results
    as the oracle, whole-model and layer-wise, in place and into another buffer."""
    n = 4
    pm = store_as(random_basis_like(D, n, seed=41), D, dtype)
    po = to_oracle(pm)
    s = torch.tensor([0.7, -1.3, 0.2, 2.1], device="cuda")
    w0 = synth.gradient(D, 0.05, seed=42, device="cuda")
    w = w0.clone()
    gt = torch.empty(D, device="cuda")
    twa.expand_update(pm, s, w, 0.1, gt)
    torch.cuda.synchronize()
    wo = w0.cpu().numpy().astype(np.float64)
    gto = orc.expand_update(po, s.cpu().numpy().astype(np.float64), wo, float(np.float32(0.1)), want_gt=True)
    assert rel_l2(gt.cpu().numpy(), gto) <= REL_L2_TOL and rel_l2(w.cpu().numpy(), wo) <= REL_L2_TOL
    off = synth.layer_offsets(synth.random_layer_sizes(D, 25, seed=6))
    plan = twa.LayerPlan(off, D)
    S = torch.randn((plan.L, n), generator=torch.Generator().manual_seed(3)).cuda()
    w = w0.clone()
    twa.expand_update_layers(pm, S, plan, w, 0.1, gt)
    torch.cuda.synchronize()
    wo = w0.cpu().numpy().astype(np.float64)
    gto = orc.expand_update_layers(po, S.cpu().numpy().astype(np.float64), off.numpy(), wo, float(np.float32(0.1)),
                                   want_gt=True)
    assert rel_l2(gt.cpu().numpy(), gto) <= REL_L2_TOL and rel_l2(w.cpu().numpy(), wo) <= REL_L2_TOL
    # into another buffer: w = wbar + P beta (the coefficient form), the old weights left untouched
    wbar = w0.clone()
    w2 = twa.weights_from_beta(pm, S, plan, wbar)
    torch.cuda.synchronize()
    w2o = orc.weights_from_beta(po, S.cpu().numpy().astype(np.float64), off.numpy(), w0.cpu().numpy().astype(np.float64))
    assert rel_l2(w2.cpu().numpy(), w2o) <= REL_L2_TOL and torch.equal(wbar, w0)


@pytest.mark.parametrize("dtype", [twa.F32, twa.I8, twa.I4], ids=["f32", "i8", "i4"])
def test_expand_launch_partition_on_a_small_grid(dtype, launch_knobs):
    """The cut of a vector into launches and of a launch into rounds, exercised with a grid of a few workgroups
    so that short vectors already need several launches: every tile count around the capacity of one launch
    (4 waves x 7 rounds x grid), remainders of every size, whole-model and layer-wise."""
    n = 3
    s = torch.tensor([0.7, -1.3, 0.2], device="cuda")
    for grid in (1, 3):
        launch_knobs(twa.KNOB_EXPAND_GRID, grid)
        cap = 4 * 7 * grid                                    # tiles of 2048 elements one launch holds
        for tiles in sorted({1, 2, 5, cap - 1, cap, cap + 1, cap + 4, 2 * cap - 3, 2 * cap, 2 * cap + 1, 3 * cap + 9}):
            D = tiles * 2048 - 5
            print("partition", dtype, "grid", grid, "tiles", tiles, flush=True)
            pm = store_as(random_basis_like(D, n, seed=tiles), D, dtype)
            po = to_oracle(pm)
            w0 = synth.gradient(D, 0.05, seed=43, device="cuda")
            w = w0.clone()
            gt = torch.full((D,), float("nan"), device="cuda")
            twa.expand_update(pm, s, w, 0.1, gt)
            torch.cuda.synchronize()
            wo = w0.cpu().numpy().astype(np.float64)
            gto = orc.expand_update(po, s.cpu().numpy().astype(np.float64), wo, float(np.float32(0.1)), want_gt=True)
            assert rel_l2(gt.cpu().numpy(), gto) <= REL_L2_TOL and rel_l2(w.cpu().numpy(), wo) <= REL_L2_TOL
            # layer-wise over a ragged table: the device divides the plan's tiles with the same rule
            off = synth.layer_offsets(synth.random_layer_sizes(D, 9, seed=tiles))
            plan = twa.LayerPlan(off, D)
            S = torch.randn((plan.L, n), generator=torch.Generator().manual_seed(tiles)).cuda()
            w = w0.clone()
            gt.fill_(float("nan"))
            twa.expand_update_layers(pm, S, plan, w, 0.1, gt)
            torch.cuda.synchronize()
            wo = w0.cpu().numpy().astype(np.float64)
            gto = orc.expand_update_layers(po, S.cpu().numpy().astype(np.float64), off.numpy(), wo,
                                           float(np.float32(0.1)), want_gt=True)
            assert rel_l2(gt.cpu().numpy(), gto) <= REL_L2_TOL and rel_l2(w.cpu().numpy(), wo) <= REL_L2_TOL


@pytest.mark.parametrize("dtype", [twa.F32, twa.I8, twa.I4], ids=["f32", "i8", "i4"])
def test_project_tile_division_on_a_small_grid(dtype, launch_knobs):
    """The division of the tiles over the workgroups of the projection (and the per-layer slots of its partial
    sums), exercised with a grid of a few workgroups: many tiles per workgroup, workgroups without tiles."""
    n = 5
    for grid in (1, 3, 7):
        launch_knobs(twa.KNOB_PROJECT_GRID, grid)
        for tiles in (1, 2, grid, grid + 1, 5 * grid - 1, 11 * grid + 2):
            D = tiles * 2048 - 3
            print("division", dtype, "grid", grid, "tiles", tiles, flush=True)
            pm = store_as(random_basis_like(D, n, seed=tiles + grid), D, dtype)
            po = to_oracle(pm)
            g = synth.gradient(D, 1e-2, seed=44, device="cuda")
            s = twa.project(pm, g)
            torch.cuda.synchronize()
            so = orc.project(po, g.cpu().numpy().astype(np.float64))
            assert rel_l2(s.cpu().numpy(), so) <= REL_L2_TOL
            off = synth.layer_offsets(synth.random_layer_sizes(D, 9, seed=tiles))
            plan = twa.LayerPlan(off, D)
            S = twa.project_layers(pm, g, plan)
            torch.cuda.synchronize()
            So = orc.project_layers(po, g.cpu().numpy().astype(np.float64), off.numpy())
            assert rel_l2(S.cpu().numpy(), So) <= REL_L2_TOL
