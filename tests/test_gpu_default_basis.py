"""Parity of the paper's default basis and of the coefficient form of the step (Sec. 4.1, 4.3, 4.5, Alg. 1)
against the fp64 oracle: wbar bit-exact (fp64 sum in checkpoint order, rounded once), E / norms / beta / w
within a relative L2 error of 1e-5."""
import numpy as np
import pytest
import torch

from oracle import twa_oracle as orc
from paper_2205_13104_amd import binding as twa
from paper_2205_13104_amd import synth
from tests.gpu_common import REL_L2_TOL, rel_l2, store_as, to_oracle

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def layer_cases(D):
    yield "one", [D]
    head = [5, 1, 1, 0, 2, 30, 64, 64, 0, 3, 2048, 1000, 4097]
    yield "hand", head + [D - sum(head) - 1, 1]
    yield "random60", synth.random_layer_sizes(D, 60, seed=4)


@pytest.mark.parametrize("D,n", [(70001, 7), (300_017, 20), (1_000_003, 100)])
def test_centre_normalise_matches_oracle(D, n):
    W = synth.trajectory(D, n, 0.95, 0.4, seed=D % 101, device="cuda")
    W[:, 39:103] = 0.25                                  # a layer of the hand-made table that never moves
    W[:, 3000:3100] = 1.0 + 1e-5 * W[:, 3000:3100]       # and a stretch that hardly moves: |w - wbar| << |wbar|
    Wd = W[:, :D].cpu().numpy().astype(np.float64)
    for name, sizes in layer_cases(D):
        off = synth.layer_offsets(sizes)
        say("centre_normalise D", D, "n", n, name, "L", len(sizes))
        plan = twa.LayerPlan(off, D)
        E, wbar, norms = twa.centre_normalise(W, D, plan)
        torch.cuda.synchronize()
        Eo, wbo, nro = orc.centre_normalise_layers(Wd, off.numpy())
        assert np.array_equal(wbar.cpu().numpy(), wbo.astype(np.float32))
        Eg = E[:, :D].cpu().numpy()
        assert rel_l2(Eg, Eo) <= REL_L2_TOL
        assert rel_l2(norms.cpu().numpy(), nro) <= REL_L2_TOL
        offs = off.numpy()
        for l in range(len(sizes)):
            a, b = int(offs[l]), int(offs[l + 1])
            if b > a:
                assert rel_l2(Eg[:, a:b], Eo[:, a:b]) <= REL_L2_TOL, (l, a, b)
                if np.all(nro[l] == 0.0):
                    assert np.all(Eg[:, a:b] == 0.0)
        assert torch.all(E[:, D:] == 0)
        # in place: same bits
        W2 = W.clone()
        E2, wbar2, _ = twa.centre_normalise(W2, D, plan, out=W2, want_norms=False)
        assert E2.data_ptr() == W2.data_ptr()
        assert torch.equal(E2, E) and torch.equal(wbar2, wbar)


@pytest.mark.parametrize("dtype", [twa.F32, twa.I8, twa.I4], ids=["f32", "i8", "i4"])
@pytest.mark.parametrize("lam", [0.0, 0.05])
def test_coefficient_form_of_the_step(dtype, lam):
    D, n, T, lr = 400_009, 24, 4, 0.1
    sizes = synth.random_layer_sizes(D, 30, seed=8)
    off = synth.layer_offsets(sizes)
    L = len(sizes)
    plan = twa.LayerPlan(off, D)
    W = synth.trajectory(D, n, 0.95, 0.4, seed=21, device="cuda")
    E, wbar, _ = twa.centre_normalise(W, D, plan)
    pm = store_as(E, D, dtype)
    po = to_oracle(pm)
    beta = torch.zeros((L, n), device="cuda")
    beta_o = np.zeros((L, n))
    wbar_o = wbar.cpu().numpy().astype(np.float64)
    w_direct = wbar.clone()                              # weight form, lambda = 0 only
    say("coefficient form", dtype, "lambda", lam)
    for t in range(T):
        g = synth.gradient(D, 1e-2, seed=5, step=t, device="cuda")
        S = twa.project_layers(pm, g, plan)
        twa.beta_update(beta, S, lr, lam)
        w = twa.weights_from_beta(pm, beta, plan, wbar)
        torch.cuda.synchronize()
        # the oracle follows its own trajectory from the same gradients
        So = orc.project_layers(po, g.cpu().numpy().astype(np.float64), off.numpy())
        orc.beta_step(beta_o, So, float(np.float32(lr)), float(np.float32(lam)))
        wo = orc.weights_from_beta(po, beta_o, off.numpy(), wbar_o)
        assert rel_l2(beta.cpu().numpy(), beta_o) <= REL_L2_TOL
        assert rel_l2(w.cpu().numpy(), wo) <= REL_L2_TOL
        # what moved, not the mean that dominates w: the displacement itself to the bar
        assert rel_l2((w - wbar).double().cpu().numpy(), wo - wbar_o) <= REL_L2_TOL
        if lam == 0.0:
            twa.expand_update_layers(pm, S, plan, w_direct, lr)
            assert rel_l2(w_direct.cpu().numpy(), wo) <= REL_L2_TOL
    # the fused call takes the same coefficient step
    b1 = beta.clone()
    b2 = beta.clone()
    g = synth.gradient(D, 1e-2, seed=5, step=T, device="cuda")
    S1 = twa.project_layers(pm, g, plan)
    twa.beta_update(b1, S1, lr, lam)
    S2 = torch.empty_like(S1)
    twa.beta_step(pm, g, plan, b2, lr, lam, S=S2)
    assert torch.equal(S1, S2) and torch.equal(b1, b2)
    b3 = beta.clone()
    twa.beta_step(pm, g, plan, b3, lr, lam)
    assert torch.equal(b1, b3)
    # w may be written over wbar's buffer
    wb2 = wbar.clone()
    w2 = twa.weights_from_beta(pm, beta, plan, wb2, w=wb2)
    assert torch.equal(w2, w)


def test_default_basis_argument_errors():
    import ctypes as C
    D, n = 5000, 4
    W = synth.trajectory(D, n, 0.9, 0.5, seed=1, device="cuda")
    plan = twa.LayerPlan([0, 100, D], D)
    wbar = torch.zeros(D, device="cuda")
    L = twa.lib()
    nb = C.c_size_t()
    assert L.twa_centre_normalise_workspace_bytes(D, n, 2, C.byref(nb)) == twa.OK
    ws = twa.Workspace(nb.value)
    ld = W.shape[1]
    args = lambda **k: [k.get("W", W.data_ptr()), D, n, ld, k.get("plan", plan.ptr), 2, wbar.data_ptr(),
                        k.get("E", W.data_ptr()), k.get("lde", ld), None, ws.ptr, k.get("wsb", ws.nbytes), None]
    assert L.twa_centre_normalise(*args(W=None)) == twa.ERR_NULL
    assert L.twa_centre_normalise(*args(plan=None)) == twa.ERR_NULL
    assert L.twa_centre_normalise(*args(wsb=16)) == twa.ERR_WORKSPACE
    assert L.twa_centre_normalise(*args(E=W.data_ptr() + 4 * ld)) == twa.ERR_SHAPE        # partial overlap
    assert L.twa_centre_normalise(*args(lde=ld + 128)) == twa.ERR_SHAPE                  # in place needs lde == ldw
    b = torch.zeros(8, device="cuda")
    assert L.twa_beta_update(None, b.data_ptr(), 8, 0.1, 0.0, None) == twa.ERR_NULL
    assert L.twa_beta_update(b.data_ptr(), b.data_ptr(), 0, 0.1, 0.0, None) == twa.ERR_SHAPE


@pytest.mark.parametrize("kind,lam", [("momentum", 0.0), ("momentum", 0.05), ("adam", 0.0), ("adam", 0.05), ("adamw", 0.05)])
def test_coefficient_step_with_the_base_optimiser(kind, lam):
    """Layer-wise training of the coefficients with momentum / Adam / AdamW (Sec. 5.1) over several steps: the
    library and the oracle each follow their own trajectory from the same gradients."""
    D, n, T, lr = 300_007, 16, 6, 0.02
    off = synth.layer_offsets(synth.random_layer_sizes(D, 20, seed=9))
    plan = twa.LayerPlan(off, D)
    L = plan.L
    W = synth.trajectory(D, n, 0.95, 0.4, seed=23, device="cuda")
    E, wbar, _ = twa.centre_normalise(W, D, plan)
    pm = store_as(E, D, twa.I8)
    po = to_oracle(pm)
    K = {"momentum": twa.OPT_MOMENTUM, "adam": twa.OPT_ADAM, "adamw": twa.OPT_ADAMW}[kind]
    Ko = {"momentum": orc.MOMENTUM, "adam": orc.ADAM, "adamw": orc.ADAMW}[kind]
    mu, b2, eps = 0.9, 0.99, 1e-8
    beta, m, v = (torch.zeros((L, n), device="cuda") for _ in range(3))
    beta_o, m_o, v_o = (np.zeros((L, n)) for _ in range(3))
    wbar_o = wbar.cpu().numpy().astype(np.float64)
    f = lambda x: float(np.float32(x))
    say("base optimiser", kind, "lambda", lam)
    for t in range(1, T + 1):
        g = synth.gradient(D, 1e-2, seed=6, step=t, device="cuda")
        S = twa.project_layers(pm, g, plan)
        twa.beta_optim(K, beta, S, m, None if kind == "momentum" else v, lr, lam, mu, b2, eps, t)
        w = twa.weights_from_beta(pm, beta, plan, wbar)
        torch.cuda.synchronize()
        So = orc.project_layers(po, g.cpu().numpy().astype(np.float64), off.numpy())
        orc.beta_optim(Ko, beta_o, So, m_o, None if kind == "momentum" else v_o, f(lr), f(lam), f(mu), f(b2), f(eps), t)
        wo = orc.weights_from_beta(po, beta_o, off.numpy(), wbar_o)
        assert rel_l2(beta.cpu().numpy(), beta_o) <= REL_L2_TOL, t
        assert rel_l2(m.cpu().numpy(), m_o) <= REL_L2_TOL, t
        if kind != "momentum":
            assert rel_l2(v.cpu().numpy(), v_o) <= REL_L2_TOL, t
        assert rel_l2(w.cpu().numpy(), wo) <= REL_L2_TOL, t
    if kind == "momentum":
        # without momentum it is Alg. 1's own step, bit for bit
        b1, b2_, m0 = beta.clone(), beta.clone(), torch.zeros_like(beta)
        twa.beta_update(b1, S, lr, lam)
        twa.beta_optim(twa.OPT_MOMENTUM, b2_, S, m0, None, lr, lam, 0.0)
        assert rel_l2(b1.cpu().numpy(), b2_.double().cpu().numpy()) <= 1e-7


def test_base_optimiser_argument_errors():
    import ctypes as C
    L = twa.lib()
    b = torch.zeros(8, device="cuda")
    mk = lambda **k: twa.OptimStruct(k.get("kind", 1), 0.1, 0.0, k.get("mu", 0.9), k.get("beta2", 0.99), k.get("eps", 1e-8),
                                     k.get("t", 1))
    p = b.data_ptr()
    assert L.twa_beta_optim(None, p, p, p, p, 8, None) == twa.ERR_NULL
    assert L.twa_beta_optim(C.byref(mk()), p, p, p, None, 8, None) == twa.ERR_NULL          # Adam needs v
    assert L.twa_beta_optim(C.byref(mk(kind=0)), p, p, p, None, 8, None) == twa.OK           # momentum does not
    assert L.twa_beta_optim(C.byref(mk(kind=7)), p, p, p, p, 8, None) == twa.ERR_DTYPE
    assert L.twa_beta_optim(C.byref(mk(t=0)), p, p, p, p, 8, None) == twa.ERR_SHAPE
    assert L.twa_beta_optim(C.byref(mk(mu=1.0)), p, p, p, p, 8, None) == twa.ERR_SHAPE
    assert L.twa_beta_optim(C.byref(mk(beta2=-0.1)), p, p, p, p, 8, None) == twa.ERR_SHAPE
    assert L.twa_beta_optim(C.byref(mk()), p, p, p, p, 0, None) == twa.ERR_SHAPE
    torch.cuda.synchronize()
