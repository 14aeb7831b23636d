"""Pins of the layer-wise part of the fp64 CPU oracle (Sec. 4.5, Alg. 1).  No HIP code is touched.

* one layer reduces to the whole-model functions; the layer rows of S add up to the whole-model s
* the layer-wise operators are the whole-model ones for the block-diagonal D x nL matrix, built
  densely here and multiplied with numpy
* with per-layer orthonormal blocks the layer-wise projected step is idempotent
* coefficient form (beta, w = wbar + P beta) == weight form over T steps for lambda = 0; for
  lambda > 0 the decay shrinks w - wbar; closed form of beta under a constant gradient
* layer-wise centre + normalise against its definition in numpy: unit norms per layer, centred
  vectors of a layer sum to zero, a layer that is equal in all checkpoints gives zero vectors
"""
import numpy as np
import pytest

from oracle import twa_oracle as orc
from paper_2205_13104_amd import synth


def rng(seed):
    return np.random.default_rng(seed)


OFFS = [0, 7, 7, 8, 300, 301, 1000, 1333]          # an empty layer, two of one element, ragged sizes


def block_diagonal(Pd, off):
    """Dense D x (L*n) matrix whose column l*n+j is basis vector j restricted to layer l."""
    n, D = Pd.shape
    L = len(off) - 1
    M = np.zeros((D, L * n))
    for l in range(L):
        M[off[l]:off[l + 1], l * n:(l + 1) * n] = Pd[:, off[l]:off[l + 1]].T
    return M


def stored(kind, P):
    P32 = P.astype(np.float32)
    if kind == "f64":
        return orc.pmat_f64(P)
    if kind == "f32":
        return orc.pmat_f32(P32)
    if kind == "bf16":
        return orc.to_bf16(P32)
    if kind == "i8":
        return orc.quantize_i8(P32)
    return orc.quantize_i4(P32)


@pytest.mark.parametrize("kind", ["f64", "f32", "bf16", "i8", "i4"])
def test_layer_operators_are_the_block_diagonal_ones(kind):
    r = rng(31)
    n, D = 5, OFFS[-1]
    pm = stored(kind, r.normal(size=(n, D)) * 0.1)
    Pd = pm.dense()[:, :D]
    M = block_diagonal(Pd, OFFS)
    g = r.normal(size=D)
    S = orc.project_layers(pm, g, OFFS)
    assert S.shape == (len(OFFS) - 1, n)
    assert np.allclose(S.reshape(-1), M.T @ g, rtol=0, atol=1e-12)
    assert np.all(S[1] == 0.0)                                  # the empty layer
    assert np.allclose(S.sum(axis=0), orc.project(pm, g), rtol=0, atol=1e-12)
    S2 = r.normal(size=S.shape)
    w0 = r.normal(size=D)
    w = w0.copy()
    gt = orc.expand_update_layers(pm, S2, OFFS, w, 0.3, want_gt=True)
    assert np.allclose(gt, M @ S2.reshape(-1), rtol=0, atol=1e-12)
    assert np.allclose(w, w0 - 0.3 * (M @ S2.reshape(-1)), rtol=0, atol=1e-12)


def test_one_layer_is_the_whole_model():
    r = rng(32)
    n, D = 4, 777
    pm = orc.pmat_f64(r.normal(size=(n, D)))
    g = r.normal(size=D)
    s = orc.project(pm, g)
    S = orc.project_layers(pm, g, [0, D])
    assert np.array_equal(S[0], s)
    wa, wb = np.ones(D), np.ones(D)
    ga = orc.expand_update(pm, s, wa, 0.1, want_gt=True)
    gb = orc.expand_update_layers(pm, S, [0, D], wb, 0.1, want_gt=True)
    assert np.array_equal(ga, gb) and np.array_equal(wa, wb)


def test_layerwise_step_is_idempotent_for_orthonormal_layer_blocks():
    r = rng(33)
    n, D = 3, 400
    off = [0, 50, 53, 200, 400]
    P = np.zeros((n, D))
    for l in range(len(off) - 1):
        q, _ = np.linalg.qr(r.normal(size=(off[l + 1] - off[l], n)))
        P[:, off[l]:off[l + 1]] = q.T
    pm = orc.pmat_f64(P)
    g = r.normal(size=D)
    S = orc.project_layers(pm, g, off)
    w = np.zeros(D)
    gt = orc.expand_update_layers(pm, S, off, w, 1.0, want_gt=True)
    assert np.allclose(w, -gt, rtol=0, atol=0)
    S_again = orc.project_layers(pm, gt, off)
    assert np.allclose(S_again, S, rtol=0, atol=1e-13)
    # and each layer's part of g~ is the orthogonal projection of that layer's part of g
    for l in range(len(off) - 1):
        sl = slice(off[l], off[l + 1])
        resid = g[sl] - gt[sl]
        assert np.max(np.abs(P[:, sl] @ resid)) <= 1e-13


def test_beta_step_closed_form():
    r = rng(34)
    s = r.normal(size=(3, 4))
    eta, lam, T = 0.1, 0.5, 12
    beta = np.zeros_like(s)
    for _ in range(T):
        orc.beta_step(beta, s, eta, lam)
    q = 1.0 - eta * lam
    assert np.allclose(beta, -eta * s * (1 - q ** T) / (1 - q), rtol=1e-13, atol=0)
    beta = np.zeros_like(s)
    for _ in range(T):
        orc.beta_step(beta, s, eta, 0.0)
    assert np.allclose(beta, -T * eta * s, rtol=1e-14, atol=0)
    one = np.array([[2.0]])
    orc.beta_step(one, np.array([[3.0]]), 0.5, 0.25)          # (1 - 0.125)*2 - 0.5*3
    assert one[0, 0] == 0.25


@pytest.mark.parametrize("lam", [0.0, 0.05])
def test_coefficient_form_equals_weight_form(lam):
    r = rng(35)
    n, D, T, eta = 4, OFFS[-1], 6, 0.2
    W = synth.trajectory(D, n, 0.9, 0.5, seed=35, ld=D).numpy().astype(np.float64)
    E, wbar, _ = orc.centre_normalise_layers(W, OFFS)
    pm = orc.pmat_f64(E)
    M = block_diagonal(E, OFFS)
    beta = np.zeros((len(OFFS) - 1, n))
    w_beta = wbar.copy()
    w_direct = wbar.copy()
    for t in range(T):
        g = r.normal(size=D)
        S = orc.project_layers(pm, g, OFFS)
        orc.beta_step(beta, S, eta, lam)
        w_beta = orc.weights_from_beta(pm, beta, OFFS, wbar)
        # the decay acts on the coefficients, i.e. on w - wbar (Alg. 1 with the offset of Sec. 4.3)
        w_direct = wbar + (1 - eta * lam) * (w_direct - wbar) - eta * (M @ (M.T @ g))
        if lam == 0.0:
            w_form = w_direct.copy()
        assert np.allclose(w_beta, w_direct, rtol=0, atol=1e-12)
    if lam == 0.0:
        # same trajectory through the oracle's own weight-space form
        r = rng(35)
        w = wbar.copy()
        for t in range(T):
            g = r.normal(size=D)
            orc.expand_update_layers(pm, orc.project_layers(pm, g, OFFS), OFFS, w, eta)
        assert np.allclose(w, w_form, rtol=0, atol=1e-12)


def test_weights_from_beta_definition():
    r = rng(36)
    n, D = 3, OFFS[-1]
    P = r.normal(size=(n, D))
    beta = r.normal(size=(len(OFFS) - 1, n))
    wbar = r.normal(size=D)
    w = orc.weights_from_beta(orc.pmat_f64(P), beta, OFFS, wbar)
    assert np.allclose(w, wbar + block_diagonal(P, OFFS) @ beta.reshape(-1), rtol=0, atol=1e-13)


def test_centre_normalise_layers_matches_definition():
    n, D = 7, OFFS[-1]
    W = synth.trajectory(D, n, 0.9, 0.5, seed=37, ld=D).numpy().astype(np.float64)
    W[:, 300:301] = 0.25                       # a one-element layer that is the same in all checkpoints
    E, wbar, nrm = orc.centre_normalise_layers(W, OFFS)
    assert np.allclose(wbar, W.mean(axis=0), rtol=0, atol=1e-16)
    C = W - W.mean(axis=0)
    for l in range(len(OFFS) - 1):
        sl = slice(OFFS[l], OFFS[l + 1])
        nr = np.linalg.norm(C[:, sl], axis=1)
        assert np.allclose(nrm[l], nr, rtol=1e-14, atol=0)
        if OFFS[l] == 300:
            assert np.all(nrm[l] == 0.0) and np.all(E[:, sl] == 0.0)
            continue
        if sl.stop > sl.start:
            assert np.allclose(np.linalg.norm(E[:, sl], axis=1), 1.0, rtol=0, atol=1e-13)
            assert np.allclose(E[:, sl] * nr[:, None], C[:, sl], rtol=0, atol=1e-15)
            # the centred vectors of a layer sum to zero: rank <= n - 1 in every layer
            assert np.linalg.norm((E[:, sl] * nrm[l][:, None]).sum(axis=0)) <= 1e-12 * nr.max()
    # a one-element layer whose entries differ: every basis vector is +1 or -1 there
    assert set(np.unique(E[:, 7:8])) <= {-1.0, 1.0}


def test_centre_normalise_one_layer_is_the_whole_model_construction():
    W = synth.trajectory(900, 5, 0.9, 0.5, seed=38, ld=900).numpy().astype(np.float64)
    E1, wbar1 = orc.centre_normalise(W)
    E2, wbar2, _ = orc.centre_normalise_layers(W, [0, 900])
    assert np.array_equal(E1, E2) and np.array_equal(wbar1, wbar2)


# ---------------------------------------------------------------- base optimiser on the coefficients (Sec. 5.1)
def test_momentum_without_momentum_is_algorithm_1():
    r = rng(40)
    s = r.normal(size=(3, 5))
    b1, b2, m = r.normal(size=(3, 5)), None, np.zeros((3, 5))
    b2 = b1.copy()
    for _ in range(4):
        orc.beta_step(b1, s, 0.1, 0.3)
        orc.beta_optim(orc.MOMENTUM, b2, s, m, None, 0.1, 0.3, 0.0)
        assert np.allclose(b1, b2, rtol=0, atol=1e-15)


def test_momentum_closed_form_under_a_constant_gradient():
    r = rng(41)
    s = r.normal(size=(2, 4))
    eta, mu, T = 0.05, 0.9, 9
    beta, m = np.zeros_like(s), np.zeros_like(s)
    for _ in range(T):
        orc.beta_optim(orc.MOMENTUM, beta, s, m, None, eta, 0.0, mu)
    # m_k = s (1 - mu^k) / (1 - mu);  beta_T = -eta sum_k m_k
    tot = sum((1 - mu ** k) / (1 - mu) for k in range(1, T + 1))
    assert np.allclose(beta, -eta * tot * s, rtol=1e-13, atol=0)
    assert np.allclose(m, s * (1 - mu ** T) / (1 - mu), rtol=1e-13, atol=0)
    # one hand-computed step with decay: d = 3 + 0.5*2 = 4; m = 0.5*1 + 4 = 4.5; beta = 2 - 0.25*4.5
    one, mm = np.array([[2.0]]), np.array([[1.0]])
    orc.beta_optim(orc.MOMENTUM, one, np.array([[3.0]]), mm, None, 0.25, 0.5, 0.5)
    assert mm[0, 0] == 4.5 and one[0, 0] == 0.875


@pytest.mark.parametrize("kind", ["adam", "adamw"])
def test_adam_closed_forms(kind):
    r = rng(42)
    s = r.normal(size=(2, 5))
    eta, b1, b2, eps, T = 0.01, 0.9, 0.999, 1e-8, 7
    K = orc.ADAM if kind == "adam" else orc.ADAMW
    # constant gradient, no decay: the bias corrections make m^ = s and v^ = s^2 at every step,
    # so every step moves by eta * s / (|s| + eps)
    beta, m, v = np.zeros_like(s), np.zeros_like(s), np.zeros_like(s)
    for t in range(1, T + 1):
        orc.beta_optim(K, beta, s, m, v, eta, 0.0, b1, b2, eps, t)
        assert np.allclose(beta, -t * eta * s / (np.abs(s) + eps), rtol=1e-12, atol=0)
    # b1 = b2 = 0: no memory, a normalised step on the current gradient alone
    beta, m, v = np.ones_like(s), np.zeros_like(s), np.zeros_like(s)
    s2 = r.normal(size=s.shape)
    orc.beta_optim(K, beta, s, m, v, eta, 0.0, 0.0, 0.0, eps, 1)
    orc.beta_optim(K, beta, s2, m, v, eta, 0.0, 0.0, 0.0, eps, 2)
    assert np.allclose(beta, 1 - eta * s / (np.abs(s) + eps) - eta * s2 / (np.abs(s2) + eps), rtol=1e-13, atol=0)
    # where the two differ: the decay.  AdamW shrinks beta by (1 - eta*lam) and leaves the gradient alone:
    # constant gradient => beta_t = q beta_{t-1} - c, a geometric series.  Adam adds lam*beta to the gradient.
    lam = 0.5
    beta, m, v = np.full_like(s, 2.0), np.zeros_like(s), np.zeros_like(s)
    for t in range(1, T + 1):
        orc.beta_optim(K, beta, s, m, v, eta, lam, b1, b2, eps, t)
    if kind == "adamw":
        q, c = 1 - eta * lam, eta * s / (np.abs(s) + eps)
        assert np.allclose(beta, q ** T * 2.0 - c * (1 - q ** T) / (1 - q), rtol=1e-12, atol=0)
    else:
        # first step by hand: d = s + lam*2, step = eta * d / (|d| + eps)
        beta1, m1, v1 = np.full_like(s, 2.0), np.zeros_like(s), np.zeros_like(s)
        orc.beta_optim(K, beta1, s, m1, v1, eta, lam, b1, b2, eps, 1)
        d = s + lam * 2.0
        assert np.allclose(beta1, 2.0 - eta * d / (np.abs(d) + eps), rtol=1e-13, atol=0)
        assert np.allclose(m1, (1 - b1) * d, rtol=1e-13, atol=0) and np.allclose(v1, (1 - b2) * d * d, rtol=1e-13, atol=0)


def test_adam_is_invariant_to_the_scale_of_the_gradient():
    """Adam's step depends on the gradient's direction per coordinate, not its scale (eps = 0):
    a property a wrong power or a missing square root would break."""
    r = rng(43)
    G = r.normal(size=(6, 3, 4))
    out = []
    for scale in (1.0, 1000.0):
        beta, m, v = np.zeros((3, 4)), np.zeros((3, 4)), np.zeros((3, 4))
        for t in range(1, 7):
            orc.beta_optim(orc.ADAM, beta, scale * G[t - 1], m, v, 0.01, 0.0, 0.9, 0.99, 0.0, t)
        out.append(beta)
    assert np.allclose(out[0], out[1], rtol=1e-12, atol=0)
