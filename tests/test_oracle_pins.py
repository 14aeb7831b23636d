"""Pins of the fp64 CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP library.  Each pin is chosen so that a plausible
mistake in ``oracle/twa_oracle.c`` (a dropped term, a wrong sign or index, a transposed
operand, a wrong tie rule) fails at least one of them:

* closed form for n = 1 (basis, projection, expansion)                       -- Sec. 4.1/4.2
* P^T P = I to 1e-12, R = P^T W upper triangular with positive diagonal, W = P R
* span(P) = span(W) by brute-force least squares with a hand-written Gaussian elimination
* idempotence and the projector identities of P P^T                          -- Sec. 4.2
* block identity P P^T g = sum_i P_i P_i^T g for column partitions           -- Sec. 4.4
* coefficient form == weight form of the update over T steps (lambda = 0)    -- Sec. 4.3, Alg. 1
* library cross-checks (numpy matmul / LAPACK QR / numpy binary16 / torch bfloat16)
* quantiser: hand-computed codes that separate half-even from half-away and truncation,
  error bound, idempotence on its own output, storage sizes of the memory table of Sec. 4.6
* the paper's own min-max quantiser (Sec. 4.6): code range, error bound a/2, end points
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import twa_oracle as orc
from paper_2205_13104_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def traj(D, n, decay=0.9, drift=0.5, seed=0):
    W = synth.trajectory(D, n, decay, drift, seed=seed, ld=D).numpy()
    return W.astype(np.float64)


# --------------------------------------------------------------------------- n = 1 closed form
def test_n1_closed_form():
    r = rng(1)
    D = 1000
    w = r.normal(size=D)
    g = r.normal(size=D)
    P, R = orc.build_basis(w[None, :])
    nw = math.sqrt(float(np.dot(w, w)))
    assert np.allclose(P[0], w / nw, rtol=0, atol=1e-14)
    assert abs(R[0, 0] - nw) <= 1e-12 * nw
    s = orc.project(orc.pmat_f64(P), g)
    assert abs(s[0] - np.dot(w, g) / nw) <= 1e-12
    w0 = r.normal(size=D)
    wv = w0.copy()
    gt = orc.expand_update(orc.pmat_f64(P), s, wv, 0.25, want_gt=True)
    expect = w * (np.dot(w, g) / nw ** 2)
    assert np.allclose(gt, expect, rtol=0, atol=1e-12)
    assert np.allclose(wv, w0 - 0.25 * expect, rtol=0, atol=1e-12)


def test_n1_negative_leading_entry_keeps_positive_R():
    # Householder picks alpha with the sign opposite to x_0: both signs must end with R_00 > 0.
    for sign in (+1.0, -1.0):
        w = np.array([sign * 3.0, 4.0, 0.0, 0.0])
        P, R = orc.build_basis(w[None, :])
        assert R[0, 0] == pytest.approx(5.0, abs=1e-14)
        assert np.allclose(P[0], w / 5.0, atol=1e-15)


# --------------------------------------------------------------------------- orthonormality, QR structure
@pytest.mark.parametrize("D,n,decay,drift", [(20000, 10, 0.9, 0.5), (6000, 100, 0.97, 0.3), (257, 7, 0.9, 0.5)])
def test_build_basis_invariants(D, n, decay, drift):
    W = traj(D, n, decay, drift, seed=3)
    P, R = orc.build_basis(W)
    G = P @ P.T
    assert np.max(np.abs(G - np.eye(n))) <= 1e-12
    # R = P^T W is upper triangular with positive diagonal (column picture: R[a, b] = p_a . w_b)
    Rchk = P @ W.T
    assert np.max(np.abs(np.tril(Rchk, -1))) <= 1e-10 * np.max(np.abs(Rchk))
    assert np.all(np.diag(R) > 0)
    assert np.max(np.abs(np.tril(R, -1))) == 0.0
    assert np.allclose(R, np.triu(Rchk), rtol=0, atol=1e-10 * np.max(np.abs(Rchk)))
    # W = P R
    assert np.linalg.norm(W - R.T @ P) <= 1e-13 * np.linalg.norm(W)
    # first basis vector is the first checkpoint, normalised (checkpoint order is kept)
    assert np.allclose(P[0], W[0] / np.linalg.norm(W[0]), rtol=0, atol=1e-12)


def test_build_basis_matches_lapack_qr():
    r = rng(5)
    n, D = 12, 500
    W = r.normal(size=(n, D))
    P, R = orc.build_basis(W)
    Q, Rl = np.linalg.qr(W.T)            # independent Householder implementation
    sg = np.sign(np.diag(Rl))
    Q = Q * sg[None, :]
    Rl = Rl * sg[:, None]
    assert np.allclose(P, Q.T, rtol=0, atol=1e-12)
    assert np.allclose(R, Rl, rtol=0, atol=1e-11)


def _solve_gauss(A, b):
    """Plain Gaussian elimination with partial pivoting on python floats."""
    m = len(A)
    M = [list(map(float, A[i])) + [float(b[i])] for i in range(m)]
    for c in range(m):
        piv = max(range(c, m), key=lambda r_: abs(M[r_][c]))
        M[c], M[piv] = M[piv], M[c]
        for r_ in range(c + 1, m):
            f = M[r_][c] / M[c][c]
            for k in range(c, m + 1):
                M[r_][k] -= f * M[c][k]
    x = [0.0] * m
    for c in range(m - 1, -1, -1):
        x[c] = (M[c][m] - sum(M[c][k] * x[k] for k in range(c + 1, m))) / M[c][c]
    return x


def _ls_residual(basis, v):
    """|| v - proj_{span(basis)} v || by normal equations solved with _solve_gauss."""
    m = len(basis)
    A = [[sum(a * b for a, b in zip(basis[i], basis[j])) for j in range(m)] for i in range(m)]
    rhs = [sum(a * b for a, b in zip(basis[i], v)) for i in range(m)]
    x = _solve_gauss(A, rhs)
    res = [v[t] - sum(x[i] * basis[i][t] for i in range(m)) for t in range(len(v))]
    return math.sqrt(sum(e * e for e in res))


@pytest.mark.parametrize("D,n", [(8, 1), (16, 3), (64, 5), (5, 5)])
def test_span_equality_brute_force(D, n):
    r = rng(10 + D + n)
    W = r.normal(size=(n, D))
    P, _ = orc.build_basis(W)
    Wl, Pl = W.tolist(), P.tolist()
    for j in range(n):
        assert _ls_residual(Pl, Wl[j]) <= 1e-10 * np.linalg.norm(W[j])
        assert _ls_residual(Wl, Pl[j]) <= 1e-10
    # and a vector outside the span is NOT reproduced (guards against a trivially passing residual)
    if n < D:
        v = r.normal(size=D).tolist()
        assert _ls_residual(Pl, v) > 1e-3


def test_rank_deficient_is_an_error():
    r = rng(2)
    W = r.normal(size=(4, 50))
    W[2] = 0.5 * W[0] - 2.0 * W[1]
    with pytest.raises(orc.OracleError) as ei:
        orc.build_basis(W)
    assert ei.value.code == orc.ERR_RANK and ei.value.column == 2


# --------------------------------------------------------------------------- projector identities
def test_projector_identities():
    D, n = 4000, 10
    W = traj(D, n, seed=4)
    P, _ = orc.build_basis(W)
    pm = orc.pmat_f64(P)
    r = rng(6)
    g = r.normal(size=D)
    s = orc.project(pm, g)
    z = np.zeros(D)
    gt = orc.expand_update(pm, s, z, 1.0, want_gt=True)
    assert np.allclose(z, -gt, rtol=0, atol=0)               # w = 0 - 1*g~
    # ||g~|| = ||s|| <= ||g||
    assert abs(np.linalg.norm(gt) - np.linalg.norm(s)) <= 1e-12 * np.linalg.norm(s)
    assert np.linalg.norm(s) <= np.linalg.norm(g)
    # P^T (g - P P^T g) = 0
    assert np.max(np.abs(orc.project(pm, g - gt))) <= 1e-12 * np.linalg.norm(g)
    # idempotence: projecting g~ again returns g~
    s2 = orc.project(pm, gt)
    gt2 = orc.expand_update(pm, s2, np.zeros(D), 1.0, want_gt=True)
    assert np.allclose(gt2, gt, rtol=0, atol=1e-12 * np.linalg.norm(gt))
    # a vector of span(W) is reproduced
    v = W[3]
    sv = orc.project(pm, v)
    vv = orc.expand_update(pm, sv, np.zeros(D), 1.0, want_gt=True)
    assert np.linalg.norm(vv - v) <= 1e-12 * np.linalg.norm(v)


def test_project_expand_match_numpy():
    r = rng(7)
    n, D, k = 13, 3001, 3
    A = r.normal(size=(n, D))
    G = r.normal(size=(k, D))
    pm = orc.pmat_f64(A)
    S = orc.project(pm, G)
    assert S.shape == (k, n)
    assert np.allclose(S, G @ A.T, rtol=1e-13, atol=1e-11)
    s = r.normal(size=n)
    w0 = r.normal(size=D)
    w = w0.copy()
    gt = orc.expand_update(pm, s, w, 0.3, want_gt=True)
    assert np.allclose(gt, s @ A, rtol=1e-13, atol=1e-12)
    assert np.allclose(w, w0 - 0.3 * (s @ A), rtol=1e-13, atol=1e-12)


def test_project_is_not_transposed_or_offset():
    # element (i, j) = 10*j + i on a 3 x 2 matrix: any index mix-up changes the numbers below
    A = np.array([[0.0, 1.0, 2.0], [10.0, 11.0, 12.0]])     # rows = basis vectors
    g = np.array([1.0, 10.0, 100.0])
    assert orc.project(orc.pmat_f64(A), g).tolist() == [210.0, 1320.0]
    w = np.zeros(3)
    gt = orc.expand_update(orc.pmat_f64(A), np.array([1.0, 2.0]), w, 1.0, want_gt=True)
    assert gt.tolist() == [20.0, 23.0, 26.0] and w.tolist() == [-20.0, -23.0, -26.0]


def test_padding_is_ignored():
    r = rng(8)
    n, D, ld = 3, 37, 64
    A = np.zeros((n, ld))
    A[:, :D] = r.normal(size=(n, D))
    A[:, D:] = 1e9                                           # poison
    g = r.normal(size=D)
    pm = orc.Pmat(orc.F64, D, A)
    assert np.allclose(orc.project(pm, g), A[:, :D] @ g, rtol=1e-13)


def test_block_identity_column_partition():
    # Sec. 4.4: P P^T g equals the sum over column blocks of P_i P_i^T g
    D, n = 3000, 12
    P, _ = orc.build_basis(traj(D, n, seed=9))
    g = rng(9).normal(size=D)
    full = orc.expand_update(orc.pmat_f64(P), orc.project(orc.pmat_f64(P), g), np.zeros(D), 1.0, want_gt=True)
    for k in (2, 4):
        acc = np.zeros(D)
        for part in np.array_split(np.arange(n), k):
            Pi = orc.pmat_f64(P[part])
            acc += orc.expand_update(Pi, orc.project(Pi, g), np.zeros(D), 1.0, want_gt=True)
        assert np.allclose(acc, full, rtol=0, atol=1e-12 * np.linalg.norm(full))


def test_beta_form_equals_weight_form():
    # Sec. 4.3 / Alg. 1 with lambda = 0: w^(t) = wbar + P beta^(t), beta^(0) = 0, and
    # beta <- beta - eta P^T g  must trace the same iterates as  w <- w - eta P P^T g.
    D, n, T, eta = 2000, 8, 25, 0.1
    W = traj(D, n, seed=11)
    P, _ = orc.build_basis(W)
    pm = orc.pmat_f64(P)
    wbar = W.mean(axis=0)
    w = wbar.copy()
    beta = np.zeros(n)
    r = rng(11)
    for _ in range(T):
        g = r.normal(size=D) * 1e-2
        s = orc.project(pm, g)
        orc.expand_update(pm, s, w, eta)
        beta = beta - eta * s
    w_beta = wbar + beta @ P
    assert np.linalg.norm(w - w_beta) <= 1e-10 * np.linalg.norm(w)
    # the iterate never leaves wbar + span(W): residual of (w - wbar) on P vanishes
    d = w - wbar
    assert np.linalg.norm(d - (P @ d) @ P) <= 1e-10 * max(np.linalg.norm(d), 1e-30)


# --------------------------------------------------------------------------- number formats
def test_binary16_conversion_matches_numpy():
    allh = np.arange(65536, dtype=np.uint16)
    vals = allh.view(np.float16).astype(np.float32)
    for h in range(0, 65536, 7):
        v = orc.f16_bits_to_f32(h)
        if math.isnan(vals[h]):
            assert math.isnan(v)
        else:
            assert v == float(vals[h])
            assert orc.f32_to_f16_bits(float(vals[h])) == h or vals[h] == 0
    r = rng(12)
    x = np.concatenate([r.normal(size=4000).astype(np.float32) * s for s in (1e-8, 1e-5, 1e-3, 1.0, 1e3, 1e5)])
    # exact ties and near-ties around binary16 quanta, incl. the subnormal range
    ties = (np.arange(1, 4000, dtype=np.float64) + 0.5) * 2.0 ** -24
    x = np.concatenate([x, ties.astype(np.float32), (ties * 1024).astype(np.float32)])
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    got = np.array([orc.f32_to_f16_bits(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(ref, got)


def test_bfloat16_conversion_matches_torch():
    r = rng(13)
    x = (r.normal(size=5000) * 10.0 ** r.integers(-6, 6, size=5000)).astype(np.float32)
    x[:6] = np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e38], dtype=np.float32)  # incl. ties
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    pm = orc.to_bf16(x[None, :])
    assert np.array_equal(pm.data[0], ref)
    assert np.array_equal(pm.dense()[0], torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy())


# --------------------------------------------------------------------------- block-absmax quantiser
def test_quantize_i8_hand_cases():
    # amax = 127 -> scale = 1, inv = 1, so the code is just the rounded value: ties go to even.
    vals = [0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 127.0, 3.49, 3.51, -127.0, 0.0]
    want = [0, 2, 2, 0, -2, -2, 126, 127, 3, 4, -127, 0]
    p = np.zeros((1, 128), dtype=np.float32)
    p[0, :len(vals)] = vals
    q = orc.quantize_i8(p)
    assert q.scales[0, 0] == 1.0
    assert q.data[0, :len(vals)].tolist() == want
    assert not q.data[0, len(vals):].any()


def test_quantize_i4_hand_cases_and_packing():
    vals = [0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 6.5, 7.0, -7.0, 3.0]
    want = [0, 2, 2, 0, -2, -2, 6, 7, -7, 3]
    p = np.zeros((1, 64), dtype=np.float32)
    p[0, :len(vals)] = vals
    q = orc.quantize_i4(p, gscale=1.0)
    assert orc.f16_bits_to_f32(int(q.scales[0, 0])) == 1.0
    by = q.data[0]
    lo = (by & 0xF).astype(int) - 8
    hi = (by >> 4).astype(int) - 8
    codes = np.stack([lo, hi], axis=1).reshape(-1)
    assert codes[:len(vals)].tolist() == want
    # explicit bytes: element 0 (q=0 -> 8) in the low nibble, element 1 (q=2 -> 10) in the high nibble
    assert by[0] == (8 | (10 << 4)) and by[1] == (10 | (8 << 4))
    assert np.all(by[5:] == 0x88)                            # zero is stored as nibble 8
    assert np.array_equal(q.dense()[0, :len(vals)], np.array(want, dtype=np.float64))


def test_quantize_blocks_run_along_D_inside_one_vector():
    # two vectors, two blocks each, different magnitudes: scales must be per (vector, block)
    p = np.zeros((2, 256), dtype=np.float32)
    p[0, :128] = 127.0
    p[0, 128:] = 254.0
    p[1, :128] = 12.7
    p[1, 128:200] = 1.27
    q = orc.quantize_i8(p, D=200)
    assert q.scales.shape == (2, 2)
    assert q.scales[0].tolist() == [1.0, 2.0]
    assert q.scales[1, 0] == np.float32(np.float32(12.7) / np.float32(127.0))
    assert np.all(q.data[0, :200] == 127) and np.all(q.data[1, :200] == 127)
    assert not q.data[:, 200:].any()                         # padding: code 0


def test_quantize_zero_block_and_ragged_tail():
    r = rng(14)
    D = 128 * 3 + 40
    p = r.normal(size=(3, D)).astype(np.float32)
    p[1, 128:256] = 0.0
    q = orc.quantize_i8(p)
    assert q.ld == 128 * 4 and q.scales.shape == (3, 4)
    assert q.scales[1, 1] == 0.0 and not q.data[1, 128:256].any()
    # the tail block's absmax only sees the 40 real elements
    assert q.scales[2, 3] == np.float32(np.abs(p[2, 384:]).max() / np.float32(127.0))
    assert not q.data[:, D:].any()
    # elements at +-amax map to +-qmax
    for j in range(3):
        for b in range(4):
            blk = p[j, b * 128:min((b + 1) * 128, D)]
            if blk.size and np.abs(blk).max() > 0:
                i = int(np.argmax(np.abs(blk)))
                assert abs(int(q.data[j, b * 128 + i])) == 127


def _numpy_f32_recipe_i8(p, block=128):
    """The recipe in numpy float32 operations (an independent evaluation of every binary32 step)."""
    n, D = p.shape
    nblk = (D + block - 1) // block
    pp = np.zeros((n, nblk * block), dtype=np.float32)
    pp[:, :D] = p
    b3 = pp.reshape(n, nblk, block)
    amax = np.abs(b3).max(axis=2)
    scale = (amax / np.float32(127.0)).astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(scale != 0, np.float32(1.0) / scale, np.float32(0)).astype(np.float32)
    t = (b3 * inv[:, :, None]).astype(np.float32)
    q = np.clip(np.rint(t), -127, 127).astype(np.int8)
    return q.reshape(n, -1), scale


@pytest.mark.parametrize("scale_mag", [1.0, 6.3e-5, 2.0e-4, 37.0])
def test_quantize_i8_equals_float32_evaluation(scale_mag):
    r = rng(15)
    p = (r.normal(size=(4, 128 * 37 + 5)) * scale_mag).astype(np.float32)
    q = orc.quantize_i8(p)
    qn, sn = _numpy_f32_recipe_i8(p)
    assert np.array_equal(q.scales, sn)
    assert np.array_equal(q.data, qn)


def test_quantize_properties_i8_i4():
    r = rng(16)
    D = 128 * 20 + 17
    p = (r.normal(size=(5, D)) / math.sqrt(D)).astype(np.float32)
    for kind in ("i8", "i4"):
        if kind == "i8":
            q = orc.quantize_i8(p)
            qmax, blk = 127, 128
            eff = q.scales.astype(np.float64)
            assert q.data.nbytes == 5 * q.ld                    # n*B*D/8 bytes of codes (Sec. 4.6 memory table), B = 8
        else:
            q = orc.quantize_i4(p)
            qmax, blk = 7, 64
            eff = q.scales.view(np.float16).astype(np.float64) * q.gscale
            assert q.data.nbytes == 5 * q.ld // 2               # B = 4: half a byte per element
            # every stored binary16 scale is a normal number and the largest sits in [2^14, 2^15)
            hs = q.scales.view(np.float16).astype(np.float64)
            assert hs.max() >= 2.0 ** 14 and hs.max() < 2.0 ** 15
            assert hs[hs > 0].min() >= 2.0 ** -14
            assert math.log2(q.gscale) == int(math.log2(q.gscale))
        dq = q.dense()
        e = np.repeat(eff, blk, axis=1)[:, :D]
        assert np.all(np.abs(dq - p.astype(np.float64)) <= 0.5 * e * (1 + 2.0 ** -10) + 1e-300)
        # quantising the dequantised values returns the same codes and scales (fixed point)
        if kind == "i8":
            q2 = orc.quantize_i8(dq.astype(np.float32))
            assert np.array_equal(q2.data, q.data) and np.array_equal(q2.scales, q.scales)
        codes = np.rint(dq / np.where(e > 0, e, 1.0))
        assert codes.min() >= -qmax and codes.max() <= qmax


def test_gscale_formula():
    p = np.zeros((2, 64), dtype=np.float32)
    assert orc.gscale_i4(p) == 1.0
    p[1, 5] = -7.0                       # max scale32 = 1 -> floor(log2) = 0 -> 2^-14
    assert orc.gscale_i4(p) == 2.0 ** -14
    p[0, 3] = 7.0 * 1.999                # still exponent 0
    assert orc.gscale_i4(p) == 2.0 ** -14
    p[0, 3] = 7.0 * 2.0
    assert orc.gscale_i4(p) == 2.0 ** -13
    p[:] = 0
    p[0, 0] = 7.0 * 2.0 ** -20
    assert orc.gscale_i4(p) == 2.0 ** -34


def test_quantized_projection_uses_dequantised_values():
    r = rng(17)
    D = 128 * 5 + 3
    p = (r.normal(size=(4, D)) / math.sqrt(D)).astype(np.float32)
    g = r.normal(size=D)
    for q in (orc.quantize_i8(p), orc.quantize_i4(p), orc.to_bf16(p)):
        dq = q.dense()
        assert np.allclose(orc.project(q, g), dq @ g, rtol=1e-13, atol=1e-15)
        s = r.normal(size=4)
        w = np.zeros(D)
        gt = orc.expand_update(q, s, w, 1.0, want_gt=True)
        assert np.allclose(gt, s @ dq, rtol=1e-13, atol=1e-15)


# --------------------------------------------------------------------------- memory table of Sec. 4.6
def test_memory_formulas_of_the_paper():
    rows = {}
    with open(os.path.join(GOLD, "memory_projection.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                rows[k.strip()] = float(v)
    n, D = int(rows["n"]), int(rows["D"])
    # 4nD bytes at 32 bits and nBD/8 at B bits (Sec. 4.6, table of memory required for P); the paper measures +6000 MB and +750 MB
    # of device memory for fp32 and 4-bit P at this shape (Sec. 5.3.2, DDP table, one GPU).
    fp32_bytes = orc.pmat_f32(np.zeros((1, 128), dtype=np.float32)).data.itemsize * n * D
    assert fp32_bytes == 4 * n * D
    assert abs(fp32_bytes / 2 ** 20 - rows["fp32_extra_MB"]) / rows["fp32_extra_MB"] < 0.03
    assert abs((n * 4 * D / 8) / 2 ** 20 - rows["int4_extra_MB"]) / rows["int4_extra_MB"] < 0.03
    assert 32 / 4 == rows["compression_at_4_bits"]


# --------------------------------------------------------------------------- the paper's min-max quantiser
@pytest.mark.parametrize("B", [1, 2, 4, 8])
def test_minmax_quantiser_properties(B):
    r = rng(18)
    n, D = 6, 500
    P = r.normal(size=(n, D))
    off = [0, 100, 101, 350, 500]
    codes, a, b = orc.quantize_minmax(P, B, off)
    assert codes.min() >= 0 and codes.max() <= 2 ** B - 1
    for l in range(4):
        seg = P[:, off[l]:off[l + 1]]
        c = codes[:, off[l]:off[l + 1]]
        assert b[l] == seg.min() and a[l] == (seg.max() - seg.min()) / (2 ** B - 1)
        rec = a[l] * c + b[l]
        assert np.max(np.abs(rec - seg)) <= 0.5 * a[l] * (1 + 1e-12)
        assert c[np.unravel_index(np.argmin(seg), seg.shape)] == 0
        assert c[np.unravel_index(np.argmax(seg), seg.shape)] == 2 ** B - 1


def test_minmax_stored_matrix_and_fused_dequantisation():
    # value = a*code + b; hence (P~^l)^T g^l = a (Q^l)^T g^l + b sum(g^l) and P~^l beta = a Q^l beta + b sum(beta)
    r = rng(41)
    n, D, B = 5, 700, 4
    off = np.array([0, 100, 100, 333, 700], dtype=np.int64)
    P = r.normal(size=(n, D)) * 0.01
    codes, a, b = orc.quantize_minmax(P, B, off)
    assert a[1] == 0.0 and b[1] == 0.0                               # the empty layer
    pm = orc.pmat_minmax(codes, a, b, off)
    a32, b32 = a.astype(np.float32).astype(np.float64), b.astype(np.float32).astype(np.float64)
    dense = pm.dense()
    g = r.normal(size=D)
    S = orc.project_layers(pm, g, off)
    beta = r.normal(size=(4, n))
    w = orc.weights_from_beta(pm, beta, off, np.zeros(D))
    for l in range(4):
        sl = slice(off[l], off[l + 1])
        Q = codes[:, sl].astype(np.float64)
        assert np.array_equal(dense[:, sl], a32[l] * Q + b32[l])
        assert np.allclose(S[l], a32[l] * (Q @ g[sl]) + b32[l] * g[sl].sum(), rtol=0, atol=1e-12)
        assert np.allclose(w[sl], a32[l] * (beta[l] @ Q) + b32[l] * beta[l].sum(), rtol=0, atol=1e-12)
    # the stored matrix is within half a step of the original, layer by layer (a in binary32: one more ulp)
    for l in (0, 2, 3):
        sl = slice(off[l], off[l + 1])
        assert np.max(np.abs(dense[:, sl] - P[:, sl])) <= 0.5 * a[l] * (1 + 1e-5)


# --------------------------------------------------------------------------- default construction (Sec. 4.1)
def test_centre_normalise_matches_definition():
    W = traj(3000, 9, seed=19)
    E, wbar = orc.centre_normalise(W)
    assert np.allclose(wbar, W.mean(axis=0), rtol=0, atol=1e-15)
    assert np.allclose(np.linalg.norm(E, axis=1), 1.0, rtol=0, atol=1e-13)
    nr = np.linalg.norm(W - wbar, axis=1)
    assert np.allclose(E * nr[:, None], W - wbar, rtol=0, atol=1e-14)
    # the centred vectors sum to zero: this basis has rank n-1
    assert np.linalg.norm((E * nr[:, None]).sum(axis=0)) <= 1e-12 * nr.max()


# --------------------------------------------------------------------------- pins added against surviving mutations
def test_householder_is_stable_for_a_column_along_a_unit_vector():
    # x nearly equal to +|x| e_0: the reflector must be built without cancellation.
    r = rng(20)
    D = 50
    w = 1e-9 * r.normal(size=D)
    w[0] = 1.0
    W = np.stack([w, r.normal(size=D)])
    P, R = orc.build_basis(W)
    assert np.allclose(P[0], w / np.linalg.norm(w), rtol=0, atol=1e-15)
    assert np.max(np.abs(P @ P.T - np.eye(2))) <= 1e-14


def test_quantize_rounds_the_product_to_binary32_before_the_integer_rounding():
    # Search for inputs whose exact product p*inv is NOT a tie while its binary32 rounding IS one;
    # the recipe rounds the binary32 product, so the code is the even neighbour.
    from fractions import Fraction
    amax = np.float32(100.0)
    scale = np.float32(amax / np.float32(127.0))
    inv = np.float32(np.float32(1.0) / scale)
    found = []
    for k in range(1, 126):
        tie = k + 0.5
        p0 = np.float32(tie * float(scale))
        for step in range(-4, 5):
            p = p0
            for _ in range(abs(step)):
                p = np.nextafter(p, np.float32(np.inf if step > 0 else -np.inf), dtype=np.float32)
            exact = Fraction(float(p)) * Fraction(float(inv))
            t32 = np.float32(p * inv)
            if float(t32) == tie and exact != Fraction(tie):
                even = k if k % 2 == 0 else k + 1
                wrong = k + 1 if exact > Fraction(tie) else k      # what rounding the exact product gives
                if wrong != even:
                    found.append((float(p), even))
    assert len(found) >= 3
    vec = np.zeros((1, 128), dtype=np.float32)
    vec[0, 0] = amax
    for i, (p, _) in enumerate(found[:100]):
        vec[0, 1 + i] = p
    q = orc.quantize_i8(vec)
    assert q.scales[0, 0] == scale
    assert q.data[0, 1:1 + min(len(found), 100)].tolist() == [e for _, e in found[:100]]


# --------------------------------------------------------------------------- int4: codes against the EFFECTIVE scale
def _numpy_recipe_i4(p, gscale, block=64):
    """The 4-bit recipe in numpy float32 / float16 operations, an independent evaluation of every step:
    amax / 7 -> / gscale -> binary16 (nearest even) -> * gscale -> 1 / e -> rint(p * inv)."""
    n, D = p.shape
    nblk = (D + block - 1) // block
    pp = np.zeros((n, nblk * block), dtype=np.float32)
    pp[:, :D] = p
    b3 = pp.reshape(n, nblk, block)
    amax = np.abs(b3).max(axis=2)
    scale = (amax / np.float32(7.0)).astype(np.float32)
    h = (scale / np.float32(gscale)).astype(np.float32).astype(np.float16)
    eff = (h.astype(np.float32) * np.float32(gscale)).astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(eff != 0, np.float32(1.0) / eff, np.float32(0)).astype(np.float32)
    t = (b3 * inv[:, :, None]).astype(np.float32)
    q = np.clip(np.rint(t), -7, 7).astype(np.int64).reshape(n, -1)
    packed = ((q[:, 0::2] + 8) | ((q[:, 1::2] + 8) << 4)).astype(np.uint8)
    return packed, h.view(np.uint16), scale, eff


@pytest.mark.parametrize("scale_mag", [1.0, 5.3e-5, 2.0e-4, 37.0, 3.1e-9])
def test_quantize_i4_equals_float32_float16_evaluation(scale_mag):
    r = rng(31)
    p = (r.normal(size=(4, 64 * 41 + 9)) * scale_mag).astype(np.float32)
    q = orc.quantize_i4(p)                                   # gscale chosen by the library's rule
    assert q.gscale != 1.0
    packed, hbits, scale, eff = _numpy_recipe_i4(p, q.gscale)
    assert np.array_equal(q.scales, hbits)
    assert np.array_equal(q.data, packed)
    # the pin bites only if rounding the scale to binary16 matters: most blocks' effective scale differs
    # from the binary32 scale, and forming the codes against the unrounded one changes some of them
    assert np.mean(eff != scale) > 0.9
    with np.errstate(divide="ignore"):
        inv_unrounded = np.where(scale != 0, np.float32(1.0) / scale, np.float32(0)).astype(np.float32)
    pp = np.zeros((4, eff.shape[1] * 64), dtype=np.float32)
    pp[:, :p.shape[1]] = p
    other = np.clip(np.rint((pp.reshape(4, -1, 64) * inv_unrounded[:, :, None]).astype(np.float32)), -7, 7)
    mine = np.stack([(q.data & 0xF).astype(np.int64) - 8, (q.data >> 4).astype(np.int64) - 8], axis=2).reshape(4, -1)
    assert np.count_nonzero(other.reshape(4, -1) != mine) > 0


def test_quantize_i4_codes_are_formed_against_the_binary16_rounded_scale():
    # One block by hand.  amax = 7.005: scale = 1.000714.., which binary16 (quantum 2^-10 above 1) rounds UP to
    # e = 1 + 2^-10 = 1.0009765625.  Elements strictly between 2.5*scale and 2.5*e (4.5*scale and 4.5*e, ...)
    # lie below the tie of the effective scale and above the tie of the unrounded one.
    from fractions import Fraction
    amax = np.float32(7.005)
    scale = Fraction(float(amax)) / 7
    eff = Fraction(1) + Fraction(1, 1024)
    assert scale > 1 + Fraction(1, 2048)                     # above the binary16 tie: rounds up to 1 + 2^-10
    vals = [2.5021, 4.5038, -2.5021, 6.5052, 0.5004, 1.5011]
    want = []
    for v in vals:
        x = Fraction(float(np.float32(v))) / eff             # the quotient against the effective scale, exactly
        y = Fraction(float(np.float32(v))) / scale           # ... against the unrounded scale
        k = math.floor(abs(x))
        assert abs(abs(x) - (k + Fraction(1, 2))) > Fraction(1, 100000)   # 20x the binary32 rounding of p*inv away from a tie
        assert abs(x) < k + Fraction(1, 2) < abs(y)          # the two scales disagree about this element
        want.append(int(math.copysign(k, v)))
    p = np.zeros((1, 64), dtype=np.float32)
    p[0, 0] = amax
    p[0, 1:1 + len(vals)] = vals
    q = orc.quantize_i4(p, gscale=1.0)
    assert orc.f16_bits_to_f32(int(q.scales[0, 0])) == float(eff)
    codes = np.stack([(q.data[0] & 0xF).astype(int) - 8, (q.data[0] >> 4).astype(int) - 8], axis=1).reshape(-1)
    assert codes[0] == 7
    assert codes[1:1 + len(vals)].tolist() == want           # [2, 4, -2, 6, 0, 1]: one less than against `scale`
    assert q.dense()[0, 1] == 2 * float(eff)                 # and the stored value uses the effective scale too


def test_quantize_i4_is_a_fixed_point_on_its_own_output():
    r = rng(32)
    D = 64 * 20 + 17
    p = (r.normal(size=(5, D)) / math.sqrt(D)).astype(np.float32)
    q = orc.quantize_i4(p)
    dq = q.dense()
    assert np.array_equal(dq.astype(np.float32).astype(np.float64), dq)       # e*q is a binary32 number
    q2 = orc.quantize_i4(dq.astype(np.float32), gscale=q.gscale)
    assert np.array_equal(q2.data, q.data) and np.array_equal(q2.scales, q.scales)


# --------------------------------------------------------------------------- min-max quantiser: tie rule, a = 0, end points
@pytest.mark.parametrize("B,top", [(1, 1.0), (2, 3.0), (3, 7.0), (4, 15.0), (4, 45.0), (8, 255.0), (8, 765.0),
                                   (16, 65535.0)])
def test_minmax_ties_go_to_the_even_code(B, top):
    # min = 0 and max = top make the step a = top / (2^B - 1) exactly 1 or 3; (k + 1/2) * a is then exactly
    # half way between the codes k and k + 1: the paper names no tie rule, the reading here is ties to even.
    levels = (1 << B) - 1
    a = top / levels
    m = min(levels, 3000)
    k = np.arange(m) if levels <= 3000 else np.concatenate([np.arange(1500), np.arange(levels - 1500, levels)])
    P = np.zeros((3, k.size + 2))
    P[0, 0], P[0, 1] = 0.0, top
    P[0, 2:] = (k + 0.5) * a
    P[1, 2:] = k * a
    P[2, 2:] = (k + 0.25) * a
    codes, ao, bo = orc.quantize_minmax(P, B, [0, P.shape[1]])
    assert ao[0] == a and bo[0] == 0.0
    assert codes[0, 0] == 0 and codes[0, 1] == levels        # the end points take the first and the last code
    assert np.array_equal(codes[0, 2:].astype(np.int64), np.where(k % 2 == 0, k, k + 1))
    assert np.array_equal(codes[1, 2:].astype(np.int64), k)
    assert np.array_equal(codes[2, 2:].astype(np.int64), k)


def test_minmax_constant_layer_and_sixteen_bit_end_points():
    r = rng(33)
    P = r.normal(size=(4, 900))
    P[:, 300:500] = -0.375                                    # a constant layer: a = 0
    off = [0, 300, 500, 900]
    codes, a, b = orc.quantize_minmax(P, 16, off)
    assert a[1] == 0.0 and b[1] == -0.375 and not codes[:, 300:500].any()
    dense = orc.pmat_minmax(codes, a, b, off).dense()
    assert np.all(dense[:, 300:500] == -0.375)
    for l in (0, 2):
        seg = P[:, off[l]:off[l + 1]]
        c = codes[:, off[l]:off[l + 1]]
        assert c[np.unravel_index(np.argmin(seg), seg.shape)] == 0
        assert c[np.unravel_index(np.argmax(seg), seg.shape)] == 65535
        assert a[l] == (seg.max() - seg.min()) / 65535.0 and b[l] == seg.min()
        # every code is the nearest level, computed independently in exact rational arithmetic on a sample
        from fractions import Fraction
        fa, fb = Fraction(float(a[l])), Fraction(float(b[l]))
        for (j, i) in [(0, 0), (1, 17), (3, seg.shape[1] - 1), (2, 123)]:
            x = (Fraction(float(seg[j, i])) - fb) / fa
            lo = math.floor(x)
            near = lo if x - lo < Fraction(1, 2) else lo + 1
            assert abs(int(c[j, i]) - near) <= (1 if abs((x - lo) - Fraction(1, 2)) < Fraction(1, 10 ** 9) else 0)


# --------------------------------------------------------------------------- pins found by a mutation sweep of the oracle
def test_stored_values_of_every_vector_are_read_from_its_own_run():
    # the value of element (i, j) sits at j*ld + i, for every storage type (a column index that collapses
    # to 0 would go unnoticed by checks that go through the oracle's own dequantiser twice)
    r = rng(51)
    n, D, ld = 5, 300, 384
    a = np.zeros((n, ld), dtype=np.float32)
    a[:, :D] = r.normal(size=(n, D)).astype(np.float32)
    assert np.array_equal(orc.Pmat(orc.F32, D, a).dense(), a[:, :D].astype(np.float64))
    a64 = a.astype(np.float64)
    assert np.array_equal(orc.Pmat(orc.F64, D, a64).dense(), a64[:, :D])
    b = orc.to_bf16(a, D=D, ld=ld)
    want = torch.from_numpy(a[:, :D]).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(b.dense(), want)
    assert not b.data[:, D:].any()                            # padding of every vector is zeroed
    g = r.normal(size=D)
    assert np.allclose(orc.project(orc.Pmat(orc.F32, D, a), g), a64[:, :D] @ g, rtol=1e-13, atol=1e-13)
    assert np.allclose(orc.project(b, g), want @ g, rtol=1e-13, atol=1e-13)
    q8 = orc.quantize_i8(a, D=D, ld=ld)
    want8 = q8.data[:, :D].astype(np.float64) * np.repeat(q8.scales.astype(np.float64), 128, axis=1)[:, :D]
    assert np.array_equal(q8.dense(), want8)
    q4 = orc.quantize_i4(a, D=D, ld=ld)
    c4 = np.stack([(q4.data & 0xF).astype(np.float64) - 8, (q4.data >> 4).astype(np.float64) - 8], axis=2).reshape(n, -1)
    e4 = q4.scales.view(np.float16).astype(np.float64) * q4.gscale
    assert np.array_equal(q4.dense(), (c4 * np.repeat(e4, 64, axis=1))[:, :D])


def test_bfloat16_keeps_infinity_and_nan_apart():
    assert orc.f32_to_bf16_bits(float("inf")) == 0x7F80 and orc.f32_to_bf16_bits(float("-inf")) == 0xFF80
    assert (orc.f32_to_bf16_bits(float("nan")) & 0x7FFF) > 0x7F80
    assert orc.f32_to_f16_bits(float("inf")) == 0x7C00 and orc.f32_to_f16_bits(1e6) == 0x7C00
    assert (orc.f32_to_f16_bits(float("nan")) & 0x7FFF) > 0x7C00


def test_rank_threshold_is_relative_to_the_largest_checkpoint_norm():
    # |R_kk| <= rank_tol * max_j ||w_j|| is the error condition (rank_tol = 1e-6 by default)
    big = np.array([1000.0, 0.0, 0.0, 0.0, 0.0, 0.0])
    ok = np.array([0.0, 2e-3, 0.0, 0.0, 0.0, 0.0])            # 2e-3 > 1e-6 * 1000
    P, R = orc.build_basis(np.stack([big, ok]))
    assert R[1, 1] == pytest.approx(2e-3, rel=1e-12) and np.allclose(P[1], [0, 1, 0, 0, 0, 0], atol=1e-15)
    small = np.array([0.0, 5e-4, 0.0, 0.0, 0.0, 0.0])         # 5e-4 <= 1e-6 * 1000
    with pytest.raises(orc.OracleError) as ei:
        orc.build_basis(np.stack([big, small]))
    assert ei.value.code == orc.ERR_RANK and ei.value.column == 1
    # the largest norm counts wherever it stands, also behind the failing column
    with pytest.raises(orc.OracleError) as ei:
        orc.build_basis(np.stack([small, big]))
    assert ei.value.column == 0
    P, _ = orc.build_basis(np.stack([small, big]), rank_tol=1e-7)
    # norms below 1: the largest NORM decides (0.6), not a squared norm and not the first one seen
    e = np.eye(6)
    with pytest.raises(orc.OracleError) as ei:
        orc.build_basis(np.stack([0.5 * e[0], 0.6 * e[1], 0.55e-6 * e[2]]))
    assert ei.value.column == 2
    orc.build_basis(np.stack([0.5 * e[0], 0.6 * e[1], 0.65e-6 * e[2]]))
    assert np.allclose(np.abs(P), [[0, 1, 0, 0, 0, 0], [1, 0, 0, 0, 0, 0]], atol=1e-15)


def test_a_checkpoint_equal_to_the_mean_gives_a_zero_vector():
    # Sec. 4.1: e = (w - wbar)/||w - wbar||; a zero centred part has no direction: the vector is zero, not NaN
    w = rng(52).normal(size=(1, 40))
    E, wbar = orc.centre_normalise(w)
    assert np.array_equal(wbar, w[0]) and not E.any()
    W = np.stack([w[0], w[0] + 1.0, w[0] - 1.0])               # the first equals the mean of the three
    E, wbar = orc.centre_normalise(W)
    assert np.allclose(wbar, w[0], atol=1e-15) and np.all(np.isfinite(E))
    assert np.max(np.abs(E[0])) <= 1e-12 or np.allclose(np.linalg.norm(E[0]), 1.0)   # rounding may leave a direction
    E2, wb2, nr2 = orc.centre_normalise_layers(np.stack([w[0], w[0]]), [0, 10, 40])
    assert not E2.any() and not nr2.any()


def test_quantize_i4_ignores_what_stands_in_the_padding_of_its_input():
    # elements [D, ld) are padding: they do not enter a block's absmax and their code is 0 (nibble 8),
    # whatever the input holds there -- also when D is even and ends inside a byte pair's neighbour
    r = rng(53)
    for D in (70, 71):
        p = np.full((2, 128), 5.0e3, dtype=np.float32)         # poison everywhere ...
        p[:, :D] = r.normal(size=(2, D)).astype(np.float32)    # ... but in the D real elements
        q = orc.quantize_i4(p, D=D, ld=128, gscale=2.0 ** -14)
        codes = np.stack([(q.data & 0xF).astype(int) - 8, (q.data >> 4).astype(int) - 8], axis=2).reshape(2, -1)
        assert not codes[:, D:].any()
        clean = np.zeros_like(p)
        clean[:, :D] = p[:, :D]
        q0 = orc.quantize_i4(clean, D=D, ld=128, gscale=2.0 ** -14)
        assert np.array_equal(q.data, q0.data) and np.array_equal(q.scales, q0.scales)
        q8, q80 = orc.quantize_i8(p, D=D, ld=128), orc.quantize_i8(clean, D=D, ld=128)
        assert np.array_equal(q8.data, q80.data) and np.array_equal(q8.scales, q80.scales) and not q8.data[:, D:].any()
