"""The projection on codes of 4 bits and fewer computes in integers: every lane rounds its 32-element slice of the gradient to
multiples of unit = 2^(e-22), where 2^e is the smallest power of two above the slice's largest |g_i|, and from there on
the products and the sums of a slice are exact (include/twa.h, TWA_I4).  These tests hold the kernel to that model
against the fp64 oracle, which projects the gradient as it is: a worst-case bound per coefficient built from the
slices' units, exactness on gradients that lie on the grid, and non-finite gradients."""
import numpy as np
import pytest
import torch

from oracle import twa_oracle as orc
from paper_2205_13104_amd import binding as twa
from tests.gpu_common import REL_L2_TOL, random_basis_like, rel_l2, to_oracle

pytestmark = pytest.mark.gpu

SLICE = 32            # consecutive elements one lane turns into fixed-point numbers together (slices start at multiples of 32)


def say(*a):
    print(*a, flush=True)


def slice_units(g: np.ndarray) -> np.ndarray:
    """unit of every element's slice, from the documented rule (numpy, fp64): 2^(e - 22), 2^e > max|g_slice| >= 2^(e-1)."""
    D = g.size
    pad = (-D) % SLICE
    a = np.abs(np.concatenate([g.astype(np.float64), np.zeros(pad)])).reshape(-1, SLICE).max(axis=1)
    e = np.where(a > 0, np.floor(np.log2(np.where(a > 0, a, 1.0))) + 1, -126 - 22)
    e = np.maximum(e, -104.0)                                  # below 2^-104 the unit stays 2^-126
    return np.repeat(np.exp2(e - 22), SLICE)[:D]


def gradients(D, seed):
    r = np.random.default_rng(seed)
    z = r.normal(size=D)
    yield "gaussian", (1e-2 * z).astype(np.float32)
    yield "magnitudes over nine decades", (z * 10.0 ** r.uniform(-6, 3, size=D)).astype(np.float32)
    spike = 1e-3 * z
    spike[::SLICE] = 1e3 * np.sign(z[::SLICE])                 # one large element in every slice
    yield "one large element per slice", spike.astype(np.float32)
    yield "tiny", (1e-30 * z).astype(np.float32)
    yield "huge", (1e30 * z).astype(np.float32)
    sparse = np.where(r.random(D) < 0.02, z, 0.0)              # most slices all zero
    yield "mostly zeros", sparse.astype(np.float32)


@pytest.mark.parametrize("D,n", [(70001, 3), (150017, 100), (40000, 61), (2048 * 3, 128)])
def test_int4_projection_stays_inside_the_fixed_point_model(D, n):
    P32 = random_basis_like(D, n, seed=5 + n)
    pm = twa.quantize(P32, D, twa.I4)
    om = to_oracle(pm)
    absP = np.abs(om.dense()[:, :D])                           # |P~_ij| of the stored matrix
    for name, g in gradients(D, seed=n):
        say("int4 fixed point", D, n, name)
        s = twa.project(pm, torch.from_numpy(g).cuda()).cpu().numpy().astype(np.float64)
        g64 = g.astype(np.float64)
        ref = orc.project(om, g64)
        # rounding of g: at most half a unit per element; the float part (one conversion, two multiplications and one
        # addition per lane, basis vector and tile, then the tree and the fp64 sum): a few 2^-24 of the terms' sizes
        bound = 0.5 * absP @ slice_units(g) + 1e-6 * (absP @ np.abs(g64))
        worst = np.max(np.abs(s - ref) / np.maximum(bound, 1e-300))
        # the same model statistically: independent rounding errors, uniform within half a unit (variance unit^2 / 12),
        # six standard deviations; a digit less in the fixed-point numbers would be 16 times that
        likely = 6.0 * np.sqrt((absP ** 2) @ (slice_units(g) ** 2) / 12.0) + 2e-6 * np.sqrt((absP ** 2) @ (g64 ** 2))
        say("   rel_l2", rel_l2(s, ref), " largest error / bound", worst, " / six sigma", np.max(np.abs(s - ref) / likely))
        assert np.all(np.isfinite(s))
        assert np.all(np.abs(s - ref) <= bound)
        assert np.all(np.abs(s - ref) <= likely)
        if name in ("gaussian", "tiny", "huge"):               # one scale throughout: the bar of every storage type
            assert rel_l2(s, ref) <= REL_L2_TOL


def test_gradients_on_the_grid_are_projected_without_rounding_them():
    D, n = 100003, 25
    P32 = random_basis_like(D, n, seed=9)
    pm = twa.quantize(P32, D, twa.I4)
    om = to_oracle(pm)
    absP = np.abs(om.dense()[:, :D])
    r = np.random.default_rng(3)
    for scale in (1.0, 2.0 ** -40, 2.0 ** 30):
        g = (r.integers(-1000, 1001, size=D) * scale).astype(np.float32)      # |g| < 2^10 * scale: unit = 2^-12 * scale
        s = twa.project(pm, torch.from_numpy(g).cuda()).cpu().numpy().astype(np.float64)
        ref = orc.project(om, g.astype(np.float64))
        float_part = 1e-6 * (absP @ np.abs(g.astype(np.float64)))
        say("int4 on-grid gradient, scale", scale, " largest error / float-part bound", np.max(np.abs(s - ref) / float_part))
        assert np.all(np.abs(s - ref) <= float_part)


@pytest.mark.parametrize("bad", [float("nan"), float("inf"), -float("inf")])
def test_a_non_finite_gradient_element_poisons_every_coefficient(bad):
    D, n = 50001, 12
    pm = twa.quantize(random_basis_like(D, n, seed=4), D, twa.I4)
    g = torch.randn(D, device="cuda") * 1e-2
    g[31337] = bad
    s = twa.project(pm, g)
    assert not torch.isfinite(s).any()
    g[31337] = 0.0
    assert torch.isfinite(twa.project(pm, g)).all()


@pytest.mark.parametrize("n,k", [(37, 3), (100, 8), (120, 2), (5, 7)])
def test_batched_and_single_int4_projections_agree_bit_for_bit(n, k):
    """A batch is projected two gradients per pass over the codes (an odd last one alone; one per pass beyond 112 basis
    vectors): the same sums in the same order as one call per gradient."""
    D = 90001
    pm = twa.quantize(random_basis_like(D, n, seed=6), D, twa.I4)
    G = torch.randn((k, D + 3), device="cuda") * 1e-2
    S = twa.project(pm, G)
    for c in range(k):
        assert torch.equal(S[c], twa.project(pm, G[c, :D].contiguous())), c


@pytest.mark.parametrize("kind", ["i4", "mm4", "mm3", "mm2", "mm1"])
def test_layerwise_projection_on_narrow_codes_follows_the_same_model(kind):
    """Layer-wise, a slice that straddles a layer boundary is rounded once per layer, the other layer's elements
    counting as zeros; the model's six-sigma bar per coefficient, for the block codes and the paper's min-max codes
    of 4, 3, 2 bits and 1 bit (all of which enter the integer dot products, the narrow ones spread to nibbles)."""
    from paper_2205_13104_amd import synth
    D, n = 120011, 20
    sizes = [5, 1, 0, 30, 64, 2049, 1000, 4097, 17]
    sizes = sizes + [(D - sum(sizes)) // 2, 0]
    sizes.append(D - sum(sizes))
    off = synth.layer_offsets(sizes)
    offs = off.numpy()
    L = len(sizes)
    plan = twa.LayerPlan(off, D)
    P32 = random_basis_like(D, n, seed=12)
    if kind == "i4":
        pm = twa.quantize(P32, D, twa.I4)
        om = to_oracle(pm)
        dense = om.dense()[:, :D]
    else:
        pm = twa.quantize_minmax(P32, D, plan, bits=int(kind[2:]))
        om = to_oracle(pm, layer_off=offs)
        dense = om.dense()[:, :D]
    bias = 8.0 if kind == "mm4" else 0.0                             # 4-bit codes enter the dot products as c - 8, narrower ones as c
    for name, g in gradients(D, seed=21):
        S = twa.project_layers(pm, torch.from_numpy(g).cuda(), plan).cpu().numpy().astype(np.float64)
        g64 = g.astype(np.float64)
        ref = orc.project_layers(om, g64, offs)
        assert S.shape == ref.shape == (L, n)
        worst = 0.0
        for l in range(L):
            a, b = int(offs[l]), int(offs[l + 1])
            if b == a:
                assert np.all(S[l] == 0.0)
                continue
            gl = np.zeros(D, dtype=np.float32)
            gl[a:b] = g[a:b]
            u = slice_units(gl)[a:b]
            if kind == "i4":
                wgt = dense[:, a:b]                                  # what multiplies a rounding error of g: the stored value
            else:
                al = float(pm.scales[l, 0])                          # min-max: the integer part is a_l * (code - bias); b_l and
                wgt = dense[:, a:b] - (float(pm.scales[l, 1]) + bias * al)  # bias * a_l multiply the float sum of g
            terms = np.sqrt((dense[:, a:b] ** 2) @ (g64[a:b] ** 2))
            likely = 6.0 * np.sqrt((wgt ** 2) @ (u ** 2) / 12.0) + 2e-6 * terms + 2e-6 * abs(float(np.sum(g64[a:b]))) * \
                (0.0 if kind == "i4" else abs(float(pm.scales[l, 1])) + bias * abs(float(pm.scales[l, 0])))
            worst = max(worst, float(np.max(np.abs(S[l] - ref[l]) / np.maximum(likely, 1e-300))))
            assert np.all(np.abs(S[l] - ref[l]) <= likely), (name, l, sizes[l])
        say("layer-wise", kind, name, " rel_l2", rel_l2(S, ref), " largest error / six sigma", worst)
        if name in ("gaussian", "tiny", "huge"):
            assert rel_l2(S, ref) <= REL_L2_TOL
