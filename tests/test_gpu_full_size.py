"""Parity at the benchmark configurations' FULL sizes, in the launch configuration bench.py times.

Up to the ResNet-50 shape the fp64 oracle evaluates a WHOLE step in about a second on the machine's host cores, so
there the comparison is exhaustive: every coefficient of s and every element of g~ and w, against the oracle on
the stored P the GPU used, by relative L2 AND per element (max-abs bars, derived from the arithmetic in
check_step_whole).  Only the largest configuration (D = 350 M, n = 128: 45 G products per pass) is
sampled: a few coefficients over the whole of D, and g~ / w on sampled blocks.  Orthonormality of the full-size
bases is checked with an fp64 library matmul over row chunks."""
import numpy as np
import pytest
import torch

from oracle import twa_oracle as orc
from oracle.bridge import to_oracle
from paper_2205_13104_amd import binding as twa
from paper_2205_13104_amd import synth
from tests.gpu_common import ORTHO_TOL, REL_L2_TOL, rel_l2

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def gram_fp64(P, D, chunk=1 << 21):
    n = P.shape[0]
    G = torch.zeros((n, n), dtype=torch.float64, device=P.device)
    for a in range(0, D, chunk):
        x = P[:, a:min(D, a + chunk)].double()
        G += x @ x.T
    return G.cpu().numpy()


def sampled_blocks_pmat(pm, block_ids, block):
    """Oracle view of rows [b*block, (b+1)*block) for b in block_ids (all n vectors): bytes only."""
    rows = torch.cat([torch.arange(b * block, (b + 1) * block) for b in block_ids]).to(pm.data.device)
    nrows = int(rows.numel())
    if pm.dtype == twa.F32:
        return rows, orc.Pmat(orc.F32, nrows, np.ascontiguousarray(pm.data[:, rows].cpu().numpy()))
    if pm.dtype == twa.BF16:
        d = pm.data[:, rows].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return rows, orc.Pmat(orc.BF16, nrows, np.ascontiguousarray(d))
    if pm.dtype == twa.I8:
        sc = pm.scales_by_vector()[:, torch.tensor(block_ids, device=pm.data.device)].cpu().numpy()
        return rows, orc.Pmat(orc.I8, nrows, np.ascontiguousarray(pm.data[:, rows].cpu().numpy()),
                              np.ascontiguousarray(sc), block, 1.0)
    raise ValueError(pm.dtype)


MAX_ABS_TOL = 1e-5         # per-element bar: max |error| <= MAX_ABS_TOL * rms(reference vector); see check_step_whole
HALF_ULP = 2.0 ** -24


def rms(x):
    x = np.asarray(x, dtype=np.float64)
    return float(np.sqrt(np.mean(x * x)))


def check_step_whole(pm, D, n, g, w, lr, label):
    """One step at full size, compared with the oracle in EVERY output: all n coefficients, all D elements of
    g~ and w.  Bars: relative L2 <= 1e-5 on each vector, and per element
        max_j |s_j - s^_j|   <= 1e-5 * rms(s^)             max_i |g~_i - g~^_i| <= 1e-5 * rms(g~^)
        |w_i - w^_i|         <= 2^-24 |w^_i| + lr * 1e-5 * rms(g~^)      (one fused multiply-add per element).
    The rounding model behind the factor: a coefficient is a sum of D products held in fp32 running sums of m
    terms each (m ~ 50..800 by storage type), whose error has standard deviation ~ 2^-24 sqrt(m/6) * |s_j| --
    2e-7..7e-7 of rms(s); the largest of n = 100 such errors stays below 3e-6 * rms(s), while ONE 2048-element
    tile dropped or attributed to the wrong workgroup moves a coefficient by ~sqrt(2048/D) * rms(s) = 9e-3 * rms(s).
    Returns the GPU's s."""
    ws = twa.Workspace(twa.project_workspace_bytes(n))
    s = torch.empty(n, device="cuda")
    w0 = w.clone()
    gt = torch.empty(D, device="cuda")
    twa.project(pm, g, s, ws)
    twa.expand_update(pm, s, w, lr, gt)
    torch.cuda.synchronize()
    po = to_oracle(pm)
    g_h = g.cpu().numpy().astype(np.float64)
    s_h = s.cpu().numpy().astype(np.float64)
    # (1) every coefficient
    so = orc.project(po, g_h)
    e_s, m_s = rel_l2(s_h, so), float(np.max(np.abs(s_h - so))) / rms(so)
    say(f"  {label}: s: rel_l2 {e_s:.2e}, max|err|/rms {m_s:.2e}")
    assert e_s <= REL_L2_TOL and m_s <= MAX_ABS_TOL
    # (2) every element of g~ and w, per call: the oracle expands the GPU's own s from the same fp32 w
    wo = w0.cpu().numpy().astype(np.float64)
    w_start = wo.copy()
    gto = orc.expand_update(po, s_h, wo, float(np.float32(lr)), want_gt=True)
    gt_h = gt.cpu().numpy().astype(np.float64)
    w_h = w.cpu().numpy().astype(np.float64)
    r_gt = rms(gto)
    e_gt, m_gt = rel_l2(gt_h, gto), float(np.max(np.abs(gt_h - gto))) / r_gt
    e_w = rel_l2(w_h, wo)
    over = np.abs(w_h - wo) - (HALF_ULP * np.abs(wo) + float(np.float32(lr)) * MAX_ABS_TOL * r_gt)
    e_d = rel_l2(w_h - w_start, wo - w_start)
    say(f"  {label}: g~: rel_l2 {e_gt:.2e}, max|err|/rms {m_gt:.2e};  w: rel_l2 {e_w:.2e}, displacement rel_l2 {e_d:.2e}, "
        f"worst excess over the per-element bar {float(over.max()):.2e}")
    assert e_gt <= REL_L2_TOL and m_gt <= MAX_ABS_TOL and e_w <= REL_L2_TOL
    assert float(over.max()) <= 0.0
    # (3) chained: the oracle's own coefficients instead of the GPU's (what a caller that trusts the library sees)
    wc = w_start.copy()
    orc.expand_update(po, so, wc, float(np.float32(lr)))
    assert rel_l2(w_h, wc) <= REL_L2_TOL
    # (4) nothing outside [0, D) is the library's to write: the tensors are exactly D long; all of it finite
    assert torch.isfinite(w).all() and torch.isfinite(gt).all()
    return s


def test_imagenet_resnet50_int8_full_size():
    wl = synth.WORKLOADS["imagenet_resnet50"]
    D, n = wl.D, wl.n
    say("full size", wl.name, D, n)
    W = synth.checkpoints(wl, seed=0, device="cuda")
    w = W[:, :D].mean(dim=0).contiguous()
    P, R = twa.build_basis(W, D, out=W)
    G = gram_fp64(P, D)
    ortho = np.max(np.abs(G - np.eye(n)))
    say("  max|PtP-I|", ortho)
    assert ortho <= ORTHO_TOL
    assert np.all(np.diag(R.numpy()) > 0) and np.max(np.abs(np.tril(R.numpy(), -1))) == 0.0
    pm = twa.quantize(P, D, twa.I8)
    # codes and scales of EVERY vector bit-exact (whole vectors through the oracle's quantiser, 20 at a time)
    sbv = pm.scales_by_vector()
    for j0 in range(0, n, 20):
        ref = orc.quantize_i8(P[j0:j0 + 20].cpu().numpy(), D=D, ld=pm.ld)
        assert np.array_equal(pm.data[j0:j0 + 20].cpu().numpy(), ref.data), j0
        assert np.array_equal(sbv[j0:j0 + 20].cpu().numpy().view(np.uint32), ref.scales.view(np.uint32)), j0
    say("  codes and scales of all", n, "vectors equal the oracle's, bit for bit")
    g = synth.gradient(D, wl.sigma_g, seed=0, step=0, device="cuda")
    # the fp32-P variant at the same shape (the configuration times it as well)
    check_step_whole(twa.wrap_f32(P, D), D, n, g, w.clone(), wl.lr, "fp32")
    del W, P, sbv, ref
    torch.cuda.empty_cache()
    s1 = check_step_whole(pm, D, n, g, w, wl.lr, "int8")
    # rerun determinism at full size
    s2 = twa.project(pm, g)
    assert torch.equal(s1, s2)
    check_layer_step_whole(pm, D, n, g, w, wl.lr, synth.workload_layers(wl.name), "int8")


def test_imagenet_resnet50_int4_full_size():
    """The same shape with 4-bit block codes (bench.py --storage i4): codes and binary16 scales of every vector bit for bit,
    then one whole step and one layer-wise step compared in every output.  The projection runs in integer dot
    products on fixed-point slices of the gradient; the bars are those of every other storage type."""
    wl = synth.WORKLOADS["imagenet_resnet50"]
    D, n = wl.D, wl.n
    say("full size", wl.name, D, n, "int4")
    W = synth.checkpoints(wl, seed=0, device="cuda")
    w = W[:, :D].mean(dim=0).contiguous()
    P, _ = twa.build_basis(W, D, out=W, want_R=False)
    pm = twa.quantize(P, D, twa.I4)
    sbv = pm.scales_by_vector().view(torch.int16)
    for j0 in range(0, n, 20):
        ref = orc.quantize_i4(P[j0:j0 + 20].cpu().numpy(), D=D, ld=pm.ld, gscale=pm.gscale)
        assert np.array_equal(pm.data[j0:j0 + 20].cpu().numpy(), ref.data), j0
        assert np.array_equal(sbv[j0:j0 + 20].cpu().numpy().view(np.uint16), ref.scales), j0
    assert pm.gscale == orc.gscale_i4(P[:, :D].cpu().numpy(), D)
    say("  codes and scales of all", n, "vectors equal the oracle's, bit for bit; gscale", pm.gscale)
    del W, P, sbv, ref
    torch.cuda.empty_cache()
    g = synth.gradient(D, wl.sigma_g, seed=0, step=0, device="cuda")
    s1 = check_step_whole(pm, D, n, g, w, wl.lr, "int4")
    assert torch.equal(s1, twa.project(pm, g))
    check_layer_step_whole(pm, D, n, g, w, wl.lr, synth.workload_layers(wl.name), "int4")


def test_imagenet_resnet50_int8_chained_steps_full_size():
    """The update rule of Sec. 4.2 iterated at the benchmark shape: T = 50 steps with a fresh gradient each, the GPU
    keeping w in fp32 in place and feeding its own coefficients forward, the oracle running its own chain in fp64
    from the same start.  Every coefficient vector on the way and the final weights are compared."""
    wl = synth.WORKLOADS["imagenet_resnet50"]
    D, n, T = wl.D, wl.n, 50
    say("chained steps at full size", wl.name, D, n, "T", T)
    W = synth.checkpoints(wl, seed=0, device="cuda")
    w = W[:, :D].mean(dim=0).contiguous()
    P, _ = twa.build_basis(W, D, out=W, want_R=False)
    pm = twa.quantize(P, D, twa.I8)
    del W, P
    torch.cuda.empty_cache()
    po = to_oracle(pm)
    wo = w.cpu().numpy().astype(np.float64)
    w_start = wo.copy()
    ws = twa.Workspace(twa.project_workspace_bytes(n))
    s = torch.empty(n, device="cuda")
    lr = float(np.float32(wl.lr))
    worst = 0.0
    for t in range(T):
        g = synth.gradient(D, wl.sigma_g, seed=0, step=t, device="cuda")
        twa.project(pm, g, s, ws)
        twa.expand_update(pm, s, w, wl.lr)
        so = orc.project(po, g.cpu().numpy().astype(np.float64))
        e = rel_l2(s.cpu().numpy(), so)
        worst = max(worst, e)
        assert e <= REL_L2_TOL, t
        orc.expand_update(po, so, wo, lr)
        if t % 10 == 9:
            say(f"  step {t + 1}: worst rel_l2(s) so far {worst:.2e}")
    w_h = w.cpu().numpy().astype(np.float64)
    e_w = rel_l2(w_h, wo)
    e_d = rel_l2(w_h - w_start, wo - w_start)
    # per element: T in-place fp32 stores, each within half an ulp of w, plus T times the per-step bar on lr * g~
    step_rms = rms(wo - w_start) / np.sqrt(T)
    over = np.abs(w_h - wo) - T * (HALF_ULP * (np.abs(wo) + np.max(np.abs(wo - w_start))) + MAX_ABS_TOL * step_rms)
    say(f"  w after {T} steps: rel_l2 {e_w:.2e}; displacement rel_l2 {e_d:.2e} (reported: every in-place fp32 store "
        f"rounds w by up to 2^-24 |w|, ~1e-3 of one step's update); worst per-element excess {float(over.max()):.2e}")
    assert e_w <= REL_L2_TOL and float(over.max()) <= 0.0


def test_tiny_configuration_as_written():
    """The small benchmark configuration with its own numbers: D = 1,000,000, n = 10, trajectory checkpoints (decay 0.9,
    drift 0.5), basis by CholeskyQR2, 100 projected steps with g ~ N(0, 1e-2^2), lr = 0.1, seed 0, P kept in fp32."""
    wl = synth.WORKLOADS["tiny"]
    D, n, T = wl.D, wl.n, wl.steps
    assert (D, n, T, wl.lr, wl.sigma_g) == (1_000_000, 10, 100, 0.1, 1e-2)
    W = synth.checkpoints(wl, seed=0, device="cuda")
    Wh = W[:, :D].cpu().numpy().astype(np.float64)
    P, R = twa.build_basis(W, D)
    Ph = P[:, :D].cpu().numpy().astype(np.float64)
    ortho = np.max(np.abs(Ph @ Ph.T - np.eye(n)))
    say("tiny as written: max|PtP-I|", ortho)
    assert ortho <= ORTHO_TOL
    Rn = R.numpy()
    assert np.all(np.diag(Rn) > 0) and np.max(np.abs(np.tril(Rn, -1))) == 0.0
    assert np.linalg.norm(Wh - Rn.T @ Ph) <= 1e-5 * np.linalg.norm(Wh)
    _, Ro = orc.build_basis(Wh)                                  # the oracle's Householder factor of the same checkpoints
    assert np.max(np.abs(Rn - Ro)) <= 1e-5 * np.max(np.abs(Ro))
    pm = twa.wrap_f32(P, D)
    po = to_oracle(pm)
    w = W[:, :D].mean(dim=0).contiguous()
    wo = w.cpu().numpy().astype(np.float64)
    w_start = wo.copy()
    ws = twa.Workspace(twa.project_workspace_bytes(n))
    s = torch.empty(n, device="cuda")
    lr = float(np.float32(wl.lr))
    for t in range(T):
        g = synth.gradient(D, wl.sigma_g, seed=0, step=t, device="cuda")
        twa.project(pm, g, s, ws)
        twa.expand_update(pm, s, w, wl.lr)
        so = orc.project(po, g.cpu().numpy().astype(np.float64))
        assert rel_l2(s.cpu().numpy(), so) <= REL_L2_TOL, t
        orc.expand_update(po, so, wo, lr)
    w_h = w.cpu().numpy().astype(np.float64)
    e_w, e_d = rel_l2(w_h, wo), rel_l2(w_h - w_start, wo - w_start)
    step_rms = rms(wo - w_start) / np.sqrt(T)
    over = np.abs(w_h - wo) - T * (HALF_ULP * (np.abs(wo) + np.max(np.abs(wo - w_start))) + MAX_ABS_TOL * step_rms)
    say(f"  w after {T} steps: rel_l2 {e_w:.2e}; displacement rel_l2 {e_d:.2e} (reported); worst per-element excess {float(over.max()):.2e}")
    assert e_w <= REL_L2_TOL and float(over.max()) <= 0.0
    # the iterate stays in wbar + span(W): what is left of the displacement after projecting on P vanishes
    d = w_h - w_start
    # (up to the fp32 rounding of the 100 in-place stores: ~sqrt(T) * 2^-24 |w| / sqrt(3) = 1e-8 per element
    #  against a displacement of 3e-5)
    assert np.linalg.norm(d - (Ph @ d) @ Ph) <= 2e-3 * np.linalg.norm(d)


def check_layer_step_whole(pm, D, n, g, w, lr, off_cpu, label):
    """The layer-wise step (Sec. 4.5) at full size with the architecture's own layer table, exhaustive: every
    entry of S (L x n) and every element of g~ and w against the oracle, same bars as check_step_whole (the
    per-element bar of S is taken against the rms of the whole-model coefficients: a short layer's own sums can
    be arbitrarily small)."""
    L = int(off_cpu.numel()) - 1
    plan = twa.LayerPlan(off_cpu, D)
    S = twa.project_layers(pm, g, plan)
    w0 = w.clone()
    gt = torch.empty(D, device="cuda")
    twa.expand_update_layers(pm, S, plan, w, lr, gt)
    torch.cuda.synchronize()
    offs = off_cpu.numpy()
    po = to_oracle(pm)
    g_h = g.cpu().numpy().astype(np.float64)
    S_h = S.cpu().numpy().astype(np.float64)
    So = orc.project_layers(po, g_h, offs)
    s_whole = So.sum(axis=0)
    e_s, m_s = rel_l2(S_h, So), float(np.max(np.abs(S_h - So))) / rms(s_whole)
    say(f"  {label}, layer-wise L={L}: S: rel_l2 {e_s:.2e}, max|err|/rms(s) {m_s:.2e}")
    assert e_s <= REL_L2_TOL and m_s <= MAX_ABS_TOL
    wo = w0.cpu().numpy().astype(np.float64)
    gto = orc.expand_update_layers(po, S_h, offs, wo, float(np.float32(lr)), want_gt=True)
    gt_h = gt.cpu().numpy().astype(np.float64)
    w_h = w.cpu().numpy().astype(np.float64)
    r_gt = rms(gto)
    # per element: the error of g~_i grows with the size of the terms it sums, i.e. with the coefficient row of ITS
    # layer; a layer whose own rms lies above the vector's takes its own rms as the scale, every other the vector's
    sizes = np.diff(offs)
    live = sizes > 0
    layer_rms = np.zeros(L)
    layer_rms[live] = np.sqrt(np.add.reduceat(gto * gto, offs[:-1][live]) / sizes[live])
    scale = np.maximum(np.repeat(layer_rms, sizes), r_gt)
    e_gt, m_gt, e_w = rel_l2(gt_h, gto), float(np.max(np.abs(gt_h - gto) / scale)), rel_l2(w_h, wo)
    over = np.abs(w_h - wo) - (HALF_ULP * np.abs(wo) + float(np.float32(lr)) * MAX_ABS_TOL * scale)
    say(f"  {label}, layer-wise: g~: rel_l2 {e_gt:.2e}, max|err|/max(rms of the layer, rms) {m_gt:.2e} "
        f"(against the vector's rms alone {float(np.max(np.abs(gt_h - gto))) / r_gt:.2e});  w: rel_l2 {e_w:.2e}, "
        f"worst excess over the per-element bar {float(over.max()):.2e}")
    assert e_gt <= REL_L2_TOL and m_gt <= MAX_ABS_TOL and e_w <= REL_L2_TOL and float(over.max()) <= 0.0
    # the rows of S add up to the whole-model coefficients
    s = twa.project(pm, g)
    assert rel_l2(S.double().sum(0).cpu().numpy(), s.double().cpu().numpy()) <= 1e-6
    assert torch.isfinite(w).all() and torch.isfinite(gt).all()


def test_cifar_resnet18_fp32_full_size():
    wl = synth.WORKLOADS["cifar_resnet18"]
    D, n = wl.D, wl.n
    say("full size", wl.name, D, n)
    W = synth.checkpoints(wl, seed=0, device="cuda")
    w = W[:, :D].mean(dim=0).contiguous()
    P, _ = twa.build_basis(W, D, out=W)
    ortho = np.max(np.abs(gram_fp64(P, D) - np.eye(n)))
    say("  max|PtP-I|", ortho)
    assert ortho <= ORTHO_TOL
    pm = twa.wrap_f32(P, D)
    g = synth.gradient(D, wl.sigma_g, seed=0, step=0, device="cuda")
    check_step_whole(pm, D, n, g, w, wl.lr, "fp32")


def test_vit_b16_bf16_batched_full_size():
    wl = synth.WORKLOADS["vit_b16_finetune"]
    D, n, k = wl.D, wl.n, wl.k
    say("full size", wl.name, D, n, "k", k)
    W = synth.checkpoints(wl, seed=0, device="cuda")
    P, _ = twa.build_basis(W, D, out=W)
    ortho = np.max(np.abs(gram_fp64(P, D) - np.eye(n)))
    say("  max|PtP-I|", ortho)
    assert ortho <= ORTHO_TOL
    pm = twa.quantize(P, D, twa.BF16)
    ref0 = orc.to_bf16(P[3:4].cpu().numpy(), D=D, ld=pm.ld)
    assert np.array_equal(pm.data[3].view(torch.int16).cpu().numpy().view(np.uint16), ref0.data[0])
    del W, P
    torch.cuda.empty_cache()
    ldg = (D + 3) // 4 * 4
    G = synth.gradient(D, wl.sigma_g, seed=0, step=0, device="cuda", k=k, ldg=ldg)
    S = twa.project(pm, G)
    torch.cuda.synchronize()
    # every one of the k x n coefficients against the oracle (S = P^T G, Sec. 4.2 with k gradients)
    po = to_oracle(pm)
    So = orc.project(po, G[:, :D].cpu().numpy().astype(np.float64))
    S_h = S.cpu().numpy().astype(np.float64)
    e, m = rel_l2(S_h, So), float(np.max(np.abs(S_h - So))) / rms(So)
    say(f"  S (all {k} x {n}): rel_l2 {e:.2e}, max|err|/rms {m:.2e}")
    assert e <= REL_L2_TOL and m <= MAX_ABS_TOL
    for c in range(k):
        assert rel_l2(S_h[c], So[c]) <= REL_L2_TOL, c
    # every gradient alone reproduces its row of the batched result
    for c in (1, 5):
        sc = twa.project(pm, G[c, :D].contiguous())
        assert rel_l2(S[c].cpu().numpy(), sc.cpu().numpy()) <= 5e-6   # two summation orders, each within the bar
    # and one whole step with the first gradient (expansion at this shape: n = 20, several launches)
    w = torch.randn(D, device="cuda", generator=torch.Generator(device="cuda").manual_seed(3)) * 0.02
    check_step_whole(pm, D, n, G[0, :D].contiguous(), w, wl.lr, "bf16")


def test_large_int4_int8_full_size():
    """D = 350 M, n = 128, as the configuration describes it: the checkpoints' rows are produced in panels of 2^24
    rows into one staging buffer (8.6 GB), three sweeps -- Gram; first pass applied + Gram; both passes applied, the
    second fused with the quantiser -- and only the 4-bit (22.4 GB) and 8-bit (44.8 GB) matrices are kept: neither
    the 179 GB checkpoint matrix nor the fp32 basis ever exists.  Sampled at this size: the codes of whole panels
    against the oracle's quantiser, coefficients over the whole of D, g~ / w on sampled blocks; orthonormality of
    what was quantised by a fourth sweep."""
    from tests.test_gpu_pipeline import pipeline
    wl = synth.WORKLOADS["large"]
    D, n, panel = wl.D, wl.n, 1 << 24
    free, total = torch.cuda.mem_get_info()
    need = 4 * n * panel + n * (D + 2048) * 3 // 2 + 40 * D + (8 << 30)
    if free < need:
        pytest.skip(f"needs {need / 2**30:.0f} GiB of device memory, {free / 2**30:.0f} GiB free")
    say("full size", wl.name, D, n, f"free {free / 2**30:.0f} GiB; panels of", panel, "rows")
    outs, R1, R2, stage, (st1, st2) = pipeline(D, n, panel, wl, seed=0, dtypes=(twa.I4, twa.I8))
    say("  pipeline done; peak device memory", f"{torch.cuda.max_memory_allocated() / 2**30:.1f} GiB")
    assert torch.cuda.max_memory_allocated() < 100 * 2**30           # far below the 179 GB of the checkpoints alone
    R1n, R2n = R1.numpy(), R2.numpy()
    assert np.all(np.diag(R1n) > 0) and np.all(np.diag(R2n) > 0)
    assert np.max(np.abs(R2n - np.eye(n))) <= 5e-3                   # the first pass left an almost orthonormal matrix
    # a fourth sweep, for the test only: the fp32 values that were quantised, panel by panel -> their Gram matrix,
    # and on three panels the oracle's quantiser on whole vectors
    st3 = twa.BasisState(n)
    R3 = torch.zeros((n, n), dtype=torch.float64)
    starts = list(range(0, D, panel))
    check_panels = {0, starts[len(starts) // 2], starts[-1]}
    w_mean = torch.empty(D, device="cuda")
    for k, r0 in enumerate(starts):
        rows = min(panel, D - r0)
        synth.trajectory_panel(rows, n, wl.decay, wl.drift, 0, r0, stage)
        w_mean[r0:r0 + rows] = stage[:, :rows].mean(dim=0)
        twa.apply_rinv(stage, rows, st1)
        twa.apply_rinv(stage, rows, st2)
        twa.gram_accumulate(stage, rows, st3, first=k == 0)
        if r0 in check_panels:
            for j in (0, 77, n - 1):
                col = np.ascontiguousarray(stage[j:j + 1, :rows].cpu().numpy())
                ldc = (rows + 2047) // 2048 * 2048
                o8 = orc.quantize_i8(col, D=rows, ld=ldc)
                assert np.array_equal(outs[twa.I8].data[j, r0:r0 + rows].cpu().numpy(), o8.data[0, :rows]), (r0, j)
                sc8 = outs[twa.I8].scales_by_vector()[j, r0 // 128:(r0 + rows + 127) // 128].cpu().numpy()
                assert np.array_equal(sc8.view(np.uint32), o8.scales[0, :sc8.size].view(np.uint32)), (r0, j)
                o4 = orc.quantize_i4(col, D=rows, ld=ldc, gscale=outs[twa.I4].gscale)
                assert np.array_equal(outs[twa.I4].data[j, r0 // 2:(r0 + rows + 1) // 2].cpu().numpy(), o4.data[0, :(rows + 1) // 2]), (r0, j)
                sc4 = outs[twa.I4].scales_by_vector()[j, r0 // 64:(r0 + rows + 63) // 64].view(torch.int16).cpu().numpy().view(np.uint16)
                assert np.array_equal(sc4, o4.scales[0, :sc4.size]), (r0, j)
            say("  panel at row", r0, ": codes and scales of sampled vectors equal the oracle's")
    twa.gram_factor(st3, R3)                                         # G3 = R3^T R3: orthonormal input gives R3 = I
    G3 = R3.numpy().T @ R3.numpy()
    ortho = np.max(np.abs(G3 - np.eye(n)))
    say("  max|PtP-I| of the quantised values' fp32 originals", ortho)
    assert ortho <= ORTHO_TOL
    del stage
    torch.cuda.empty_cache()
    g = synth.gradient(D, wl.sigma_g, seed=0, step=0, device="cuda")
    w = w_mean
    for dtype in (twa.I4, twa.I8):
        pm = outs[dtype]
        # one step: sampled coefficients over the whole of D, g~ / w on sampled blocks
        ws = twa.Workspace(twa.project_workspace_bytes(n))
        s = torch.empty(n, device="cuda")
        w1 = w.clone()
        gt = torch.empty(D, device="cuda")
        twa.project(pm, g, s, ws)
        twa.expand_update(pm, s, w1, wl.lr, gt)
        torch.cuda.synchronize()
        cols = [0, n - 1]
        so = orc.project(to_oracle(pm, cols=cols), g.cpu().numpy().astype(np.float64))
        e_s = rel_l2(s[cols].cpu().numpy(), so)
        say("  dtype", dtype, "rel_l2 s[sampled]", e_s)
        assert e_s <= REL_L2_TOL
        blk = pm.block
        nb = D // blk
        r = np.random.default_rng(5)
        ids = sorted(set([0, nb - 1] + r.integers(0, nb, size=32).tolist()))
        rows = torch.cat([torch.arange(b * blk, (b + 1) * blk) for b in ids]).cuda()
        scv = pm.scales_by_vector()[:, torch.tensor(ids, device="cuda")]
        if dtype == twa.I8:
            po = orc.Pmat(orc.I8, int(rows.numel()), np.ascontiguousarray(pm.data[:, rows].cpu().numpy()),
                          np.ascontiguousarray(scv.cpu().numpy()), blk, 1.0)
        else:
            bytes_ = torch.cat([torch.arange(b * blk // 2, (b + 1) * blk // 2) for b in ids]).cuda()
            po = orc.Pmat(orc.I4, int(rows.numel()), np.ascontiguousarray(pm.data[:, bytes_].cpu().numpy()),
                          np.ascontiguousarray(scv.view(torch.int16).cpu().numpy().view(np.uint16)), blk, pm.gscale)
        wo = w[rows].cpu().numpy().astype(np.float64)
        gto = orc.expand_update(po, s.cpu().numpy().astype(np.float64), wo, wl.lr, want_gt=True)
        e_gt, e_w = rel_l2(gt[rows].cpu().numpy(), gto), rel_l2(w1[rows].cpu().numpy(), wo)
        say("  dtype", dtype, "rel_l2 g~[sampled]", e_gt, "w[sampled]", e_w)
        assert e_gt <= REL_L2_TOL and e_w <= REL_L2_TOL
        del w1, gt, ws
        torch.cuda.empty_cache()


def _minmax_codes_at(pm, idx):
    """Codes of all vectors at the elements `idx` (a device tensor of indices), read from the packed storage."""
    if pm.dtype == twa.U4MM:
        by = pm.data[:, idx // 2]
        return ((by >> (4 * (idx & 1)).to(torch.uint8)) & 0xF).cpu().numpy().astype(np.uint16)
    if pm.dtype in (twa.U2MM, twa.U1MM):                   # B-bit fields, low bits first
        B = 2 if pm.dtype == twa.U2MM else 1
        per = 8 // B
        by = pm.data[:, idx // per]
        return ((by >> (B * (idx % per)).to(torch.uint8)) & ((1 << B) - 1)).cpu().numpy().astype(np.uint16)
    if pm.dtype in (twa.U8MM, twa.U16MM):                  # the container holds code - 2^(B-1)
        return (pm.data[:, idx].to(torch.int32) + (1 << (pm.block - 1))).cpu().numpy().astype(np.uint16)
    assert pm.dtype == twa.U3MM
    # groups of 32 elements in three 32-bit words: element e = 16h + 4k + m has its low two bits in word h at
    # bit 2(4k + m), its high bit in word 2 at bit 8k + m + 4h
    words = pm.data.view(torch.int32)
    g, e = idx // 32, idx % 32
    h, f = e // 16, e % 16
    low = (words[:, 3 * g + h] >> (2 * f).to(torch.int32)) & 3
    high = (words[:, 3 * g + 2] >> (8 * (f // 4) + f % 4 + 4 * h).to(torch.int32)) & 1
    return (low | (high << 2)).cpu().numpy().astype(np.uint16)


@pytest.mark.parametrize("bits", [4, 3, 2, 1, 8, 16])
def test_imagenet_resnet50_algorithm_1_minmax_full_size(bits):
    """The paper's default configuration at the benchmark shape, as bench.py --mode layerwise --storage mm4 runs it
    (and the same with 3-bit codes, --storage mm3):
    layer-wise centre+normalise basis (Sec. 4.1, 4.5), 4-bit per-layer min-max codes (Sec. 4.6), coefficient step
    with weight decay and w = wbar + P beta (Alg. 1).  Sampled: wbar and E on blocks, codes and factors of whole
    layers through the oracle's quantiser, coefficient columns over all of D, w on blocks next to layer boundaries."""
    wl = synth.WORKLOADS["imagenet_resnet50"]
    D, n = wl.D, wl.n
    off_cpu = synth.workload_layers(wl.name)
    offs = off_cpu.numpy()
    L = len(offs) - 1
    say("full size, Alg. 1, min-max codes of", bits, "bits", wl.name, D, n, "L", L)
    W = synth.checkpoints(wl, seed=0, device="cuda")
    plan = twa.LayerPlan(off_cpu, D)
    # ---- basis: mean bit-exact and centred/normalised vectors within the bar, on sampled layers (whole layers)
    sizes = np.diff(offs)
    order = np.argsort(sizes)
    layers = sorted(set(order[:6].tolist() + order[L // 2 - 2:L // 2 + 2].tolist() + [0, L - 1]
                        + [int(np.argmin(np.abs(sizes - 590_000)))]))
    W_host = {l: W[:, offs[l]:offs[l + 1]].cpu().numpy().astype(np.float64) for l in layers}
    E, wbar, _ = twa.centre_normalise(W, D, plan, out=W, want_norms=False)
    torch.cuda.synchronize()
    for l in layers:
        a, b = int(offs[l]), int(offs[l + 1])
        Eo, wbo, _ = orc.centre_normalise_layers(W_host[l], np.array([0, b - a], dtype=np.int64))
        assert np.array_equal(wbar[a:b].cpu().numpy(), wbo.astype(np.float32)), l
        assert rel_l2(E[:, a:b].cpu().numpy(), Eo) <= REL_L2_TOL, l
    # ---- codes and factors of those layers, bit-exact
    E_host = {l: E[:, offs[l]:offs[l + 1]].cpu().numpy().astype(np.float64) for l in layers}
    pm = twa.quantize_minmax(E, D, plan, bits=bits)
    torch.cuda.synchronize()
    ab = pm.scales.cpu().numpy()
    for l in layers:
        a, b = int(offs[l]), int(offs[l + 1])
        co, ao, bo = orc.quantize_minmax(E_host[l], bits, np.array([0, b - a], dtype=np.int64))
        codes = _minmax_codes_at(pm, torch.arange(a, b, device="cuda"))
        assert np.array_equal(codes, co), l
        assert ab[l, 0] == np.float32(ao[0]) and ab[l, 1] == np.float32(bo[0]), l
    del W, E, W_host, E_host
    torch.cuda.empty_cache()
    # ---- one step of Alg. 1 from beta = 0
    lr, lam = wl.lr, 1e-4
    g = synth.gradient(D, wl.sigma_g, seed=0, step=0, device="cuda")
    beta = torch.zeros((L, n), device="cuda")
    S = torch.empty((L, n), device="cuda")
    twa.beta_step(pm, g, plan, beta, lr, lam, S=S)
    w = twa.weights_from_beta(pm, beta, plan, wbar)
    torch.cuda.synchronize()
    cols = [0, 57, n - 1]
    So = orc.project_layers(to_oracle(pm, cols=cols, layer_off=offs), g.cpu().numpy().astype(np.float64), offs)
    e_s = rel_l2(S[:, cols].cpu().numpy(), So)
    say("  rel_l2 S[:, sampled]", e_s)
    assert e_s <= REL_L2_TOL
    beta_o = np.zeros((L, n))
    orc.beta_step(beta_o, S.cpu().numpy().astype(np.float64), float(np.float32(lr)), float(np.float32(lam)))
    assert rel_l2(beta.cpu().numpy(), beta_o) <= REL_L2_TOL
    # w on sampled 128-element blocks: next to layer boundaries, first, last, random
    block = 128
    nb = D // block
    r = np.random.default_rng(7)
    near = [int(o) // block for o in offs[1:-1]] + [max(0, int(o) // block - 1) for o in offs[1:-1]]
    ids = sorted(set([0, nb - 1] + r.integers(0, nb, size=48).tolist() + r.choice(near, size=40).tolist()))
    rows = torch.cat([torch.arange(b * block, (b + 1) * block) for b in ids]).cuda()
    codes = _minmax_codes_at(pm, rows)
    rows_np = rows.cpu().numpy()
    off_sub = np.searchsorted(rows_np, offs, side="left").astype(np.int64)
    po = orc.Pmat(orc.MM, int(rows.numel()), np.ascontiguousarray(codes), np.ascontiguousarray(ab, dtype=np.float32), 0, 1.0,
                  off_sub)
    wo = orc.weights_from_beta(po, beta.cpu().numpy().astype(np.float64), off_sub, wbar[rows].cpu().numpy().astype(np.float64))
    e_w = rel_l2(w[rows].cpu().numpy(), wo)
    e_d = rel_l2((w[rows] - wbar[rows]).double().cpu().numpy(), wo - wbar[rows].cpu().numpy().astype(np.float64))
    say("  rel_l2 w[sampled]", e_w, "displacement", e_d)
    assert e_w <= REL_L2_TOL and e_d <= REL_L2_TOL
    assert torch.isfinite(w).all()
    if bits != 4:
        return
    # the paper's default width once more, exhaustively: every entry of S and every element of w against the oracle
    # on the whole stored matrix (codes spread out to one per element on the host)
    del po
    po = to_oracle(pm, layer_off=offs)
    g_h = g.cpu().numpy().astype(np.float64)
    So = orc.project_layers(po, g_h, offs)
    S_h = S.cpu().numpy().astype(np.float64)
    e_s, m_s = rel_l2(S_h, So), float(np.max(np.abs(S_h - So))) / rms(So.sum(axis=0))
    say(f"  whole: S: rel_l2 {e_s:.2e}, max|err|/rms(s) {m_s:.2e}")
    assert e_s <= REL_L2_TOL and m_s <= MAX_ABS_TOL
    wbar_h = wbar.cpu().numpy().astype(np.float64)
    wo = orc.weights_from_beta(po, beta.cpu().numpy().astype(np.float64), offs, wbar_h)
    w_h = w.cpu().numpy().astype(np.float64)
    d_ref = wo - wbar_h
    e_w, e_d = rel_l2(w_h, wo), rel_l2(w_h - wbar_h, d_ref)
    # per element: the displacement P beta within the bar of g~, w itself within half an ulp more (one addition).
    # The basis is normalised PER LAYER, so the size of the displacement differs by orders of magnitude between a
    # 64-element normalisation vector and a 2.4 M-element convolution: the bar is taken against the layer's own rms.
    sizes = np.diff(offs)
    live = sizes > 0
    layer_ms = np.zeros(L)
    layer_ms[live] = np.add.reduceat(d_ref * d_ref, offs[:-1][live]) / sizes[live]
    bar = MAX_ABS_TOL * np.repeat(np.sqrt(layer_ms), sizes)
    over = np.abs(w_h - wo) - (HALF_ULP * np.abs(wo) + bar)
    say(f"  whole: w: rel_l2 {e_w:.2e}, displacement rel_l2 {e_d:.2e}, worst excess over the per-element bar {float(over.max()):.2e}")
    assert e_w <= REL_L2_TOL and float(over.max()) <= 0.0
