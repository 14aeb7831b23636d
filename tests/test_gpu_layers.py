"""Parity of the layer-wise calls (Sec. 4.5, Alg. 1) of the HIP library against the fp64 oracle on the
same stored P: S (L x n), g~ and w within a relative L2 error of 1e-5, for every storage type, with
layer tables that put boundaries at odd positions, several boundaries into one tile and into one
128-bit vector, one-element and empty layers, and layers that span many tiles and workgroups."""
import numpy as np
import pytest
import torch

from oracle import twa_oracle as orc
from paper_2205_13104_amd import binding as twa
from paper_2205_13104_amd import synth
from tests.gpu_common import REL_L2_TOL, random_basis_like, rel_l2, store_as, to_oracle

pytestmark = pytest.mark.gpu

DTYPES = [twa.F32, twa.BF16, twa.I8, twa.I4]
NAMES = {twa.F32: "f32", twa.BF16: "bf16", twa.I8: "i8", twa.I4: "i4"}


def say(*a):
    print(*a, flush=True)


def hand_made_sizes(D):
    """Boundaries inside one 128-bit vector, one-element and empty layers, then long layers."""
    head = [5, 1, 1, 0, 2, 30, 64, 64, 0, 0, 3, 2048, 1000, 4097, 17]
    assert D > sum(head) + 10
    rest = D - sum(head)
    return head + [rest // 2, 0, rest - rest // 2 - 1, 1]


def layer_tables(D):
    yield "hand", hand_made_sizes(D)
    yield "random40", synth.random_layer_sizes(D, 40, seed=D % 97)
    yield "random700", synth.random_layer_sizes(D, 700, seed=5)
    yield "one", [D]
    yield "ends_empty", [0, D, 0]


def check_layers(D, n, dtype, name, sizes, seed):
    off_cpu = synth.layer_offsets(sizes)
    L = len(sizes)
    off = twa.LayerPlan(off_cpu, D)
    P32 = random_basis_like(D, n, seed=seed)
    pm = store_as(P32, D, dtype)
    po = to_oracle(pm)
    g = synth.gradient(D, 1e-2, seed=seed, device="cuda")
    say("layers", NAMES[dtype], "D", D, "n", n, name, "L", L)

    S = twa.project_layers(pm, g, off)
    torch.cuda.synchronize()
    S_ref = orc.project_layers(po, g.cpu().numpy().astype(np.float64), off_cpu.numpy())
    Sg = S.cpu().numpy()
    assert Sg.shape == (L, n)
    assert rel_l2(Sg, S_ref) <= REL_L2_TOL
    scale = np.abs(S_ref).max()
    for l in range(L):
        if sizes[l] == 0:
            assert np.all(Sg[l] == 0.0)
        else:
            # row by row, against the row's own size or (for rows that cancel to almost nothing) the largest entry
            assert np.linalg.norm(Sg[l] - S_ref[l]) <= REL_L2_TOL * max(np.linalg.norm(S_ref[l]), scale), (l, sizes[l])

    # expansion with coefficients of its own (not the projection's output): every row matters
    gen = torch.Generator().manual_seed(seed + 1)
    S2 = torch.randn((L, n), generator=gen, dtype=torch.float32).cuda()
    w0 = synth.gradient(D, 0.05, seed=seed + 2, device="cuda")
    for want_gt in (True, False):
        w = w0.clone()
        gt = torch.full((D,), float("nan"), device="cuda") if want_gt else None
        twa.expand_update_layers(pm, S2, off, w, 0.1, gt)
        torch.cuda.synchronize()
        w_ref = w0.cpu().numpy().astype(np.float64)
        gt_ref = orc.expand_update_layers(po, S2.cpu().numpy().astype(np.float64), off_cpu.numpy(), w_ref,
                                          float(np.float32(0.1)), want_gt=True)
        if want_gt:
            assert rel_l2(gt.cpu().numpy(), gt_ref) <= REL_L2_TOL
            # layer by layer as well: a wrong row for a small layer must not hide in the total
            # (against the layer's own norm, or for a few elements that cancel to almost nothing the typical size)
            gg = gt.cpu().numpy()
            rms = float(np.sqrt(np.mean(gt_ref ** 2)))
            for l in range(L):
                a, b = int(off_cpu[l]), int(off_cpu[l + 1])
                if b > a:
                    bound = max(np.linalg.norm(gt_ref[a:b]), rms * (b - a) ** 0.5)
                    assert np.linalg.norm(gg[a:b] - gt_ref[a:b]) <= REL_L2_TOL * bound, (l, a, b)
        assert rel_l2(w.cpu().numpy(), w_ref) <= REL_L2_TOL


@pytest.mark.parametrize("dtype", DTYPES, ids=[NAMES[d] for d in DTYPES])
@pytest.mark.parametrize("D,n", [(70001, 7), (300_017, 100), (1_234_567, 33)])
def test_layers_match_oracle(dtype, D, n):
    for name, sizes in layer_tables(D):
        check_layers(D, n, dtype, name, sizes, seed=D % 1000 + n)


@pytest.mark.parametrize("dtype", DTYPES, ids=[NAMES[d] for d in DTYPES])
def test_layers_n128_many_workgroups(dtype):
    D = 9_000_011
    check_layers(D, 128, dtype, "random40", synth.random_layer_sizes(D, 40, seed=3), seed=77)


@pytest.mark.parametrize("dtype", [twa.F32, twa.I8, twa.I4], ids=["f32", "i8", "i4"])
def test_the_largest_layer_table(dtype):
    """TWA_MAX_LAYERS layers: mostly one to a few elements each, some empty, so that nearly every tile holds
    the boundaries of hundreds of layers."""
    D, n, L = 150_001, 5, 65536
    gen = np.random.default_rng(12)
    cuts = np.sort(gen.integers(0, D + 1, size=L - 1))
    sizes = np.diff(np.concatenate([[0], cuts, [D]])).tolist()
    assert len(sizes) == L and sum(sizes) == D
    check_layers(D, n, dtype, "max", sizes, seed=5)


@pytest.mark.parametrize("dtype", DTYPES, ids=[NAMES[d] for d in DTYPES])
def test_one_layer_reproduces_the_whole_model_calls_bit_for_bit(dtype):
    D, n = 2_000_003, 100
    pm = store_as(random_basis_like(D, n, seed=9), D, dtype)
    g = synth.gradient(D, 1e-2, seed=9, device="cuda")
    off = twa.LayerPlan([0, D], D)
    s = twa.project(pm, g)
    S = twa.project_layers(pm, g, off)
    assert torch.equal(S[0], s)
    w1 = synth.gradient(D, 0.05, seed=10, device="cuda")
    w2 = w1.clone()
    twa.expand_update(pm, s, w1, 0.25)
    twa.expand_update_layers(pm, S, off, w2, 0.25)
    assert torch.equal(w1, w2)


def test_layer_rows_add_up_to_the_whole_model_projection():
    D, n = 3_000_017, 100
    pm = store_as(random_basis_like(D, n, seed=12), D, twa.I8)
    g = synth.gradient(D, 1e-2, seed=12, device="cuda")
    off = twa.LayerPlan(synth.layer_offsets(synth.random_layer_sizes(D, 300, seed=1)), D)
    S = twa.project_layers(pm, g, off)
    s = twa.project(pm, g)
    assert rel_l2(S.double().sum(0).cpu().numpy(), s.double().cpu().numpy()) <= 1e-6
    # deterministic: same bits on every call
    assert torch.equal(S, twa.project_layers(pm, g, off))


@pytest.mark.parametrize("bits,D,n", [(8, 70001, 7), (8, 300_017, 100), (8, 1_234_567, 33), (4, 70001, 7),
                                      (4, 300_017, 100), (4, 1_234_567, 33), (1, 300_017, 20), (2, 300_017, 20),
                                      (3, 70001, 7), (6, 70001, 7), (16, 70001, 7), (16, 300_017, 100),
                                      (16, 1_234_567, 33), (12, 70001, 7), (9, 300_017, 20), (5, 300_017, 20),
                                      (2, 70001, 7), (2, 1_234_567, 100), (1, 70001, 7), (1, 1_234_567, 100),
                                      (3, 300_017, 100), (3, 1_234_567, 33)])
def test_minmax_format_matches_oracle(bits, D, n):
    """The paper's own quantiser (Sec. 4.6): codes and factors bit-exact against the fp64 oracle, then the
    layer-wise step on the stored matrix within the bar."""
    for name, sizes in layer_tables(D):
        off_cpu = synth.layer_offsets(sizes)
        L = len(sizes)
        plan = twa.LayerPlan(off_cpu, D)
        P32 = random_basis_like(D, n, seed=D % 1000 + n + bits)
        P32[0, :64] = 3.0 * P32[0, :64]                         # an outlier decides a layer's range
        say("minmax", bits, "D", D, "n", n, name, "L", L)
        pm = twa.quantize_minmax(P32, D, plan, bits=bits)
        torch.cuda.synchronize()
        codes_o, a_o, b_o = orc.quantize_minmax(P32[:, :D].cpu().numpy().astype(np.float64), bits, off_cpu.numpy())
        po = to_oracle(pm, layer_off=off_cpu.numpy())
        assert np.array_equal(po.data[:, :D], codes_o)
        ab = pm.scales.cpu().numpy()
        assert np.array_equal(ab[:, 0], a_o.astype(np.float32)) and np.array_equal(ab[:, 1], b_o.astype(np.float32))
        # the stored values stay within half a step of the original
        g = synth.gradient(D, 1e-2, seed=3, device="cuda")
        S = twa.project_layers(pm, g, plan)
        S_ref = orc.project_layers(po, g.cpu().numpy().astype(np.float64), off_cpu.numpy())
        assert rel_l2(S.cpu().numpy(), S_ref) <= REL_L2_TOL
        scale = np.abs(S_ref).max()
        Sg = S.cpu().numpy()
        for l in range(L):
            assert np.linalg.norm(Sg[l] - S_ref[l]) <= REL_L2_TOL * max(np.linalg.norm(S_ref[l]), scale), (l, sizes[l])
        gen = torch.Generator().manual_seed(D + bits)
        S2 = torch.randn((L, n), generator=gen, dtype=torch.float32).cuda()
        w0 = synth.gradient(D, 0.05, seed=9, device="cuda")
        w = w0.clone()
        gt = torch.full((D,), float("nan"), device="cuda")
        twa.expand_update_layers(pm, S2, plan, w, 0.1, gt)
        torch.cuda.synchronize()
        w_ref = w0.cpu().numpy().astype(np.float64)
        gt_ref = orc.expand_update_layers(po, S2.cpu().numpy().astype(np.float64), off_cpu.numpy(), w_ref,
                                          float(np.float32(0.1)), want_gt=True)
        assert rel_l2(gt.cpu().numpy(), gt_ref) <= REL_L2_TOL
        assert rel_l2(w.cpu().numpy(), w_ref) <= REL_L2_TOL
        gg = gt.cpu().numpy()
        rms = float(np.sqrt(np.mean(gt_ref ** 2)))
        for l in range(L):
            a, b = int(off_cpu[l]), int(off_cpu[l + 1])
            if b > a:
                bound = max(np.linalg.norm(gt_ref[a:b]), rms * (b - a) ** 0.5)
                assert np.linalg.norm(gg[a:b] - gt_ref[a:b]) <= REL_L2_TOL * bound, (l, a, b)
    # the whole-model calls do not take this format
    with pytest.raises(twa.TwaError) as e:
        twa.project(pm, g)
    assert e.value.code == twa.ERR_DTYPE


@pytest.mark.parametrize("bits,top", [(4, 15.0), (4, 45.0), (8, 255.0), (8, 765.0), (2, 3.0), (16, 65535.0), (3, 7.0),
                                      (3, 21.0)])
def test_minmax_codes_at_exact_ties(bits, top):
    """Values whose quotient (p - b) / a is exactly half way between two codes, for a step a that is and is not a
    power of two: the quantiser takes these through the true quotient and rounds them to even, as the oracle does."""
    D, n = 6000, 3
    levels = (1 << bits) - 1
    a = top / levels                                       # 1 or 3: min 0, max top
    P32 = torch.zeros((n, 6144), dtype=torch.float32)
    k = torch.arange(0, 2000) % levels
    P32[0, :2000] = (k.float() + 0.5) * a                  # ties k + 1/2
    P32[1, :2000] = k.float() * a                          # exact codes
    P32[2, :2000] = (k.float() + 0.25) * a
    P32[0, 0], P32[0, 1] = 0.0, top                        # the layer's range
    gen = torch.Generator().manual_seed(4)
    P32[:, 2000:D] = torch.randn((n, D - 2000), generator=gen)
    P32 = P32.cuda()
    off = np.array([0, 2000, D], dtype=np.int64)
    plan = twa.LayerPlan(off, D)
    pm = twa.quantize_minmax(P32, D, plan, bits=bits)
    torch.cuda.synchronize()
    codes_o, a_o, b_o = orc.quantize_minmax(P32[:, :D].cpu().numpy().astype(np.float64), bits, off)
    po = to_oracle(pm, layer_off=off)
    assert a_o[0] == a and b_o[0] == 0.0
    assert np.array_equal(po.data[:, :D], codes_o)
    # and they are ties indeed: rounded to even
    q = codes_o[0, 2:2000].astype(np.int64)
    kk = k[2:2000].numpy()
    assert np.array_equal(q, np.where(kk % 2 == 0, kk, kk + 1))


def test_plan_tables():
    D = 10_000
    plan = twa.LayerPlan([0, 5, 5, 40, 2100, 2100, 9000, D], D)
    off, f2048, f1024 = plan.tables()
    assert off.tolist() == [0, 5, 5, 40, 2100, 2100, 9000, D]
    # tiles start at the layer's first element rounded down to 2048 elements
    assert f2048.tolist() == [0, 1, 1, 2, 4, 4, 8, 9]
    assert f1024.tolist() == [0, 1, 1, 2, 5, 5, 12, 14]
    # a table that breaks the rules is clamped into one that keeps them
    bad = twa.LayerPlan([7, 50, 20, -3, 99999, D], D)
    off, f2048, _ = bad.tables()
    assert off.tolist() == [0, 50, 50, 50, D, D]
    assert f2048.tolist()[-1] == 1 + 5


def test_layer_argument_errors():
    import ctypes as C
    D, n = 5000, 4
    pm = store_as(random_basis_like(D, n, seed=1), D, twa.F32)
    g = torch.zeros(D, device="cuda")
    plan = twa.LayerPlan([0, 100, D], D)
    S = torch.zeros((2, n), device="cuda")
    ws = twa.Workspace(twa.project_layers_workspace_bytes(n, 2))
    st = pm.c_struct()
    L = twa.lib()
    assert L.twa_project_layers(C.byref(st), g.data_ptr(), None, 2, S.data_ptr(), ws.ptr, ws.nbytes, None) == twa.ERR_NULL
    assert L.twa_project_layers(C.byref(st), g.data_ptr(), plan.ptr, 0, S.data_ptr(), ws.ptr, ws.nbytes,
                                None) == twa.ERR_SHAPE
    assert L.twa_project_layers(C.byref(st), g.data_ptr(), plan.ptr, twa.MAX_LAYERS + 1, S.data_ptr(), ws.ptr,
                                ws.nbytes, None) == twa.ERR_SHAPE
    assert L.twa_project_layers(C.byref(st), g.data_ptr(), plan.ptr, 2, S.data_ptr(), ws.ptr, 64,
                                None) == twa.ERR_WORKSPACE
    assert L.twa_expand_update_layers(C.byref(st), S.data_ptr(), None, 2, g.data_ptr(), 0.1, None, None) == twa.ERR_NULL
    assert L.twa_expand_update_layers(C.byref(st), S.data_ptr(), plan.ptr + 4, 2, g.data_ptr(), 0.1, None,
                                      None) == twa.ERR_ALIGN
    assert L.twa_layer_plan(plan.layer_off.data_ptr(), 2, D, plan.ptr, 8, None) == twa.ERR_WORKSPACE
    assert L.twa_layer_plan(None, 2, D, plan.ptr, 1 << 20, None) == twa.ERR_NULL


def test_a_plan_of_another_layer_table_poisons_the_result_and_touches_nothing_else():
    """A plan carries the L and D it was built for.  Handed to a call with another L or another D (the host cannot
    see into device memory, the status is TWA_OK) every kernel refuses to read its tables: the coefficients come
    back as NaN, the expansion marks w[0] and leaves everything else as it was, the quantiser's factors are NaN."""
    import ctypes as C
    D, n = 70_001, 5
    P32 = random_basis_like(D, n, seed=3, ld=(D + 2047) // 2048 * 2048)
    pm = store_as(P32, D, twa.I8)
    g = synth.gradient(D, 1e-2, seed=3, device="cuda")
    good = twa.LayerPlan([0, 100, 5000, D], D)                        # L = 3
    other_L = twa.LayerPlan([0, 100, D], D)                           # L = 2, same D
    other_D = twa.LayerPlan([0, 100, 5000, D - 2048], D - 2048)       # L = 3, another D
    lib, st = twa.lib(), pm.c_struct()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    ws = twa.Workspace(twa.project_layers_workspace_bytes(n, 3))
    S_good = twa.project_layers(pm, g, good)
    assert torch.isfinite(S_good).all()
    for bad in (other_L, other_D):
        S = torch.zeros((3, n), device="cuda")
        guard = torch.full((64,), 7.0, device="cuda")                 # right behind S in no particular place: canaries
        assert lib.twa_project_layers(C.byref(st), C.c_void_p(g.data_ptr()), C.c_void_p(bad.ptr), 3,
                                      C.c_void_p(S.data_ptr()), C.c_void_p(ws.ptr), ws.nbytes, stream) == twa.OK
        w = torch.full((D,), 0.25, device="cuda")
        gt = torch.full((D,), 0.5, device="cuda")
        assert lib.twa_expand_update_layers(C.byref(st), C.c_void_p(S_good.data_ptr()), C.c_void_p(bad.ptr), 3,
                                            C.c_void_p(w.data_ptr()), C.c_float(0.1), C.c_void_p(gt.data_ptr()),
                                            stream) == twa.OK
        beta = torch.zeros((3, n), device="cuda")
        assert lib.twa_beta_step(C.byref(st), C.c_void_p(g.data_ptr()), C.c_void_p(bad.ptr), 3,
                                 C.c_void_p(beta.data_ptr()), C.c_float(0.1), C.c_float(0.0), None, C.c_void_p(ws.ptr),
                                 ws.nbytes, stream) == twa.OK
        torch.cuda.synchronize()
        assert torch.isnan(S).all() and torch.isnan(beta).all() and torch.all(guard == 7.0)
        assert torch.isnan(w[0]) and torch.all(w[1:] == 0.25)
        assert torch.isnan(gt[0]) and torch.all(gt[1:] == 0.5)
    # the one-time producers say so as well
    E = P32.clone()
    out = twa.alloc_pmat(twa.U8MM, D, n)
    ab = torch.zeros((3, 2), device="cuda")
    st_mm = twa._Pmat(twa.U8MM, n, D, out.ld, out.data.data_ptr(), ab.data_ptr(), 8, 1.0)
    nb = C.c_size_t()
    assert lib.twa_quantize_minmax_workspace_bytes(3, C.byref(nb)) == twa.OK
    wsq = twa.Workspace(nb.value + 8)
    assert lib.twa_quantize_minmax(C.c_void_p(E.data_ptr()), D, n, E.shape[1], C.c_void_p(other_L.ptr), 3, 8, C.byref(st_mm),
                                   C.c_void_p(wsq.ptr), wsq.nbytes, stream) == twa.OK
    nbc = C.c_size_t()
    assert lib.twa_centre_normalise_workspace_bytes(D, n, 3, C.byref(nbc)) == twa.OK
    wsc = twa.Workspace(nbc.value)
    wbar = torch.zeros(D, device="cuda")
    norms = torch.zeros((3, n), device="cuda")
    E2 = torch.full_like(P32, 3.0)
    assert lib.twa_centre_normalise(C.c_void_p(P32.data_ptr()), D, n, P32.shape[1], C.c_void_p(other_L.ptr), 3,
                                    C.c_void_p(wbar.data_ptr()), C.c_void_p(E2.data_ptr()), E2.shape[1],
                                    C.c_void_p(norms.data_ptr()), C.c_void_p(wsc.ptr), wsc.nbytes, stream) == twa.OK
    torch.cuda.synchronize()
    assert torch.isnan(ab).all() and torch.isnan(norms).all()
    assert torch.isnan(E2[0, 0]) and torch.all(E2.flatten()[1:] == 3.0)
    # and the good plan still works afterwards
    assert torch.equal(twa.project_layers(pm, g, good), S_good)
