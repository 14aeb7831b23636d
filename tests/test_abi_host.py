"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol that
include/twa.h declares, sizes buffers as the paper's memory table says, and rejects bad arguments
with the documented status codes before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2205_13104_amd import binding as twa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "twa.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(twa_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    L = twa.lib()
    names = declared_symbols()
    assert {"twa_build_basis", "twa_quantize", "twa_project", "twa_expand_update"} <= set(names)
    for nm in names:
        assert hasattr(L, nm), nm
    assert L.twa_version() >= 100
    assert twa.strerror(0) == "success" and "NULL" in twa.strerror(twa.ERR_NULL)


def test_pmat_bytes_follow_the_memory_table():
    # Sec. 4.6: 4nD bytes at 32 bits, nBD/8 bytes of codes at B bits (here D is padded to a multiple of 128)
    D, n = 25_557_032, 100
    ld, db, sb = twa.pmat_bytes(twa.F32, D, n)
    assert ld == (D + 127) // 128 * 128 and db == 4 * n * ld and sb == 0
    ld, db, sb = twa.pmat_bytes(twa.I8, D, n, 128)
    assert ld == (D + 2047) // 2048 * 2048 and db == n * 8 * ld // 8 and sb == n * (ld // 128) * 4
    ld, db, sb = twa.pmat_bytes(twa.I4, D, n, 64)
    assert ld == (D + 2047) // 2048 * 2048 and db == n * 4 * ld // 8 and sb == n * (ld // 64) * 2
    ld, db, sb = twa.pmat_bytes(twa.BF16, D, n)
    assert db == 2 * n * ld
    with pytest.raises(twa.TwaError) as e:
        twa.pmat_bytes(twa.I8, D, n, 100)          # block must be a power of two
    assert e.value.code == twa.ERR_SHAPE
    with pytest.raises(twa.TwaError) as e:
        twa.pmat_bytes(99, D, n)
    assert e.value.code == twa.ERR_DTYPE
    # the paper's formats at B bits: nBD/8 bytes of codes (the 8L bytes of factors are the caller's)
    for dt, B in ((twa.U16MM, 16), (twa.U8MM, 8), (twa.U4MM, 4), (twa.U3MM, 3), (twa.U2MM, 2), (twa.U1MM, 1)):
        ld, db, sb = twa.pmat_bytes(dt, D, n)
        assert ld == (D + 2047) // 2048 * 2048 and db == n * B * ld // 8 and sb == 0
    with pytest.raises(twa.TwaError) as e:
        twa.pmat_bytes(twa.F32, D, 129)
    assert e.value.code == twa.ERR_SHAPE
    with pytest.raises(twa.TwaError) as e:
        twa.pmat_bytes(twa.F32, 2 ** 31, 1)        # one fp32 vector must stay below 4 GiB
    assert e.value.code == twa.ERR_SHAPE


def _pm(dtype=twa.F32, n=4, D=1000, ld=1024, data=0x1000, scales=0, block=0, gscale=1.0):
    return twa._Pmat(dtype, n, D, ld, data, scales, block, gscale)


def _project(pm, g=0x2000, k=1, ldg=0, s=0x3000, ws=0x4000, wsb=None):
    if wsb is None:
        wsb = twa.project_workspace_bytes(max(1, min(pm.n, 128)), max(1, min(k, 8)))
    return twa.lib().twa_project(C.byref(pm), g, k, ldg, s, ws, wsb, None)


def test_project_argument_errors():
    assert twa.lib().twa_project(None, 0x2000, 1, 0, 0x3000, 0x4000, 1 << 30, None) == twa.ERR_NULL
    assert _project(_pm(data=0)) == twa.ERR_NULL
    assert _project(_pm(), g=0) == twa.ERR_NULL
    assert _project(_pm(), s=0) == twa.ERR_NULL
    assert _project(_pm(dtype=99)) == twa.ERR_DTYPE
    assert _project(_pm(n=0)) == twa.ERR_SHAPE
    assert _project(_pm(n=129)) == twa.ERR_SHAPE
    assert _project(_pm(D=0)) == twa.ERR_SHAPE
    assert _project(_pm(D=2000)) == twa.ERR_SHAPE            # ld < D
    assert _project(_pm(ld=1000)) == twa.ERR_ALIGN           # ld not a multiple of 128
    assert _project(_pm(data=0x1004)) == twa.ERR_ALIGN
    assert _project(_pm(), g=0x2004) == twa.ERR_ALIGN
    assert _project(_pm(), k=0) == twa.ERR_SHAPE
    assert _project(_pm(), k=9) == twa.ERR_SHAPE
    assert _project(_pm(), k=2, ldg=999) == twa.ERR_SHAPE    # ldg < D
    assert _project(_pm(), ws=0) == twa.ERR_WORKSPACE
    assert _project(_pm(), wsb=16) == twa.ERR_WORKSPACE
    assert _project(_pm(dtype=twa.I8, block=128, ld=2048)) == twa.ERR_NULL          # scales missing
    assert _project(_pm(dtype=twa.I8, block=100, scales=0x5000, ld=2048)) == twa.ERR_SHAPE
    assert _project(_pm(dtype=twa.I8, block=128, scales=0x5000, ld=1024)) == twa.ERR_ALIGN    # ld % 2048 for int8
    assert _project(_pm(dtype=twa.I4, block=64, scales=0x5000, ld=2048, gscale=3.0)) == twa.ERR_SHAPE   # not 2^k
    assert _project(_pm(dtype=twa.I4, block=64, scales=0x5000, ld=2048, gscale=0.0)) == twa.ERR_SHAPE


def test_other_entry_points_argument_errors():
    L = twa.lib()
    pm = _pm()
    assert L.twa_expand_update(C.byref(pm), 0, 0x3000, 0.1, None, None) == twa.ERR_NULL
    assert L.twa_expand_update(C.byref(pm), 0x2000, 0, 0.1, None, None) == twa.ERR_NULL
    assert L.twa_expand_update(C.byref(pm), 0x2000, 0x3004, 0.1, None, None) == twa.ERR_ALIGN
    out = _pm(dtype=twa.I8, block=128, scales=0x5000, ld=2048)
    assert L.twa_quantize(None, 1000, 4, 1024, C.byref(out), None) == twa.ERR_NULL
    assert L.twa_quantize(0x6000, 1000, 5, 1024, C.byref(out), None) == twa.ERR_SHAPE     # n mismatch
    assert L.twa_quantize(0x6000, 1000, 4, 1000, C.byref(out), None) == twa.ERR_ALIGN     # ldp
    bad = _pm(dtype=twa.I4, block=64, scales=0x5000, ld=2048, gscale=0.3)
    assert L.twa_quantize(0x6000, 1000, 4, 1024, C.byref(bad), None) == twa.ERR_SHAPE
    wsb = twa.build_basis_workspace_bytes(4)
    assert L.twa_build_basis(None, 1000, 4, 1024, 0x7000, 1024, None, 0x8000, wsb, None) == twa.ERR_NULL
    assert L.twa_build_basis(0x6000, 3, 4, 128, 0x7000, 128, None, 0x8000, wsb, None) == twa.ERR_SHAPE   # n > D
    assert L.twa_build_basis(0x6000, 1000, 4, 1024, 0x7000, 1024, None, 0x8000, 8, None) == twa.ERR_WORKSPACE
    assert L.twa_build_basis(0x6000, 1000, 4, 1024, 0x6000, 2048, None, 0x8000, wsb, None) == twa.ERR_SHAPE  # alias


def test_layerwise_entry_points_argument_errors():
    L = twa.lib()
    nb = C.c_size_t()
    assert L.twa_layer_plan_bytes(161, C.byref(nb)) == twa.OK and nb.value == 16 + 162 * 16      # header {magic, L, D} + three tables
    assert L.twa_layer_plan_bytes(0, C.byref(nb)) == twa.ERR_SHAPE
    assert L.twa_layer_plan_bytes(twa.MAX_LAYERS + 1, C.byref(nb)) == twa.ERR_SHAPE
    assert L.twa_layer_plan(None, 3, 1000, 0x9000, 1 << 20, None) == twa.ERR_NULL
    assert L.twa_layer_plan(0x8000, 3, 1000, 0x9000, 8, None) == twa.ERR_WORKSPACE
    assert L.twa_layer_plan(0x8004, 3, 1000, 0x9000, 1 << 20, None) == twa.ERR_ALIGN
    assert L.twa_layer_plan(0x8000, 3, 0, 0x9000, 1 << 20, None) == twa.ERR_SHAPE
    assert L.twa_project_layers_workspace_bytes(100, 161, C.byref(nb)) == twa.OK
    assert nb.value == (2048 + 161) * 101 * 4            # partial sums per (workgroup + layer) slot, n + 1 numbers each
    pm = _pm()
    wsb = nb.value
    assert L.twa_project_layers(C.byref(pm), 0x2000, None, 2, 0x3000, 0x4000, wsb, None) == twa.ERR_NULL
    assert L.twa_project_layers(C.byref(pm), 0x2000, 0x9000, 2, None, 0x4000, wsb, None) == twa.ERR_NULL
    assert L.twa_project_layers(C.byref(pm), 0x2000, 0x9000, 0, 0x3000, 0x4000, wsb, None) == twa.ERR_SHAPE
    assert L.twa_project_layers(C.byref(pm), 0x2000, 0x9004, 2, 0x3000, 0x4000, wsb, None) == twa.ERR_ALIGN
    assert L.twa_project_layers(C.byref(pm), 0x2000, 0x9000, 2, 0x3000, 0x4000, 64, None) == twa.ERR_WORKSPACE
    assert L.twa_beta_step(C.byref(pm), 0x2000, 0x9000, 2, None, 0.1, 0.0, None, 0x4000, wsb, None) == twa.ERR_NULL
    assert L.twa_expand_update_layers(C.byref(pm), None, 0x9000, 2, 0x3000, 0.1, None, None) == twa.ERR_NULL
    assert L.twa_expand_update_layers(C.byref(pm), 0x2000, 0x9000, 2, 0x3004, 0.1, None, None) == twa.ERR_ALIGN
    assert L.twa_weights_from_beta(C.byref(pm), 0x2000, 0x9000, 2, None, 0x3000, None) == twa.ERR_NULL
    assert L.twa_beta_update(0x2000, 0x3000, -1, 0.1, 0.0, None) == twa.ERR_SHAPE
    # the coefficient step with the base optimiser
    opt = lambda **k: C.byref(twa.OptimStruct(k.get("kind", twa.OPT_ADAM), 0.1, 0.0, k.get("mu", 0.9), k.get("beta2", 0.99),
                                              k.get("eps", 1e-8), k.get("t", 1)))
    assert L.twa_beta_optim(None, 0x2000, 0x3000, 0x4000, 0x5000, 8, None) == twa.ERR_NULL
    assert L.twa_beta_optim(opt(), 0x2000, 0x3000, None, 0x5000, 8, None) == twa.ERR_NULL
    assert L.twa_beta_optim(opt(), 0x2000, 0x3000, 0x4000, None, 8, None) == twa.ERR_NULL
    assert L.twa_beta_optim(opt(kind=9), 0x2000, 0x3000, 0x4000, 0x5000, 8, None) == twa.ERR_DTYPE
    assert L.twa_beta_optim(opt(t=0), 0x2000, 0x3000, 0x4000, 0x5000, 8, None) == twa.ERR_SHAPE
    assert L.twa_beta_optim(opt(mu=1.5), 0x2000, 0x3000, 0x4000, 0x5000, 8, None) == twa.ERR_SHAPE
    assert L.twa_beta_optim(opt(eps=-1.0), 0x2000, 0x3000, 0x4000, 0x5000, 8, None) == twa.ERR_SHAPE
    assert L.twa_beta_optim(opt(), 0x2000, 0x3002, 0x4000, 0x5000, 8, None) == twa.ERR_ALIGN
    # the paper's min-max format: layer-wise calls only, factors required
    mm = _pm(dtype=twa.U4MM, ld=2048, scales=0)
    assert L.twa_project_layers(C.byref(mm), 0x2000, 0x9000, 2, 0x3000, 0x4000, wsb, None) == twa.ERR_NULL
    mm = _pm(dtype=twa.U8MM, ld=2048, scales=0x5000, block=9)            # a byte holds codes of at most 8 bits
    assert L.twa_project_layers(C.byref(mm), 0x2000, 0x9000, 2, 0x3000, 0x4000, wsb, None) == twa.ERR_SHAPE
    mm = _pm(dtype=twa.U4MM, ld=1024, scales=0x5000)
    assert L.twa_project_layers(C.byref(mm), 0x2000, 0x9000, 2, 0x3000, 0x4000, wsb, None) == twa.ERR_ALIGN
    out = _pm(dtype=twa.I8, block=128, scales=0x5000, ld=2048)
    assert L.twa_quantize_minmax(0x6000, 1000, 4, 1024, 0x9000, 2, 8, C.byref(out), 0x4000, 1 << 20, None) == twa.ERR_DTYPE
    out = _pm(dtype=twa.U8MM, scales=0x5000, ld=2048)
    assert L.twa_quantize_minmax(0x6000, 1000, 4, 1024, 0x9000, 2, 8, C.byref(out), 0x4000, 8, None) == twa.ERR_WORKSPACE
    assert L.twa_quantize_minmax(0x6000, 1000, 5, 1024, 0x9000, 2, 8, C.byref(out), 0x4000, 1 << 20, None) == twa.ERR_SHAPE
    assert L.twa_quantize_minmax(0x6000, 1000, 4, 1024, 0x9000, 2, 9, C.byref(out), 0x4000, 1 << 20, None) == twa.ERR_SHAPE
    out = _pm(dtype=twa.U4MM, scales=0x5000, ld=2048)
    assert L.twa_quantize_minmax(0x6000, 1000, 4, 1024, 0x9000, 2, 5, C.byref(out), 0x4000, 1 << 20, None) == twa.ERR_SHAPE
    out = _pm(dtype=twa.U16MM, scales=0x5000, ld=2048)
    assert L.twa_quantize_minmax(0x6000, 1000, 4, 1024, 0x9000, 2, 17, C.byref(out), 0x4000, 1 << 20, None) == twa.ERR_SHAPE
    assert L.twa_centre_normalise(0x6000, 1000, 4, 1024, 0x9000, 2, None, 0x7000, 1024, None, 0x4000, 1 << 30,
                                  None) == twa.ERR_NULL
    assert L.twa_centre_normalise(0x6000, 1000, 4, 1000, 0x9000, 2, 0xa000, 0x7000, 1024, None, 0x4000, 1 << 30,
                                  None) == twa.ERR_ALIGN


def test_valid_call_without_a_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    # every argument is acceptable, so the only thing missing is the device: no silent fallback
    assert _project(_pm()) == twa.ERR_NO_DEVICE


def test_panel_calls_argument_errors():
    L = twa.lib()
    gb, rb, wb = C.c_size_t(), C.c_size_t(), C.c_size_t()
    assert L.twa_basis_state_bytes(100, C.byref(gb), C.byref(rb), C.byref(wb)) == twa.OK
    assert gb.value == 112 * 112 * 8 and rb.value == 112 * 112 * 4 and wb.value == 512 * 112 * 112 * 8
    assert L.twa_basis_state_bytes(129, C.byref(gb), C.byref(rb), C.byref(wb)) == twa.ERR_SHAPE
    assert L.twa_basis_state_bytes(4, None, C.byref(rb), C.byref(wb)) == twa.ERR_NULL
    big = 1 << 30
    assert L.twa_gram_accumulate(None, 1000, 4, 1024, 0x2000, 0, 0x4000, big, None) == twa.ERR_NULL
    assert L.twa_gram_accumulate(0x1000, 1000, 4, 1024, None, 0, 0x4000, big, None) == twa.ERR_NULL
    assert L.twa_gram_accumulate(0x1000, 1000, 4, 999, 0x2000, 0, 0x4000, big, None) == twa.ERR_SHAPE     # stride < rows
    assert L.twa_gram_accumulate(0x1000, 1000, 4, 1002, 0x2000, 0, 0x4000, big, None) == twa.ERR_ALIGN     # stride % 4
    assert L.twa_gram_accumulate(0x1004, 1000, 4, 1024, 0x2000, 0, 0x4000, big, None) == twa.ERR_ALIGN
    assert L.twa_gram_accumulate(0x1000, 1000, 4, 1024, 0x2000, 0, 0x4000, 64, None) == twa.ERR_WORKSPACE
    assert L.twa_gram_accumulate(0x1000, 1000, 4, 1024, 0x2000, 4, 0x4000, big, None) == twa.ERR_SHAPE     # unknown flag
    assert L.twa_gram_factor(None, 4, 0x3000, None, 0, None) == twa.ERR_NULL
    assert L.twa_gram_factor(0x2000, 4, 0x3000, None, 1, None) == twa.ERR_NULL                            # compose needs R
    assert L.twa_gram_factor(0x2000, 0, 0x3000, None, 0, None) == twa.ERR_SHAPE
    assert L.twa_apply_rinv(0x1000, 1000, 4, 1024, None, 0x5000, 1024, None) == twa.ERR_NULL
    assert L.twa_apply_rinv(0x1000, 1000, 4, 1024, 0x3000, 0x5000, 996, None) == twa.ERR_SHAPE
    assert L.twa_apply_rinv(0x1000, 1000, 4, 1024, 0x3000, 0x1000, 2048, None) == twa.ERR_SHAPE            # in place: same stride


def test_read_probe_argument_errors():
    L = twa.lib()
    assert L.twa_probe_read(None, 1 << 20, 0x2000, None) == twa.ERR_NULL
    assert L.twa_probe_read(0x1000, 1 << 20, None, None) == twa.ERR_NULL
    assert L.twa_probe_read(0x1000, 8, 0x2000, None) == twa.ERR_SHAPE
    assert L.twa_probe_read(0x1008, 1 << 20, 0x2000, None) == twa.ERR_ALIGN


def test_project_noalloc_argument_errors():
    """The entry point that allocates nothing: its size limit and the usual argument errors, all on the host."""
    L = twa.lib()

    def call(pm, g=0x2000, k=1, ldg=0, s=0x3000):
        return L.twa_project_noalloc(C.byref(pm), g, k, ldg, s, None)

    assert L.twa_project_noalloc(None, 0x2000, 1, 0, 0x3000, None) == twa.ERR_NULL
    assert call(_pm(), g=0) == twa.ERR_NULL and call(_pm(), s=0) == twa.ERR_NULL
    assert call(_pm(dtype=99)) == twa.ERR_DTYPE
    assert call(_pm(), k=9) == twa.ERR_SHAPE
    assert call(_pm(), g=0x2004) == twa.ERR_ALIGN
    assert call(_pm(n=100), k=8, ldg=1024) == twa.ERR_LIMIT          # n * k = 800 > 512
    assert call(_pm(n=128), k=5, ldg=1024) == twa.ERR_LIMIT
    assert call(_pm(n=64), k=8, ldg=1024) in (twa.ERR_NO_DEVICE, twa.ERR_HIP)      # at the limit: goes on to the device
    assert call(_pm(n=128), k=4, ldg=996) == twa.ERR_SHAPE           # inside the limit; ldg < D
    assert "fixed device array" in twa.strerror(twa.ERR_LIMIT)


def test_launch_knobs_are_explicit_and_bounded():
    """The library reads no environment variable; its launch geometry changes only through this call."""
    L = twa.lib()
    assert L.twa_set_launch_knob(twa.KNOB_PROJECT_GRID, 7) == twa.OK
    assert L.twa_set_launch_knob(twa.KNOB_PROJECT_GRID, 0) == twa.OK
    assert L.twa_set_launch_knob(twa.KNOB_EXPAND_GRID, 2048) == twa.OK
    assert L.twa_set_launch_knob(twa.KNOB_EXPAND_GRID, 0) == twa.OK
    assert L.twa_set_launch_knob(twa.KNOB_EXPAND_GRID, 2049) == twa.ERR_SHAPE
    assert L.twa_set_launch_knob(twa.KNOB_BASIS_WGS_PER_CU, -1) == twa.ERR_SHAPE
    assert L.twa_set_launch_knob(3, 1) == twa.ERR_DTYPE and L.twa_set_launch_knob(-1, 1) == twa.ERR_DTYPE
    src = "".join(open(os.path.join(ROOT, "paper_2205_13104_amd", "csrc", f)).read()
                  for f in os.listdir(os.path.join(ROOT, "paper_2205_13104_amd", "csrc")))
    assert "getenv" not in src


def test_fused_second_pass_and_absmax_argument_errors():
    L = twa.lib()
    out = _pm(dtype=twa.I8, n=4, D=5000, ld=6144, data=0x100000, scales=0x200000, block=128)

    def call(W=0x6000, rows=5000, n=4, ldw=6144, rinv=0x7000, desc=out, row0=0):
        return L.twa_apply_rinv_quantize(W, rows, n, ldw, rinv, C.byref(desc), row0, None)

    assert call(W=None) == twa.ERR_NULL and call(rinv=None) == twa.ERR_NULL
    assert L.twa_apply_rinv_quantize(0x6000, 5000, 4, 6144, 0x7000, None, 0, None) == twa.ERR_NULL
    assert call(n=5) == twa.ERR_SHAPE                                   # the descriptor says 4 vectors
    assert call(rows=2048, row0=1024) == twa.ERR_ALIGN                  # panels start on multiples of 2048 rows ...
    assert call(rows=1000) == twa.ERR_ALIGN                             # ... and end there unless they end the matrix
    assert call(rows=4096, row0=2048) == twa.ERR_SHAPE                  # past the end of the matrix
    assert call(desc=_pm(dtype=twa.I8, n=4, D=5000, ld=6144, data=0x100000, scales=0, block=128)) == twa.ERR_NULL
    assert call(desc=_pm(dtype=twa.I8, n=4, D=5000, ld=6144, data=0x100000, scales=0x200000, block=256)) == twa.ERR_SHAPE
    assert call(desc=_pm(dtype=twa.I4, n=4, D=5000, ld=6144, data=0x100000, scales=0x200000, block=64, gscale=0.0)) == twa.ERR_SHAPE
    assert call(desc=_pm(dtype=twa.U4MM, n=4, D=5000, ld=6144, data=0x100000, scales=0x200000)) == twa.ERR_DTYPE
    assert call(desc=_pm(dtype=twa.I8, n=4, D=5000, ld=6144, data=0x6000 + 64, scales=0x200000, block=128)) == twa.ERR_SHAPE  # overlap
    assert call() == twa.ERR_NO_DEVICE                                  # a valid call goes on to the device
    assert L.twa_absmax_accumulate(None, 100, 4, 128, 0x9000, 0, None) == twa.ERR_NULL
    assert L.twa_absmax_accumulate(0x6000, 100, 4, 128, None, 0, None) == twa.ERR_NULL
    assert L.twa_absmax_accumulate(0x6000, 100, 4, 64, 0x9000, 0, None) == twa.ERR_SHAPE      # ld < rows
    assert L.twa_absmax_accumulate(0x6000, 100, 4, 128, 0x9002, 0, None) == twa.ERR_ALIGN


def test_gscale_for_absmax_is_the_rule_of_the_four_bit_format():
    # 2^(floor(log2(amax / 7)) - 14); the oracle states the same rule from its own code
    import numpy as np
    from oracle import twa_oracle as orc
    assert twa.gscale_for_absmax(0.0) == 1.0
    assert twa.gscale_for_absmax(7.0) == 2.0 ** -14 and twa.gscale_for_absmax(13.99) == 2.0 ** -14
    assert twa.gscale_for_absmax(14.0) == 2.0 ** -13
    for amax in (3.1e-4, 5.5e-5, 0.02, 1.0, 6.9999, 123.0):
        p = np.zeros((1, 64), dtype=np.float32)
        p[0, 3] = -amax
        assert twa.gscale_for_absmax(float(np.float32(amax))) == orc.gscale_i4(p)


def test_async_basis_argument_errors():
    L = twa.lib()
    wsb = twa.build_basis_workspace_bytes(4)
    assert L.twa_build_basis_async(None, 1000, 4, 1024, 0x7000, 1024, None, 0x9000, 0x8000, wsb, None) == twa.ERR_NULL
    assert L.twa_build_basis_async(0x6000, 1000, 4, 1024, 0x7000, 1024, None, None, 0x8000, wsb, None) == twa.ERR_NULL   # status
    assert L.twa_build_basis_async(0x6000, 3, 4, 128, 0x7000, 128, None, 0x9000, 0x8000, wsb, None) == twa.ERR_SHAPE    # n > D
    assert L.twa_build_basis_async(0x6000, 1000, 4, 1024, 0x7000, 1024, 0xA004, 0x9000, 0x8000, wsb, None) == twa.ERR_ALIGN
    assert L.twa_build_basis_async(0x6000, 1000, 4, 1024, 0x7000, 1024, None, 0x9000, 0x8000, 8, None) == twa.ERR_WORKSPACE
    assert L.twa_build_basis_async(0x6000, 1000, 4, 1024, 0x7000, 1024, None, 0x9000, 0x8000, wsb, None) == twa.ERR_NO_DEVICE
    assert L.twa_gram_factor_async(None, 4, 0x7000, None, 0x9000, None) == twa.ERR_NULL
    assert L.twa_gram_factor_async(0x6000, 4, 0x7000, None, None, None) == twa.ERR_NULL
    assert L.twa_gram_factor_async(0x6000, 129, 0x7000, None, 0x9000, None) == twa.ERR_SHAPE
    assert L.twa_gram_factor_async(0x6000, 4, 0x7000, None, 0x9000, None) == twa.ERR_NO_DEVICE
