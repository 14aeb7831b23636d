"""Thin ctypes binding of ``libtwa.so`` (the C ABI declared in ``include/twa.h``).

Argument marshalling only: torch tensors provide device memory and the current stream, every
step of the path runs in the library's HIP kernels.  There is no fallback: if the library has
not been built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtwa.so")

F32, BF16, I8, I4, U8MM, U4MM, U16MM, U2MM, U1MM, U3MM = 0, 1, 2, 3, 4, 5, 6, 7, 8, 9
GRAM_ADD, GRAM_ORTHONORMAL_INPUT = 1, 2         # flags of twa_gram_accumulate
MINMAX_TYPES = (U8MM, U4MM, U16MM, U2MM, U1MM, U3MM)
BITS_OF = {F32: 32, BF16: 16, I8: 8, I4: 4, U8MM: 8, U4MM: 4, U16MM: 16, U2MM: 2, U1MM: 1, U3MM: 3}
MAX_N, MAX_K, LD_MULTIPLE, SCALE_SPAN, MAX_LAYERS = 128, 8, 128, 2048, 65536
DEFAULT_BLOCK = {I8: 128, I4: 64}

OK = 0
ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_DTYPE, ERR_WORKSPACE, ERR_RANK, ERR_HIP, ERR_NO_DEVICE, ERR_LIMIT = range(-1, -10, -1)
NOALLOC_MAX_NK = 512


class TwaError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        msg = f"{where}: {strerror(code)} (status {code})"
        if code == ERR_HIP:
            msg += f", hipError {lib().twa_last_hip_error()}"
        super().__init__(msg + (f" {detail}" if detail else ""))


OPT_MOMENTUM, OPT_ADAM, OPT_ADAMW = 0, 1, 2


class OptimStruct(C.Structure):
    """twa_optim of include/twa.h."""
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("lam", C.c_float), ("mu", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("t", C.c_int32)]


class _Pmat(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("n", C.c_int32), ("D", C.c_int64), ("ld", C.c_int64),
                ("data", C.c_void_p), ("scales", C.c_void_p), ("block", C.c_int32), ("gscale", C.c_float)]


_lib = None


def lib():
    """Load the library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2205_13104_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        L.twa_version.restype = C.c_int
        L.twa_strerror.restype = C.c_char_p
        L.twa_strerror.argtypes = [C.c_int]
        L.twa_last_hip_error.restype = C.c_int
        L.twa_pmat_bytes.argtypes = [i32, i64, i32, i32, C.POINTER(i64), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.twa_project_workspace_bytes.argtypes = [i32, i32, C.POINTER(C.c_size_t)]
        L.twa_build_basis_workspace_bytes.argtypes = [i32, C.POINTER(C.c_size_t)]
        L.twa_build_basis.argtypes = [vp, i64, i32, i64, vp, i64, vp, vp, C.c_size_t, vp]
        L.twa_probe_read.argtypes = [vp, C.c_size_t, vp, vp]
        L.twa_basis_state_bytes.argtypes = [i32, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.twa_gram_accumulate.argtypes = [vp, i64, i32, i64, vp, i32, vp, C.c_size_t, vp]
        L.twa_gram_factor.argtypes = [vp, i32, vp, vp, i32, vp]
        L.twa_apply_rinv.argtypes = [vp, i64, i32, i64, vp, vp, i64, vp]
        L.twa_quantize.argtypes = [vp, i64, i32, i64, C.POINTER(_Pmat), vp]
        L.twa_project.argtypes = [C.POINTER(_Pmat), vp, i32, i64, vp, vp, C.c_size_t, vp]
        L.twa_expand_update.argtypes = [C.POINTER(_Pmat), vp, vp, f32, vp, vp]
        L.twa_project_noalloc.argtypes = [C.POINTER(_Pmat), vp, i32, i64, vp, vp]
        L.twa_project_noalloc.restype = C.c_int
        L.twa_apply_rinv_quantize.argtypes = [vp, i64, i32, i64, vp, C.POINTER(_Pmat), i64, vp]
        L.twa_apply_rinv_quantize.restype = C.c_int
        L.twa_absmax_accumulate.argtypes = [vp, i64, i32, i64, vp, i32, vp]
        L.twa_absmax_accumulate.restype = C.c_int
        L.twa_gscale_for_absmax.argtypes = [f32]
        L.twa_gscale_for_absmax.restype = C.c_float
        L.twa_build_basis_async.argtypes = [vp, i64, i32, i64, vp, i64, vp, vp, vp, C.c_size_t, vp]
        L.twa_build_basis_async.restype = C.c_int
        L.twa_gram_factor_async.argtypes = [vp, i32, vp, vp, vp, vp]
        L.twa_gram_factor_async.restype = C.c_int
        L.twa_set_launch_knob.argtypes = [i32, i32]
        L.twa_set_launch_knob.restype = C.c_int
        L.twa_project_layers_workspace_bytes.argtypes = [i32, i32, C.POINTER(C.c_size_t)]
        L.twa_project_layers.argtypes = [C.POINTER(_Pmat), vp, vp, i32, vp, vp, C.c_size_t, vp]
        L.twa_expand_update_layers.argtypes = [C.POINTER(_Pmat), vp, vp, i32, vp, f32, vp, vp]
        L.twa_layer_plan_bytes.argtypes = [i32, C.POINTER(C.c_size_t)]
        L.twa_layer_plan.argtypes = [vp, i32, i64, vp, C.c_size_t, vp]
        L.twa_quantize_minmax_workspace_bytes.argtypes = [i32, C.POINTER(C.c_size_t)]
        L.twa_quantize_minmax.argtypes = [vp, i64, i32, i64, vp, i32, i32, C.POINTER(_Pmat), vp, C.c_size_t, vp]
        L.twa_quantize_minmax_workspace_bytes.restype = C.c_int
        L.twa_quantize_minmax.restype = C.c_int
        L.twa_centre_normalise_workspace_bytes.argtypes = [i64, i32, i32, C.POINTER(C.c_size_t)]
        L.twa_centre_normalise.argtypes = [vp, i64, i32, i64, vp, i32, vp, vp, i64, vp, vp, C.c_size_t, vp]
        L.twa_beta_update.argtypes = [vp, vp, i64, f32, f32, vp]
        L.twa_beta_optim.argtypes = [C.POINTER(OptimStruct), vp, vp, vp, vp, i64, vp]
        L.twa_beta_step.argtypes = [C.POINTER(_Pmat), vp, vp, i32, vp, f32, f32, vp, vp, C.c_size_t, vp]
        L.twa_beta_step.restype = C.c_int
        L.twa_weights_from_beta.argtypes = [C.POINTER(_Pmat), vp, vp, i32, vp, vp, vp]
        for f in (L.twa_project_layers_workspace_bytes, L.twa_project_layers, L.twa_expand_update_layers,
                  L.twa_layer_plan_bytes, L.twa_layer_plan, L.twa_centre_normalise_workspace_bytes,
                  L.twa_centre_normalise, L.twa_beta_update, L.twa_beta_optim, L.twa_weights_from_beta,
                  L.twa_basis_state_bytes, L.twa_gram_accumulate, L.twa_gram_factor, L.twa_apply_rinv,
                  L.twa_probe_read):
            f.restype = C.c_int
        for f in (L.twa_pmat_bytes, L.twa_project_workspace_bytes, L.twa_build_basis_workspace_bytes,
                  L.twa_build_basis, L.twa_quantize, L.twa_project, L.twa_expand_update):
            f.restype = C.c_int
        _lib = L
    return _lib


KNOB_PROJECT_GRID, KNOB_EXPAND_GRID, KNOB_BASIS_WGS_PER_CU = 0, 1, 2


def set_launch_knob(knob: int, value: int) -> None:
    """twa_set_launch_knob: launch geometry for tests and tuning runs (0 = the library's own choice)."""
    _check(lib().twa_set_launch_knob(int(knob), int(value)), "twa_set_launch_knob")


def strerror(code: int) -> str:
    return lib().twa_strerror(int(code)).decode()


def _check(rc: int, where: str):
    if rc != OK:
        raise TwaError(rc, where)


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def pmat_bytes(dtype: int, D: int, n: int, block: int = 0):
    """(ld, data_bytes, scale_bytes) of the smallest admissible buffers."""
    ld, db, sb = C.c_int64(), C.c_size_t(), C.c_size_t()
    _check(lib().twa_pmat_bytes(dtype, D, n, block or DEFAULT_BLOCK.get(dtype, 0), C.byref(ld), C.byref(db),
                                C.byref(sb)), "twa_pmat_bytes")
    return int(ld.value), int(db.value), int(sb.value)


def project_workspace_bytes(n: int, k: int = 1) -> int:
    b = C.c_size_t()
    _check(lib().twa_project_workspace_bytes(n, k, C.byref(b)), "twa_project_workspace_bytes")
    return int(b.value)


def build_basis_workspace_bytes(n: int) -> int:
    b = C.c_size_t()
    _check(lib().twa_build_basis_workspace_bytes(n, C.byref(b)), "twa_build_basis_workspace_bytes")
    return int(b.value)


_TORCH_OF = {F32: torch.float32, BF16: torch.bfloat16, I8: torch.int8, I4: torch.uint8, U8MM: torch.int8,
             U4MM: torch.uint8, U16MM: torch.int16, U2MM: torch.uint8, U1MM: torch.uint8, U3MM: torch.uint8}


@dataclass
class Pmat:
    """A projection matrix stored on the device: the tensors plus the C descriptor."""
    dtype: int
    D: int
    n: int
    ld: int
    data: torch.Tensor                      # (n, ld) values/codes; sub-byte codes: (n, ld * bits // 8) bytes
    scales: Optional[torch.Tensor] = None   # (ld // 2048, n, 2048 // block): float32 (I8) / float16 (I4);
                                            # min-max types: (L, 2) float32 = (a_l, b_l) per layer
    block: int = 0
    gscale: float = 1.0

    def scales_by_vector(self) -> Optional[torch.Tensor]:
        """The scales re-ordered (a copy, pure data movement) as (n, ld // block): row j = vector j."""
        if self.scales is None:
            return None
        return self.scales.permute(1, 0, 2).reshape(self.n, -1).contiguous()

    def c_struct(self) -> _Pmat:
        return _Pmat(self.dtype, self.n, self.D, self.ld, _ptr(self.data), _ptr(self.scales), self.block,
                     float(self.gscale))

    @property
    def stream_bytes(self) -> int:
        """Bytes of P one pass over the matrix has to move (codes/values of the D logical elements + scales)."""
        bits = BITS_OF[self.dtype]
        b = self.n * self.D * bits // 8
        if self.dtype in MINMAX_TYPES:
            return b + self.scales.numel() * 4
        if self.scales is not None:
            b += self.n * ((self.D + self.block - 1) // self.block) * self.scales.element_size()
        return b


def wrap_f32(P: torch.Tensor, D: Optional[int] = None) -> Pmat:
    """Describe an existing (n, ld) float32 device tensor as an F32 projection matrix."""
    assert P.dtype == torch.float32 and P.dim() == 2 and P.is_contiguous()
    return Pmat(F32, P.shape[1] if D is None else D, P.shape[0], P.shape[1], P)


def alloc_pmat(dtype: int, D: int, n: int, block: int = 0, device="cuda") -> Pmat:
    block = block or DEFAULT_BLOCK.get(dtype, 0)
    ld, _, _ = pmat_bytes(dtype, D, n, block)
    cols = ld // 2 if dtype == I4 else ld
    data = torch.empty((n, cols), dtype=_TORCH_OF[dtype], device=device)
    scales = None
    if dtype in (I8, I4):
        scales = torch.empty((ld // SCALE_SPAN, n, SCALE_SPAN // block),
                             dtype=torch.float32 if dtype == I8 else torch.float16, device=device)
    return Pmat(dtype, D, n, ld, data, scales, block if dtype in (I8, I4) else 0, 0.0 if dtype == I4 else 1.0)


def quantize(P: torch.Tensor, D: int, dtype: int, block: int = 0, gscale: float = 0.0,
             out: Optional[Pmat] = None) -> Pmat:
    """twa_quantize: store the fp32 matrix P ((n, ldp) device tensor) as `dtype`."""
    assert P.dtype == torch.float32 and P.dim() == 2 and P.is_contiguous()
    n, ldp = P.shape
    if out is None:
        out = alloc_pmat(dtype, D, n, block, device=P.device)
    if dtype == I4:
        out.gscale = float(gscale)
    st = out.c_struct()
    _check(lib().twa_quantize(_ptr(P), D, n, ldp, C.byref(st), _stream()), "twa_quantize")
    out.gscale = float(st.gscale)
    return out


class Workspace:
    """Device scratch of a fixed size, owned by the caller of the library."""

    def __init__(self, nbytes: int, device="cuda"):
        self.nbytes = int(nbytes)
        self.buf = torch.empty(max(self.nbytes, 16), dtype=torch.uint8, device=device)

    @property
    def ptr(self) -> int:
        return int(self.buf.data_ptr())


def project(P: Pmat, g: torch.Tensor, s: Optional[torch.Tensor] = None, ws: Optional[Workspace] = None) -> torch.Tensor:
    """twa_project: s = P^T g.  g: (D,) or (k, ldg) float32 on the device.  Returns s: (n,) or (k, n)."""
    assert g.dtype == torch.float32 and g.is_contiguous()
    if g.dim() == 1:
        k, ldg = 1, 0
    else:
        k, ldg = int(g.shape[0]), int(g.shape[1])
    if s is None:
        s = torch.empty((P.n,) if g.dim() == 1 else (k, P.n), dtype=torch.float32, device=g.device)
    if ws is None:
        ws = Workspace(project_workspace_bytes(P.n, k), device=g.device)
    st = P.c_struct()
    _check(lib().twa_project(C.byref(st), _ptr(g), k, ldg, _ptr(s), ws.ptr, ws.nbytes, _stream()), "twa_project")
    return s


def project_noalloc(P: Pmat, g: torch.Tensor, s: torch.Tensor) -> torch.Tensor:
    """twa_project_noalloc: s = P^T g into the caller's `s`, partial sums in the library's fixed device array
    (n * k <= NOALLOC_MAX_NK); neither this wrapper nor the call allocates."""
    assert g.dtype == torch.float32 and g.is_contiguous() and s.dtype == torch.float32 and s.is_contiguous()
    k, ldg = (1, 0) if g.dim() == 1 else (int(g.shape[0]), int(g.shape[1]))
    assert s.numel() == k * P.n
    st = P.c_struct()
    _check(lib().twa_project_noalloc(C.byref(st), _ptr(g), k, ldg, _ptr(s), _stream()), "twa_project_noalloc")
    return s


def expand_update(P: Pmat, s: torch.Tensor, w: torch.Tensor, lr: float, g_tilde: Optional[torch.Tensor] = None) -> None:
    """twa_expand_update: g~ = P s; w -= lr * g~ (in place); g~ stored if a tensor is given."""
    assert s.dtype == torch.float32 and w.dtype == torch.float32 and w.is_contiguous() and s.is_contiguous()
    st = P.c_struct()
    _check(lib().twa_expand_update(C.byref(st), _ptr(s), _ptr(w), float(lr), _ptr(g_tilde), _stream()),
           "twa_expand_update")


def project_layers_workspace_bytes(n: int, L: int) -> int:
    b = C.c_size_t()
    _check(lib().twa_project_layers_workspace_bytes(n, L, C.byref(b)), "twa_project_layers_workspace_bytes")
    return int(b.value)


class LayerPlan:
    """twa_layer_plan: the device-side plan of a layer table (L+1 int64 offsets on the device, or any
    sequence of ints, which is copied there).  Built once per model; valid for every stored matrix
    of the same D."""

    def __init__(self, layer_off, D: int, device="cuda"):
        if not isinstance(layer_off, torch.Tensor):
            layer_off = torch.tensor(list(layer_off), dtype=torch.int64)
        assert layer_off.dtype == torch.int64 and layer_off.dim() == 1
        self.layer_off = layer_off.to(device).contiguous()
        self.L = int(self.layer_off.numel()) - 1
        self.D = int(D)
        nb = C.c_size_t()
        _check(lib().twa_layer_plan_bytes(self.L, C.byref(nb)), "twa_layer_plan_bytes")
        self.buf = torch.empty(int(nb.value) // 8 + 1, dtype=torch.int64, device=device)
        _check(lib().twa_layer_plan(_ptr(self.layer_off), self.L, self.D, _ptr(self.buf), self.buf.numel() * 8,
                                    _stream()), "twa_layer_plan")

    @property
    def ptr(self) -> int:
        return int(self.buf.data_ptr())

    def tables(self):
        """(off, first2048, first1024) copied to the host, for inspection."""
        raw = self.buf.cpu()[2:]                       # behind the 16-byte header {magic, L, D}
        n = self.L + 1
        off = raw[:n].clone()
        rest = raw[n:].view(torch.int32)
        return off, rest[:n].clone(), rest[n:2 * n].clone()


def project_layers(P: Pmat, g: torch.Tensor, plan: LayerPlan, S: Optional[torch.Tensor] = None,
                   ws: Optional[Workspace] = None) -> torch.Tensor:
    """twa_project_layers: S[l] = (P^l)^T g^l.  Returns S: (L, n)."""
    assert g.dtype == torch.float32 and g.is_contiguous() and g.dim() == 1
    assert plan.D == P.D
    L = plan.L
    if S is None:
        S = torch.empty((L, P.n), dtype=torch.float32, device=g.device)
    if ws is None:
        ws = Workspace(project_layers_workspace_bytes(P.n, L), device=g.device)
    st = P.c_struct()
    _check(lib().twa_project_layers(C.byref(st), _ptr(g), plan.ptr, L, _ptr(S), ws.ptr, ws.nbytes, _stream()),
           "twa_project_layers")
    return S


def expand_update_layers(P: Pmat, S: torch.Tensor, plan: LayerPlan, w: torch.Tensor, lr: float,
                         g_tilde: Optional[torch.Tensor] = None) -> None:
    """twa_expand_update_layers: g~_i = sum_j P_ij S[l(i), j]; w -= lr * g~ (in place)."""
    L = plan.L
    assert plan.D == P.D
    assert S.dtype == torch.float32 and S.is_contiguous() and tuple(S.shape) == (L, P.n)
    assert w.dtype == torch.float32 and w.is_contiguous()
    st = P.c_struct()
    _check(lib().twa_expand_update_layers(C.byref(st), _ptr(S), plan.ptr, L, _ptr(w), float(lr),
                                          _ptr(g_tilde), _stream()), "twa_expand_update_layers")


def quantize_minmax(P: torch.Tensor, D: int, plan: LayerPlan, bits: int = 4) -> Pmat:
    """twa_quantize_minmax: the paper's per-layer min-max format (Sec. 4.6), B = 1..16 bits, in the
    smallest container that holds them (1, 2, 3 and 4 bits packed at that width, up to 8 in bytes, else words)."""
    assert P.dtype == torch.float32 and P.dim() == 2 and P.is_contiguous() and plan.D == D
    assert 1 <= bits <= 16
    dtype = (U1MM if bits == 1 else U2MM if bits == 2 else U3MM if bits == 3 else U4MM if bits == 4
             else U8MM if bits <= 8 else U16MM)
    n, ldp = P.shape
    ld, _, _ = pmat_bytes(dtype, D, n)
    cols = ld * BITS_OF[dtype] // 8 if BITS_OF[dtype] < 8 else ld
    data = torch.empty((n, cols), dtype=_TORCH_OF[dtype], device=P.device)
    ab = torch.empty((plan.L, 2), dtype=torch.float32, device=P.device)
    out = Pmat(dtype, D, n, ld, data, ab, bits, 1.0)       # block carries B for these types
    nb = C.c_size_t()
    _check(lib().twa_quantize_minmax_workspace_bytes(plan.L, C.byref(nb)), "twa_quantize_minmax_workspace_bytes")
    ws = Workspace(int(nb.value) + 8, device=P.device)
    st = out.c_struct()
    _check(lib().twa_quantize_minmax(_ptr(P), D, n, ldp, plan.ptr, plan.L, bits, C.byref(st), ws.ptr, ws.nbytes,
                                     _stream()), "twa_quantize_minmax")
    return out


def centre_normalise(W: torch.Tensor, D: int, plan: LayerPlan, out: Optional[torch.Tensor] = None,
                     want_norms: bool = True):
    """twa_centre_normalise: the paper's default (layer-wise) basis.  W: (n, ldw) float32 device tensor.

    out=None allocates E; out=W works in place.  Returns (E, wbar (D,), norms (L, n) or None)."""
    assert W.dtype == torch.float32 and W.dim() == 2 and W.is_contiguous() and plan.D == D
    n, ldw = W.shape
    E = torch.empty_like(W) if out is None else out
    wbar = torch.empty(D, dtype=torch.float32, device=W.device)
    norms = torch.empty((plan.L, n), dtype=torch.float32, device=W.device) if want_norms else None
    nb = C.c_size_t()
    _check(lib().twa_centre_normalise_workspace_bytes(D, n, plan.L, C.byref(nb)), "twa_centre_normalise_workspace_bytes")
    ws = Workspace(int(nb.value), device=W.device)
    _check(lib().twa_centre_normalise(_ptr(W), D, n, ldw, plan.ptr, plan.L, _ptr(wbar), _ptr(E), int(E.shape[1]),
                                      _ptr(norms), ws.ptr, ws.nbytes, _stream()), "twa_centre_normalise")
    return E, wbar, norms


def beta_update(beta: torch.Tensor, s: torch.Tensor, lr: float, lam: float = 0.0) -> None:
    """twa_beta_update: beta <- (1 - lr*lam) * beta - lr * s, in place."""
    assert beta.dtype == torch.float32 and s.dtype == torch.float32 and beta.shape == s.shape
    assert beta.is_contiguous() and s.is_contiguous()
    _check(lib().twa_beta_update(_ptr(beta), _ptr(s), beta.numel(), float(lr), float(lam), _stream()),
           "twa_beta_update")


def beta_optim(kind: int, beta: torch.Tensor, s: torch.Tensor, m: torch.Tensor, v: Optional[torch.Tensor], lr: float,
               lam: float = 0.0, mu: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, t: int = 1) -> None:
    """twa_beta_optim: one coefficient step with momentum (OPT_MOMENTUM), Adam or AdamW, in place on beta, m, v."""
    for a in (beta, s, m) + (() if v is None else (v,)):
        assert a.dtype == torch.float32 and a.is_contiguous() and a.shape == beta.shape
    o = OptimStruct(int(kind), float(lr), float(lam), float(mu), float(beta2), float(eps), int(t))
    _check(lib().twa_beta_optim(C.byref(o), _ptr(beta), _ptr(s), _ptr(m), _ptr(v), beta.numel(), _stream()),
           "twa_beta_optim")


def beta_step(P: Pmat, g: torch.Tensor, plan: LayerPlan, beta: torch.Tensor, lr: float, lam: float = 0.0,
              S: Optional[torch.Tensor] = None, ws: Optional[Workspace] = None) -> None:
    """twa_beta_step: s = (P^l)^T g^l and beta <- (1 - lr*lam) * beta - lr * s in one call (s stored in S if given)."""
    assert g.dtype == torch.float32 and g.is_contiguous() and g.dim() == 1 and plan.D == P.D
    assert beta.dtype == torch.float32 and beta.is_contiguous() and tuple(beta.shape) == (plan.L, P.n)
    if ws is None:
        ws = Workspace(project_layers_workspace_bytes(P.n, plan.L), device=g.device)
    st = P.c_struct()
    _check(lib().twa_beta_step(C.byref(st), _ptr(g), plan.ptr, plan.L, _ptr(beta), float(lr), float(lam), _ptr(S),
                               ws.ptr, ws.nbytes, _stream()), "twa_beta_step")


def weights_from_beta(P: Pmat, beta: torch.Tensor, plan: LayerPlan, wbar: torch.Tensor,
                      w: Optional[torch.Tensor] = None) -> torch.Tensor:
    """twa_weights_from_beta: w = wbar + P beta, layer by layer."""
    assert beta.dtype == torch.float32 and beta.is_contiguous() and tuple(beta.shape) == (plan.L, P.n)
    assert wbar.dtype == torch.float32 and wbar.is_contiguous() and wbar.numel() == P.D and plan.D == P.D
    if w is None:
        w = torch.empty_like(wbar)
    st = P.c_struct()
    _check(lib().twa_weights_from_beta(C.byref(st), _ptr(beta), plan.ptr, plan.L, _ptr(wbar), _ptr(w), _stream()),
           "twa_weights_from_beta")
    return w


def build_basis(W: torch.Tensor, D: int, out: Optional[torch.Tensor] = None, want_R: bool = True,
                ws: Optional[Workspace] = None):
    """twa_build_basis: orthonormal P with W = P R.  W: (n, ldw) float32 device tensor.

    out=None allocates P; out=W orthonormalises in place.  Returns (P tensor, R as an (n, n) float64 CPU tensor
    or None)."""
    assert W.dtype == torch.float32 and W.dim() == 2 and W.is_contiguous()
    n, ldw = W.shape
    P = torch.empty_like(W) if out is None else out
    R = torch.zeros((n, n), dtype=torch.float64) if want_R else None
    if ws is None:
        ws = Workspace(build_basis_workspace_bytes(n), device=W.device)
    rc = lib().twa_build_basis(_ptr(W), D, n, ldw, _ptr(P), int(P.shape[1]), _ptr(R), ws.ptr, ws.nbytes, _stream())
    if rc == ERR_RANK and R is not None:
        raise TwaError(rc, "twa_build_basis", f"(checkpoint {int(R[0, 0].item())})")
    _check(rc, "twa_build_basis")
    return P, R


def build_basis_async(W: torch.Tensor, D: int, out: Optional[torch.Tensor] = None, R: Optional[torch.Tensor] = None,
                      status: Optional[torch.Tensor] = None, ws: Optional[Workspace] = None):
    """twa_build_basis_async: as build_basis, without any synchronisation.  R: optional (n, n) float64 DEVICE tensor;
    status: one int32 on the device (0, or 1 + the index of a dependent checkpoint).  Returns (P, R, status)."""
    assert W.dtype == torch.float32 and W.dim() == 2 and W.is_contiguous()
    n, ldw = W.shape
    P = torch.empty_like(W) if out is None else out
    if status is None:
        status = torch.empty(1, dtype=torch.int32, device=W.device)
    if ws is None:
        ws = Workspace(build_basis_workspace_bytes(n), device=W.device)
    _check(lib().twa_build_basis_async(_ptr(W), D, n, ldw, _ptr(P), int(P.shape[1]), _ptr(R), _ptr(status), ws.ptr,
                                       ws.nbytes, _stream()), "twa_build_basis_async")
    return P, R, status


def build_basis_panels(W: torch.Tensor, D: int, panel_rows: int, out: Optional[torch.Tensor] = None):
    """CholeskyQR2 through the panel calls (twa_gram_accumulate / twa_gram_factor / twa_apply_rinv): the rows of
    W ((n, ldw) float32 device tensor) are visited `panel_rows` at a time.  Returns (P, R as (n, n) float64 CPU)."""
    assert W.dtype == torch.float32 and W.dim() == 2 and W.is_contiguous() and panel_rows % 4 == 0
    n, ldw = W.shape
    P = torch.empty_like(W) if out is None else out
    if P.data_ptr() != W.data_ptr():
        P[:, D:].zero_()                               # the panel calls leave the padding alone
    ldp = int(P.shape[1])
    gb, rb, wb = C.c_size_t(), C.c_size_t(), C.c_size_t()
    _check(lib().twa_basis_state_bytes(n, C.byref(gb), C.byref(rb), C.byref(wb)), "twa_basis_state_bytes")
    gram, rinv, ws = Workspace(gb.value, device=W.device), Workspace(rb.value, device=W.device), Workspace(wb.value, device=W.device)
    R = torch.zeros((n, n), dtype=torch.float64)
    src, lds = W, ldw
    for p in range(2):
        for k, r0 in enumerate(range(0, D, panel_rows)):
            rows = min(panel_rows, D - r0)
            flags = (GRAM_ADD if k else 0) | (GRAM_ORTHONORMAL_INPUT if p else 0)     # second pass: fp32 products
            _check(lib().twa_gram_accumulate(src.data_ptr() + 4 * r0, rows, n, lds, gram.ptr, flags, ws.ptr,
                                             ws.nbytes, _stream()), "twa_gram_accumulate")
        rc = lib().twa_gram_factor(gram.ptr, n, rinv.ptr, _ptr(R), p, _stream())
        if rc == ERR_RANK:
            raise TwaError(rc, "twa_gram_factor", f"(checkpoint {int(R[0, 0].item())})")
        _check(rc, "twa_gram_factor")
        for r0 in range(0, D, panel_rows):
            rows = min(panel_rows, D - r0)
            _check(lib().twa_apply_rinv(src.data_ptr() + 4 * r0, rows, n, lds, rinv.ptr, P.data_ptr() + 4 * r0, ldp,
                                        _stream()), "twa_apply_rinv")
        src, lds = P, ldp
    return P, R


class BasisState:
    """The device buffers of a panel-wise CholeskyQR pass (twa_basis_state_bytes): Gram matrix, R^-1, workspace."""

    def __init__(self, n: int, device="cuda"):
        gb, rb, wb = C.c_size_t(), C.c_size_t(), C.c_size_t()
        _check(lib().twa_basis_state_bytes(n, C.byref(gb), C.byref(rb), C.byref(wb)), "twa_basis_state_bytes")
        self.n = n
        self.gram, self.rinv, self.ws = Workspace(gb.value, device), Workspace(rb.value, device), Workspace(wb.value, device)


def gram_accumulate(panel: torch.Tensor, rows: int, st: BasisState, first: bool, orthonormal_input: bool = False) -> None:
    """twa_gram_accumulate on a panel ((n, ld) float32 device tensor or view whose row j starts ld elements after row j-1)."""
    n, ld = panel.shape[0], panel.stride(0)
    flags = (0 if first else GRAM_ADD) | (GRAM_ORTHONORMAL_INPUT if orthonormal_input else 0)
    _check(lib().twa_gram_accumulate(panel.data_ptr(), rows, n, ld, st.gram.ptr, flags, st.ws.ptr, st.ws.nbytes, _stream()),
           "twa_gram_accumulate")


def gram_factor(st: BasisState, R: Optional[torch.Tensor] = None, compose: bool = False) -> None:
    """twa_gram_factor: R^-1 of the accumulated Gram matrix to the device (synchronises); R (n, n) float64 CPU optional."""
    rc = lib().twa_gram_factor(st.gram.ptr, st.n, st.rinv.ptr, _ptr(R), 1 if compose else 0, _stream())
    if rc == ERR_RANK and R is not None:
        raise TwaError(rc, "twa_gram_factor", f"(checkpoint {int(R[0, 0].item())})")
    _check(rc, "twa_gram_factor")


def apply_rinv(panel: torch.Tensor, rows: int, st: BasisState, out: Optional[torch.Tensor] = None) -> None:
    """twa_apply_rinv on a panel (in place by default)."""
    dst = panel if out is None else out
    _check(lib().twa_apply_rinv(panel.data_ptr(), rows, panel.shape[0], panel.stride(0), st.rinv.ptr, dst.data_ptr(),
                                dst.stride(0), _stream()), "twa_apply_rinv")


def apply_rinv_quantize(panel: torch.Tensor, rows: int, st: BasisState, out: Pmat, row0: int) -> None:
    """twa_apply_rinv_quantize: rows [row0, row0 + rows) of the stored matrix `out` from a panel of the first pass."""
    c = out.c_struct()
    _check(lib().twa_apply_rinv_quantize(panel.data_ptr(), rows, panel.shape[0], panel.stride(0), st.rinv.ptr, C.byref(c),
                                         row0, _stream()), "twa_apply_rinv_quantize")


def absmax_accumulate(panel: torch.Tensor, rows: int, amax: torch.Tensor, first: bool) -> None:
    """twa_absmax_accumulate: amax (1 float32 on the device) = largest |entry| seen so far."""
    _check(lib().twa_absmax_accumulate(panel.data_ptr(), rows, panel.shape[0], panel.stride(0), amax.data_ptr(),
                                       0 if first else 1, _stream()), "twa_absmax_accumulate")


def gscale_for_absmax(amax: float) -> float:
    return float(lib().twa_gscale_for_absmax(C.c_float(amax)))


def probe_read(buf: torch.Tensor, sink: torch.Tensor) -> None:
    """twa_probe_read: one plain read pass over `buf` (measurement aid)."""
    assert buf.is_contiguous() and sink.numel() >= 1 and sink.element_size() == 4
    _check(lib().twa_probe_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream()), "twa_probe_read")
