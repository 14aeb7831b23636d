"""ctypes front end of the fp64 CPU oracle (``twa_oracle.c``).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; the product package never does.
It only marshals numpy arrays into the C functions -- all arithmetic is in the C file,
next to the citations of the passages of arXiv 2205.13104 it follows.

Layout convention (shared with nothing): a D x n matrix is a numpy array of shape
``(n, ld)`` with ``ld >= D`` -- row j is basis vector / checkpoint j.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "twa_oracle.c")
_LIB = os.path.join(_HERE, "libtwa_oracle.so")

F64, F32, BF16, I8, I4, MM = -1, 0, 1, 2, 3, 4
ERR_ARG, ERR_RANK, ERR_NOMEM = -1, -6, -8


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _PmatStruct(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("n", C.c_int32), ("D", C.c_int64), ("ld", C.c_int64),
                ("data", C.c_void_p), ("scales", C.c_void_p), ("block", C.c_int32),
                ("gscale", C.c_float), ("layer_off", C.c_void_p), ("L", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.twa_oracle_threads.restype = C.c_int
        L.twa_oracle_set_threads.argtypes = [C.c_int]
        L.twa_oracle_f32_to_f16.argtypes = [C.c_float]
        L.twa_oracle_f32_to_f16.restype = C.c_uint16
        L.twa_oracle_f16_to_f32.argtypes = [C.c_uint16]
        L.twa_oracle_f16_to_f32.restype = C.c_float
        L.twa_oracle_f32_to_bf16.argtypes = [C.c_float]
        L.twa_oracle_f32_to_bf16.restype = C.c_uint16
        L.twa_oracle_bf16_to_f32.argtypes = [C.c_uint16]
        L.twa_oracle_bf16_to_f32.restype = C.c_float
        L.twa_oracle_gscale_i4.restype = C.c_float
        L.twa_oracle_gscale_i4.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64]
        P = C.POINTER(_PmatStruct)
        L.twa_oracle_dequant.argtypes = [P, C.c_void_p, C.c_int64]
        L.twa_oracle_project.argtypes = [P, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p]
        L.twa_oracle_expand_update.argtypes = [P, C.c_void_p, C.c_void_p, C.c_double, C.c_void_p]
        L.twa_oracle_build_basis.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_void_p,
                                             C.c_int64, C.c_void_p, C.c_double, C.POINTER(C.c_int32)]
        L.twa_oracle_centre_normalise.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64,
                                                  C.c_void_p, C.c_int64, C.c_void_p]
        L.twa_oracle_quantize_i8.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_void_p,
                                             C.c_int64, C.c_void_p, C.c_int32]
        L.twa_oracle_quantize_i4.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_void_p,
                                             C.c_int64, C.c_void_p, C.c_int32, C.c_float]
        L.twa_oracle_to_bf16.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_void_p, C.c_int64]
        L.twa_oracle_quantize_minmax.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_int32,
                                                 C.c_void_p, C.c_int32, C.c_void_p, C.c_int64,
                                                 C.c_void_p, C.c_void_p]
        L.twa_oracle_project_layers.argtypes = [P, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.twa_oracle_expand_update_layers.argtypes = [P, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                                      C.c_double, C.c_void_p]
        L.twa_oracle_beta_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_double, C.c_double]
        L.twa_oracle_beta_optim.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                            C.c_double, C.c_double, C.c_double, C.c_double, C.c_double, C.c_int32]
        L.twa_oracle_weights_from_beta.argtypes = [P, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.twa_oracle_centre_normalise_layers.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64,
                                                         C.c_void_p, C.c_int32, C.c_void_p, C.c_int64,
                                                         C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def threads() -> int:
    return int(lib().twa_oracle_threads())


def set_threads(t: int) -> None:
    lib().twa_oracle_set_threads(int(t))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise OracleError(rc, what)


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: oracle error {code}")
        self.code = code


_NP = {F64: np.float64, F32: np.float32, BF16: np.uint16, I8: np.int8, I4: np.uint8, MM: np.uint16}


@dataclass
class Pmat:
    """A stored projection matrix as the oracle sees it (host numpy arrays)."""
    dtype: int
    D: int
    data: np.ndarray                 # (n, ld) values/codes; I4: (n, ld//2) bytes
    scales: Optional[np.ndarray] = None   # (n, ld//block): float32 (I8) / uint16 binary16 bits (I4)
    block: int = 0
    gscale: float = 1.0
    layer_off: Optional[np.ndarray] = None   # MM (the paper's min-max format): L+1 int64 offsets; scales = (L, 2) float32 (a, b)

    def __post_init__(self):
        assert self.data.ndim == 2 and self.data.flags.c_contiguous
        assert self.data.dtype == _NP[self.dtype], (self.data.dtype, self.dtype)
        if self.dtype == MM:
            assert self.layer_off is not None and self.layer_off.dtype == np.int64 and self.layer_off.flags.c_contiguous
            assert self.scales is not None and self.scales.dtype == np.float32 and self.scales.flags.c_contiguous
            assert self.scales.shape == (self.layer_off.size - 1, 2)
            assert self.layer_off[0] == 0 and self.layer_off[-1] == self.D
        if self.dtype in (I8, I4):
            assert self.scales is not None and self.scales.flags.c_contiguous and self.block > 0
            assert self.scales.dtype == (np.float32 if self.dtype == I8 else np.uint16)
            assert self.scales.shape == (self.n, self.ld // self.block)
        assert self.ld >= self.D

    @property
    def n(self) -> int:
        return int(self.data.shape[0])

    @property
    def ld(self) -> int:
        return int(self.data.shape[1]) * (2 if self.dtype == I4 else 1)

    def _struct(self) -> _PmatStruct:
        return _PmatStruct(self.dtype, self.n, self.D, self.ld, self.data.ctypes.data,
                           0 if self.scales is None else self.scales.ctypes.data,
                           self.block, float(self.gscale),
                           0 if self.layer_off is None else self.layer_off.ctypes.data,
                           0 if self.layer_off is None else self.layer_off.size - 1)

    def dense(self) -> np.ndarray:
        """(n, D) float64 array of the exact stored values."""
        out = np.empty((self.n, self.D), dtype=np.float64)
        st = self._struct()
        _check(lib().twa_oracle_dequant(C.byref(st), _ptr(out), self.D), "dequant")
        return out


def pmat_f64(a: np.ndarray, D: Optional[int] = None) -> Pmat:
    a = np.ascontiguousarray(a, dtype=np.float64)
    return Pmat(F64, a.shape[1] if D is None else D, a)


def pmat_f32(a: np.ndarray, D: Optional[int] = None) -> Pmat:
    a = np.ascontiguousarray(a, dtype=np.float32)
    return Pmat(F32, a.shape[1] if D is None else D, a)


def project(P: Pmat, G: np.ndarray) -> np.ndarray:
    """S[c, j] = sum_i P[i, j] * G[c, i] -- Sec. 4.2 (gradient w.r.t. the coefficients).

    G: (D,) or (k, >=D) float64.  Returns (n,) or (k, n)."""
    G = np.asarray(G, dtype=np.float64)
    one = G.ndim == 1
    G2 = np.ascontiguousarray(G.reshape(1, -1) if one else G)
    k, ldg = G2.shape
    S = np.empty((k, P.n), dtype=np.float64)
    st = P._struct()
    _check(lib().twa_oracle_project(C.byref(st), _ptr(G2), k, ldg, _ptr(S)), "project")
    return S[0] if one else S


def expand_update(P: Pmat, s: np.ndarray, w: np.ndarray, eta: float, want_gt: bool = False):
    """g~ = P s; w <- w - eta g~ in place (w float64, length D) -- Sec. 4.2, lambda = 0."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    assert s.shape == (P.n,)
    assert w.dtype == np.float64 and w.flags.c_contiguous and w.shape == (P.D,)
    gt = np.empty(P.D, dtype=np.float64) if want_gt else None
    st = P._struct()
    _check(lib().twa_oracle_expand_update(C.byref(st), _ptr(s), _ptr(w), float(eta), _ptr(gt)),
           "expand_update")
    return gt


def build_basis(W: np.ndarray, rank_tol: float = 1e-6):
    """Thin QR with positive diagonal of the (n, D) checkpoint array W (rows = checkpoints).

    Returns (P (n, D) float64, R (n, n) float64 upper triangular) with W^T = P^T R in the
    column picture, i.e. W[b] = sum_a R[a, b] P[a]."""
    W = np.ascontiguousarray(W, dtype=np.float64)
    n, D = W.shape
    P = np.empty((n, D), dtype=np.float64)
    R = np.empty((n, n), dtype=np.float64)
    bad = C.c_int32(-1)
    rc = lib().twa_oracle_build_basis(_ptr(W), D, n, D, _ptr(P), D, _ptr(R), float(rank_tol), C.byref(bad))
    if rc == ERR_RANK:
        e = OracleError(rc, f"build_basis: rank deficient at column {bad.value}")
        e.column = bad.value
        raise e
    _check(rc, "build_basis")
    return P, R


def centre_normalise(W: np.ndarray):
    W = np.ascontiguousarray(W, dtype=np.float64)
    n, D = W.shape
    E = np.empty((n, D), dtype=np.float64)
    wbar = np.empty(D, dtype=np.float64)
    _check(lib().twa_oracle_centre_normalise(_ptr(W), D, n, D, _ptr(E), D, _ptr(wbar)), "centre_normalise")
    return E, wbar


def _off(layer_off, D: int) -> np.ndarray:
    off = np.ascontiguousarray(layer_off, dtype=np.int64)
    assert off.ndim == 1 and off.size >= 2 and off[0] == 0 and off[-1] == D
    return off


def project_layers(P: Pmat, g: np.ndarray, layer_off) -> np.ndarray:
    """S[l, j] = sum over the elements i of layer l of P[i, j] g[i] -- Sec. 4.5 / Alg. 1.  Returns (L, n)."""
    g = np.ascontiguousarray(g, dtype=np.float64)
    assert g.shape == (P.D,)
    off = _off(layer_off, P.D)
    S = np.empty((off.size - 1, P.n), dtype=np.float64)
    st = P._struct()
    _check(lib().twa_oracle_project_layers(C.byref(st), _ptr(g), _ptr(off), off.size - 1, _ptr(S)), "project_layers")
    return S


def expand_update_layers(P: Pmat, S: np.ndarray, layer_off, w: np.ndarray, eta: float, want_gt: bool = False):
    """g~_i = sum_j P[i, j] S[l(i), j]; w <- w - eta g~ in place -- Sec. 4.5, lambda = 0."""
    off = _off(layer_off, P.D)
    S = np.ascontiguousarray(S, dtype=np.float64)
    assert S.shape == (off.size - 1, P.n)
    assert w.dtype == np.float64 and w.flags.c_contiguous and w.shape == (P.D,)
    gt = np.empty(P.D, dtype=np.float64) if want_gt else None
    st = P._struct()
    _check(lib().twa_oracle_expand_update_layers(C.byref(st), _ptr(S), _ptr(off), off.size - 1, _ptr(w), float(eta),
                                                 _ptr(gt)), "expand_update_layers")
    return gt


def beta_step(beta: np.ndarray, s: np.ndarray, eta: float, lam: float) -> None:
    """beta <- (1 - eta*lam) beta - eta s in place -- Alg. 1, "update variables"."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    assert beta.dtype == np.float64 and beta.flags.c_contiguous and beta.shape == s.shape
    _check(lib().twa_oracle_beta_step(_ptr(beta), _ptr(s), beta.size, float(eta), float(lam)), "beta_step")


MOMENTUM, ADAM, ADAMW = 0, 1, 2


def beta_optim(kind: int, beta: np.ndarray, s: np.ndarray, m: np.ndarray, v, eta: float, lam: float,
               mu_or_b1: float, b2: float = 0.0, eps: float = 0.0, t: int = 1) -> None:
    """One coefficient step with the base optimiser (Sec. 5.1) in place: heavy-ball momentum, Adam (decay as an
    L2 term) or AdamW (decoupled decay) on beta, state m (and v) updated in place.  t counts from 1."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    for a in (beta, m) + (() if v is None else (v,)):
        assert a.dtype == np.float64 and a.flags.c_contiguous and a.shape == s.shape
    _check(lib().twa_oracle_beta_optim(int(kind), _ptr(beta), _ptr(s), _ptr(m), None if v is None else _ptr(v),
                                       beta.size, float(eta), float(lam), float(mu_or_b1), float(b2), float(eps),
                                       int(t)), "beta_optim")


def weights_from_beta(P: Pmat, beta: np.ndarray, layer_off, wbar: np.ndarray) -> np.ndarray:
    """w^l = wbar^l + P^l beta^l -- Alg. 1, "update weights".  beta: (L, n).  Returns w (D,)."""
    off = _off(layer_off, P.D)
    beta = np.ascontiguousarray(beta, dtype=np.float64)
    wbar = np.ascontiguousarray(wbar, dtype=np.float64)
    assert beta.shape == (off.size - 1, P.n) and wbar.shape == (P.D,)
    w = np.empty(P.D, dtype=np.float64)
    st = P._struct()
    _check(lib().twa_oracle_weights_from_beta(C.byref(st), _ptr(beta), _ptr(off), off.size - 1, _ptr(wbar), _ptr(w)),
           "weights_from_beta")
    return w


def centre_normalise_layers(W: np.ndarray, layer_off):
    """Layer-wise basis of Sec. 4.5: returns (E (n, D), wbar (D,), norms (L, n))."""
    W = np.ascontiguousarray(W, dtype=np.float64)
    n, D = W.shape
    off = _off(layer_off, D)
    E = np.empty((n, D), dtype=np.float64)
    wbar = np.empty(D, dtype=np.float64)
    nrm = np.empty((off.size - 1, n), dtype=np.float64)
    _check(lib().twa_oracle_centre_normalise_layers(_ptr(W), D, n, D, _ptr(off), off.size - 1, _ptr(E), D,
                                                    _ptr(wbar), _ptr(nrm)), "centre_normalise_layers")
    return E, wbar, nrm


def _pad_ld(D: int, mult: int) -> int:
    return (D + mult - 1) // mult * mult


def quantize_i8(P32: np.ndarray, D: Optional[int] = None, block: int = 128, ld: Optional[int] = None) -> Pmat:
    P32 = np.ascontiguousarray(P32, dtype=np.float32)
    n, ldp = P32.shape
    D = ldp if D is None else D
    ld = _pad_ld(D, block) if ld is None else ld
    codes = np.empty((n, ld), dtype=np.int8)
    scales = np.empty((n, ld // block), dtype=np.float32)
    _check(lib().twa_oracle_quantize_i8(_ptr(P32), D, n, ldp, _ptr(codes), ld, _ptr(scales), block), "quantize_i8")
    return Pmat(I8, D, codes, scales, block, 1.0)


def gscale_i4(P32: np.ndarray, D: Optional[int] = None) -> float:
    P32 = np.ascontiguousarray(P32, dtype=np.float32)
    n, ldp = P32.shape
    return float(lib().twa_oracle_gscale_i4(_ptr(P32), ldp if D is None else D, n, ldp))


def quantize_i4(P32: np.ndarray, D: Optional[int] = None, block: int = 64, ld: Optional[int] = None,
                gscale: Optional[float] = None) -> Pmat:
    P32 = np.ascontiguousarray(P32, dtype=np.float32)
    n, ldp = P32.shape
    D = ldp if D is None else D
    ld = _pad_ld(D, block) if ld is None else ld
    if gscale is None:
        gscale = gscale_i4(P32, D)
    codes = np.empty((n, ld // 2), dtype=np.uint8)
    scales = np.empty((n, ld // block), dtype=np.uint16)
    _check(lib().twa_oracle_quantize_i4(_ptr(P32), D, n, ldp, _ptr(codes), ld, _ptr(scales), block,
                                        float(gscale)), "quantize_i4")
    return Pmat(I4, D, codes, scales, block, float(gscale))


def to_bf16(P32: np.ndarray, D: Optional[int] = None, ld: Optional[int] = None) -> Pmat:
    P32 = np.ascontiguousarray(P32, dtype=np.float32)
    n, ldp = P32.shape
    D = ldp if D is None else D
    ld = D if ld is None else ld
    out = np.empty((n, ld), dtype=np.uint16)
    _check(lib().twa_oracle_to_bf16(_ptr(P32), D, n, ldp, _ptr(out), ld), "to_bf16")
    return Pmat(BF16, D, out)


def quantize_minmax(P: np.ndarray, B: int, layer_off):
    """The paper's per-layer min-max quantiser (Sec. 4.6).  Returns (codes uint16 (n, D), a (L,), b (L,))."""
    P = np.ascontiguousarray(P, dtype=np.float64)
    n, D = P.shape
    off = np.ascontiguousarray(layer_off, dtype=np.int64)
    L = off.size - 1
    codes = np.empty((n, D), dtype=np.uint16)
    a = np.empty(L, dtype=np.float64)
    b = np.empty(L, dtype=np.float64)
    _check(lib().twa_oracle_quantize_minmax(_ptr(P), D, n, D, B, _ptr(off), L, _ptr(codes), D, _ptr(a), _ptr(b)),
           "quantize_minmax")
    return codes, a, b


def pmat_minmax(codes: np.ndarray, a, b, layer_off, D: Optional[int] = None) -> Pmat:
    """The stored matrix of the paper's min-max format (Sec. 4.6): value = a_l * code + b_l, with the two
    factors of every layer kept as binary32 (8L bytes in the memory table of that section)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    ab = np.ascontiguousarray(np.stack([np.asarray(a), np.asarray(b)], axis=1).astype(np.float32))
    off = np.ascontiguousarray(layer_off, dtype=np.int64)
    return Pmat(MM, codes.shape[1] if D is None else D, codes, ab, 0, 1.0, off)


def f32_to_f16_bits(x: float) -> int:
    return int(lib().twa_oracle_f32_to_f16(C.c_float(x)))


def f16_bits_to_f32(h: int) -> float:
    return float(lib().twa_oracle_f16_to_f32(C.c_uint16(h)))


def f32_to_bf16_bits(x: float) -> int:
    return int(lib().twa_oracle_f32_to_bf16(C.c_float(x)))
