"""Copy a device-resident projection matrix to the host as the oracle's `Pmat`.

Test infrastructure (see twa_oracle.py).  The argument is duck-typed -- any object with the
fields of the C descriptor (dtype code, D, block, gscale) whose `data` / `scales` are torch
tensors -- so that nothing of the HIP path is imported here.  Only stored bytes are moved and re-encoded
(scales permuted into the oracle's order, packed integer codes spread out); none of the method's arithmetic.
"""
import numpy as np
import torch

from . import twa_oracle as orc


U8MM, U4MM, U16MM, U2MM, U1MM, U3MM = 4, 5, 6, 7, 8, 9      # dtype codes of the paper's min-max format in the C descriptor


def to_oracle(pm, cols=None, layer_off=None) -> orc.Pmat:
    """The oracle's view of the stored matrix `pm` (optionally only the basis vectors in `cols`).

    The min-max formats need the layer table (`layer_off`, L+1 offsets) the matrix was quantised with;
    their packed codes are spread out to one unsigned 16-bit code per element, as the oracle keeps them."""
    data = pm.data if cols is None else pm.data[cols]
    if pm.dtype in (U8MM, U4MM, U16MM, U2MM, U1MM, U3MM):
        raw = data.cpu().numpy()
        if pm.dtype == U3MM:
            # groups of 32 elements = three little-endian 32-bit words: element e = 16h + 4k + m has its two low
            # bits in word h at bit 2(4k + m), its high bit in word 2 at bit 8k + m + 4h
            w = np.ascontiguousarray(raw).view(np.uint32).reshape(raw.shape[0], -1, 3).astype(np.uint64)
            codes = np.empty((w.shape[0], w.shape[1], 32), dtype=np.uint16)
            for e in range(32):
                h, f = e >> 4, e & 15
                k, m = f >> 2, f & 3
                codes[:, :, e] = ((w[:, :, h] >> np.uint64(2 * f)) & np.uint64(3)) | \
                                 (((w[:, :, 2] >> np.uint64(8 * k + m + 4 * h)) & np.uint64(1)) << np.uint64(2))
            codes = codes.reshape(w.shape[0], -1)
        elif pm.dtype in (U2MM, U1MM):
            bits = 2 if pm.dtype == U2MM else 1
            per = 8 // bits                                                     # codes per byte, low bits first
            b = raw.astype(np.uint16)
            codes = np.empty((b.shape[0], per * b.shape[1]), dtype=np.uint16)
            for k in range(per):
                codes[:, k::per] = (b >> (bits * k)) & ((1 << bits) - 1)
        elif pm.dtype in (U16MM, U8MM):
            B = pm.block or (16 if pm.dtype == U16MM else 8)                   # bits of the codes
            codes = (raw.astype(np.int32) + (1 << (B - 1))).astype(np.uint16)  # the container holds code - 2^(B-1)
        else:
            b = raw.astype(np.uint16)
            codes = np.empty((b.shape[0], 2 * b.shape[1]), dtype=np.uint16)
            codes[:, 0::2] = b & 0xF                                            # even element in the low nibble
            codes[:, 1::2] = b >> 4
        ab = np.ascontiguousarray(pm.scales.cpu().numpy(), dtype=np.float32)
        off = np.ascontiguousarray(np.asarray(layer_off), dtype=np.int64)
        return orc.Pmat(orc.MM, pm.D, np.ascontiguousarray(codes), ab, 0, 1.0, off)
    scales = None
    if pm.scales is not None:
        # the device keeps the scales as [span][vector][scale in span]; the oracle wants one row of
        # scales per vector: a permutation of the stored values, nothing else
        sc = pm.scales if cols is None else pm.scales[:, cols, :]
        scales = sc.permute(1, 0, 2).reshape(sc.shape[1], -1).contiguous()
    if pm.dtype == orc.F32:
        return orc.Pmat(orc.F32, pm.D, np.ascontiguousarray(data.cpu().numpy()))
    if pm.dtype == orc.BF16:
        return orc.Pmat(orc.BF16, pm.D, np.ascontiguousarray(data.view(torch.int16).cpu().numpy().view(np.uint16)))
    if pm.dtype == orc.I8:
        return orc.Pmat(orc.I8, pm.D, np.ascontiguousarray(data.cpu().numpy()),
                        np.ascontiguousarray(scales.cpu().numpy()), pm.block, 1.0)
    if pm.dtype == orc.I4:
        return orc.Pmat(orc.I4, pm.D, np.ascontiguousarray(data.cpu().numpy()),
                        np.ascontiguousarray(scales.view(torch.int16).cpu().numpy().view(np.uint16)), pm.block,
                        pm.gscale)
    raise ValueError(pm.dtype)
