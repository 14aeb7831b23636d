"""Copy a device-resident projection matrix to the host as the oracle's `Pmat`.

Test infrastructure (see twa_oracle.py).  The argument is duck-typed -- any object with the
fields of the C descriptor (dtype code, D, block, gscale) whose `data` / `scales` are torch
tensors -- so that nothing of the HIP path is imported here.  Only bytes are moved; no arithmetic.
"""
import numpy as np
import torch

from . import twa_oracle as orc


def to_oracle(pm, cols=None) -> orc.Pmat:
    """The oracle's view of the stored matrix `pm` (optionally only the basis vectors in `cols`)."""
    data = pm.data if cols is None else pm.data[cols]
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
