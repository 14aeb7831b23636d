"""Basis construction for checkpoints whose rows arrive in panels: the order of the C-ABI calls, nothing else.

The checkpoint matrix of the largest configuration (D = 350 M, n = 128: 179 GB in fp32) is never held, and neither
is the fp32 basis: a caller-supplied function produces rows [r0, r0 + rows) of all n checkpoints into ONE staging
buffer, as often as it is asked, and three sweeps over the panels leave only the low-bit projection matrix
(arXiv 2205.13104, Sec. 4.1 for the basis, Sec. 4.6 for its storage):

    sweep 1   panel -> twa_gram_accumulate                          G1 = W^T W        -> twa_gram_factor -> R1^-1
    sweep 2   panel -> twa_apply_rinv (R1^-1, in place)
                    -> twa_gram_accumulate (orthonormal input)      G2 = Q1^T Q1      -> twa_gram_factor -> R2^-1
                    -> twa_absmax_accumulate                        largest |entry| (for the 4-bit scales)
    sweep 3   panel -> twa_apply_rinv (R1^-1, in place)
                    -> twa_apply_rinv_quantize (R2^-1)              rows [r0, r0 + rows) of every stored matrix

Every step of the arithmetic runs in the library's kernels; this module only sequences them.
"""
from __future__ import annotations

from typing import Callable, Dict, Optional, Sequence

import torch

from . import binding as twa


def stored_basis_from_panels(make_panel: Callable[[int, int, torch.Tensor], None], D: int, n: int, panel_rows: int,
                             dtypes: Sequence[int], device="cuda", on_first_sweep: Optional[Callable] = None):
    """Orthonormal basis of the span of n checkpoints of length D, stored in every format of `dtypes`.

    make_panel(r0, rows, stage) writes rows [r0, r0 + rows) of all n checkpoints to stage[:, :rows]; it is called
    three times per panel and must produce the same values each time.  panel_rows: a multiple of 2048.
    on_first_sweep(r0, rows, stage), if given, sees every panel of the first sweep (e.g. to form the mean).
    Returns (dict dtype -> binding.Pmat, R1, R2 as (n, n) float64 CPU tensors: W = P (R2 R1)), and the staging buffer."""
    assert panel_rows % twa.SCALE_SPAN == 0
    stage = torch.empty((n, panel_rows), dtype=torch.float32, device=device)
    starts = list(range(0, D, panel_rows))
    st1, st2 = twa.BasisState(n, device), twa.BasisState(n, device)
    R1 = torch.zeros((n, n), dtype=torch.float64)
    R2 = torch.zeros((n, n), dtype=torch.float64)
    amax = torch.zeros(1, dtype=torch.float32, device=device)
    for k, r0 in enumerate(starts):
        rows = min(panel_rows, D - r0)
        make_panel(r0, rows, stage)
        if on_first_sweep is not None:
            on_first_sweep(r0, rows, stage)
        twa.gram_accumulate(stage, rows, st1, first=k == 0)
    twa.gram_factor(st1, R1)
    for k, r0 in enumerate(starts):
        rows = min(panel_rows, D - r0)
        make_panel(r0, rows, stage)
        twa.apply_rinv(stage, rows, st1)
        twa.gram_accumulate(stage, rows, st2, first=k == 0, orthonormal_input=True)
        twa.absmax_accumulate(stage, rows, amax, first=k == 0)
    twa.gram_factor(st2, R2)
    gscale = twa.gscale_for_absmax(float(amax.item()))
    outs: Dict[int, twa.Pmat] = {}
    for dt in dtypes:
        outs[dt] = twa.alloc_pmat(dt, D, n, device=device)
        outs[dt].gscale = gscale if dt == twa.I4 else 1.0
    for r0 in starts:
        rows = min(panel_rows, D - r0)
        make_panel(r0, rows, stage)
        twa.apply_rinv(stage, rows, st1)
        for dt in dtypes:
            twa.apply_rinv_quantize(stage, rows, st2, outs[dt], r0)
    return outs, R1, R2, stage, (st1, st2)
