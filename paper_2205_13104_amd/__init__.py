"""MI355X-native projected-gradient step of Trainable Weight Averaging (arXiv 2205.13104).

The work is done by hand-written HIP kernels for gfx950 behind a C-ABI shared library
(``include/twa.h``); :mod:`.binding` marshals torch device pointers into it and
:mod:`.synth` draws the seeded synthetic inputs, :mod:`.panels` sequences the calls of a
basis construction whose checkpoints arrive in panels of rows.  Importing the package loads nothing;
the library is loaded on first use of a binding call and a missing library is an error.
"""
__all__ = ["binding", "synth", "build", "panels"]
