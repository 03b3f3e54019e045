"""LAPLEX apply for MI355X: y = L(a, b) x with L_ij = exp(-|a_i - b_j|).

The work is done by hand-written HIP kernels behind a C-ABI library
(``include/laplex.h``); :mod:`paper_2605_24584_amd.binding` marshals
arguments to it and nothing else.  Importing the package loads nothing: the
shared library is opened on the first call and a missing library is an error,
never a fallback.
"""

__all__ = ["binding", "synth"]
