"""Asynchronous Tsetlin machine hot path for MI355X (gfx950).

`binding` is the thin Python layer over the C boundary declared in
include/tm.h; `synth` generates the seeded synthetic workloads; `build`
compiles the HIP library.  Importing the package loads nothing: the HIP
library is opened on first use and its absence is an error, never a fallback.
"""
