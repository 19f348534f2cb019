"""CPU oracle for the per-device hot path of the 2D (SUMMA) transformer scheme.

TEST INFRASTRUCTURE ONLY.  Plain numpy in fp64, written from the paper's
definitions; deliberately slow and unblocked so it can be checked against the
paper by eye.  It shares no code with the HIP library and must never be
imported by the product package: only ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py`` may use it.

Pins (see tests/test_oracle_*.py): brute-force loops on tiny inputs, the
reassembly invariant of Algorithms 1-3 for q in {1, 2, 4}, transpose
identities, closed forms, Eq. 1-3 and every backward formula against central
finite differences.

Parity unpinned (conventions the paper leaves open, fixed by the readings in
the design notes and shared by both sides): row order of M = b*s, head-major
column order of the 3h projection, pre-LayerNorm wiring with two residuals,
exact-erf GeLU, eps = 1e-5.
"""
from . import blocks, summa, layernorm, attention, layer, metrics, flops, stack, model_ends  # noqa: F401
