"""SABlock prefill-time KV-cache compression hot path for MI355X (gfx950).

The package holds the HIP kernels and C-ABI library (``csrc/``), the thin
Python binding (``binding``) and the seeded synthetic-input generators
(``synth``).  Importing the package loads nothing native; the binding loads
``libsablock.so`` on first use and raises if it has not been built.
"""

__all__ = ["binding", "synth", "build"]
