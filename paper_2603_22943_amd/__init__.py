"""libtaq: Trigger-Aware Quantized cross-attention (PersonalQ, Section III-B) for MI355X.

The compute path is the HIP library ``libtaq.so`` built from ``csrc/``; this
package holds its thin ctypes binding (``paper_2603_22943_amd.taq``) and the
seeded synthetic-input generators (``paper_2603_22943_amd.synth``). Importing
the package loads nothing; the binding loads the shared library on first use
and raises if it is missing.
"""
__all__ = ["synth", "taq"]
