"""MI355X-native leaf kernels for the dense tensor-algebra expressions of DISTAL.

Importing the package is cheap and works without a GPU; the HIP library is
loaded on first use of ``paper_2203_08069_amd.binding`` and its absence is an
error, never a fallback.
"""
__all__ = ["binding", "inputs"]
__version__ = "0.6.0"   # distal_version() of the library reports the same (600)
