"""MI355X-native shifted sparse attention (LongLoRA S2-Attn): HIP kernels behind a
C-ABI library, plus a thin ctypes binding.  Importing the package loads nothing;
the shared library is opened on the first call and its absence is an error."""

__all__ = ["binding", "inputs"]
