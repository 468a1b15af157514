"""MI355X-native dilated flash attention forward (SAM-Lightening, section 3.1).

`synth` makes the seeded synthetic workloads; `binding` is the thin ctypes layer over
libdfa.so (argument marshalling only - every step runs in the HIP kernels).  Importing
the package loads nothing; the library is loaded on first use and its absence is an error.
"""
__all__ = ["synth", "binding", "build"]
