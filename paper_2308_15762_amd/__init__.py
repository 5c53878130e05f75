"""Per-rank hot path of a Hanayo wave pipeline on one MI355X.

`hanayo` is the ctypes binding of libhanayo.so (argument marshalling only:
every step runs in the library's own host code and HIP kernels); `synth`
holds the seeded synthetic workloads.  Importing `hanayo` raises if the
library has not been built (python -m paper_2308_15762_amd.build).
"""
