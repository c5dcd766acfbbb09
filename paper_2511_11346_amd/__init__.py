"""MtPC head on MI355X: HIP kernels behind a C ABI (csrc/, include/mtpc.h) and a
thin ctypes binding.  Importing the package does not load the shared library;
the first call does, and raises if it has not been built."""
from .binding import (BF16, F32, FAMILY, Head, MtpcError, lib, n_latents, philox_uniforms,  # noqa: F401
                      profile_circuit, profile_unembed)
