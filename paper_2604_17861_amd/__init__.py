"""MI355X-native GPUOS hot path: persistent worker kernel + host-fed task ring + dual-slot
operator table, behind the C ABI declared in include/gpuos.h.

`runtime` is the thin ctypes binding (argument marshalling only); `streams` holds the seeded
synthetic task-stream generators.  Importing this package does not load the HIP library; the
binding loads it on first use and fails loudly if it has not been built.
"""
__all__ = ["runtime", "streams", "build"]
