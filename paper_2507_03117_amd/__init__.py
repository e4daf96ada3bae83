"""MI355X-native block-sparse MLP (BLaST hot path): HIP kernels behind a C ABI.

`synth` (seeded input generators) is importable without the HIP library;
everything in `api` loads the compiled library on first use and raises if it is
missing: there is no CPU fallback.
"""
__all__ = ["synth", "api"]
