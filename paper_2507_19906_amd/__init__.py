"""MI355X-native CaliDrop hot path: prefill-time KV compression with calibration-state
precompute (Alg. 1) and calibrated decode attention (Alg. 2, Eq. 1-2) as hand-written HIP
kernels behind a C-ABI library.  ``binding`` holds the thin ctypes layer; ``synth`` the seeded
input generators.  Nothing here computes on the CPU."""
