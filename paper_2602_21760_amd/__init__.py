"""MI355X-native hot path of conditional-guidance hybrid parallelism (one guidance branch's
denoiser step, CFG combine, branch discrepancy, Euler update) behind a C-ABI HIP library.

`synth` holds the seeded input generators; `binding` loads libhyb.so (and fails loudly if it
is missing).  Nothing is loaded at import time of the package itself."""
__all__ = ["synth", "binding"]
