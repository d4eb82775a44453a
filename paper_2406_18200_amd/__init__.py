"""MI355X (gfx950) library for the batched target-model verification step of scheduled speculative
decoding: thin Python binding over the C ABI declared in include/seed_verify.h and include/seed_sched.h.

The binding only marshals arguments (PyTorch tensors supply device memory and the stream); every step
of the path runs in the library's HIP kernels.  There is no CPU fallback: importing works anywhere, but
any call raises if libseed_verify.so is missing.
"""
from .binding import (SeedError, VerifyContext, accept_resample, sample_probs, load_library,  # noqa: F401
                      library_path, ModelShape, sched_run, uniform_philox)
