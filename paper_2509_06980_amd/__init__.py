"""MI355X-native batched multi-turn rollout engine (Python binding of librl_rollout.so).

The binding only marshals arguments; every step of the rollout path runs in the HIP
library.  Importing this package does not load the library; the first use does, and it
fails loudly if the library has not been built (python paper_2509_06980_amd/build.py).
"""
from .binding import (RolloutEngine, RolloutError, sample_from_logits, sample_device_logits, uniform_u32,  # noqa: F401
                      measure_stream_read, load_library, LIB_PATH, EXPORTED_SYMBOLS,
                      FLAG_GENERIC_KERNELS, FLAG_SHARED_PREFIX_ATTENTION, FLAG_FP8_KV_CACHE)
