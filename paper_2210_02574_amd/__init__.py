"""MI355X-native RNS-CKKS ciphertext arithmetic: HIP kernels behind a C ABI (include/he.h)
with a thin ctypes binding.  Importing the binding requires the built library; nothing here
falls back to a CPU implementation."""
from .binding import HE, EvalKey, HeError, SecretKey, load_library, LIB_PATH, SYMBOLS  # noqa: F401
from .ciphertext import Ciphertext, Evaluator  # noqa: F401
