"""MI355X-native Shamir-secret-sharing inference arithmetic (p = 2^61 - 1).

`SSNet` wraps the C ABI of libssnet.so (include/ssnet.h); `fixedpoint` holds
the plaintext-side encode/decode helpers of the harness; `chain` runs a
sequential stack of linear layers on shares.
"""
from .binding import (P45, P61, SSNet, SSNetError, load_library, rng_draw, rng_field, rng_key)  # noqa: F401
from . import fixedpoint  # noqa: F401
