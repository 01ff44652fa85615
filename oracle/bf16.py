"""bfloat16 storage rounding (oracle side; test infrastructure).

The bf16 configurations keep weights and activations in bfloat16 and accumulate in higher precision
(the paper trains in mixed precision, section 5; the task's configurations say "bf16 weights/activations
with fp32 accumulate").  bfloat16 is the upper 16 bits of an IEEE binary32 number: 1 sign, 8 exponent and 7
fraction bits.  ``round_bf16`` maps every value to the nearest bfloat16 value, ties to the one whose last
fraction bit is even, and returns it as fp64 (every bfloat16 value is exact in fp64).

With ``storage=round_bf16`` the layer oracle rounds each tensor that the method keeps in storage precision
(activations handed from one step to the next, gradients of activations) at the point where it is produced;
sums and matrix products stay in fp64 and parameter gradients stay unrounded, as they accumulate in fp32
outside storage.  Nothing else changes: the default path of the oracle performs no rounding at all.
"""
import numpy as np


def round_bf16(x):
    """Nearest bfloat16 (ties to even) of every element of x, as fp64.  The value is first brought to
    binary32, as the accumulators of a mixed-precision run are, then cut to 16 bits."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float64).astype(np.float32))
    bits = f.view(np.uint32)
    last = (bits >> np.uint32(16)) & np.uint32(1)                    # last bit that is kept
    rounded = (bits + np.uint32(0x7FFF) + last) & np.uint32(0xFFFF0000)
    out = rounded.view(np.float32).astype(np.float64)
    nan = np.isnan(f)
    if nan.any():
        out = np.where(nan, np.nan, out)
    return out.reshape(np.shape(x))
