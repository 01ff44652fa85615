"""Counter-based dropout mask (oracle side).

The paper fuses bias + dropout + add (section 4.2) but does not say how the
random bits are drawn.  This build fixes a counter-based generator so that the
mask is a pure function of (seed, layer, site, microbatch, element index) and
the backward pass can recompute it instead of storing it:

* mixing function: the SplitMix64 output function (Steele, Lea, Flood 2014;
  public domain): two xor-shift-multiply rounds and a final xor-shift over a
  64-bit state;
* stream key: the seed, then (2*layer + site + 1), then (microbatch + 1) are
  absorbed one after the other, each as ``mix(key + GOLDEN * word)``;
* one 64-bit word per group of four consecutive elements:
  ``r = mix(key + GOLDEN * group)`` with ``group = index >> 2``; element
  ``index`` takes the 16-bit field ``(r >> 16*(index & 3)) & 0xFFFF``;
* the element is KEPT iff ``field >= floor(p*65536 + 0.5)``; kept values are
  scaled by ``1/(1-p)`` (inverted dropout); ``p == 0`` keeps everything.

``index`` is the flat row-major index into the ``[s, b, h]`` tensor at the
dropout site (site 0: after the attention output projection, site 1: after the
second MLP GEMM).

Everything is integer arithmetic modulo 2**64; numpy's uint64 wraps silently.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_MUL_A = np.uint64(0xBF58476D1CE4E5B9)
_MUL_B = np.uint64(0x94D049BB133111EB)


def mix64(z):
    """SplitMix64 output function on a uint64 array (or scalar)."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _MUL_A
        z = (z ^ (z >> np.uint64(27))) * _MUL_B
        z = z ^ (z >> np.uint64(31))
    return z


def stream_key(seed, layer, site, microbatch):
    """64-bit key of one dropout site of one layer for one microbatch."""
    with np.errstate(over="ignore"):
        k = mix64(np.uint64(seed))
        k = mix64(k + _GOLDEN * np.uint64(2 * int(layer) + int(site) + 1))
        k = mix64(k + _GOLDEN * np.uint64(int(microbatch) + 1))
    return np.uint64(k)


def hash_word(seed, layer, site, microbatch, group):
    """The 64-bit word that serves elements 4*group .. 4*group+3."""
    key = stream_key(seed, layer, site, microbatch)
    with np.errstate(over="ignore"):
        return mix64(key + _GOLDEN * np.asarray(group, dtype=np.uint64))


def threshold(p):
    """Drop threshold on the 16-bit field, from the fp32 value of p."""
    return int(np.floor(float(np.float32(p)) * 65536.0 + 0.5))


def keep_mask(seed, layer, site, microbatch, n, p, start=0):
    """Boolean keep-mask for flat element indices start .. start+n-1."""
    if p == 0:
        return np.ones(n, dtype=bool)
    idx = np.arange(start, start + n, dtype=np.uint64)
    word = hash_word(seed, layer, site, microbatch, idx >> np.uint64(2))
    field = (word >> (np.uint64(16) * (idx & np.uint64(3)))) & np.uint64(0xFFFF)
    return field >= np.uint64(threshold(p))


def keep_scale(p):
    """1/(1-p) with p taken at its fp32 value."""
    return 1.0 / (1.0 - float(np.float32(p)))
