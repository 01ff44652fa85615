"""Pins for oracle/dropout_hash.py (CPU only)."""
import os

import numpy as np

from oracle import dropout_hash as D

GOLDEN = 0x9E3779B97F4A7C15
HERE = os.path.dirname(__file__)


def test_mix64_matches_published_splitmix64_sequence():
    want = [int(l, 16) for l in open(os.path.join(HERE, "golden", "splitmix64_seed0.txt"))
            if l.strip() and not l.startswith("#")]
    got = [int(D.mix64(np.uint64((GOLDEN * (i + 1)) % 2 ** 64))) for i in range(len(want))]
    assert got == want


def test_mix64_against_python_bigint():
    def ref(z):
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) % 2 ** 64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) % 2 ** 64
        return z ^ (z >> 31)
    rng = np.random.default_rng(1)
    zs = rng.integers(0, 2 ** 64, size=200, dtype=np.uint64)
    assert [int(v) for v in D.mix64(zs)] == [ref(int(z)) for z in zs]


def test_keep_rate_within_binomial_bound():
    n = 1 << 20
    for p in (0.1, 0.5, 0.25):
        m = D.keep_mask(0, 3, 1, 7, n, p)
        q = 1.0 - D.threshold(p) / 65536.0
        assert abs(m.mean() - q) < 4 * np.sqrt(q * (1 - q) / n)
        assert abs(q - (1 - p)) < 1e-4


def test_p_zero_keeps_everything_and_threshold_rounding():
    assert D.keep_mask(0, 0, 0, 0, 1000, 0.0).all()
    assert D.threshold(0.1) == 6554 and D.threshold(0.5) == 32768


def test_mask_is_function_of_its_five_arguments_only():
    base = D.keep_mask(5, 2, 0, 3, 4096, 0.3)
    assert (base == D.keep_mask(5, 2, 0, 3, 4096, 0.3)).all()
    # a window of the stream equals the same indices of the full stream
    assert (D.keep_mask(5, 2, 0, 3, 100, 0.3, start=1001) == base[1001:1101]).all()
    for other in (D.keep_mask(6, 2, 0, 3, 4096, 0.3), D.keep_mask(5, 3, 0, 3, 4096, 0.3),
                  D.keep_mask(5, 2, 1, 3, 4096, 0.3), D.keep_mask(5, 2, 0, 4, 4096, 0.3)):
        agree = (other == base).mean()
        assert 0.45 < agree < 0.72          # independent masks agree with prob 0.58
    # (layer, site) pairs do not alias: layer 1 site 0 differs from layer 0 site 1 etc.
    keys = {int(D.stream_key(0, l, s, mb)) for l in range(8) for s in range(2) for mb in range(8)}
    assert len(keys) == 128


def test_four_fields_of_a_word_are_used_in_order():
    w = int(D.hash_word(9, 1, 1, 2, np.uint64(17)))
    thr = D.threshold(0.4)
    want = [((w >> (16 * i)) & 0xFFFF) >= thr for i in range(4)]
    got = D.keep_mask(9, 1, 1, 2, 4, 0.4, start=68)
    assert list(got) == want


def test_avalanche_of_counter():
    g = np.arange(4096, dtype=np.uint64)
    a = D.hash_word(0, 0, 0, 0, g)
    b = D.hash_word(0, 0, 0, 0, g ^ np.uint64(1))
    flips = np.array([bin(int(x)).count("1") for x in (a ^ b)])
    assert 28 < flips.mean() < 36
