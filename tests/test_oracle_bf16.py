"""Pins of the bfloat16 storage rounding and of the oracle's storage-rounded mode (CPU only)."""
import numpy as np
import torch

from oracle import bf16
from oracle import gpt_layer as L


def test_round_bf16_hand_values():
    """bfloat16 keeps 7 fraction bits: spacing 2^-7 in [1, 2).  Ties go to the even neighbour."""
    u = 2.0 ** -7
    r = bf16.round_bf16
    assert r(1.0) == 1.0 and r(-2.5) == -2.5 and r(0.0) == 0.0
    assert r(1.0 + u) == 1.0 + u                         # representable
    assert r(1.0 + u / 2) == 1.0                         # tie: 1.0 has an even last bit
    assert r(1.0 + 3 * u / 2) == 1.0 + 2 * u             # tie: rounds up to the even one
    assert r(1.0 + u / 2 + 2.0 ** -20) == 1.0 + u        # just above the tie
    assert r(1.0 + u / 2 - 2.0 ** -20) == 1.0            # just below
    assert r(-(1.0 + 3 * u / 2)) == -(1.0 + 2 * u)       # sign-symmetric
    assert r(2.0 - u / 4) == 2.0                         # carries into the exponent
    assert r(3.0e38) == float(torch.tensor(3.0e38).to(torch.bfloat16).double())
    assert np.isinf(r(np.inf)) and np.isnan(r(np.nan))
    assert r(np.float64(2.0 ** -130)) == 2.0 ** -130     # subnormal of binary32, representable in bfloat16


def test_round_bf16_matches_library_conversion_and_error_bound():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(200000), rng.standard_normal(1000) * 1e-30, rng.standard_normal(1000) * 1e30,
                        np.ldexp(rng.integers(128, 256, 5000) + 0.5, rng.integers(-20, 20, 5000))])   # many exact ties
    got = bf16.round_bf16(x)
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, want)
    assert np.array_equal(bf16.round_bf16(got), got)                          # idempotent
    assert (np.abs(got - x) <= np.abs(x) * 2.0 ** -8 + 1e-45).all()          # half a unit in the last place
    assert got.shape == x.shape and bf16.round_bf16(x.reshape(4, -1)).shape == (4, x.size // 4)


def tiny():
    cfg = L.LayerConfig(h=32, a=4, t=2, s=12, b=2, p_hidden=0.1, seed=3)
    rng = np.random.default_rng(1)
    P = {k: rng.standard_normal(shp) * (0.2 if len(shp) == 2 else 0.1) for k, shp in L.param_shapes(cfg).items()}
    P["ln1_g"] += 1.0; P["ln2_g"] += 1.0
    x = rng.standard_normal((cfg.s, cfg.b, cfg.h)); dy = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    return cfg, P, x, dy


def test_storage_none_and_identity_are_the_exact_path():
    cfg, P, x, dy = tiny()
    y0, c0 = L.layer_forward(x, P, cfg, 1, 2)
    y1, c1 = L.layer_forward(x, P, cfg, 1, 2, storage=lambda a: a)
    assert np.array_equal(y0, y1)
    dx0, g0 = L.layer_backward(dy, P, cfg, c0)
    dx1, g1 = L.layer_backward(dy, P, cfg, c1)
    assert np.array_equal(dx0, dx1) and all(np.array_equal(g0[k], g1[k]) for k in g0)


def test_storage_rounding_is_applied_where_tensors_are_handed_on():
    """Every cached activation and both outputs are bfloat16 values; parameter gradients are not rounded; and
    the rounded run stays within a few units of bfloat16 precision of the exact one (mild softmax here)."""
    cfg, P, x, dy = tiny()
    Pb = {k: bf16.round_bf16(v) for k, v in P.items()}
    xb, dyb = bf16.round_bf16(x), bf16.round_bf16(dy)
    y, c = L.layer_forward(xb, Pb, cfg, 1, 2, storage=bf16.round_bf16)
    dx, g = L.layer_backward(dyb, Pb, cfg, c)
    is_bf16 = lambda a: np.array_equal(bf16.round_bf16(a), a)
    for k in ("u", "qkv", "ctx", "o", "x1", "u2", "g", "mo"):
        assert is_bf16(c[k]), k
    assert np.array_equal(c["z"], bf16.round_bf16(c["u2"] @ Pb["w_1"]) + Pb["b_1"])      # stored before its bias
    assert is_bf16(y) and is_bf16(dx)
    assert not is_bf16(g["w_1"]) and not is_bf16(g["ln1_g"])
    ye, ce = L.layer_forward(xb, Pb, cfg, 1, 2)
    dxe, ge = L.layer_backward(dyb, Pb, cfg, ce)
    rel = lambda a, b: np.linalg.norm(a - b) / np.linalg.norm(b)
    assert 1e-4 < rel(y, ye) < 1e-2 and 1e-4 < rel(dx, dxe) < 2e-2
    for k in ge:
        assert rel(g[k], ge[k]) < 2e-2, k
    # a chunk carries the rounding through its layers
    y2, caches = L.chunk_forward(xb, [Pb, Pb], cfg, 0, 0, storage=bf16.round_bf16)
    assert is_bf16(y2) and all(cc["storage"] is bf16.round_bf16 for cc in caches)
    dx2, _ = L.chunk_backward(dyb, [Pb, Pb], cfg, caches)
    assert is_bf16(dx2)
