"""Pins of the activation-recomputation oracle (section 3.5)."""
import numpy as np
import pytest

from oracle import gpt_layer as L
from oracle import recompute as R


def _params(cfg, n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        P = {}
        for k, shp in L.param_shapes(cfg).items():
            if k.endswith("_g"):
                P[k] = 1.0 + 0.1 * rng.standard_normal(shp)
            elif k.startswith("w_"):
                P[k] = 0.05 * rng.standard_normal(shp)
            else:
                P[k] = 0.1 * rng.standard_normal(shp)
        out.append(P)
    return out


@pytest.mark.parametrize("l,a_in,a_int", [(80, 1.0, 17.0), (96, 2.0, 5.0), (4, 3.0, 40.0), (128, 7.0, 7.0)])
def test_optimum_closed_form_vs_brute_force(l, a_in, a_int):
    c_star = R.optimal_checkpoints(l, a_in, a_int)
    grid = np.linspace(0.05, 4 * l, 400001)
    brute = grid[np.argmin(R.kept_bytes(grid, l, a_in, a_int))]
    assert abs(brute - c_star) <= 2 * (grid[1] - grid[0])
    # stationarity: d/dc (c A_in + l A_int / c) = A_in - l A_int / c^2 = 0
    assert abs(a_in - l * a_int / c_star ** 2) < 1e-12 * a_in
    # the minimum value is 2 sqrt(l A_in A_int) (both terms equal there)
    assert np.isclose(R.kept_bytes(c_star, l, a_in, a_int), 2 * np.sqrt(l * a_in * a_int), rtol=1e-13)
    assert np.isclose(c_star * a_in, (l / c_star) * a_int, rtol=1e-13)


def test_extremes_of_the_memory_model():
    # one checkpoint = the stage input only; l checkpoints = every layer's input + one layer of intermediates
    assert R.kept_bytes(1, 12, 3.0, 10.0) == 3.0 + 12 * 10.0
    assert R.kept_bytes(12, 12, 3.0, 10.0) == 12 * 3.0 + 10.0


@pytest.mark.parametrize("n,seg", [(4, 1), (4, 2), (4, 4), (5, 2), (3, 3)])
def test_recompute_backward_is_the_plain_backward(n, seg):
    cfg = L.LayerConfig(h=16, a=2, t=1, s=5, b=2, p_hidden=0.25, seed=11)
    Ps = _params(cfg, n, 3)
    rng = np.random.default_rng(5)
    x = rng.standard_normal((cfg.s, cfg.b, cfg.h)); dy = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    y0, caches = L.chunk_forward(x, Ps, cfg, first_layer=6, microbatch=3)
    dx0, g0 = L.chunk_backward(dy, Ps, cfg, caches)
    y1, ck = R.chunk_forward_checkpoints(x, Ps, cfg, seg, first_layer=6, microbatch=3)
    ledger = []
    dx1, g1 = R.chunk_backward_recompute(dy, Ps, cfg, ck, seg, first_layer=6, microbatch=3, ledger=ledger)
    assert np.array_equal(y0, y1) and np.array_equal(dx0, dx1)
    for a, b in zip(g0, g1):
        for k in a:
            assert np.array_equal(a[k], b[k]), k
    # live arrays follow c*A_in + (l/c)*A_int: all c checkpoints exist when the last segment runs,
    # and never more than seg layer caches
    c = len(ck)
    assert c == -(-n // seg)
    assert ledger[0][0] == c and max(m for _, m in ledger) == min(seg, n)
    if n % seg == 0:
        a_in, a_int = 1.0, 9.0
        assert ledger[0][0] * a_in + ledger[0][1] * a_int == R.kept_bytes(c, n, a_in, a_int)


def test_wrong_microbatch_in_the_rerun_changes_the_gradients():
    """The rerun must use the forward's dropout stream: a different microbatch index is a different mask."""
    cfg = L.LayerConfig(h=16, a=2, t=1, s=5, b=2, p_hidden=0.25, seed=11)
    Ps = _params(cfg, 2, 4)
    rng = np.random.default_rng(6)
    x = rng.standard_normal((cfg.s, cfg.b, cfg.h)); dy = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    _, ck = R.chunk_forward_checkpoints(x, Ps, cfg, 1, microbatch=0)
    dx_ok, _ = R.chunk_backward_recompute(dy, Ps, cfg, ck, 1, microbatch=0)
    dx_bad, _ = R.chunk_backward_recompute(dy, Ps, cfg, ck, 1, microbatch=1)
    assert not np.allclose(dx_ok, dx_bad)
