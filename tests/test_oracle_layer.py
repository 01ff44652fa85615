"""Pins for oracle/gpt_layer.py (CPU only): finite differences, an independent
derivation with torch CPU fp64 library routines + autograd, invariants and
degenerate cases."""
import math

import numpy as np
import pytest
import torch

from oracle import dropout_hash
from oracle import flops as F
from oracle import gpt_layer as L


def rand_params(cfg, rng, scale=0.3):
    P = {}
    for k, shp in L.param_shapes(cfg).items():
        if k in ("ln1_g", "ln2_g"):
            P[k] = 1.0 + 0.2 * rng.standard_normal(shp)
        else:
            P[k] = scale * rng.standard_normal(shp)
    return P


TINY = dict(h=16, a=2, s=8, b=2, p_hidden=0.1, seed=3)


@pytest.mark.parametrize("t", [1, 2])
@pytest.mark.parametrize("tanh", [False, True])
def test_backward_by_central_differences(t, tanh):
    cfg = L.LayerConfig(t=t, gelu_tanh=tanh, **TINY)
    rng = np.random.default_rng(10 + t)
    P = rand_params(cfg, rng)
    x = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    w = rng.standard_normal((cfg.s, cfg.b, cfg.h))     # loss = <w, y>
    y, cache = L.layer_forward(x, P, cfg, layer=5, microbatch=2)
    dx, G = L.layer_backward(w, P, cfg, cache)
    loss = lambda xx, PP: float((L.layer_forward(xx, PP, cfg, layer=5, microbatch=2)[0] * w).sum())
    eps = 1e-6

    def check(arr, grad, setter):
        flat = arr.reshape(-1)
        picks = rng.choice(flat.size, size=min(flat.size, 24), replace=False)
        for i in picks:
            old = flat[i]
            flat[i] = old + eps
            lp = setter()
            flat[i] = old - eps
            lm = setter()
            flat[i] = old
            fd = (lp - lm) / (2 * eps)
            assert fd == pytest.approx(grad.reshape(-1)[i], rel=2e-5, abs=2e-7)

    check(x, dx, lambda: loss(x, P))
    for name in L.PARAM_NAMES:
        check(P[name], G[name], lambda: loss(x, P))


def torch_layer(x, P, cfg, keep1, keep2):
    """The same ten steps through torch library routines (independent code)."""
    tf = torch.nn.functional
    h, hp, dh, al = cfg.h, cfg.hp, cfg.dh, cfg.heads_local
    scale = 1.0 / (1.0 - float(np.float32(cfg.p_hidden)))
    u = tf.layer_norm(x, (h,), P["ln1_g"], P["ln1_b"], cfg.ln_eps)
    qkv = tf.linear(u, P["w_qkv"].T, P["b_qkv"])
    q, k, v = qkv.split(hp, dim=-1)
    # [s, b, heads, dh] -> [b, heads, s, dh]
    f = lambda z: z.reshape(cfg.s, cfg.b, al, dh).permute(1, 2, 0, 3)
    ctx = tf.scaled_dot_product_attention(f(q), f(k), f(v), is_causal=True)
    ctx = ctx.permute(2, 0, 1, 3).reshape(cfg.s, cfg.b, hp)
    o = ctx @ P["w_o"]
    x1 = x + (o + P["b_o"]) * keep1 * scale
    u2 = tf.layer_norm(x1, (h,), P["ln2_g"], P["ln2_b"], cfg.ln_eps)
    g = tf.gelu(tf.linear(u2, P["w_1"].T, P["b_1"]), approximate="tanh" if cfg.gelu_tanh else "none")
    return x1 + (g @ P["w_2"] + P["b_2"]) * keep2 * scale


@pytest.mark.parametrize("t,tanh", [(1, False), (2, False), (4, True)])
def test_against_torch_autograd(t, tanh):
    cfg = L.LayerConfig(h=32, a=4, t=t, s=12, b=3, p_hidden=0.2, seed=1, gelu_tanh=tanh)
    rng = np.random.default_rng(4)
    P = rand_params(cfg, rng)
    x = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    w = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    y, cache = L.layer_forward(x, P, cfg, layer=2, microbatch=9)
    dx, G = L.layer_backward(w, P, cfg, cache)

    tP = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in P.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    n = cfg.s * cfg.b * cfg.h
    k1 = torch.tensor(dropout_hash.keep_mask(1, 2, 0, 9, n, 0.2).reshape(x.shape), dtype=torch.float64)
    k2 = torch.tensor(dropout_hash.keep_mask(1, 2, 1, 9, n, 0.2).reshape(x.shape), dtype=torch.float64)
    ty = torch_layer(tx, tP, cfg, k1, k2)
    (ty * torch.tensor(w)).sum().backward()
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-9, atol=1e-11)
    for name in L.PARAM_NAMES:
        np.testing.assert_allclose(G[name], tP[name].grad.numpy(), rtol=1e-9, atol=1e-11, err_msg=name)


def test_softmax_rows_sum_to_one_and_future_is_zero():
    cfg = L.LayerConfig(h=24, a=3, s=10, b=2)
    rng = np.random.default_rng(0)
    qkv = rng.standard_normal((cfg.s, cfg.b, 3 * cfg.hp)) * 3
    ctx, probs, lse = L.attention_core(qkv, cfg)
    np.testing.assert_allclose(probs.sum(axis=-1), 1.0, rtol=1e-13)
    assert (probs[..., np.triu_indices(cfg.s, 1)[0], np.triu_indices(cfg.s, 1)[1]] == 0).all()
    assert (probs[..., 0, 0] == 1).all()                       # row 0 attends only to itself
    # lse is the log of the softmax denominator of the scaled masked scores
    q = qkv[:, 1, 0:cfg.dh]; k = qkv[:, 1, cfg.hp:cfg.hp + cfg.dh]
    i = 6
    sc = (k[: i + 1] @ q[i]) / math.sqrt(cfg.dh)
    assert lse[1, 0, i] == pytest.approx(math.log(np.exp(sc).sum()), rel=1e-12)
    rows, lse_rows = L.attention_rows(qkv, cfg, 1, 2, [0, 3, 9])
    np.testing.assert_allclose(rows, ctx[[0, 3, 9], 1, 2 * cfg.dh:3 * cfg.dh], rtol=1e-12)
    np.testing.assert_allclose(lse_rows, lse[1, 2, [0, 3, 9]], rtol=1e-12)


def test_causal_invariance_is_bit_exact():
    cfg = L.LayerConfig(h=32, a=4, s=16, b=2, p_hidden=0.1, seed=7)
    rng = np.random.default_rng(2)
    P = rand_params(cfg, rng)
    x = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    y, _ = L.layer_forward(x, P, cfg)
    i = 9
    x2 = x.copy()
    x2[i + 1:] += rng.standard_normal(x2[i + 1:].shape)
    y2, _ = L.layer_forward(x2, P, cfg)
    assert np.array_equal(y[: i + 1], y2[: i + 1])
    assert not np.array_equal(y[i + 1:], y2[i + 1:])


def test_tensor_parallel_sum_equals_unsharded():
    full = L.LayerConfig(h=32, a=4, t=1, s=9, b=2)
    rng = np.random.default_rng(5)
    P = rand_params(full, rng)
    x = rng.standard_normal((full.s, full.b, full.h))
    o_full = L.attention_block_partial(x, P, full)
    mo_full = L.mlp_block_partial(x, P, full)
    for t in (2, 4):
        cfg = L.LayerConfig(h=32, a=4, t=t, s=9, b=2)
        shards = [L.shard_params(P, full, t, r) for r in range(t)]
        np.testing.assert_allclose(sum(L.attention_block_partial(x, S, cfg) for S in shards), o_full, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(sum(L.mlp_block_partial(x, S, cfg) for S in shards), mo_full, rtol=1e-11, atol=1e-13)
        # column-parallel outputs concatenate: [Y1, Y2] = [GeLU(X A1), GeLU(X A2)]
        u2, _, _ = L.layernorm(x, P["ln2_g"], P["ln2_b"], 1e-5)
        cat = np.concatenate([L.gelu(u2 @ S["w_1"] + S["b_1"]) for S in shards], axis=-1)
        np.testing.assert_allclose(cat, L.gelu(u2 @ P["w_1"] + P["b_1"]), rtol=1e-12)
    # backward: input gradients of the column-parallel GEMMs sum over shards (operator f)
    w = rng.standard_normal(x.shape)
    full_p0 = L.LayerConfig(h=32, a=4, t=1, s=9, b=2, p_hidden=0.0)
    y, c = L.layer_forward(x, P, full_p0)
    dx_full, G_full = L.layer_backward(w, P, full_p0, c)
    # with p = 0 and zero row-parallel biases, y - x = sum over shards of (y_shard - x) is NOT
    # linear across the two blocks, so compare block-wise instead:
    t = 2
    cfg = L.LayerConfig(h=32, a=4, t=t, s=9, b=2)
    shards = [L.shard_params(P, full, t, r) for r in range(t)]
    for block, key in ((L.attention_block_partial, "w_o"), (L.mlp_block_partial, "w_2")):
        eps = 1e-6
        d = rng.standard_normal(x.shape)
        fd_full = ((block(x + eps * d, P, full) - block(x - eps * d, P, full)) / (2 * eps))
        fd_sum = sum((block(x + eps * d, S, cfg) - block(x - eps * d, S, cfg)) / (2 * eps) for S in shards)
        np.testing.assert_allclose(fd_sum, fd_full, rtol=1e-6, atol=1e-8)


def test_parameter_count_matches_eq2_per_layer_term():
    for h, a in ((256, 4), (12288, 96)):
        cfg = L.LayerConfig(h=h, a=a)
        n = sum(int(np.prod(s)) for s in L.param_shapes(cfg).values())
        assert n == 12 * h * h + 13 * h
        assert F.parameters(3, h, 0, 0) == 3 * n
    # one of t shards holds 1/t of every matrix
    cfg = L.LayerConfig(h=64, a=8, t=4)
    shp = L.param_shapes(cfg)
    assert sum(int(np.prod(shp[k])) for k in ("w_qkv", "w_o", "w_1", "w_2")) == 12 * 64 * 64 // 4


def test_degenerate_cases():
    rng = np.random.default_rng(8)
    # s = 1: ctx = v
    cfg = L.LayerConfig(h=16, a=2, s=1, b=3)
    qkv = rng.standard_normal((1, 3, 48))
    ctx, _, lse = L.attention_core(qkv, cfg)
    np.testing.assert_allclose(ctx, qkv[..., 32:], rtol=1e-14)
    # all matrices zero: y = x + D1(b_o) + D2(b_2)
    cfg = L.LayerConfig(h=16, a=2, s=5, b=2, p_hidden=0.25, seed=11)
    P = {k: np.zeros(s) for k, s in L.param_shapes(cfg).items()}
    P["b_o"] = rng.standard_normal(16); P["b_2"] = rng.standard_normal(16)
    P["ln1_g"][:] = 1; P["ln2_g"][:] = 1
    x = rng.standard_normal((5, 2, 16))
    y, c = L.layer_forward(x, P, cfg, layer=1, microbatch=4)
    k1 = dropout_hash.keep_mask(11, 1, 0, 4, x.size, 0.25).reshape(x.shape)
    k2 = dropout_hash.keep_mask(11, 1, 1, 4, x.size, 0.25).reshape(x.shape)
    sc = 1 / (1 - float(np.float32(0.25)))
    np.testing.assert_allclose(y, x + P["b_o"] * k1 * sc + P["b_2"] * k2 * sc, rtol=1e-14)
    # p = 0: dropout is the identity
    cfg0 = L.LayerConfig(h=16, a=2, s=5, b=2, p_hidden=0.0)
    y0, c0 = L.layer_forward(x, P, cfg0)
    np.testing.assert_allclose(y0, x + P["b_o"] + P["b_2"], rtol=1e-14)
    assert c0["keep1"].all() and c0["keep2"].all()
    # LayerNorm: gain 1, bias 0 -> rows with mean 0 and variance var/(var+eps); constant row -> bias
    u, mu, rstd = L.layernorm(x, np.ones(16), np.zeros(16), 1e-5)
    np.testing.assert_allclose(u.mean(-1), 0, atol=1e-14)
    np.testing.assert_allclose(u.var(-1), x.var(-1) / (x.var(-1) + 1e-5), rtol=1e-12)
    beta = rng.standard_normal(16)
    u, _, _ = L.layernorm(np.full((2, 16), 3.7), rng.standard_normal(16), beta, 1e-5)
    np.testing.assert_allclose(u, np.broadcast_to(beta, (2, 16)), atol=1e-9)


def test_gelu_values_and_derivative():
    assert L.gelu(np.array([0.0]))[0] == 0
    assert L.gelu(np.array([1.0]))[0] == pytest.approx(0.8413447460685429, rel=1e-14)   # Phi(1)
    assert L.gelu(np.array([-1.0]))[0] == pytest.approx(-0.15865525393145707, rel=1e-13)
    z = np.linspace(-4, 4, 41)
    for tanh in (False, True):
        fd = (L.gelu(z + 1e-6, tanh) - L.gelu(z - 1e-6, tanh)) / 2e-6
        np.testing.assert_allclose(L.gelu_grad(z, tanh), fd, rtol=1e-7, atol=1e-9)
    assert np.abs(L.gelu(z, True) - L.gelu(z, False)).max() < 1e-3


def test_flop_count_of_the_six_products():
    # count 2mkn over the matrix products the oracle actually performs on one shard
    cfg = L.LayerConfig(h=64, a=8, t=2, s=32, b=3)
    T = cfg.s * cfg.b
    n = (2 * T * cfg.h * 3 * cfg.hp + cfg.b * cfg.heads_local * (2 * cfg.s * cfg.dh * cfg.s) * 2
         + 2 * T * cfg.hp * cfg.h + 2 * T * cfg.h * cfg.fp + 2 * T * cfg.fp * cfg.h)
    assert n == F.layer_forward_flops(cfg.b, cfg.s, cfg.h) // cfg.t
    assert 3 * n == F.shard_layer_flops(cfg.b, cfg.s, cfg.h, cfg.t)


def test_chunk_is_composition_and_grads_accumulate():
    cfg = L.LayerConfig(h=16, a=2, s=6, b=2, p_hidden=0.1, seed=2)
    rng = np.random.default_rng(3)
    Ps = [rand_params(cfg, rng) for _ in range(3)]
    x = rng.standard_normal((6, 2, 16))
    y, caches = L.chunk_forward(x, Ps, cfg, first_layer=4, microbatch=1)
    z = x
    for i, P in enumerate(Ps):
        z, _ = L.layer_forward(z, P, cfg, layer=4 + i, microbatch=1)
    assert np.array_equal(y, z)
    w = rng.standard_normal(y.shape)
    dx, grads = L.chunk_backward(w, Ps, cfg, caches)
    eps = 1e-6
    d = rng.standard_normal(x.shape)
    fd = ((L.chunk_forward(x + eps * d, Ps, cfg, 4, 1)[0] - L.chunk_forward(x - eps * d, Ps, cfg, 4, 1)[0]) * w).sum() / (2 * eps)
    assert fd == pytest.approx((dx * d).sum(), rel=1e-6)
