"""Pins of the general-mask attention of the oracle (section 4.2: the fused scale + mask + softmax
kernel with a general mask)."""
import numpy as np
import torch

from oracle import gpt_layer as L


def _case(seed=0, s=9, b=2, h=32, a=4):
    cfg = L.LayerConfig(h=h, a=a, t=1, s=s, b=b, causal=False)
    rng = np.random.default_rng(seed)
    qkv = rng.standard_normal((s, b, 3 * h))
    mask = (rng.random((b, s, s)) < 0.35).astype(np.uint8)
    for j in range(b):
        np.fill_diagonal(mask[j], 0)                   # every query sees itself: no empty rows here
    return cfg, rng, qkv, mask


def test_against_library_attention_with_boolean_mask():
    cfg, rng, qkv, mask = _case()
    ctx, probs, lse = L.attention_core(qkv, cfg, mask)
    t = torch.tensor(qkv)
    h, dh = cfg.h, cfg.dh
    q, k, v = [t[:, :, i * h:(i + 1) * h].reshape(cfg.s, cfg.b, cfg.a, dh).permute(1, 2, 0, 3) for i in range(3)]
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=torch.tensor(mask == 0)[:, None])
    assert np.allclose(ctx, want.permute(2, 0, 1, 3).reshape(cfg.s, cfg.b, h).numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(probs.sum(axis=-1), 1.0) and np.all(probs[np.broadcast_to(mask[:, None] != 0, probs.shape)] == 0.0)


def test_no_mask_is_plain_softmax_and_all_but_causal_mask_matches_causal_path():
    cfg, rng, qkv, _ = _case(1)
    ctx0, p0, lse0 = L.attention_core(qkv, cfg, None)
    sc = np.einsum("id,kd->ik", qkv[:, 0, :cfg.dh], qkv[:, 0, cfg.h:cfg.h + cfg.dh]) / np.sqrt(cfg.dh)
    e = np.exp(sc - sc.max(axis=1, keepdims=True))
    assert np.allclose(p0[0, 0], e / e.sum(axis=1, keepdims=True), rtol=1e-13)
    upper = np.triu(np.ones((cfg.s, cfg.s), dtype=np.uint8), 1)
    ctx1, p1, lse1 = L.attention_core(qkv, cfg, np.broadcast_to(upper, (cfg.b, cfg.s, cfg.s)))
    ccfg = L.LayerConfig(h=cfg.h, a=cfg.a, t=1, s=cfg.s, b=cfg.b, causal=True)
    ctx2, p2, lse2 = L.attention_core(qkv, ccfg)
    assert np.allclose(ctx1, ctx2, rtol=1e-13) and np.allclose(lse1, lse2, rtol=1e-13) and np.array_equal(p1 == 0, p2 == 0)


def test_row_with_no_visible_key_attends_uniformly():
    cfg, rng, qkv, mask = _case(2)
    mask[1, 4, :] = 1
    ctx, probs, lse = L.attention_core(qkv, cfg, mask)
    assert np.allclose(probs[1, :, 4, :], 1.0 / cfg.s)
    v = qkv[:, 1, 2 * cfg.h:]
    assert np.allclose(ctx[4, 1], v.mean(axis=0))
    assert np.allclose(lse[1, :, 4], L.MASK_FILL + np.log(cfg.s))


def test_gradients_by_finite_differences_including_an_empty_row():
    cfg, rng, qkv, mask = _case(3, s=6, b=1, h=16, a=2)
    mask[0, 2, :] = 1
    w = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    f = lambda z: (L.attention_core(z, cfg, mask)[0] * w).sum()
    ctx, probs, _ = L.attention_core(qkv, cfg, mask)
    g = L.attention_core_backward(w, qkv, probs, cfg, mask)
    eps = 1e-6
    flat = qkv.reshape(-1)
    for idx in rng.choice(flat.size, size=60, replace=False):
        old = flat[idx]
        flat[idx] = old + eps; fp = f(qkv)
        flat[idx] = old - eps; fm = f(qkv)
        flat[idx] = old
        assert abs((fp - fm) / (2 * eps) - g.reshape(-1)[idx]) < 1e-7, idx
    # the empty row's query gets no gradient at all
    assert np.all(g[2, 0, :cfg.h] == 0.0)


def test_layer_with_general_mask_runs_forward_and_backward_consistently():
    cfg, rng, qkv, mask = _case(4, s=5, b=2, h=16, a=2)
    P = {}
    for k, shp in L.param_shapes(cfg).items():
        P[k] = (1.0 + 0.1 * rng.standard_normal(shp)) if k.endswith("_g") else 0.1 * rng.standard_normal(shp)
    x = rng.standard_normal((cfg.s, cfg.b, cfg.h)); dy = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    y, cache = L.layer_forward(x, P, cfg, mask=mask)
    dx, G = L.layer_backward(dy, P, cfg, cache)
    eps = 1e-6
    for idx in rng.choice(x.size, size=10, replace=False):
        xp = x.copy().reshape(-1); xm = x.copy().reshape(-1)
        xp[idx] += eps; xm[idx] -= eps
        fp = (L.layer_forward(xp.reshape(x.shape), P, cfg, mask=mask)[0] * dy).sum()
        fm = (L.layer_forward(xm.reshape(x.shape), P, cfg, mask=mask)[0] * dy).sum()
        assert abs((fp - fm) / (2 * eps) - dx.reshape(-1)[idx]) < 1e-6
