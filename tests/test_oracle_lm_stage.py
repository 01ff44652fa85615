"""Pins of the first/last-stage oracle (embeddings, final LayerNorm, logit layer, loss)."""
import numpy as np
import pytest
import torch

from oracle import flops as F
from oracle import gpt_layer as L
from oracle import lm_stage as S


def _setup(p=0.0, s=6, b=2, h=16, V=40, seed=0):
    cfg = L.LayerConfig(h=h, a=2, t=1, s=s, b=b, p_hidden=p, seed=5)
    rng = np.random.default_rng(seed)
    tokens = rng.integers(0, V, size=(s, b))
    tokens[1, 0] = tokens[0, 0]                       # a repeated id: its rows' gradients must add up
    targets = rng.integers(0, V, size=(s, b))
    e_word = 0.3 * rng.standard_normal((V, h)); e_pos = 0.3 * rng.standard_normal((s, h))
    gain = 1.0 + 0.1 * rng.standard_normal(h); bias = 0.1 * rng.standard_normal(h)
    return cfg, rng, tokens, targets, e_word, e_pos, gain, bias


def _loss(tokens, targets, e_word, e_pos, gain, bias, cfg):
    x = S.embedding_forward(tokens, e_word, e_pos, cfg, microbatch=2)
    return S.head_forward(x, gain, bias, e_word, targets, cfg)[0]


@pytest.mark.parametrize("p", [0.0, 0.3])
def test_finite_differences_through_embedding_and_head(p):
    """loss(tokens -> embedding -> final LN -> logits -> loss) with the word table used twice."""
    cfg, rng, tokens, targets, e_word, e_pos, gain, bias = _setup(p)
    x = S.embedding_forward(tokens, e_word, e_pos, cfg, microbatch=2)
    loss, cache = S.head_forward(x, gain, bias, e_word, targets, cfg)
    dy, dgain, dbias, dw_head = S.head_backward(cache, gain, e_word)
    dw_emb, dpos = S.embedding_backward(dy, tokens, e_word.shape[0], cfg, microbatch=2)
    grads = {"e_word": dw_head + dw_emb, "e_pos": dpos, "gain": dgain, "bias": dbias}
    vals = {"e_word": e_word, "e_pos": e_pos, "gain": gain, "bias": bias}
    eps = 1e-6
    for name, arr in vals.items():
        flat = arr.reshape(-1)
        for idx in rng.choice(flat.size, size=min(12, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + eps; lp = _loss(tokens, targets, e_word, e_pos, gain, bias, cfg)
            flat[idx] = old - eps; lm = _loss(tokens, targets, e_word, e_pos, gain, bias, cfg)
            flat[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grads[name].reshape(-1)[idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx)


def test_against_torch_autograd():
    cfg, rng, tokens, targets, e_word, e_pos, gain, bias = _setup(0.0, s=5, b=3, h=24, V=31, seed=3)
    tw = torch.tensor(e_word, requires_grad=True); tp = torch.tensor(e_pos, requires_grad=True)
    tg = torch.tensor(gain, requires_grad=True); tb = torch.tensor(bias, requires_grad=True)
    tok = torch.tensor(tokens); tgt = torch.tensor(targets)
    x = torch.nn.functional.embedding(tok, tw) + tp[:, None, :]
    u = torch.nn.functional.layer_norm(x, (cfg.h,), tg, tb, cfg.ln_eps)
    logits = u.reshape(-1, cfg.h) @ tw.T
    loss = torch.nn.functional.cross_entropy(logits, tgt.reshape(-1))
    loss.backward()
    x0 = S.embedding_forward(tokens, e_word, e_pos, cfg)
    l0, cache = S.head_forward(x0, gain, bias, e_word, targets, cfg)
    dy, dgain, dbias, dwh = S.head_backward(cache, gain, e_word)
    dwe, dpos = S.embedding_backward(dy, tokens, e_word.shape[0], cfg)
    assert np.isclose(l0, loss.item(), rtol=1e-12)
    for got, want in [(dwh + dwe, tw.grad), (dpos, tp.grad), (dgain, tg.grad), (dbias, tb.grad)]:
        assert np.allclose(got, want.numpy(), rtol=1e-9, atol=1e-12)


def test_uniform_logits_give_log_of_row_count():
    cfg, rng, tokens, targets, e_word, e_pos, gain, bias = _setup()
    y = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    loss, cache = S.head_forward(y, gain, bias, np.zeros_like(e_word), targets, cfg)
    assert np.isclose(loss, np.log(e_word.shape[0]), rtol=1e-14)
    dy, dgain, dbias, dw = S.head_backward(cache, gain, np.zeros_like(e_word))
    assert np.allclose(dy, 0.0) and np.allclose(dw.sum(axis=0), 0.0, atol=1e-15)   # rows of softmax - onehot sum to 0


def test_vocabulary_shards():
    """Partial embeddings of the shards add up to the unsharded embedding; a shard that holds no
    target of a token leaves that token's gradient row a plain softmax."""
    cfg, rng, tokens, targets, e_word, e_pos, gain, bias = _setup()
    V = e_word.shape[0]
    full = S.embedding_forward(tokens, e_word, np.zeros_like(e_pos), cfg)
    parts = sum(S.embedding_forward(tokens, e_word[v0:v0 + V // 4], np.zeros_like(e_pos), cfg, v0=v0)
                for v0 in range(0, V, V // 4))
    assert np.allclose(full, parts, rtol=0, atol=0)
    y = rng.standard_normal((cfg.s, cfg.b, cfg.h))
    v0 = V // 2
    loss, cache = S.head_forward(y, gain, bias, e_word[v0:], targets, cfg, v0=v0)
    outside = ~cache["inside"]
    assert outside.any() and cache["inside"].any()
    p = np.exp(cache["logits"] - cache["m"]) / cache["z"]
    dl = S.head_backward(cache, gain, e_word[v0:])
    assert np.allclose(cache["per_token"][outside], (np.log(cache["z"]) + cache["m"])[outside, 0])
    assert np.allclose(p.sum(axis=1), 1.0)


def test_embedding_dropout_uses_its_own_stream():
    cfg, rng, tokens, targets, e_word, e_pos, gain, bias = _setup(0.5)
    x = S.embedding_forward(tokens, e_word, e_pos, cfg, microbatch=1)
    keep_layer0 = L.dropout_keep(cfg, 0, 0, 1)
    kept = x != 0
    assert 0.3 < kept.mean() < 0.7 and (kept != (keep_layer0 != 0)).any()
    assert np.allclose(x[kept], (2.0 * (e_word[tokens] + e_pos[:, None, :]))[kept])


def test_logit_flops_closed_form():
    B, s, h, V = 3, 7, 16, 40
    fwd, bwd = S.logit_flops(B, s, h, V)
    assert fwd == 2 * B * s * h * V and bwd == 4 * B * s * h * V
    # eq. (3) = 4 x the layers' forward + the logit layer's 6 B s h V
    l = 5
    assert F.iteration_flops(B, s, l, h, V) == 4 * l * F.layer_forward_flops(B, s, h) + fwd + bwd
