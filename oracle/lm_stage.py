"""First- and last-stage extras of the GPT model, oracle side (test infrastructure only).

The paper fixes little here: eq. (2) counts (V + s) h embedding parameters (a
V x h word table and an s x h position table) and the appendix counts the
logit layer, which maps features of size h to the vocabulary (2 B s h V FLOPs
forward, 4 B s h V backward).  Everything else below is a stated reading:

* input: x[i, j, :] = E_word[token[i, j]] + E_pos[i], then hidden dropout
  (stream of layer id EMBED_LAYER, site 0);
* output: u = LayerNorm(y) (gain, bias), logits = u E_word^T (the word table is
  shared between input and output), loss = mean over the s*b tokens of
  log(sum_v exp(logit_v)) - logit_target;
* one tensor-parallel shard holds vocabulary rows [v0, v0 + rows): tokens and
  targets outside the range contribute zero rows / zero target logits, and the
  maximum and the sum of exponentials are taken over the shard's rows (the
  cross-shard reductions are the identity on one shard, exactly as for the
  layer's f and g operators).

Pins (tests/test_oracle_lm_stage.py): central finite differences of the loss
w.r.t. every input, an independent derivation through torch's embedding,
layer_norm and cross_entropy with autograd, uniform logits -> log(rows),
shards' partial embeddings summing to the unsharded one, the FLOP closed form
against the products actually performed.
"""
import numpy as np

from . import dropout_hash
from . import gpt_layer as L

EMBED_LAYER = (1 << 31) - 1   # layer id of the embedding's dropout stream


def embedding_forward(tokens, e_word, e_pos, cfg, v0=0, microbatch=0):
    """tokens [s, b] int; e_word [rows, h] = vocabulary rows v0..v0+rows-1; e_pos [s, h]."""
    s, b = tokens.shape
    rows, h = e_word.shape
    local = tokens - v0
    inside = (local >= 0) & (local < rows)
    x = np.where(inside[..., None], e_word[np.clip(local, 0, rows - 1)], 0.0)
    x = x + e_pos[:s, None, :]
    keep = dropout_hash.keep_mask(cfg.seed, EMBED_LAYER, 0, microbatch, s * b * h, cfg.p_hidden).reshape(s, b, h)
    return x * keep * dropout_hash.keep_scale(cfg.p_hidden)


def embedding_backward(dx, tokens, rows, cfg, v0=0, microbatch=0):
    """Returns (d e_word [rows, h], d e_pos [s, h])."""
    s, b, h = dx.shape
    keep = dropout_hash.keep_mask(cfg.seed, EMBED_LAYER, 0, microbatch, s * b * h, cfg.p_hidden).reshape(s, b, h)
    d = dx * keep * dropout_hash.keep_scale(cfg.p_hidden)
    d_pos = d.sum(axis=1)
    d_word = np.zeros((rows, h))
    for i in range(s):
        for j in range(b):
            r = tokens[i, j] - v0
            if 0 <= r < rows:
                d_word[r] += d[i, j]
    return d_word, d_pos


def head_forward(y, gain, bias, e_word, targets, cfg, v0=0):
    """Final LayerNorm, logits against the shard's rows, mean token loss.  Returns (loss, cache)."""
    s, b, h = y.shape
    rows = e_word.shape[0]
    u, mu, rstd = L.layernorm(y, gain, bias, cfg.ln_eps)
    logits = u.reshape(s * b, h) @ e_word.T                      # [T, rows]
    m = logits.max(axis=1, keepdims=True)
    z = np.exp(logits - m).sum(axis=1, keepdims=True)
    local = targets.reshape(-1) - v0
    inside = (local >= 0) & (local < rows)
    picked = np.where(inside, logits[np.arange(s * b), np.clip(local, 0, rows - 1)], 0.0)
    per_token = np.log(z[:, 0]) + m[:, 0] - picked
    return per_token.mean(), dict(y=y, u=u, mu=mu, rstd=rstd, logits=logits, m=m, z=z, local=local, inside=inside,
                                  per_token=per_token)


def head_backward(cache, gain, e_word, dloss=1.0):
    """Gradients of dloss * loss: returns (dy, dgain, dbias, d e_word)."""
    y, u = cache["y"], cache["u"]
    s, b, h = y.shape
    T = s * b
    p = np.exp(cache["logits"] - cache["m"]) / cache["z"]
    idx = np.arange(T)[cache["inside"]]
    p[idx, cache["local"][cache["inside"]]] -= 1.0
    dlogits = p * (dloss / T)
    du = (dlogits @ e_word).reshape(s, b, h)
    d_word = dlogits.T @ u.reshape(T, h)
    dy, dgain, dbias = L.layernorm_backward(du, y, gain, cache["mu"], cache["rstd"])
    return dy, dgain, dbias, d_word


def logit_flops(B, s, h, V):
    """Appendix: the logit layer's forward product and its two backward products."""
    fwd = 2 * (B * s) * h * V
    return fwd, 2 * fwd
