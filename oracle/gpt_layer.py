"""One tensor-parallel shard of a GPT transformer layer, forward and backward,
written out from its definition in fp64 (oracle side; test infrastructure).

What is computed follows the paper's description of the layer (section 2.3):
a self-attention block (Q, K, V projections split by heads across the ``t``
tensor-parallel ranks, output projection split by rows) followed by a
two-layer MLP ``Y = GeLU(XA)``, ``Z = Dropout(YB)`` with ``A`` split by
columns and ``B`` by rows, the partial results of the row-split GEMMs being
summed over ranks *before* bias and dropout.  The fused element-wise groups
named in section 4.2 (bias + GeLU, bias + dropout + add, scale + causal mask
+ softmax) fix where biases, dropout and the residual additions sit.  The
parameter count of eq. (2) (12 h^2 + 13 h per layer) fixes that all four
linear maps have a bias and that there are two LayerNorms with gain and bias.
The activation layout is ``[s, b, h]`` (section 4.2).

Points the paper leaves open, and the reading taken here:

* pre-LayerNorm residual blocks (GPT-2/3 style), eps = 1e-5, biased variance;
* exact (erf) GeLU by default, tanh form on request;
* attention scale 1/sqrt(dh); causal mask gives exactly zero probability;
  no dropout on attention probabilities;
* inverted dropout with the counter-based mask of ``dropout_hash``;
* on a single shard the all-reduce operators ``f`` and ``g`` are the identity
  (the other ranks contribute zero), so the forward pass continues from the
  shard's own partial sum.

Parameters of one shard (all numpy arrays, any float dtype, used as fp64):
  ln1_g, ln1_b [h]; w_qkv [h, 3*hp], b_qkv [3*hp]; w_o [hp, h], b_o [h];
  ln2_g, ln2_b [h]; w_1 [h, fp], b_1 [fp]; w_2 [fp, h], b_2 [h]
with ``hp = h/t`` (local heads * dh) and ``fp = 4h/t``.  The columns of
``w_qkv`` are ordered [Q of all local heads | K | V], each head contiguous.
Weights are stored [in, out] so that ``Y = X A`` is a plain matmul.

No blocking, fusion or reordering: every step is the textbook formula, with
``numpy.matmul`` as the matrix-product primitive.
"""
import math
from dataclasses import dataclass

import numpy as np
from scipy.special import erf

from . import dropout_hash

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


@dataclass
class LayerConfig:
    h: int            # full hidden size
    a: int            # full number of attention heads
    t: int = 1        # tensor-parallel degree
    s: int = 1        # sequence length
    b: int = 1        # microbatch size
    p_hidden: float = 0.0   # dropout probability at the two hidden sites
    ln_eps: float = 1e-5
    gelu_tanh: bool = False
    seed: int = 0
    causal: bool = True     # False: general mask (section 4.2, the kernel "used in models such as BERT")

    @property
    def dh(self):
        return self.h // self.a

    @property
    def heads_local(self):
        return self.a // self.t

    @property
    def hp(self):
        return self.h // self.t

    @property
    def fp(self):
        return 4 * self.h // self.t


def param_shapes(cfg):
    h, hp, fp = cfg.h, cfg.hp, cfg.fp
    return {"ln1_g": (h,), "ln1_b": (h,), "w_qkv": (h, 3 * hp), "b_qkv": (3 * hp,),
            "w_o": (hp, h), "b_o": (h,), "ln2_g": (h,), "ln2_b": (h,),
            "w_1": (h, fp), "b_1": (fp,), "w_2": (fp, h), "b_2": (h,)}


def shard_params(full, cfg_full, t, rank):
    """Shard ``rank`` of ``t`` of an unsharded (t=1) parameter set (section 2.3):
    Q/K/V columns by heads, output projection by rows, first MLP matrix by
    columns, second by rows; LayerNorm parameters and the biases of the
    row-split GEMMs are replicated."""
    h, a = cfg_full.h, cfg_full.a
    dh = h // a
    al = a // t
    cols = np.arange(rank * al * dh, (rank + 1) * al * dh)
    qkv_cols = np.concatenate([cols, h + cols, 2 * h + cols])
    f0, f1 = rank * 4 * h // t, (rank + 1) * 4 * h // t
    return {"ln1_g": full["ln1_g"], "ln1_b": full["ln1_b"],
            "w_qkv": full["w_qkv"][:, qkv_cols], "b_qkv": full["b_qkv"][qkv_cols],
            "w_o": full["w_o"][cols, :], "b_o": full["b_o"],
            "ln2_g": full["ln2_g"], "ln2_b": full["ln2_b"],
            "w_1": full["w_1"][:, f0:f1], "b_1": full["b_1"][f0:f1],
            "w_2": full["w_2"][f0:f1, :], "b_2": full["b_2"]}


# ---------------------------------------------------------------- pieces

def layernorm(x, gain, bias, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    return gain * ((x - mu) * rstd) + bias, mu, rstd


def layernorm_backward(dout, x, gain, mu, rstd):
    """Gradient of ``layernorm`` w.r.t. x, gain, bias."""
    xhat = (x - mu) * rstd
    dgain = (dout * xhat).reshape(-1, x.shape[-1]).sum(axis=0)
    dbias = dout.reshape(-1, x.shape[-1]).sum(axis=0)
    dxhat = dout * gain
    dx = rstd * (dxhat - dxhat.mean(axis=-1, keepdims=True)
                 - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True))
    return dx, dgain, dbias


def gelu(z, tanh_form=False):
    if tanh_form:
        return 0.5 * z * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (z + 0.044715 * z ** 3)))
    return 0.5 * z * (1.0 + erf(z / math.sqrt(2.0)))


def gelu_grad(z, tanh_form=False):
    if tanh_form:
        c = math.sqrt(2.0 / math.pi)
        th = np.tanh(c * (z + 0.044715 * z ** 3))
        return 0.5 * (1.0 + th) + 0.5 * z * (1.0 - th * th) * c * (1.0 + 3 * 0.044715 * z * z)
    return 0.5 * (1.0 + erf(z / math.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)


def causal_softmax_rows(scores):
    """Row softmax of an [s, s] score matrix with entries above the diagonal
    masked out (they get probability exactly 0)."""
    s = scores.shape[0]
    masked = np.where(np.tril(np.ones((s, s), dtype=bool)), scores, -np.inf)
    masked = masked - masked.max(axis=1, keepdims=True)
    e = np.exp(masked)
    return e / e.sum(axis=1, keepdims=True)


MASK_FILL = -10000.0   # value a hidden score is replaced with under the general mask (a stated reading)


def masked_softmax_rows(scores, hidden):
    """Row softmax under a general mask: hidden[q, k] True replaces the scaled score by MASK_FILL before
    the softmax, so a row with some visible key gives hidden keys probability exp(-10000 - max) = 0 and a
    row with no visible key attends uniformly.  Returns (probs, log-sum-exp)."""
    sc = np.where(hidden, MASK_FILL, scores)
    mx = sc.max(axis=1, keepdims=True)
    e = np.exp(sc - mx)
    z = e.sum(axis=1, keepdims=True)
    return e / z, (mx + np.log(z))[:, 0]


def attention_core(qkv, cfg, mask=None):
    """Per (sample, local head): ctx = softmax(mask(q k^T / sqrt(dh))) v.
    qkv: [s, b, 3*hp].  Returns ctx [s, b, hp], probs [b, heads, s, s] and the
    log-sum-exp of the scaled, masked scores [b, heads, s].
    cfg.causal: implicit causal mask.  Otherwise mask [b, s, s] (nonzero = key hidden from query;
    None = nothing hidden) is applied as in masked_softmax_rows."""
    s, b, al, dh, hp = cfg.s, cfg.b, cfg.heads_local, cfg.dh, cfg.hp
    ctx = np.zeros((s, b, hp))
    probs = np.zeros((b, al, s, s))
    lse = np.zeros((b, al, s))
    for j in range(b):
        for e in range(al):
            q = qkv[:, j, e * dh:(e + 1) * dh]
            k = qkv[:, j, hp + e * dh: hp + (e + 1) * dh]
            v = qkv[:, j, 2 * hp + e * dh: 2 * hp + (e + 1) * dh]
            sc = (q @ k.T) / math.sqrt(dh)
            if cfg.causal:
                p = causal_softmax_rows(sc)
                scm = np.where(np.tril(np.ones((s, s), dtype=bool)), sc, -np.inf)
                mx = scm.max(axis=1)
                lse[j, e] = mx + np.log(np.exp(scm - mx[:, None]).sum(axis=1))
            else:
                hidden = np.zeros((s, s), dtype=bool) if mask is None else (np.asarray(mask[j]) != 0)
                p, lse[j, e] = masked_softmax_rows(sc, hidden)
            probs[j, e] = p
            ctx[:, j, e * dh:(e + 1) * dh] = p @ v
    return ctx, probs, lse


def attention_core_backward(dctx, qkv, probs, cfg, mask=None):
    """Under the general mask a hidden score is a constant, so no gradient reaches q and k through it
    (its probability still weighs v: that matters only for rows with no visible key)."""
    s, b, al, dh, hp = cfg.s, cfg.b, cfg.heads_local, cfg.dh, cfg.hp
    dqkv = np.zeros_like(qkv)
    for j in range(b):
        for e in range(al):
            q = qkv[:, j, e * dh:(e + 1) * dh]
            k = qkv[:, j, hp + e * dh: hp + (e + 1) * dh]
            v = qkv[:, j, 2 * hp + e * dh: 2 * hp + (e + 1) * dh]
            p = probs[j, e]
            dc = dctx[:, j, e * dh:(e + 1) * dh]
            dv = p.T @ dc
            dp = dc @ v.T
            ds = p * (dp - (dp * p).sum(axis=1, keepdims=True))
            if not cfg.causal and mask is not None:
                ds = np.where(np.asarray(mask[j]) != 0, 0.0, ds)
            dq = (ds @ k) / math.sqrt(dh)
            dk = (ds.T @ q) / math.sqrt(dh)
            dqkv[:, j, e * dh:(e + 1) * dh] = dq
            dqkv[:, j, hp + e * dh: hp + (e + 1) * dh] = dk
            dqkv[:, j, 2 * hp + e * dh: 2 * hp + (e + 1) * dh] = dv
    return dqkv


def dropout_keep(cfg, layer, site, microbatch):
    """Keep-mask [s, b, h] of one dropout site (all ones when p == 0)."""
    n = cfg.s * cfg.b * cfg.h
    m = dropout_hash.keep_mask(cfg.seed, layer, site, microbatch, n, cfg.p_hidden)
    return m.reshape(cfg.s, cfg.b, cfg.h)


# ------------------------------------------------------- partial blocks

def attention_block_partial(x, P, cfg):
    """LayerNorm-1, QKV projection, attention, output projection WITHOUT bias:
    this shard's summand of the row-split output projection."""
    u, _, _ = layernorm(x, P["ln1_g"], P["ln1_b"], cfg.ln_eps)
    qkv = u @ P["w_qkv"] + P["b_qkv"]
    ctx, _, _ = attention_core(qkv, cfg)
    return ctx @ P["w_o"]


def mlp_block_partial(x1, P, cfg):
    """LayerNorm-2, first GEMM + bias + GeLU, second GEMM WITHOUT bias: this
    shard's summand of the row-split second GEMM."""
    u2, _, _ = layernorm(x1, P["ln2_g"], P["ln2_b"], cfg.ln_eps)
    g = gelu(u2 @ P["w_1"] + P["b_1"], cfg.gelu_tanh)
    return g @ P["w_2"]


# ------------------------------------------------------------ the layer

def _f64(P):
    return {k: np.asarray(v, dtype=np.float64) for k, v in P.items()}


def _keep(a):
    return a


def layer_forward(x, P, cfg, layer=0, microbatch=0, mask=None, storage=None):
    """x [s, b, h] -> (y [s, b, h], cache).  ``layer`` is the global layer
    index and ``microbatch`` the microbatch id; both only select the dropout
    stream.  ``mask`` [b, s, s]: general attention mask, used when cfg.causal is False.
    ``storage``: None (exact fp64 throughout), or a rounding function applied to every activation at the
    point where the method hands it on in storage precision (see ``oracle.bf16``); the first MLP GEMM's
    output is kept before its bias is added, as the bias + GeLU group of section 4.2 consumes it."""
    r = storage or _keep
    P = _f64(P)
    x = np.asarray(x, dtype=np.float64)
    c = {"x": x, "storage": storage}
    u, c["mu1"], c["rstd1"] = layernorm(x, P["ln1_g"], P["ln1_b"], cfg.ln_eps)
    c["u"] = r(u)
    c["qkv"] = r(c["u"] @ P["w_qkv"] + P["b_qkv"])
    c["mask"] = mask
    ctx, c["probs"], c["lse"] = attention_core(c["qkv"], cfg, mask)
    c["ctx"] = r(ctx)
    c["o"] = r(c["ctx"] @ P["w_o"])
    c["keep1"] = dropout_keep(cfg, layer, 0, microbatch)
    scale = dropout_hash.keep_scale(cfg.p_hidden)
    c["x1"] = r(x + (c["o"] + P["b_o"]) * c["keep1"] * scale)
    u2, c["mu2"], c["rstd2"] = layernorm(c["x1"], P["ln2_g"], P["ln2_b"], cfg.ln_eps)
    c["u2"] = r(u2)
    c["z"] = r(c["u2"] @ P["w_1"]) + P["b_1"]
    c["g"] = r(gelu(c["z"], cfg.gelu_tanh))
    c["mo"] = r(c["g"] @ P["w_2"])
    c["keep2"] = dropout_keep(cfg, layer, 1, microbatch)
    y = r(c["x1"] + (c["mo"] + P["b_2"]) * c["keep2"] * scale)
    return y, c


def layer_backward(dy, P, cfg, cache):
    """Gradient of ``layer_forward`` at the cached point: returns
    (dx [s, b, h], grads dict with one array per parameter).  Under a storage rounding (taken from the
    cache) every gradient of an activation is rounded where it is produced; parameter gradients are not."""
    P = _f64(P)
    c = cache
    r = c.get("storage") or _keep
    h = cfg.h
    dy = np.asarray(dy, dtype=np.float64)
    scale = dropout_hash.keep_scale(cfg.p_hidden)
    G = {}
    flat = lambda a: a.reshape(-1, a.shape[-1])

    dmo = r(dy * c["keep2"] * scale)                # grad w.r.t. (mo + b_2)
    G["b_2"] = flat(dmo).sum(axis=0)
    dx1 = dy.copy()                                 # residual branch
    dg = r(dmo @ P["w_2"].T)
    G["w_2"] = flat(c["g"]).T @ flat(dmo)
    dz = r(dg * gelu_grad(c["z"], cfg.gelu_tanh))
    G["b_1"] = flat(dz).sum(axis=0)
    du2 = r(dz @ P["w_1"].T)
    G["w_1"] = flat(c["u2"]).T @ flat(dz)
    d, G["ln2_g"], G["ln2_b"] = layernorm_backward(du2, c["x1"], P["ln2_g"], c["mu2"], c["rstd2"])
    dx1 = r(dx1 + d)

    do = r(dx1 * c["keep1"] * scale)                # grad w.r.t. (o + b_o)
    G["b_o"] = flat(do).sum(axis=0)
    dx = dx1.copy()                                 # residual branch
    dctx = r(do @ P["w_o"].T)
    G["w_o"] = flat(c["ctx"]).T @ flat(do)
    dqkv = r(attention_core_backward(dctx, c["qkv"], c["probs"], cfg, c.get("mask")))
    G["b_qkv"] = flat(dqkv).sum(axis=0)
    du = r(dqkv @ P["w_qkv"].T)
    G["w_qkv"] = flat(c["u"]).T @ flat(dqkv)
    d, G["ln1_g"], G["ln1_b"] = layernorm_backward(du, c["x"], P["ln1_g"], c["mu1"], c["rstd1"])
    dx = r(dx + d)
    assert dx.shape[-1] == h
    return dx, G


def chunk_forward(x, params_list, cfg, first_layer=0, microbatch=0, storage=None):
    """A model chunk = consecutive layers (section 2.2).  Returns (y, caches)."""
    caches = []
    for i, P in enumerate(params_list):
        x, c = layer_forward(x, P, cfg, first_layer + i, microbatch, storage=storage)
        caches.append(c)
    return x, caches


def chunk_backward(dy, params_list, cfg, caches):
    grads = [None] * len(params_list)
    for i in reversed(range(len(params_list))):
        dy, grads[i] = layer_backward(dy, params_list[i], cfg, caches[i])
    return dy, grads


# ------------------------------------------------ sampled definitions
# Used for parity at full size: each function evaluates the definition of one
# step at a few output positions from that step's actual inputs.

def attention_rows(qkv, cfg, sample, head, rows):
    """ctx rows and lse for the given query positions of one (sample, head)."""
    dh, hp = cfg.dh, cfg.hp
    qkv = np.asarray(qkv, dtype=np.float64)
    k = qkv[:, sample, hp + head * dh: hp + (head + 1) * dh]
    v = qkv[:, sample, 2 * hp + head * dh: 2 * hp + (head + 1) * dh]
    out, lse = [], []
    for i in rows:
        q = qkv[i, sample, head * dh:(head + 1) * dh]
        sc = (k[: i + 1] @ q) / math.sqrt(dh)
        mx = sc.max()
        e = np.exp(sc - mx)
        out.append((e / e.sum()) @ v[: i + 1])
        lse.append(mx + math.log(e.sum()))
    return np.array(out), np.array(lse)
