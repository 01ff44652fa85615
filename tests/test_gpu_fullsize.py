"""Parity at the full shapes that bench.py times (GPT-3-shaped and 1T-shaped shards), in the same launch
configuration, on sampled outputs: every sampled value is recomputed by the oracle's definition in
fp64 from the inputs the GPU step actually consumed (stash fields are read back from the device)."""
import ctypes as C
import math

import numpy as np
import pytest
import torch

from oracle import dropout_hash
from oracle import gpt_layer as L
from paper_2104_04473_amd import binding as B
from paper_2104_04473_amd import synth
from gpu_util import assert_close, np64, oracle_cfg, stream, sync

pytestmark = pytest.mark.gpu

SHAPES = {"c3": dict(h=12288, a=96, t=8, s=2048, b=1), "c4": dict(h=25600, a=160, t=8, s=2048, b=1),
          "c2": dict(h=2048, a=16, t=1, s=2048, b=4)}


def field(stash, offs, name, shape, dt=torch.bfloat16):
    n = int(np.prod(shape)) * torch.empty((), dtype=dt).element_size()
    return stash[offs[name]:offs[name] + n].view(dt).view(*shape)


@pytest.mark.parametrize("name", ["c3", "c4", "c2"])
def test_layer_sampled_parity_at_full_size(name):
    w = SHAPES[name]
    h, a, t, s, b = w["h"], w["a"], w["t"], w["s"], w["b"]
    hp, fp, dh, al, T = h // t, 4 * h // t, h // a, a // t, s * b
    layer, mb, p, seed = 3, 5, 0.1, 11
    cfg = B.make_cfg(h=h, a=a, t=t, s=s, b=b, dtype=B.BF16, p_hidden=p, seed=seed)
    P = synth.layer_params(h, a, t, B.BF16, seed=1, device="cuda")
    G = synth.zero_grads(h, a, t, "cuda")
    ch = B.Chunk(cfg, 1, layer)
    ch.bind(0, P, G)
    x = synth.activations(s, b, h, B.BF16, 2, "cuda")
    dy = synth.activations(s, b, h, B.BF16, 3, "cuda")
    y = torch.empty_like(x); dx = torch.empty_like(x)
    stash = torch.empty(ch.stash_bytes(), dtype=torch.uint8, device="cuda")
    ws = torch.empty(ch.workspace_bytes(), dtype=torch.uint8, device="cuda")
    B.check(ch.forward(mb, x.data_ptr(), y.data_ptr(), stash.data_ptr(), ws.data_ptr()), "forward")
    B.check(ch.backward(mb, dy.data_ptr(), dx.data_ptr(), stash.data_ptr(), ws.data_ptr()), "backward")
    sync()
    offs = B.stash_offsets(cfg)
    rng = np.random.default_rng(0)
    ocfg = oracle_cfg(cfg)
    scale = dropout_hash.keep_scale(p)
    tok = np.sort(rng.choice(T, size=24, replace=False))          # sampled tokens (rows of [T, .])
    f = lambda name_, width, dt=torch.bfloat16: field(stash, offs, name_, (T, width), dt)
    X, U, QKV, CTX, X1, U2, Z, Gs = (f("X", h), f("U", h), f("QKV", 3 * hp), f("CTX", hp), f("X1", h),
                                     f("U2", h), f("Z", fp), f("G", fp))
    Pn = {k: np64(v) for k, v in P.items()}
    rows = lambda tns: np64(tns[torch.as_tensor(tok, device="cuda")])

    # F1 LayerNorm-1 on sampled rows; stash X is the input
    assert torch.equal(X.view(s, b, h), x)
    wu, wmu, wrstd = L.layernorm(rows(X), Pn["ln1_g"], Pn["ln1_b"], ocfg.ln_eps)
    assert_close(rows(U), wu, B.BF16, "u rows")
    mu1 = field(stash, offs, "MU1", (T,), torch.float32)
    assert_close(np64(mu1)[tok], wmu[:, 0], B.F32, "mu1", 100)
    # F2 QKV GEMM + bias on sampled rows (from the device's u)
    assert_close(rows(QKV), rows(U) @ Pn["w_qkv"] + Pn["b_qkv"], B.BF16, "qkv rows")
    # F3 attention on sampled (sample, head, query) triples from the device's qkv
    qkv_np = np64(QKV).reshape(s, b, 3 * hp)
    lse = np64(field(stash, offs, "LSE", (b, al, s), torch.float32))
    ctx_np = np64(CTX).reshape(s, b, hp)
    for (j, e) in {(0, 0), (b - 1, al - 1), (b // 2, al // 2)}:
        qs = [0, 1, 63, 64, 127, 128, 1000, s - 1]
        wr, wl = L.attention_rows(qkv_np, ocfg, j, e, qs)
        assert_close(ctx_np[qs, j, e * dh:(e + 1) * dh], wr, B.BF16, "ctx rows")
        assert_close(lse[j, e, qs], wl, B.F32, "lse", 300)
    # F4 + F5: x1 = x + keep*(ctx Wo + bo)/(1-p) on sampled rows; the mask is the oracle's
    keep = lambda site: np.stack([dropout_hash.keep_mask(seed, layer, site, mb, h, p, start=int(r) * h) for r in tok])
    o = rows(CTX) @ Pn["w_o"] + Pn["b_o"]
    assert_close(rows(X1), rows(X) + o * keep(0) * scale, B.BF16, "x1 rows")
    # F6..F10
    wu2, _, _ = L.layernorm(rows(X1), Pn["ln2_g"], Pn["ln2_b"], ocfg.ln_eps)
    assert_close(rows(U2), wu2, B.BF16, "u2 rows")
    assert_close(rows(Z), rows(U2) @ Pn["w_1"], B.BF16, "z rows")
    assert_close(rows(Gs), L.gelu(rows(Z) + Pn["b_1"]), B.BF16, "g rows")
    mo = rows(Gs) @ Pn["w_2"] + Pn["b_2"]
    assert_close(np64(y.view(T, h)[torch.as_tensor(tok, device="cuda")]), rows(X1) + mo * keep(1) * scale, B.BF16, "y rows")

    # backward, MLP block, from dy (everything below is a definition evaluated in fp64):
    #   dmo = dy*keep2*scale; db2 = colsum(dmo); dW2[i,j] = sum_t g[t,i] dmo[t,j];
    #   dz[:,i] = (dmo W2[i,:]) * GeLU'(z[:,i]+b1[i]); db1[i] = sum_t dz[t,i]; dW1[k,i] = sum_t u2[t,k] dz[t,i]
    keep2 = dropout_hash.keep_mask(seed, layer, 1, mb, T * h, p).reshape(T, h)
    dmo = np64(dy.view(T, h)) * keep2 * scale
    assert_close(np64(G["b_2"]), dmo.sum(axis=0), B.BF16, "db2")
    cols_i = rng.choice(fp, size=6, replace=False)
    cols_j = rng.choice(h, size=64, replace=False)
    g_np = np64(Gs[:, torch.as_tensor(cols_i, device="cuda")])                          # [T, 6]
    want = g_np.T @ dmo[:, cols_j]
    got = np64(G["w_2"][torch.as_tensor(cols_i, device="cuda")][:, torch.as_tensor(cols_j, device="cuda")])
    assert_close(got, want, B.BF16, "dW2 samples")
    w2_rows = Pn["w_2"][cols_i]                                                          # [6, h]
    z_cols = np64(Z[:, torch.as_tensor(cols_i, device="cuda")]) + Pn["b_1"][cols_i]
    dz = (dmo @ w2_rows.T) * L.gelu_grad(z_cols)                                         # [T, 6]
    assert_close(np64(G["b_1"])[cols_i], dz.sum(axis=0), B.BF16, "db1 samples", 1.5)
    rows_k = rng.choice(h, size=64, replace=False)
    want = np64(U2[:, torch.as_tensor(rows_k, device="cuda")]).T @ dz                    # [64, 6]
    got = np64(G["w_1"][torch.as_tensor(rows_k, device="cuda")][:, torch.as_tensor(cols_i, device="cuda")])
    assert_close(got, want, B.BF16, "dW1 samples", 1.5)
    # properties that hold at any size: finite outputs, residual path present, gradients touched everywhere
    assert torch.isfinite(dx.float()).all() and torch.isfinite(y.float()).all()
    for k in B.PARAM_NAMES:
        assert torch.isfinite(G[k]).all(), k
        assert (G[k] != 0).float().mean() > 0.99, k
    ch.close()


@pytest.mark.parametrize("dh,heads", [(160, 20), (128, 12)])
def test_attention_backward_at_full_sequence(dh, heads):
    """s = 2048 through the exported attention kernels; two (sample, head) pairs checked in full."""
    s, b = 2048, 1
    hp = heads * dh
    qkv = synth.activations(s, b, 3 * hp, B.BF16, 4, "cuda")
    dctx = synth.activations(s, b, hp, B.BF16, 5, "cuda")
    ctx = torch.empty((s, b, hp), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((b, heads, s), device="cuda")
    dqkv = torch.empty_like(qkv)
    delta = torch.empty((b, heads, s), device="cuda")
    B.check(B.ptdp_attn_fwd(B.BF16, qkv.data_ptr(), ctx.data_ptr(), lse.data_ptr(), s, b, heads, dh, stream()), "fwd")
    B.check(B.ptdp_attn_bwd(B.BF16, qkv.data_ptr(), ctx.data_ptr(), lse.data_ptr(), dctx.data_ptr(), dqkv.data_ptr(),
                            delta.data_ptr(), s, b, heads, dh, stream()), "bwd")
    sync()
    one = L.LayerConfig(h=dh, a=1, t=1, s=s, b=1)
    for e in (0, heads - 1):
        sl = lambda base: slice(base + e * dh, base + (e + 1) * dh)
        q1 = np.concatenate([np64(qkv[:, :, sl(0)]), np64(qkv[:, :, sl(hp)]), np64(qkv[:, :, sl(2 * hp)])], axis=-1)
        wctx, probs, wlse = L.attention_core(q1, one)
        assert_close(np64(ctx[:, :, sl(0)]), wctx, B.BF16, "ctx head %d" % e)
        want = L.attention_core_backward(np64(dctx[:, :, sl(0)]), q1, probs, one)
        for i, nm in enumerate(("dq", "dk", "dv")):
            assert_close(np64(dqkv[:, :, sl(i * hp)]), want[..., i * dh:(i + 1) * dh], B.BF16, "%s head %d" % (nm, e))


def test_interleaved_share_at_gpt3_shape_accounting():
    """Config 5's stash accounting (host only arithmetic on the real sizes): peak in-flight slots x slot bytes."""
    cfg = B.make_cfg(h=12288, a=96, t=8, s=2048, b=1, dtype=B.BF16, p_hidden=0.1)
    per_layer = B.ptdp_layer_stash_bytes(C.byref(cfg))
    T, h, hp, fp = 2048, 12288, 1536, 6144
    payload = 2 * T * (4 * h + 3 * hp + hp + 2 * fp) + 4 * 4 * T + 4 * 12 * 2048
    assert payload <= per_layer <= payload + 13 * 256
    peak = B.ptdp_schedule_peak_inflight(4, 2, 8, 0)
    assert peak == 11
    assert abs(peak * 4 * per_layer / 2 ** 30 - 11 * 4 * payload / 2 ** 30) < 0.01
