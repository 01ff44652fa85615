"""General-mask attention (section 4.2's fused softmax with a general mask) through the C ABI against
the oracle: the attention op alone and a whole layer with cfg.causal = 0."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import gpt_layer as L
from paper_2104_04473_amd import binding as B
from gpu_util import LayerRig, assert_close, np64, oracle_cfg, params_np, randn, stream, sync, tdt

pytestmark = pytest.mark.gpu


def make_mask(b, s, seed, frac=0.3, empty_rows=()):
    rng = np.random.default_rng(seed)
    m = (rng.random((b, s, s)) < frac).astype(np.uint8)
    for j in range(b):
        np.fill_diagonal(m[j], 0)
    for (j, q) in empty_rows:
        m[j, q, :] = 1
    return m


CASES = [  # dtype, s, b, heads, dh, masked?, empty rows
    (B.F32, 50, 2, 2, 32, True, [(1, 7)]),
    (B.F32, 33, 1, 1, 64, False, []),
    (B.BF16, 128, 2, 2, 64, True, [(0, 5), (1, 127)]),
    (B.BF16, 333, 1, 2, 160, True, [(0, 300)]),
    (B.BF16, 200, 2, 3, 128, True, []),
    (B.BF16, 130, 1, 2, 96, False, []),
    (B.BF16, 64, 1, 1, 32, True, []),
    (B.BF16, 257, 1, 1, 128, True, [(0, 256)]),
    # more than 512 (query block, sample, head) triples: one-pair form of the backward kernels
    (B.BF16, 130, 6, 30, 64, True, [(2, 129)]),
    (B.BF16, 140, 4, 44, 160, True, []),
]


@pytest.mark.parametrize("dtype,s,b,heads,dh,masked,empty", CASES)
def test_masked_attention_forward_backward(dtype, s, b, heads, dh, masked, empty):
    hp = heads * dh
    qkv = randn((s, b, 3 * hp), dtype, 1)
    mask = make_mask(b, s, 2, empty_rows=empty) if masked else None
    mask_d = torch.from_numpy(mask).cuda() if masked else None
    mp = mask_d.data_ptr() if masked else None
    ctx = torch.zeros((s, b, hp), dtype=tdt(dtype), device="cuda")
    lse = torch.zeros((b, heads, s), device="cuda")
    B.check(B.ptdp_attn_masked_fwd(dtype, qkv.data_ptr(), mp, ctx.data_ptr(), lse.data_ptr(), s, b, heads, dh, stream()),
            "attn_masked_fwd")
    sync()
    cfg = L.LayerConfig(h=hp, a=heads, t=1, s=s, b=b, causal=False)
    wctx, probs, wlse = L.attention_core(np64(qkv), cfg, mask)
    assert_close(np64(ctx), wctx, dtype, "ctx")
    assert np.allclose(np64(lse), wlse, rtol=0, atol=3e-2 if dtype == B.BF16 else 1e-3)
    for (j, q) in empty:        # a query that sees no key averages V
        assert_close(np64(ctx)[q, j], np64(qkv)[:, j, 2 * hp:].mean(axis=0), dtype, "empty row")
    dctx = randn((s, b, hp), dtype, 7)
    dqkv = torch.zeros_like(qkv)
    delta = torch.zeros((b, heads, s), device="cuda")
    B.check(B.ptdp_attn_masked_bwd(dtype, qkv.data_ptr(), mp, ctx.data_ptr(), lse.data_ptr(), dctx.data_ptr(),
                                   dqkv.data_ptr(), delta.data_ptr(), s, b, heads, dh, stream()), "attn_masked_bwd")
    sync()
    want = L.attention_core_backward(np64(dctx), np64(qkv), probs, cfg, mask)
    got = np64(dqkv)
    for name, lo in (("dq", 0), ("dk", hp), ("dv", 2 * hp)):
        assert_close(got[..., lo:lo + hp], want[..., lo:lo + hp], dtype, name)
    for (j, q) in empty:
        assert np.all(got[q, j, :hp] == 0.0)      # no gradient reaches the query of an empty row


def test_upper_triangular_mask_equals_the_causal_kernels():
    s, b, heads, dh = 192, 1, 2, 128
    hp = heads * dh
    qkv = randn((s, b, 3 * hp), B.BF16, 3)
    mask = torch.from_numpy(np.triu(np.ones((b, s, s), dtype=np.uint8), 1)).cuda()
    outs = []
    for general in (False, True):
        ctx = torch.zeros((s, b, hp), dtype=torch.bfloat16, device="cuda"); lse = torch.zeros((b, heads, s), device="cuda")
        if general:
            B.check(B.ptdp_attn_masked_fwd(B.BF16, qkv.data_ptr(), mask.data_ptr(), ctx.data_ptr(), lse.data_ptr(), s, b,
                                           heads, dh, stream()), "masked")
        else:
            B.check(B.ptdp_attn_fwd(B.BF16, qkv.data_ptr(), ctx.data_ptr(), lse.data_ptr(), s, b, heads, dh, stream()), "causal")
        sync()
        outs.append((ctx, lse))
    assert_close(np64(outs[1][0]), np64(outs[0][0]), B.BF16, "ctx", 0.05)
    assert np.allclose(np64(outs[1][1]), np64(outs[0][1]), atol=1e-4)


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
def test_layer_with_general_mask(dtype):
    cfg = B.make_cfg(h=256, a=4, t=2, s=72, b=2, dtype=dtype, p_hidden=0.1, seed=2, causal=0)
    rig = LayerRig(cfg, 2, first_layer=1, seed=30)
    mask = make_mask(cfg.b, cfg.s, 5, empty_rows=[(1, 3)])
    mask_d = torch.from_numpy(mask).cuda()
    assert B.ptdp_chunk_set_mask(rig.chunk.handle, mask_d.data_ptr() + 1) == B.E_INVALID_ARG     # alignment
    B.check(B.ptdp_chunk_set_mask(rig.chunk.handle, mask_d.data_ptr()), "set_mask")
    shape = (cfg.s, cfg.b, cfg.h)
    x = randn(shape, dtype, 1); dy = randn(shape, dtype, 2)
    y = torch.empty_like(x); dx = torch.empty_like(x)
    B.check(rig.chunk.forward(3, x.data_ptr(), y.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "fwd")
    B.check(rig.chunk.backward(3, dy.data_ptr(), dx.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "bwd")
    sync()
    ocfg = oracle_cfg(cfg)
    ocfg.causal = False
    Ps = [params_np(P) for P in rig.params]
    cur = np64(x); caches = []
    for l, P in enumerate(Ps):
        cur, c = L.layer_forward(cur, P, ocfg, 1 + l, 3, mask=mask)
        caches.append(c)
    assert_close(np64(y), cur, dtype, "y")
    wdx, wg = L.chunk_backward(np64(dy), Ps, ocfg, caches)
    assert_close(np64(dx), wdx, dtype, "dx")
    for l in range(2):
        for k in B.PARAM_NAMES:
            assert_close(np64(rig.grads[l][k]), wg[l][k], dtype, "layer %d grad %s" % (l, k))
    # a causal chunk refuses a mask
    crig = LayerRig(B.make_cfg(h=256, a=4, t=1, s=8, b=1, dtype=dtype), 1)
    assert B.ptdp_chunk_set_mask(crig.chunk.handle, mask_d.data_ptr()) == B.E_INVALID_ARG
