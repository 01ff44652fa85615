"""First/last-stage extras through the C ABI against the oracle: embedding forward/backward, and the
head step (final LayerNorm, logit GEMM, loss, all gradients)."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import lm_stage as S
from paper_2104_04473_amd import binding as B
from gpu_util import TOL, assert_close, dev_bytes, np64, oracle_cfg, randn, stream, sync, tdt

pytestmark = pytest.mark.gpu


def _tokens(s, b, lo, hi, seed):
    rng = np.random.default_rng(seed)
    t = rng.integers(lo, hi, size=(s, b)).astype(np.int32)
    t[1 % s, 0] = t[0, 0]          # a repeated id
    if s > 3:
        t[3, b - 1] = t[0, 0]
    return t


CASES = [  # dtype, s, b, h, V, v0, rows, p
    (B.F32, 12, 2, 64, 96, 0, 96, 0.1),
    (B.F32, 9, 3, 128, 200, 40, 80, 0.0),
    (B.BF16, 40, 2, 256, 512, 0, 512, 0.1),
    (B.BF16, 130, 1, 512, 4096, 1024, 2048, 0.1),
    (B.BF16, 33, 4, 1024, 6400, 0, 6400, 0.0),
]


@pytest.mark.parametrize("dtype,s,b,h,V,v0,rows,p", CASES)
def test_embedding_forward_backward(dtype, s, b, h, V, v0, rows, p):
    cfg = B.make_cfg(h=h, a=h // 64, t=1, s=s, b=b, dtype=dtype, p_hidden=p, seed=3)
    ocfg = oracle_cfg(cfg)
    tok = _tokens(s, b, 0, V, 1)
    e_word = randn((rows, h), dtype, 2, 0.5); e_pos = randn((s, h), dtype, 3, 0.5)
    tok_d = torch.from_numpy(tok).cuda()
    x = torch.empty((s, b, h), dtype=tdt(dtype), device="cuda")
    mb = 4
    B.check(B.ptdp_embedding_forward(C.byref(cfg), v0, rows, tok_d.data_ptr(), e_word.data_ptr(), e_pos.data_ptr(),
                                     x.data_ptr(), mb, stream()), "embedding_forward")
    sync()
    want = S.embedding_forward(tok.astype(np.int64), np64(e_word), np64(e_pos), ocfg, v0=v0, microbatch=mb)
    assert_close(np64(x), want, dtype, "x")
    assert np.array_equal(np64(x) == 0, want == 0)          # dropped elements and out-of-shard rows exactly

    dx = randn((s, b, h), dtype, 5)
    dw = torch.full((rows, h), 0.25, dtype=torch.float32, device="cuda")
    dp = torch.full((s, h), -0.5, dtype=torch.float32, device="cuda")
    ws = dev_bytes(B.ptdp_lm_workspace_bytes(C.byref(cfg), rows))
    B.check(B.ptdp_embedding_backward(C.byref(cfg), v0, rows, tok_d.data_ptr(), dx.data_ptr(), dw.data_ptr(),
                                      dp.data_ptr(), ws.data_ptr(), mb, stream()), "embedding_backward")
    sync()
    wdw, wdp = S.embedding_backward(np64(dx), tok.astype(np.int64), rows, ocfg, v0=v0, microbatch=mb)
    assert_close(np64(dw), wdw + 0.25, dtype, "d e_word (+= on 0.25)")
    assert_close(np64(dp), wdp - 0.5, dtype, "d e_pos (+= on -0.5)")
    untouched = np.ones(rows, dtype=bool)
    inside = (tok >= v0) & (tok < v0 + rows)
    untouched[(tok[inside] - v0)] = False
    assert np.all(np64(dw)[untouched] == 0.25)               # rows no token names are not written
    # a second run gives the same bits (fixed summation order)
    dw2 = torch.full_like(dw, 0.25); dp2 = torch.full_like(dp, -0.5)
    B.check(B.ptdp_embedding_backward(C.byref(cfg), v0, rows, tok_d.data_ptr(), dx.data_ptr(), dw2.data_ptr(),
                                      dp2.data_ptr(), ws.data_ptr(), mb, stream()), "embedding_backward")
    sync()
    assert torch.equal(dw, dw2) and torch.equal(dp, dp2)


@pytest.mark.parametrize("dtype,s,b,h,V,v0,rows,p", CASES)
def test_head_step(dtype, s, b, h, V, v0, rows, p):
    cfg = B.make_cfg(h=h, a=h // 64, t=1, s=s, b=b, dtype=dtype, p_hidden=p, seed=3)
    ocfg = oracle_cfg(cfg)
    T = s * b
    tgt = _tokens(s, b, 0, V, 7)
    y = randn((s, b, h), dtype, 8)
    g = (1.0 + 0.1 * randn((h,), B.F32, 9)).to(tdt(dtype)); bb = randn((h,), dtype, 10, 0.1)
    e_word = randn((rows, h), dtype, 2, 0.05)
    tgt_d = torch.from_numpy(tgt).cuda()
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    tl = torch.zeros(T, dtype=torch.float32, device="cuda")
    dy = torch.empty_like(y)
    dg = torch.zeros(h, dtype=torch.float32, device="cuda"); db = torch.zeros_like(dg)
    dw = torch.zeros((rows, h), dtype=torch.float32, device="cuda")
    ws = dev_bytes(B.ptdp_lm_workspace_bytes(C.byref(cfg), rows))
    scale = 2.0
    B.check(B.ptdp_lm_head_step(C.byref(cfg), v0, rows, y.data_ptr(), g.data_ptr(), bb.data_ptr(), e_word.data_ptr(),
                                tgt_d.data_ptr(), scale, loss.data_ptr(), tl.data_ptr(), dy.data_ptr(), dg.data_ptr(),
                                db.data_ptr(), dw.data_ptr(), ws.data_ptr(), stream()), "lm_head_step")
    sync()
    wl, cache = S.head_forward(np64(y), np64(g), np64(bb), np64(e_word), tgt.astype(np.int64), ocfg, v0=v0)
    wdy, wdg, wdb, wdw = S.head_backward(cache, np64(g), np64(e_word), dloss=scale)
    assert abs(loss.item() - wl) <= TOL[dtype] * abs(wl)
    assert_close(np64(tl), cache["per_token"], dtype, "token losses")
    assert_close(np64(dy), wdy, dtype, "dy")
    assert_close(np64(dg), wdg, dtype, "d gain")
    assert_close(np64(db), wdb, dtype, "d bias")
    assert_close(np64(dw), wdw, dtype, "d e_word")


def test_lm_stage_argument_errors():
    cfg = B.make_cfg(h=64, a=1, t=1, s=4, b=1, dtype=B.F32)
    assert B.ptdp_lm_workspace_bytes(C.byref(cfg), 12) == 0           # rows % 8
    assert B.ptdp_logit_flops_fwd(C.byref(cfg), 16) == 2 * 4 * 64 * 16
    assert B.ptdp_embedding_forward(C.byref(cfg), 0, 12, 256, 256, 256, 256, 0, None) == B.E_INVALID_ARG
    assert B.ptdp_embedding_forward(C.byref(cfg), -1, 16, 256, 256, 256, 256, 0, None) == B.E_INVALID_ARG
    assert B.ptdp_embedding_forward(C.byref(cfg), 0, 16, None, 256, 256, 256, 0, None) == B.E_NULL_PTR
    assert B.ptdp_embedding_backward(C.byref(cfg), 0, 16, 256, 256, 256, 256, None, 0, None) == B.E_NULL_PTR
    assert B.ptdp_lm_head_step(C.byref(cfg), 0, 16, 256, 256, 256, 256, 256, float("nan"), 256, 256, 256, 256, 256,
                               256, 256, None) == B.E_INVALID_ARG
