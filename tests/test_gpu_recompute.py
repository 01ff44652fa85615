"""Activation recomputation (section 3.5) through the C ABI: results equal the stash-everything path
bit for bit, match the oracle, and the kept bytes follow c*A_input + (l/c)*A_intermediate."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import gpt_layer as L
from oracle import recompute as R
from paper_2104_04473_amd import binding as B
from gpu_util import LayerRig, assert_close, dev_bytes, np64, oracle_cfg, params_np, randn, stream, sync

pytestmark = pytest.mark.gpu


def _clone_grads(rig):
    return [{k: g.clone() for k, g in G.items()} for G in rig.grads]


def _zero_grads(rig):
    for G in rig.grads:
        for g in G.values():
            g.zero_()


@pytest.mark.parametrize("dtype,n,seg", [(B.F32, 3, 1), (B.F32, 3, 2), (B.BF16, 3, 3), (B.BF16, 4, 2), (B.BF16, 5, 2)])
def test_chunk_recompute_matches_plain_path_and_oracle(dtype, n, seg):
    cfg = B.make_cfg(h=256, a=4, t=2, s=40, b=2, dtype=dtype, p_hidden=0.1, seed=9)
    rig = LayerRig(cfg, n, first_layer=3, seed=70)
    shape = (cfg.s, cfg.b, cfg.h)
    x = randn(shape, dtype, 1); dy = randn(shape, dtype, 2)
    y0 = torch.empty_like(x); dx0 = torch.empty_like(x)
    mb = 5
    B.check(rig.chunk.forward(mb, x.data_ptr(), y0.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "fwd")
    B.check(rig.chunk.backward(mb, dy.data_ptr(), dx0.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "bwd")
    sync()
    g0 = _clone_grads(rig)
    _zero_grads(rig)

    n_ck = B.ptdp_chunk_n_checkpoints(rig.chunk.handle, seg)
    assert n_ck == -(-n // seg)
    ck_bytes = B.ptdp_checkpoint_bytes(C.byref(cfg))
    assert ck_bytes >= x.numel() * x.element_size() and ck_bytes % 256 == 0
    ckpt = dev_bytes(n_ck * ck_bytes)
    seg_stash = dev_bytes(seg * rig.layer_stash_bytes)
    y1 = torch.empty_like(x); dx1 = torch.empty_like(x)
    xc = x.clone()
    B.check(rig.chunk.forward_ckpt(mb, xc.data_ptr(), y1.data_ptr(), ckpt.data_ptr(), seg, seg_stash.data_ptr(),
                                   rig.ws.data_ptr()), "fwd_ckpt")
    sync()
    xc.fill_(7.0)            # the input buffer is free once the forward returns
    seg_stash.fill_(0x5a)    # and so is the segment scratch (another microbatch would overwrite it)
    B.check(rig.chunk.backward_ckpt(mb, dy.data_ptr(), dx1.data_ptr(), ckpt.data_ptr(), seg, seg_stash.data_ptr(),
                                    rig.ws.data_ptr()), "bwd_ckpt")
    sync()
    assert torch.equal(y0, y1) and torch.equal(dx0, dx1)
    for l in range(n):
        for k in B.PARAM_NAMES:
            assert torch.equal(g0[l][k], rig.grads[l][k]), (l, k)

    # kept bytes: c checkpoints + l/c layer stashes (exact when seg divides n)
    if n % seg == 0:
        kept = n_ck * ck_bytes + seg * rig.layer_stash_bytes
        assert kept == R.kept_bytes(n_ck, n, ck_bytes, rig.layer_stash_bytes)
        assert kept <= n * rig.layer_stash_bytes + ck_bytes

    # against the oracle's recompute path
    ocfg = oracle_cfg(cfg)
    Ps = [params_np(P) for P in rig.params]
    wy, ck = R.chunk_forward_checkpoints(np64(x), Ps, ocfg, seg, first_layer=3, microbatch=mb)
    wdx, wg = R.chunk_backward_recompute(np64(dy), Ps, ocfg, ck, seg, first_layer=3, microbatch=mb)
    assert_close(np64(y1), wy, dtype, "y")
    assert_close(np64(dx1), wdx, dtype, "dx")
    for l in range(n):
        for k in B.PARAM_NAMES:
            assert_close(np64(rig.grads[l][k]), wg[l][k], dtype, "layer %d grad %s" % (l, k))
    # checkpoint contents are the segment inputs
    for sg in range(n_ck):
        got = ckpt[sg * ck_bytes: sg * ck_bytes + x.numel() * x.element_size()].view(x.dtype).view(*shape)
        assert_close(np64(got), ck[sg], dtype, "checkpoint %d" % sg)


def test_recompute_argument_errors():
    cfg = B.make_cfg(h=256, a=4, t=1, s=16, b=1, dtype=B.BF16)
    rig = LayerRig(cfg, 2)
    x = randn((cfg.s, cfg.b, cfg.h), cfg.dtype, 1); y = torch.empty_like(x)
    ckpt = dev_bytes(2 * B.ptdp_checkpoint_bytes(C.byref(cfg)))
    for seg in (0, 3, -1):
        assert B.ptdp_chunk_n_checkpoints(rig.chunk.handle, seg) == B.E_INVALID_ARG
        assert rig.chunk.forward_ckpt(0, x.data_ptr(), y.data_ptr(), ckpt.data_ptr(), seg, rig.stash.data_ptr(),
                                      rig.ws.data_ptr()) == B.E_INVALID_ARG
        assert rig.chunk.backward_ckpt(0, x.data_ptr(), y.data_ptr(), ckpt.data_ptr(), seg, rig.stash.data_ptr(),
                                       rig.ws.data_ptr()) == B.E_INVALID_ARG
    assert rig.chunk.forward_ckpt(0, x.data_ptr(), y.data_ptr(), None, 1, rig.stash.data_ptr(),
                                  rig.ws.data_ptr()) == B.E_NULL_PTR
    sync()


def test_schedule_run_with_recompute():
    """The interleaved order with checkpoints only: outputs equal the stash-everything run bit for bit,
    and the pool holds peak_inflight checkpoint sets instead of peak_inflight chunk stashes."""
    p, v, m, rank = 4, 2, 4, 2
    cfg = B.make_cfg(h=256, a=4, t=1, s=24, b=2, dtype=B.BF16, p_hidden=0.1, seed=4)
    rigs = [LayerRig(cfg, 2, first_layer=2 * (c * p + rank), seed=50 + 10 * c) for c in range(v)]
    steps = B.schedule_build(p, v, m, rank)
    peak = B.ptdp_schedule_peak_inflight(p, v, m, rank)
    shape = (cfg.s, cfg.b, cfg.h)
    xin = [randn(shape, cfg.dtype, 300 + i) for i in range(v * m)]
    dout = [randn(shape, cfg.dtype, 400 + i) for i in range(v * m)]
    arr = lambda ts: (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
    handles = (C.c_void_p * v)(*[r.chunk.handle for r in rigs])
    results = []
    for seg in (0, 1, 2):
        for r in rigs:
            _zero_grads(r)
        yout = [torch.empty_like(xin[0]) for _ in range(v * m)]
        din = [torch.empty_like(xin[0]) for _ in range(v * m)]
        args = (handles, v, m, steps, len(steps), arr(xin), arr(yout), arr(dout), arr(din))
        if seg == 0:
            slot = rigs[0].chunk.stash_bytes()
            pool = dev_bytes(slot * peak)
            B.check(B.ptdp_schedule_run(*args, pool.data_ptr(), slot, peak, rigs[0].ws.data_ptr(), stream()), "run")
        else:
            slot = rigs[0].chunk.checkpoint_bytes(seg)
            pool = dev_bytes(slot * peak)
            seg_stash = dev_bytes(seg * rigs[0].layer_stash_bytes)
            assert B.ptdp_schedule_run_ckpt(*args, pool.data_ptr(), slot - 256, peak, seg, seg_stash.data_ptr(),
                                            rigs[0].ws.data_ptr(), stream()) == B.E_TOO_SMALL
            assert B.ptdp_schedule_run_ckpt(*args, pool.data_ptr(), slot, peak - 1, seg, seg_stash.data_ptr(),
                                            rigs[0].ws.data_ptr(), stream()) == B.E_TOO_SMALL
            B.check(B.ptdp_schedule_run_ckpt(*args, pool.data_ptr(), slot, peak, seg, seg_stash.data_ptr(),
                                             rigs[0].ws.data_ptr(), stream()), "run_ckpt")
            assert slot * peak < rigs[0].chunk.stash_bytes() * peak
        sync()
        results.append((yout, din, [_clone_grads(r) for r in rigs]))
    for yout, din, grads in results[1:]:
        for i in range(v * m):
            assert torch.equal(yout[i], results[0][0][i]) and torch.equal(din[i], results[0][1][i])
        for c in range(v):
            for l in range(2):
                for k in B.PARAM_NAMES:
                    assert torch.equal(grads[c][l][k], results[0][2][c][l][k]), (c, l, k)
