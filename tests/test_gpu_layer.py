"""GPU parity of whole layers, chunks and the schedule runner against the oracle (C ABI)."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import gpt_layer as L
from oracle import schedule as S
from paper_2104_04473_amd import binding as B
from gpu_util import LayerRig, assert_close, dev_bytes, np64, oracle_cfg, params_np, randn, stream, sync, tdt

pytestmark = pytest.mark.gpu


def check_layer(cfg, n_layers=1, first_layer=0, microbatches=(0,), factor=1.0):
    rig = LayerRig(cfg, n_layers, first_layer)
    ocfg = oracle_cfg(cfg)
    Ps = [params_np(P) for P in rig.params]
    want_grads = [None] * n_layers
    errs = {}
    for mb in microbatches:
        x = randn((cfg.s, cfg.b, cfg.h), cfg.dtype, 1000 + mb)
        dy = randn((cfg.s, cfg.b, cfg.h), cfg.dtype, 2000 + mb)
        y = torch.empty_like(x); dx = torch.empty_like(x)
        B.check(rig.chunk.forward(mb, x.data_ptr(), y.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "forward")
        B.check(rig.chunk.backward(mb, dy.data_ptr(), dx.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "backward")
        sync()
        wy, caches = L.chunk_forward(np64(x), Ps, ocfg, first_layer, mb)
        wdx, grads = L.chunk_backward(np64(dy), Ps, ocfg, caches)
        errs["y"] = assert_close(np64(y), wy, cfg.dtype, "y (mb %d)" % mb, factor)
        errs["dx"] = assert_close(np64(dx), wdx, cfg.dtype, "dx (mb %d)" % mb, factor)
        # stashed intermediates of the last layer (what the backward pass consumed)
        T = cfg.s * cfg.b
        last = n_layers - 1
        for name, key, shape in (("U", "u", (cfg.s, cfg.b, cfg.h)), ("QKV", "qkv", (cfg.s, cfg.b, 3 * cfg.h // cfg.t)),
                                 ("CTX", "ctx", (cfg.s, cfg.b, cfg.h // cfg.t)), ("X1", "x1", (cfg.s, cfg.b, cfg.h)),
                                 ("G", "g", (cfg.s, cfg.b, 4 * cfg.h // cfg.t))):
            assert_close(np64(rig.field(last, name, shape)), caches[last][key], cfg.dtype, "stash " + name, factor)
        assert_close(np64(rig.field(last, "LSE", (cfg.b, cfg.a // cfg.t, cfg.s), torch.float32)), caches[last]["lse"],
                     cfg.dtype, "lse", factor)
        for i in range(n_layers):
            want_grads[i] = grads[i] if want_grads[i] is None else {k: want_grads[i][k] + grads[i][k] for k in grads[i]}
    for i in range(n_layers):
        for name in B.PARAM_NAMES:
            errs[name] = assert_close(np64(rig.grads[i][name]), want_grads[i][name], cfg.dtype,
                                      "grad %s layer %d" % (name, i), factor)
    return errs


def test_config1_fp32_layer():
    """1 GPT layer fp32, h=256, a=4, s=128, b=2, t=1, dropout 0.1 seed 0: forward + backward."""
    cfg = B.make_cfg(h=256, a=4, t=1, s=128, b=2, dtype=B.F32, p_hidden=0.1, seed=0)
    errs = check_layer(cfg)
    print({k: "%.2e" % v for k, v in errs.items()})


@pytest.mark.parametrize("kw", [
    dict(h=256, a=4, t=1, s=72, b=3, dtype=B.F32, p_hidden=0.25, seed=5, gelu_mode=B.GELU_TANH),
    dict(h=512, a=8, t=2, s=96, b=2, dtype=B.F32, p_hidden=0.0, seed=1),
    dict(h=512, a=8, t=1, s=200, b=2, dtype=B.BF16, p_hidden=0.1, seed=2),
    dict(h=1024, a=8, t=2, s=136, b=1, dtype=B.BF16, p_hidden=0.1, seed=3),
    dict(h=1280, a=8, t=4, s=264, b=2, dtype=B.BF16, p_hidden=0.1, seed=4),          # dh = 160
])
def test_layer_variants(kw):
    check_layer(B.make_cfg(**kw))


def test_chunk_of_layers_and_gradient_accumulation():
    cfg = B.make_cfg(h=256, a=4, t=1, s=40, b=2, dtype=B.F32, p_hidden=0.1, seed=9)
    check_layer(cfg, n_layers=3, first_layer=4, microbatches=(0, 3))
    cfg = B.make_cfg(h=512, a=4, t=2, s=136, b=1, dtype=B.BF16, p_hidden=0.1, seed=9)
    check_layer(cfg, n_layers=2, first_layer=2, microbatches=(1, 2))


def test_layer_is_deterministic():
    cfg = B.make_cfg(h=512, a=4, t=1, s=136, b=2, dtype=B.BF16, p_hidden=0.1, seed=1)
    outs = []
    for _ in range(2):
        rig = LayerRig(cfg)
        x = randn((cfg.s, cfg.b, cfg.h), cfg.dtype, 1); dy = randn((cfg.s, cfg.b, cfg.h), cfg.dtype, 2)
        y = torch.empty_like(x); dx = torch.empty_like(x)
        B.check(rig.chunk.forward(0, x.data_ptr(), y.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "f")
        B.check(rig.chunk.backward(0, dy.data_ptr(), dx.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "b")
        sync()
        outs.append((y.clone(), dx.clone(), {k: v.clone() for k, v in rig.grads[0].items()}))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    for k in outs[0][2]:
        assert torch.equal(outs[0][2][k], outs[1][2][k]), k


def test_schedule_run_interleaved():
    """One device's interleaved order (p=4, v=2, m=4, rank 1) on tiny chunks: every (chunk, microbatch)
    result is bit-identical to running it alone, gradients are the sum over microbatches, and the
    stash pool never needs more slots than the order's peak."""
    p, v, m, rank = 4, 2, 4, 1
    cfg = B.make_cfg(h=256, a=4, t=1, s=24, b=2, dtype=B.BF16, p_hidden=0.1, seed=4)
    rigs = [LayerRig(cfg, 2, first_layer=2 * (c * p + rank), seed=50 + 10 * c) for c in range(v)]
    steps = B.schedule_build(p, v, m, rank)
    peak = B.ptdp_schedule_peak_inflight(p, v, m, rank)
    slot_bytes = rigs[0].chunk.stash_bytes()
    pool = dev_bytes(slot_bytes * peak)
    shape = (cfg.s, cfg.b, cfg.h)
    xin = [randn(shape, cfg.dtype, 300 + i) for i in range(v * m)]
    dout = [randn(shape, cfg.dtype, 400 + i) for i in range(v * m)]
    yout = [torch.empty_like(xin[0]) for _ in range(v * m)]
    din = [torch.empty_like(xin[0]) for _ in range(v * m)]
    arr = lambda ts: (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
    handles = (C.c_void_p * v)(*[r.chunk.handle for r in rigs])
    args = (handles, v, m, steps, len(steps), arr(xin), arr(yout), arr(dout), arr(din))
    assert B.ptdp_schedule_run(*args, pool.data_ptr(), slot_bytes, peak - 1, rigs[0].ws.data_ptr(), stream()) == B.E_TOO_SMALL
    B.check(B.ptdp_schedule_run(*args, pool.data_ptr(), slot_bytes, peak, rigs[0].ws.data_ptr(), stream()), "run")
    sync()
    sched_grads = [[{k: g.clone() for k, g in G.items()} for G in r.grads] for r in rigs]
    # the same work, one (chunk, microbatch) at a time, in plain order
    for r in rigs:
        for G in r.grads:
            for g in G.values():
                g.zero_()
    for c in range(v):
        for mb in range(m):
            y = torch.empty_like(xin[0]); dx = torch.empty_like(xin[0])
            i = c * m + mb
            B.check(rigs[c].chunk.forward(mb, xin[i].data_ptr(), y.data_ptr(), rigs[c].stash.data_ptr(), rigs[c].ws.data_ptr()), "f")
            B.check(rigs[c].chunk.backward(mb, dout[i].data_ptr(), dx.data_ptr(), rigs[c].stash.data_ptr(), rigs[c].ws.data_ptr()), "b")
            sync()
            assert torch.equal(y, yout[i]) and torch.equal(dx, din[i])
    # gradient sums: same addends, but the schedule adds them in a different microbatch order
    for c in range(v):
        for l in range(2):
            for k in B.PARAM_NAMES:
                assert_close(np64(sched_grads[c][l][k]), np64(rigs[c].grads[l][k]), B.F32, "grad " + k, 0.1)
    # and against the oracle for one pair
    ocfg = oracle_cfg(cfg)
    Ps = [params_np(P) for P in rigs[1].params]
    wy, _ = L.chunk_forward(np64(xin[1 * m + 2]), Ps, ocfg, 2 * (1 * p + rank), 2)
    assert_close(np64(yout[1 * m + 2]), wy, cfg.dtype, "y of (chunk 1, microbatch 2)")


def test_chunk_forward_backward_replays_from_a_hip_graph():
    """The library allocates nothing, clears nothing with memsets and never synchronises, so a step can be
    captured into a HIP graph.  Every replay (with eager work and synchronisations in between) must give the
    bits of the eager step, including the += into the gradient buffers."""
    cfg = B.make_cfg(h=256, a=4, t=1, s=64, b=2, dtype=B.BF16, p_hidden=0.1, seed=6)
    rig = LayerRig(cfg, 2, first_layer=0, seed=90)
    shape = (cfg.s, cfg.b, cfg.h)
    x = randn(shape, cfg.dtype, 1); dy = randn(shape, cfg.dtype, 2)
    y = torch.empty_like(x); dx = torch.empty_like(x)

    def step():
        B.check(rig.chunk.forward(1, x.data_ptr(), y.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "fwd")
        B.check(rig.chunk.backward(1, dy.data_ptr(), dx.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "bwd")

    step()                      # eager reference (also sets the kernels' one-time attributes before capture)
    sync()
    y_ref, dx_ref = y.clone(), dx.clone()
    g1 = [{k: v.clone() for k, v in G.items()} for G in rig.grads]       # gradients after one step
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()                  # captured on the capture stream (torch's current stream inside the context)
    sync()
    for G in rig.grads:
        for v in G.values():
            v.zero_()
    for replay in range(1, 4):
        y.zero_(); dx.zero_()
        graph.replay()
        sync()
        assert torch.equal(y, y_ref) and torch.equal(dx, dx_ref), "replay %d" % replay
        scratch = randn(shape, cfg.dtype, 10 + replay) * 2.0            # unrelated eager work between replays
        sync()
        del scratch
        if replay == 1:
            for l in range(2):
                for k in B.PARAM_NAMES:
                    assert torch.equal(rig.grads[l][k], g1[l][k]), (l, k)
    # three replays accumulated three times the same addend, in the order an eager loop would
    for G in rig.grads:
        for v in G.values():
            v.zero_()
    for _ in range(3):
        step()
    sync()
    eager3 = [{k: v.clone() for k, v in G.items()} for G in rig.grads]
    for G in rig.grads:
        for v in G.values():
            v.zero_()
    for _ in range(3):
        graph.replay()
    sync()
    for l in range(2):
        for k in B.PARAM_NAMES:
            assert torch.equal(rig.grads[l][k], eager3[l][k]), (l, k)
