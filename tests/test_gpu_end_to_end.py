"""Whole-chunk parity against the full oracle at the configurations' real widths, the interleaved schedule at its
real shape with the memory accounting of section 3.5, and the microbatch sweep of section 3.4 (all through the C ABI).

The slow cases here spend their time in the fp64 oracle on the host (minutes); each prints a line per layer
so that a run is never silent for long."""
import ctypes as C
import time

import numpy as np
import pytest
import torch

from oracle import flops as F
from oracle import gpt_layer as L
from paper_2104_04473_amd import binding as B
from paper_2104_04473_amd import microbatch_sweep
from paper_2104_04473_amd import synth
from gpu_util import LayerRig, assert_close, np64, oracle_cfg, params_np, randn, stream, sync

pytestmark = pytest.mark.gpu


def run_chunk_against_oracle(cfg, n_layers, say, first_layer=0, mb=0):
    """Forward + backward of a chunk on the GPU and in the oracle, same bits in; every output, every layer
    boundary and every parameter gradient is compared in full."""
    rig = LayerRig(cfg, n_layers, first_layer)
    ocfg = oracle_cfg(cfg)
    shape = (cfg.s, cfg.b, cfg.h)
    x = randn(shape, cfg.dtype, 1000 + mb)
    dy = randn(shape, cfg.dtype, 2000 + mb)
    y = torch.empty_like(x); dx = torch.empty_like(x)
    B.check(rig.chunk.forward(mb, x.data_ptr(), y.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "forward")
    B.check(rig.chunk.backward(mb, dy.data_ptr(), dx.data_ptr(), rig.stash.data_ptr(), rig.ws.data_ptr()), "backward")
    sync()
    got_in = [np64(rig.field(l, "X", shape)) for l in range(n_layers)]      # input of every layer
    got_y, got_dx = np64(y), np64(dx)
    got_grads = [{k: np64(v) for k, v in G.items()} for G in rig.grads]
    Ps = [params_np(P) for P in rig.params]
    del rig
    torch.cuda.empty_cache()
    errs, failed = {}, []

    def close(key, got, want, what):
        try:
            errs[key] = assert_close(got, want, cfg.dtype, what)
        except AssertionError as e:                                           # keep going: report every tensor at the end
            failed.append(str(e).splitlines()[0])

    t0 = time.time()
    cur = np64(x)
    caches = []
    for l in range(n_layers):
        close("x%d" % l, got_in[l], cur, "input of layer %d" % l)
        cur, c = L.layer_forward(cur, Ps[l], ocfg, first_layer + l, mb)
        caches.append(c)
        say("oracle forward layer %d done (%.0f s)" % (l, time.time() - t0))
    close("y", got_y, cur, "y")
    d = np64(dy)
    for l in reversed(range(n_layers)):
        d, g = L.layer_backward(d, Ps[l], ocfg, caches[l])
        caches[l] = None                                                      # frees that layer's probabilities
        for k in B.PARAM_NAMES:
            close("%s[%d]" % (k, l), got_grads[l][k], g[k], "grad %s of layer %d" % (k, l))
        say("oracle backward layer %d done (%.0f s)" % (l, time.time() - t0))
    close("dx", got_dx, d, "dx")
    for msg in failed:
        say("FAILED " + msg)
    say("errors: " + " ".join("%s=%.1e" % kv for kv in errs.items()))
    assert not failed, failed
    say("largest relative L2 error %.3e (%s)" % (max(errs.values()), max(errs, key=errs.get)))
    return errs


@pytest.fixture
def say(capsys):
    def _say(msg):
        with capsys.disabled():
            print("    [end-to-end] " + msg, flush=True)
    return _say


def test_one_layer_at_full_width_short_sequence(say):
    """The 1T-shaped shard's widths (h = 25600, 20 local heads of 160, MLP 25600 -> 12800 -> 25600) with s = 256:
    every GEMM runs with the tile, panel and round counts of its full-size k and n extents, and every output
    and gradient is compared with the oracle in full."""
    cfg = B.make_cfg(h=25600, a=160, t=8, s=256, b=1, dtype=B.BF16, p_hidden=0.1, seed=3)
    run_chunk_against_oracle(cfg, 1, say, first_layer=2, mb=1)


@pytest.mark.timeout(1100)
@pytest.mark.parametrize("name,kw,n_layers", [
    ("c3", dict(h=12288, a=96, t=8, s=2048, b=1), 2),
    ("c2", dict(h=2048, a=16, t=1, s=2048, b=4), 4),
])
def test_configuration_end_to_end_against_oracle(name, kw, n_layers, say):
    """Configurations 3 (GPT-3-shaped shard, 2 layers) and 2 (h = 2048, b = 4, 4 layers) exactly as stated, the
    whole chunk forward and backward against the oracle."""
    cfg = B.make_cfg(dtype=B.BF16, p_hidden=0.1, seed=0, **kw)
    run_chunk_against_oracle(cfg, n_layers, say)


# ------------------------------------------------------------------------------- interleaved schedule, real shape
@pytest.mark.timeout(600)
@pytest.mark.parametrize("recompute", [0, 2])
def test_interleaved_share_at_gpt3_shape(recompute, say):
    """Section 2.2.2's example (4 devices, 2 chunks per device, 8 microbatches) on device 0 with GPT-3-shaped
    chunks of 4 layers: the 32 passes run in the interleaved order; sampled (chunk, microbatch) results are
    bit-identical to running that pair alone; one output is checked on sampled rows against the oracle; and the
    device memory the run needed is exactly parameters + fp32 gradients + workspace + (peak chunk-microbatches
    in flight) x chunk stash -- with recomputation: checkpoints per in-flight pair plus one segment stash
    (section 3.5: c A_input + (l/c) A_intermediate)."""
    p, v, m, rank, n_layers = 4, 2, 8, 0, 4
    w = dict(h=12288, a=96, t=8, s=2048, b=1)
    cfg = B.make_cfg(dtype=B.BF16, p_hidden=0.1, seed=0, **w)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    base = torch.cuda.memory_allocated()
    chunks, params, grads = [], [], []
    for c in range(v):
        first = n_layers * (c * p + rank)
        ch = B.Chunk(cfg, n_layers, first)
        for l in range(n_layers):
            P = synth.layer_params(w["h"], w["a"], w["t"], B.BF16, seed=1000 + first + l, device="cuda")
            G = synth.zero_grads(w["h"], w["a"], w["t"], "cuda")
            ch.bind(l, P, G)
            params.append(P); grads.append(G)
        chunks.append(ch)
    n_par = sum(int(np.prod(sh)) for sh in synth.param_shapes(w["h"], w["a"], w["t"]).values())
    shape = (w["s"], w["b"], w["h"])
    xin = [synth.activations(*shape, B.BF16, 10 + i, "cuda") for i in range(v * m)]
    dout = [synth.activations(*shape, B.BF16, 500 + i, "cuda") for i in range(v * m)]
    yout = [torch.empty_like(xin[0]) for _ in range(v * m)]
    din = [torch.empty_like(xin[0]) for _ in range(v * m)]
    io_bytes = 4 * v * m * xin[0].numel() * 2
    before_pool = torch.cuda.memory_allocated()
    steps = B.schedule_build(p, v, m, rank)
    assert len(steps) == 2 * v * m == 32
    peak = B.ptdp_schedule_peak_inflight(p, v, m, rank)
    assert peak == 11
    layer_stash = B.ptdp_layer_stash_bytes(C.byref(cfg))
    ws = torch.empty(chunks[0].workspace_bytes(), dtype=torch.uint8, device="cuda")
    if recompute:
        slot_bytes = chunks[0].checkpoint_bytes(recompute)
        seg_stash = torch.empty(recompute * layer_stash, dtype=torch.uint8, device="cuda")
    else:
        slot_bytes = chunks[0].stash_bytes()
    pool = torch.empty(slot_bytes * peak, dtype=torch.uint8, device="cuda")
    arr = lambda ts: (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
    handles = (C.c_void_p * v)(*[c.handle for c in chunks])
    args = (handles, v, m, steps, len(steps), arr(xin), arr(yout), arr(dout), arr(din))
    torch.cuda.reset_peak_memory_stats()
    if recompute:
        B.check(B.ptdp_schedule_run_ckpt(*args, pool.data_ptr(), slot_bytes, peak, recompute, seg_stash.data_ptr(),
                                         ws.data_ptr(), stream()), "schedule_run_ckpt")
    else:
        B.check(B.ptdp_schedule_run(*args, pool.data_ptr(), slot_bytes, peak, ws.data_ptr(), stream()), "schedule_run")
    sync()
    # ---- memory accounting (section 3.5): nothing was allocated during the run, and what is resident is the sum
    resident = torch.cuda.max_memory_allocated() - base
    assert torch.cuda.max_memory_allocated() == torch.cuda.memory_allocated(), "the run allocated device memory"
    weights = v * n_layers * n_par * 2
    gradients = v * n_layers * n_par * 4
    a_in = B.ptdp_checkpoint_bytes(C.byref(cfg))
    if recompute:
        n_ckpt = n_layers // recompute
        activations = peak * n_ckpt * a_in + recompute * layer_stash          # c A_in per pair + one segment's intermediates
    else:
        activations = peak * n_layers * layer_stash
    want = weights + gradients + io_bytes + chunks[0].workspace_bytes() + activations
    # torch's allocator hands out blocks a little larger than asked for (512-byte granules, unsplit remainders
    # below 1 MiB): allow 0.1 %
    assert want <= resident <= want * 1.001, (resident, want)
    assert before_pool - base >= weights + gradients + io_bytes
    say("resident %.2f GiB = weights %.2f + fp32 grads %.2f + stage io %.2f + workspace %.2f + activations %.2f GiB "
        "(%d pairs in flight)" % (resident / 2 ** 30, weights / 2 ** 30, gradients / 2 ** 30, io_bytes / 2 ** 30,
                                  chunks[0].workspace_bytes() / 2 ** 30, activations / 2 ** 30, peak))
    # ---- sampled pairs alone: same bits
    stash1 = torch.empty(chunks[0].stash_bytes(), dtype=torch.uint8, device="cuda")
    for (c, mb) in ((0, 0), (1, 5)):
        i = c * m + mb
        y1 = torch.empty_like(xin[0]); dx1 = torch.empty_like(xin[0])
        B.check(chunks[c].forward(mb, xin[i].data_ptr(), y1.data_ptr(), stash1.data_ptr(), ws.data_ptr()), "f")
        B.check(chunks[c].backward(mb, dout[i].data_ptr(), dx1.data_ptr(), stash1.data_ptr(), ws.data_ptr()), "b")
        sync()
        assert torch.equal(y1, yout[i]) and torch.equal(dx1, din[i]), (c, mb)
    # ---- one output against the oracle on sampled rows: the last layer of (chunk 1, microbatch 5), recomputed
    # from that layer's own input on the device (stash1 still holds the pair's stash)
    c, mb, l = 1, 5, n_layers - 1
    offs = B.stash_offsets(cfg)
    T, h = w["s"] * w["b"], w["h"]
    xl = stash1[l * layer_stash + offs["X"]: l * layer_stash + offs["X"] + T * h * 2].view(torch.bfloat16).view(*shape)
    small = 192                                                               # causal: the first rows need no later token
    ocfg = L.LayerConfig(h=w["h"], a=w["a"], t=w["t"], s=small, b=1, p_hidden=float(np.float32(0.1)), seed=0)
    Pn = params_np(params[c * n_layers + l])
    wy, _ = L.layer_forward(np64(xl[:small]), Pn, ocfg, n_layers * (c * p + rank) + l, mb)
    assert_close(np64(yout[c * m + mb][:small]), wy, B.BF16, "first %d rows of y of (chunk 1, microbatch 5)" % small)
    for ch in chunks:
        ch.close()


# ---------------------------------------------------------------------------------------------- microbatch sweep
def test_microbatch_sweep_and_eq1():
    """Section 3.4: t_f(b), t_b(b) measured on a small chunk, eq. (1) evaluated by the library from those very
    measurements equals the closed form."""
    w = dict(h=1024, a=8, t=1, s=256, layers=2, desc="test chunk")
    rows, summary = microbatch_sweep.sweep(w, [1, 2, 4], iters=3, p=4, batches=[8, 32])
    assert [r["b"] for r in rows] == [1, 2, 4]
    for r in rows:
        assert r["t_f_ms"] > 0 and r["t_b_ms"] > r["t_f_ms"] * 0.8          # backward is about twice the forward
        for bp in (8, 32):
            want = F.batch_time(bp, r["b"], 4, r["t_f_ms"], r["t_b_ms"])
            got = B.ptdp_batch_time(bp, r["b"], 4, r["t_f_ms"], r["t_b_ms"])
            assert abs(got - want) <= 1e-12 * want
            assert abs(summary["eq1"][str(bp)]["batch_time_ms"][str(r["b"])] - want) <= 1e-3
    for bp in ("8", "32"):
        e = summary["eq1"][bp]
        assert e["best_b"] == min((1, 2, 4), key=lambda b: e["batch_time_ms"][str(b)])
        assert max(e["normalized_throughput"].values()) == 1.0
