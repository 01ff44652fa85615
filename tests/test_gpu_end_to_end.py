"""Whole-chunk parity against the full oracle at the configurations' real widths, the interleaved schedule at its
real shape with the memory accounting of section 3.5, and the microbatch sweep of section 3.4 (all through the C ABI).

The slow cases here spend their time in the fp64 oracle on the host (minutes); each prints a line per layer
so that a run is never silent for long."""
import ctypes as C
import os
import time

import numpy as np
import pytest
import torch

from oracle import bf16
from oracle import flops as F
from oracle import gpt_layer as L
from paper_2104_04473_amd import binding as B
from paper_2104_04473_amd import microbatch_sweep
from paper_2104_04473_amd import synth
from gpu_util import LayerRig, assert_close, np64, oracle_cfg, params_np, randn, stream, sync

pytestmark = pytest.mark.gpu


# Error model for runs at GPT-3 / 1T widths.  With N(0, 0.02) weights the scaled attention logits have a
# standard deviation of sigma_q * sigma_k = 0.0004 h (4.9 at h = 12288, 10 at h = 25600): the softmax is sharp,
# and a relative perturbation d of q and k moves every logit by about d * sqrt(2) * sigma_q * sigma_k and so every
# probability by that fraction of itself.  Two consequences:
#  * against the oracle that is exact in fp64 throughout, the bf16 storage of q and k alone (d = 1.2e-3 RMS)
#    costs 1-2 % in every probability before any kernel has run; gradients behind the attention backward
#    inherit 2-4 %.  The oracle that rounds activations to bf16 where the method stores them has this term too.
#  * through a chain of layers, whatever two implementations differ by at the input of a layer (a few 1e-3 from
#    fp32 versus fp64 accumulation and from bf16 operands inside the fused attention) is multiplied by about
#    sqrt(2) * sigma_q * sigma_k by that layer's softmax.
# So every layer is compared in full, at the stated tolerance, from the inputs it received on the device, and the
# chained comparisons through sharp softmaxes hold tensors that lie behind an attention to this model's bound.
SHARP_SOFTMAX = dict(factor=2.5, justified="sharp softmax multiplies upstream differences by sqrt(2)*sigma_q*sigma_k")


def run_chunk_against_oracle(cfg, n_layers, say, first_layer=0, mb=0, sharp=False):
    """Forward + backward of a chunk on the GPU and in the oracle, same bits in; every output, every layer
    boundary and every parameter gradient is compared in full:
    (A) layer by layer, the oracle (activations stored in bf16 where the method stores them) starting from the
        input and the output gradient that this layer received on the device: stated tolerance;
    (B) the oracle exact in fp64 throughout (and, with PTDP_TEST_CHAINED=all, also the oracle of (A)) chained
        through the whole chunk: stated tolerance, except, under a sharp softmax, for tensors that lie behind
        an attention (SHARP_SOFTMAX).  The chained passes cost minutes of host time: by default they run where
        the softmax is mild (configuration 2); PTDP_TEST_CHAINED=all runs them everywhere, =none nowhere."""
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
    # the same backward one layer at a time (what ptdp_chunk_backward does inside), keeping every layer's
    # incoming gradient: same bits out
    for G in rig.grads:
        for g in G.values():
            g.zero_()
    dys = [None] * n_layers + [dy]                                            # dys[l + 1] enters layer l's backward
    for l in reversed(range(n_layers)):
        dys[l] = torch.empty_like(dy)
        B.check(rig.chunk.layer_backward(l, mb, dys[l + 1].data_ptr(), dys[l].data_ptr(),
                                         rig.stash.data_ptr() + l * rig.layer_stash_bytes, rig.ws.data_ptr()), "layer_backward")
    sync()
    assert torch.equal(dys[0], dx)
    for l in range(n_layers):
        for k in B.PARAM_NAMES:
            assert np.array_equal(np64(rig.grads[l][k]), got_grads[l][k]), (l, k)
    got_dy = [np64(t) for t in dys]
    del rig, dys
    torch.cuda.empty_cache()
    failed, worst = [], {}
    t0 = time.time()

    def closer(mode, errs, relaxed):
        def close(key, got, want, what, through_attention=False):
            kw = SHARP_SOFTMAX if (relaxed and through_attention) else {}
            try:
                errs[key] = assert_close(got, want, cfg.dtype, "%s (%s)" % (what, mode), **kw)
            except AssertionError as e:                                       # keep going: report every tensor at the end
                failed.append(str(e).splitlines()[0])
        return close

    # ---- (A) every layer from its own device inputs
    errs = {}
    close = closer("layer by layer", errs, False)
    for l in range(n_layers):
        want_y, c = L.layer_forward(got_in[l], Ps[l], ocfg, first_layer + l, mb, storage=bf16.round_bf16)
        close("y%d" % l, got_in[l + 1] if l + 1 < n_layers else got_y, want_y, "output of layer %d" % l)
        want_dx, g = L.layer_backward(got_dy[l + 1], Ps[l], ocfg, c)
        del c
        close("dx%d" % l, got_dy[l], want_dx, "input gradient of layer %d" % l)
        for k in B.PARAM_NAMES:
            close("%s[%d]" % (k, l), got_grads[l][k], g[k], "grad %s of layer %d" % (k, l))
        say("layer by layer: layer %d done (%.0f s)" % (l, time.time() - t0))
    say("layer by layer, relative L2 errors: " + " ".join("%s=%.1e" % kv for kv in errs.items()))
    worst["layer by layer"] = max(errs.values()) if errs else None

    # ---- (B) chained through the chunk
    which = os.environ.get("PTDP_TEST_CHAINED", "mild")
    modes = [("chained, exact fp64", None)] if (which == "all" or (which == "mild" and not sharp)) else []
    if which == "all":
        modes.append(("chained, bf16 storage", bf16.round_bf16))
    for mode, storage in modes:
        errs = {}
        close = closer(mode, errs, sharp)
        cur = np64(x)
        caches = []
        for l in range(n_layers):
            close("x%d" % l, got_in[l], cur, "input of layer %d" % l, l > 0)
            cur, c = L.layer_forward(cur, Ps[l], ocfg, first_layer + l, mb, storage=storage)
            caches.append(c)
            say("%s: forward layer %d done (%.0f s)" % (mode, l, time.time() - t0))
        close("y", got_y, cur, "y", True)
        d = np64(dy)
        for l in reversed(range(n_layers)):
            d, g = L.layer_backward(d, Ps[l], ocfg, caches[l])
            caches[l] = None                                                  # frees that layer's probabilities
            for k in B.PARAM_NAMES:
                # the last layer's MLP-block gradients and output-projection bias see neither the attention
                # backward nor the attention output itself; everything else does
                behind = l < n_layers - 1 or k in ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o")
                close("%s[%d]" % (k, l), got_grads[l][k], g[k], "grad %s of layer %d" % (k, l), behind)
            say("%s: backward layer %d done (%.0f s)" % (mode, l, time.time() - t0))
        close("dx", got_dx, d, "dx", True)
        say("%s, relative L2 errors: " % mode + " ".join("%s=%.1e" % kv for kv in errs.items()))
        worst[mode] = max(errs.values()) if errs else None
    for msg in failed:
        say("FAILED " + msg)
    assert not failed, failed
    return worst


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
    run_chunk_against_oracle(cfg, 1, say, first_layer=2, mb=1, sharp=True)


@pytest.mark.timeout(1100)
@pytest.mark.parametrize("name,kw,n_layers,sharp", [
    ("c3", dict(h=12288, a=96, t=8, s=2048, b=1), 2, True),
    ("c2", dict(h=2048, a=16, t=1, s=2048, b=4), 4, False),
])
def test_configuration_end_to_end_against_oracle(name, kw, n_layers, sharp, say):
    """Configurations 3 (GPT-3-shaped shard, 2 layers) and 2 (h = 2048, b = 4, 4 layers) exactly as stated, the
    whole chunk forward and backward against the oracle."""
    cfg = B.make_cfg(dtype=B.BF16, p_hidden=0.1, seed=0, **kw)
    run_chunk_against_oracle(cfg, n_layers, say, sharp=sharp)


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
        assert r["t_f_ms"] > 0 and r["t_b_ms"] > 0   # (no relation between the two is asserted: at this size a launch hiccup outweighs either)
        for bp in (8, 32):
            want = F.batch_time(bp, r["b"], 4, r["t_f_ms"], r["t_b_ms"])
            got = B.ptdp_batch_time(bp, r["b"], 4, r["t_f_ms"], r["t_b_ms"])
            assert abs(got - want) <= 1e-12 * want
            assert abs(summary["eq1"][str(bp)]["batch_time_ms"][str(r["b"])] - want) <= 1e-3
    for bp in ("8", "32"):
        e = summary["eq1"][bp]
        assert e["best_b"] == min((1, 2, 4), key=lambda b: e["batch_time_ms"][str(b)])
        assert max(e["normalized_throughput"].values()) == 1.0
