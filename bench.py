#!/usr/bin/env python3
"""Benchmark of the per-GPU PTD-P compute path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4|c3|c2|c5] [--no-cpu-baseline]
                    [--recompute SEG] [--stage middle|first|last]

A step is one pass of the whole hot path over one microbatch of synthetic input: forward of every
layer of the stage shard, then backward of every layer (for c5: the whole interleaved 1F1B order of
one device, 2 chunks x 8 microbatches).  Inputs, parameters, gradient accumulators, stash and
workspace are resident in HBM before the timed region.  Prints ONE JSON line.

value       model TFLOP/s = 3 x (24 b s h^2 + 4 b s^2 h)/t per layer and microbatch (paper appendix) / wall
            time.  The paper's factor 4 is used only with --recompute, where the rerun forward is really
            executed; --stage last adds the logit layer's 6 b s h V / t.  Both carry their own metric name.
roofline    the GEMM family with the largest share of the step, timed live with HIP events on the
            launch stream in a second pass over the same steps (event pairs around every launch)
cpu_baseline the fp64 numpy oracle, one full layer forward+backward at the workload's shape (one of the
            step's identical layer passes; about two minutes at c4), on the host cores of this machine
measured_ceilings  a register-resident MFMA loop (constant and random operands) and a 1 GiB copy
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

WORKLOADS = {
    # name: (h, a, t, s, b, layers, description)
    "c2": dict(h=2048, a=16, t=1, s=2048, b=4, layers=4, desc="4 GPT layers h=2048 a=16 s=2048 b=4 t=1"),
    "c3": dict(h=12288, a=96, t=8, s=2048, b=1, layers=2, desc="GPT-3 175B-shaped shard, 2 layers, t=8"),
    "c4": dict(h=25600, a=160, t=8, s=2048, b=1, layers=4, desc="1T-parameter-shaped stage shard, 4 layers, t=8"),
    "c5": dict(h=12288, a=96, t=8, s=2048, b=1, layers=4, chunks=2, m=8, p=4, rank=0,
               desc="interleaved 1F1B share of one device: 2 chunks x 4 layers, m=8, p=4, rank 0"),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c4", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--recompute", type=int, default=0, metavar="SEG",
                    help="activation recomputation with a checkpoint every SEG layers (section 3.5); the rerun "
                         "forward is executed and counted: FLOP factor 4 instead of 3.  Not the default metric.")
    ap.add_argument("--stage", default="middle", choices=["middle", "first", "last"],
                    help="first: embedding forward/backward around the layers; last: final LayerNorm, logit layer "
                         "(V=51200 split over t) and loss after them.  Not the default metric.")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="first run a plain 1 GiB read + 1 GiB write kernel (scale reference for FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--cpu-sample-positions", type=int, default=0,
                    help="restrict the oracle sample to the first N sequence positions (default: the whole layer)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build covers one GPU's share of the work only (no collectives are built); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2104_04473_amd import binding as B      # raises if libptdp.so is missing: no fallback
    from paper_2104_04473_amd import synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = WORKLOADS[args.workload]
    n_chunks = w.get("chunks", 1)
    m = w.get("m", 1)
    cfg = B.make_cfg(h=w["h"], a=w["a"], t=w["t"], s=w["s"], b=w["b"], dtype=B.BF16, p_hidden=0.1, seed=0)
    B.check(B.ptdp_cfg_validate(C.byref(cfg)), "cfg")
    shape = (w["s"], w["b"], w["h"])
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream

    if args.pmc_calibrate:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        for _ in range(3):
            dst = src * 1.0                                              # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # ---- resident state -------------------------------------------------------------------------
    chunks, params, grads = [], [], []
    for c in range(n_chunks):
        first = w["layers"] * (c * w.get("p", 1) + w.get("rank", 0))
        ch = B.Chunk(cfg, w["layers"], first)
        for l in range(w["layers"]):
            P = synth.layer_params(w["h"], w["a"], w["t"], B.BF16, seed=1000 + first + l, device=dev, zero_bias=True,
                                   ln_jitter=0.0)
            G = synth.zero_grads(w["h"], w["a"], w["t"], dev)
            ch.bind(l, P, G)
            params.append(P)
            grads.append(G)
        chunks.append(ch)
    slot_bytes = chunks[0].stash_bytes()
    ws = torch.empty(chunks[0].workspace_bytes(), dtype=torch.uint8, device=dev)
    n_pairs = n_chunks * m
    xin = [synth.activations(*shape, B.BF16, seed=10 + i, device=dev) for i in range(n_pairs)]
    dout = [synth.activations(*shape, B.BF16, seed=500 + i, device=dev) for i in range(n_pairs)]
    yout = [torch.empty_like(xin[0]) for _ in range(n_pairs)]
    din = [torch.empty_like(xin[0]) for _ in range(n_pairs)]

    seg = args.recompute
    if seg:
        slot_bytes = chunks[0].checkpoint_bytes(seg)
        seg_stash = torch.empty(seg * B.ptdp_layer_stash_bytes(C.byref(cfg)), dtype=torch.uint8, device=dev)
    if args.workload == "c5" and (args.stage != "middle"):
        print("bench.py: --stage first/last is measured on the single-chunk workloads", file=sys.stderr)
        sys.exit(2)
    if args.workload == "c5":
        steps = B.schedule_build(w["p"], n_chunks, m, w["rank"])
        n_slots = B.ptdp_schedule_peak_inflight(w["p"], n_chunks, m, w["rank"])
        pool = torch.empty(slot_bytes * n_slots, dtype=torch.uint8, device=dev)
        arr = lambda ts: (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
        handles = (C.c_void_p * n_chunks)(*[c.handle for c in chunks])
        a_in, a_out, a_dout, a_din = arr(xin), arr(yout), arr(dout), arr(din)

        def step():
            if seg:
                B.check(B.ptdp_schedule_run_ckpt(handles, n_chunks, m, steps, len(steps), a_in, a_out, a_dout, a_din,
                                                 pool.data_ptr(), slot_bytes, n_slots, seg, seg_stash.data_ptr(),
                                                 ws.data_ptr(), sh), "schedule_run_ckpt")
            else:
                B.check(B.ptdp_schedule_run(handles, n_chunks, m, steps, len(steps), a_in, a_out, a_dout, a_din,
                                            pool.data_ptr(), slot_bytes, n_slots, ws.data_ptr(), sh), "schedule_run")
        passes_per_step = n_pairs
    else:
        pool = torch.empty(slot_bytes, dtype=torch.uint8, device=dev)

        V = 51200
        vrows = V // w["t"]
        if args.stage != "middle":
            lm_ws = torch.empty(B.ptdp_lm_workspace_bytes(C.byref(cfg), vrows), dtype=torch.uint8, device=dev)
            e_word = (0.02 * torch.randn((vrows, w["h"]), device=dev)).to(torch.bfloat16)
            e_pos = (0.02 * torch.randn((w["s"], w["h"]), device=dev)).to(torch.bfloat16)
            d_e_word = torch.zeros((vrows, w["h"]), dtype=torch.float32, device=dev)
            d_e_pos = torch.zeros((w["s"], w["h"]), dtype=torch.float32, device=dev)
            gen = torch.Generator(device="cpu"); gen.manual_seed(7)
            ids = torch.randint(0, V, (w["s"], w["b"]), generator=gen, dtype=torch.int32).to(dev)
            lnf_g = torch.ones(w["h"], dtype=torch.bfloat16, device=dev); lnf_b = torch.zeros_like(lnf_g)
            d_lnf_g = torch.zeros(w["h"], dtype=torch.float32, device=dev); d_lnf_b = torch.zeros_like(d_lnf_g)
            loss = torch.zeros(1, dtype=torch.float32, device=dev)
            token_loss = torch.zeros(w["s"] * w["b"], dtype=torch.float32, device=dev)

        def step():
            x, y, dy, dx = xin[0].data_ptr(), yout[0].data_ptr(), dout[0].data_ptr(), din[0].data_ptr()
            if args.stage == "first":
                B.check(B.ptdp_embedding_forward(C.byref(cfg), 0, vrows, ids.data_ptr(), e_word.data_ptr(),
                                                 e_pos.data_ptr(), x, 0, sh), "embedding_forward")
            if seg:
                B.check(chunks[0].forward_ckpt(0, x, y, pool.data_ptr(), seg, seg_stash.data_ptr(), ws.data_ptr(),
                                               stream), "chunk_forward_ckpt")
                if args.stage == "last":
                    B.check(B.ptdp_lm_head_step(C.byref(cfg), 0, vrows, y, lnf_g.data_ptr(), lnf_b.data_ptr(),
                                                e_word.data_ptr(), ids.data_ptr(), 1.0, loss.data_ptr(),
                                                token_loss.data_ptr(), dy, d_lnf_g.data_ptr(), d_lnf_b.data_ptr(),
                                                d_e_word.data_ptr(), lm_ws.data_ptr(), sh), "lm_head_step")
                B.check(chunks[0].backward_ckpt(0, dy, dx, pool.data_ptr(), seg, seg_stash.data_ptr(), ws.data_ptr(),
                                                stream), "chunk_backward_ckpt")
            else:
                B.check(chunks[0].forward(0, x, y, pool.data_ptr(), ws.data_ptr(), stream), "chunk_forward")
                if args.stage == "last":
                    B.check(B.ptdp_lm_head_step(C.byref(cfg), 0, vrows, y, lnf_g.data_ptr(), lnf_b.data_ptr(),
                                                e_word.data_ptr(), ids.data_ptr(), 1.0, loss.data_ptr(),
                                                token_loss.data_ptr(), dy, d_lnf_g.data_ptr(), d_lnf_b.data_ptr(),
                                                d_e_word.data_ptr(), lm_ws.data_ptr(), sh), "lm_head_step")
                B.check(chunks[0].backward(0, dy, dx, pool.data_ptr(), ws.data_ptr(), stream), "chunk_backward")
            if args.stage == "first":
                B.check(B.ptdp_embedding_backward(C.byref(cfg), 0, vrows, ids.data_ptr(), dx, d_e_word.data_ptr(),
                                                  d_e_pos.data_ptr(), lm_ws.data_ptr(), 0, sh), "embedding_backward")
        passes_per_step = 1

    flop_factor = 4 if seg else 3
    flops_step = flop_factor * B.ptdp_layer_flops_fwd(C.byref(cfg)) * w["layers"] * passes_per_step
    if args.stage == "last":
        flops_step += 3 * B.ptdp_logit_flops_fwd(C.byref(cfg), 51200 // w["t"])      # 6 b s h V / t
    torch.cuda.synchronize()
    peak_hbm_bytes = torch.cuda.memory_allocated()

    # ---- timed region ---------------------------------------------------------------------------
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # recorded, never waited on
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(args.steps):
        step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    tflops = flops_step * args.steps / dt / 1e12
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    step_ms = {"median": round(per_step[len(per_step) // 2], 3), "min": round(per_step[0], 3),
               "max": round(per_step[-1], 3)}

    # ---- per-kernel pass: HIP event pairs on the launch stream around every launch ------------------
    B.ptdp_prof_enable(1)
    prof_steps = max(1, min(args.steps, 3))
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = B.prof_collect()
    B.ptdp_prof_enable(0)
    kernels = {}
    for name, (ms, work, launches) in prof.items():
        if launches == 0:
            continue
        is_flops = name.startswith("gemm") or name.startswith("attn")
        rate = work / (ms * 1e-3) / (1e12 if is_flops else 1e9)
        peak = PEAK_BF16_TFLOPS if is_flops else PEAK_HBM_GBS
        kernels[name] = {"ms_per_step": round(ms / prof_steps, 4), "launches_per_step": launches // prof_steps,
                         "avg_launch_ms": round(ms / launches, 5), "achieved": round(rate, 2),
                         "unit": "TFLOP/s" if is_flops else "GB/s", "frac": round(rate / peak, 4)}
    gemm = {k: v for k, v in prof.items() if k.startswith("gemm") and v[2] > 0}
    dom = max(gemm, key=lambda k: gemm[k][0])
    dms, dwork, dl = gemm[dom]
    all_ms = sum(v[0] for v in gemm.values())
    all_work = sum(v[1] for v in gemm.values())
    traffic = measured_traffic(args.workload, dom)
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(dwork / (dms * 1e-3) / 1e12, 2),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(dwork / (dms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                "traffic": traffic,
                "traffic_source": None if traffic is None else "profiles/%s_hbm_traffic.txt: rocprofv3 FETCH_SIZE + WRITE_SIZE per "
                                  "library launch of this family, two separate counter runs of this script (not this run)" % args.workload,
                "flops_per_launch": dwork / dl, "avg_launch_ms": round(dms / dl, 5),
                "all_gemm_achieved": round(all_work / (all_ms * 1e-3) / 1e12, 2),
                "all_gemm_share_of_step": round(all_ms / prof_steps / ms_per_step, 4)}

    # ---- measured ceilings: register-resident MFMA loop, 1 GiB copy (events on the launch stream) ---------------
    def timed(fn, n):
        fn()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / n
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    fl = C.c_double(0.0)
    t_m = timed(lambda: B.check(B.ptdp_ceiling_mfma(sink.data_ptr(), 256 * 4, 20000, 0, C.byref(fl), sh), "ceiling_mfma"), 3)
    t_r = timed(lambda: B.check(B.ptdp_ceiling_mfma(sink.data_ptr(), 256 * 4, 20000, 1, C.byref(fl), sh), "ceiling_mfma"), 3)
    t_r16 = timed(lambda: B.check(B.ptdp_ceiling_mfma(sink.data_ptr(), 256 * 4, 20000, 3, C.byref(fl), sh), "ceiling_mfma"), 3)
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev); dst = torch.empty_like(src)
    t_c = timed(lambda: B.check(B.ptdp_ceiling_copy(src.data_ptr(), dst.data_ptr(), src.numel(), sh), "ceiling_copy"), 5)
    ceilings = {"mfma_bf16_register_loop_tflops": round(fl.value / t_m / 1e12, 1),
                "mfma_bf16_register_loop_random_operands_tflops": round(fl.value / t_r / 1e12, 1),
                "mfma_bf16_16x16x32_register_loop_random_operands_tflops": round(fl.value / t_r16 / 1e12, 1),
                "copy_1gib_read_plus_write_gbs": round(2 * src.numel() / t_c / 1e9, 1)}
    del src, dst

    # ---- CPU oracle on a bounded sample of the same workload ------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, params[0], args.cpu_sample_positions)

    out = {
        "metric": "model_tflops_per_gpu_fwd_bwd" + ("_recompute" if seg else "") + ("" if args.stage == "middle" else "_%s_stage" % args.stage), "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "step_ms": step_ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "config": {"workload": "%s: %s" % (args.workload, w["desc"]), "h": w["h"], "a": w["a"], "t": w["t"],
                   "s": w["s"], "b": w["b"], "layers": w["layers"], "chunks": n_chunks, "microbatches": m,
                   "dropout_p": 0.1, "model_flops_per_step": flops_step, "flop_factor": flop_factor,
                   "recompute_segment_layers": seg, "stage": args.stage, "activation_pool_gb": round(pool.numel() / 2 ** 30, 3),
                   "resident_hbm_gb": round(peak_hbm_bytes / 2 ** 30, 2)},
        "roofline": roofline, "cpu_baseline": cpu, "measured_ceilings": ceilings, "kernels": kernels,
        "context": "paper: 163 TFLOP/s per A100 = 52% of peak, end-to-end on 3072 GPUs, recompute counted (x4)",
    }
    print(json.dumps(out))


def measured_traffic(workload, family):
    """HBM bytes per library call of `family` from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this
    workload (profiles/<workload>_hbm_traffic.txt), or None when no summary exists."""
    path = os.path.join(ROOT, "profiles", "%s_hbm_traffic.txt" % workload)
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 6 and f[0] == "family" and f[1] == family:
                return int((float(f[3]) + float(f[5])) * 2 ** 20)
    except OSError:
        pass
    return None


def cpu_baseline(w, params_dev, positions):
    """Times the oracle (fp64 numpy, as it stands) on ONE full layer forward+backward of the workload (all s
    positions; the workload's layers are identical in cost, so the whole step is `layers` times this), on the
    host cores of this machine.  `positions` > 0 restricts the sample to the first `positions` sequence positions."""
    import numpy as np
    from oracle import gpt_layer as L
    from oracle import flops as F
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    if positions <= 0 or positions > w["s"]:
        positions = w["s"]
    cfg = L.LayerConfig(h=w["h"], a=w["a"], t=w["t"], s=positions, b=w["b"], p_hidden=0.1, seed=0)
    P = {k: v.float().cpu().numpy() for k, v in params_dev.items()}
    rng = np.random.default_rng(0)
    x = rng.standard_normal((positions, w["b"], w["h"]))
    dy = rng.standard_normal((positions, w["b"], w["h"]))
    print("bench.py: timing the CPU oracle on one layer (%d positions, %d threads) ..." % (positions, cores),
          file=sys.stderr, flush=True)
    t0 = time.perf_counter()
    y, cache = L.layer_forward(x, P, cfg, 0, 0)
    print("bench.py: oracle forward done after %.0f s" % (time.perf_counter() - t0), file=sys.stderr, flush=True)
    dx, G = L.layer_backward(dy, P, cfg, cache)
    dt = time.perf_counter() - t0
    fl = F.shard_layer_flops(w["b"], positions, w["h"], w["t"])
    n_layers = w["layers"] * w.get("chunks", 1) * w.get("m", 1)
    whole = "all %d" % w["s"] if positions == w["s"] else "first %d of %d" % (positions, w["s"])
    return {"value": round(fl / dt / 1e12, 5), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": "1 layer forward+backward of the step's %d layer passes (identical in cost: the whole step would "
                      "take %d x %.0f s), fp64 numpy, %s sequence positions, same h/a/t/b" % (n_layers, n_layers, dt, whole)}


if __name__ == "__main__":
    main()
