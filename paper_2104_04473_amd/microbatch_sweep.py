"""Microbatch-size sweep (section 3.4): measures t_f(b) and t_b(b) of a model chunk on one GPU and
evaluates eq. (1), (b'/b + p - 1)(t_f(b) + t_b(b)), for the batch sizes of the paper's figure.

    python -m paper_2104_04473_amd.microbatch_sweep [--model 1b|gpt3-shard] [--b 1 2 4 8] [--iters 5]

Default model: the paper's single-GPU example (hidden size 4096, 128 heads, 4 layers, sequence 2048,
t = 1).  Prints one JSON object per microbatch size, then one summary object.  Every timed step runs in
the HIP library (this script only allocates device memory, times with events on the launch stream and
calls ptdp_batch_time for eq. (1)).
"""
import argparse
import ctypes as C
import json
import sys

MODELS = {
    "1b": dict(h=4096, a=128, t=1, s=2048, layers=4, desc="h=4096, 128 heads, 4 layers, s=2048, t=1 (about 1 B parameters)"),
    "gpt3-shard": dict(h=12288, a=96, t=8, s=2048, layers=1, desc="GPT-3-shaped layer shard: h=12288, 96 heads, t=8, s=2048"),
}


def sweep(w, bs, iters, p, batches, emit=None):
    """Measures t_f(b), t_b(b) of the chunk described by `w` (keys h, a, t, s, layers, desc) for every b in
    `bs` and evaluates eq. (1) for every per-replica batch size b' in `batches`.  Returns (rows, summary)."""
    import torch
    from . import binding as B
    from . import synth
    if not torch.cuda.is_available():
        raise RuntimeError("microbatch_sweep: no GPU visible")
    dev = "cuda:0"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    rows = []
    params = [synth.layer_params(w["h"], w["a"], w["t"], B.BF16, seed=1000 + l, device=dev, zero_bias=True, ln_jitter=0.0)
              for l in range(w["layers"])]
    grads = [synth.zero_grads(w["h"], w["a"], w["t"], dev) for _ in range(w["layers"])]
    for b in bs:
        cfg = B.make_cfg(h=w["h"], a=w["a"], t=w["t"], s=w["s"], b=b, dtype=B.BF16, p_hidden=0.1, seed=0)
        B.check(B.ptdp_cfg_validate(C.byref(cfg)), "cfg")
        ch = B.Chunk(cfg, w["layers"], 0)
        for l in range(w["layers"]):
            ch.bind(l, params[l], grads[l])
        stash = torch.empty(ch.stash_bytes(), dtype=torch.uint8, device=dev)
        ws = torch.empty(ch.workspace_bytes(), dtype=torch.uint8, device=dev)
        shape = (w["s"], b, w["h"])
        x = synth.activations(*shape, B.BF16, seed=10, device=dev)
        dy = synth.activations(*shape, B.BF16, seed=11, device=dev)
        y = torch.empty_like(x)
        dx = torch.empty_like(x)

        def fwd():
            B.check(ch.forward(0, x.data_ptr(), y.data_ptr(), stash.data_ptr(), ws.data_ptr(), stream), "forward")

        def bwd():
            B.check(ch.backward(0, dy.data_ptr(), dx.data_ptr(), stash.data_ptr(), ws.data_ptr(), stream), "backward")

        for _ in range(2):
            fwd()
            bwd()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        tf = tb = 0.0
        for _ in range(iters):
            ev[0].record(stream)
            fwd()
            ev[1].record(stream)
            bwd()
            ev[2].record(stream)
            torch.cuda.synchronize()
            tf += ev[0].elapsed_time(ev[1]) / iters
            tb += ev[1].elapsed_time(ev[2]) / iters
        flops = 3 * B.ptdp_layer_flops_fwd(C.byref(cfg)) * w["layers"]
        row = {"b": b, "t_f_ms": round(tf, 4), "t_b_ms": round(tb, 4),
               "tflops_per_gpu": round(flops / ((tf + tb) * 1e-3) / 1e12, 2),
               "ms_per_sample": round((tf + tb) / b, 4)}
        rows.append(row)
        if emit:
            emit(row)
        ch.close()
        del stash, ws, x, dy, y, dx

    base = rows[0]["tflops_per_gpu"]
    summary = {"model": w["desc"], "dtype": "bf16", "p": p,
               "single_gpu_speedup_vs_smallest_b": {str(r["b"]): round(r["tflops_per_gpu"] / base, 3) for r in rows},
               "eq1": {}}
    for bp in batches:
        est = {}
        for r in rows:
            if bp % r["b"] == 0:
                est[r["b"]] = B.ptdp_batch_time(bp, r["b"], p, r["t_f_ms"], r["t_b_ms"])
        best = min(est, key=est.get)
        summary["eq1"][str(bp)] = {"batch_time_ms": {str(k): round(v, 4) for k, v in est.items()},
                                   "normalized_throughput": {str(k): round(est[best] / v, 3) for k, v in est.items()},
                                   "best_b": best}
    return rows, summary


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="1b", choices=sorted(MODELS))
    ap.add_argument("--b", type=int, nargs="+", default=[1, 2, 4, 8])
    ap.add_argument("--iters", type=int, default=5)
    ap.add_argument("--p", type=int, default=8, help="pipeline stages for eq. (1)")
    ap.add_argument("--batch", type=int, nargs="+", default=[128, 512], help="per-replica batch sizes b' for eq. (1)")
    args = ap.parse_args()
    try:
        _, summary = sweep(MODELS[args.model], args.b, args.iters, args.p, args.batch,
                           emit=lambda row: print(json.dumps(row), flush=True))
    except RuntimeError as e:
        print(e, file=sys.stderr)
        sys.exit(2)
    print(json.dumps(summary))


if __name__ == "__main__":
    main()
