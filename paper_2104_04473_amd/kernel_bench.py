"""Each exported kernel alone at the shapes of a workload, against its roofline.

    python -m paper_2104_04473_amd.kernel_bench [--shape c4|c3|c2] [--iters 10] [--only elementwise|attention]

Element-wise kernels rotate over enough distinct buffers (> 512 MB in total) that the 256 MB memory-side
cache cannot serve them; GEMMs and attention run on one buffer set (their operands exceed the caches or
are compute-bound).  Times are HIP events on the launch stream; median and minimum over the iterations.
Prints one JSON object per kernel.  Everything timed runs in the HIP library.
"""
import argparse
import ctypes as C
import json
import sys

SHAPES = {"c4": dict(h=25600, a=160, t=8, s=2048, b=1), "c3": dict(h=12288, a=96, t=8, s=2048, b=1),
          "c2": dict(h=2048, a=16, t=1, s=2048, b=4)}
PEAK_TFLOPS, PEAK_GBS = 2500.0, 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", default="c4", choices=sorted(SHAPES))
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--only", default="all", choices=["all", "elementwise", "attention"])
    args = ap.parse_args()
    import torch
    from . import binding as B
    if not torch.cuda.is_available():
        print("kernel_bench: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dev = "cuda:0"
    w = SHAPES[args.shape]
    T, h, hp, fp = w["s"] * w["b"], w["h"], w["h"] // w["t"], 4 * w["h"] // w["t"]
    heads, dh = w["a"] // w["t"], w["h"] // w["a"]
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    bf = torch.bfloat16

    def rnd(*shape, dtype=bf, scale=1.0):
        return (scale * torch.randn(shape, device=dev)).to(dtype)

    def timed(calls):
        """calls: list of closures (one per rotating buffer set); returns (median_ms, min_ms)."""
        for f in calls[:2]:
            f()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.iters + 1)]
        ev[0].record(stream)
        for i in range(args.iters):
            B.check(calls[i % len(calls)](), "kernel")
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        ts = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(args.iters))
        return ts[len(ts) // 2], ts[0]

    def report(name, work, unit, calls):
        med, mn = timed(calls)
        rate = work / (med * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9)
        peak = PEAK_TFLOPS if unit == "TFLOP/s" else PEAK_GBS
        print(json.dumps({"kernel": name, "shape": args.shape, "median_ms": round(med, 4), "min_ms": round(mn, 4),
                          "achieved": round(rate, 1), "unit": unit, "frac_of_peak": round(rate / peak, 4)}), flush=True)

    def sets(width, n_tensors):
        """Number of rotating buffer sets so that the sets total more than 512 MB."""
        per = T * width * 2 * n_tensors
        return max(2, -(-(600 << 20) // per))

    if args.only in ("all", "elementwise"):
        # ---- element-wise kernels (bytes = algorithmic bytes of the bf16 path) ------------------------------
        g = torch.ones(h, dtype=bf, device=dev); be = torch.zeros(h, dtype=bf, device=dev)
        n = sets(h, 2)
        xs = [rnd(T, h) for _ in range(n)]; us = [torch.empty(T, h, dtype=bf, device=dev) for _ in range(n)]
        mu = torch.empty(T, device=dev); rstd = torch.empty(T, device=dev)
        report("layernorm_fwd", T * h * 4, "GB/s",
               [lambda i=i: B.ptdp_layernorm_fwd(B.BF16, xs[i].data_ptr(), g.data_ptr(), be.data_ptr(), us[i].data_ptr(),
                                                 mu.data_ptr(), rstd.data_ptr(), None, T, h, 1e-5, sh) for i in range(n)])
        dg = torch.zeros(h, device=dev); db = torch.zeros(h, device=dev)
        scratch = torch.empty(max(B.ptdp_layernorm_bwd_scratch_bytes(T, h), B.ptdp_colsum_scratch_bytes(T, max(h, fp))), dtype=torch.uint8, device=dev)
        B.ptdp_layernorm_fwd(B.BF16, xs[0].data_ptr(), g.data_ptr(), be.data_ptr(), us[0].data_ptr(), mu.data_ptr(),
                             rstd.data_ptr(), None, T, h, 1e-5, sh)
        report("layernorm_bwd (dx + parameter gradients, with residual)", T * h * 12, "GB/s",
               [lambda i=i: B.ptdp_layernorm_bwd(B.BF16, us[i].data_ptr(), xs[i].data_ptr(), g.data_ptr(), mu.data_ptr(),
                                                 rstd.data_ptr(), xs[(i + 1) % n].data_ptr(), us[i].data_ptr(), dg.data_ptr(),
                                                 db.data_ptr(), scratch.data_ptr(), T, h, sh) for i in range(n)])
        report("bias_dropout_add_fwd", T * h * 6, "GB/s",
               [lambda i=i: B.ptdp_bias_dropout_add_fwd(B.BF16, xs[i].data_ptr(), be.data_ptr(), xs[(i + 1) % n].data_ptr(),
                                                        us[i].data_ptr(), T, h, 0.1, 0, 0, 0, 0, sh) for i in range(n)])
        report("bias_dropout_add_bwd", T * h * 4, "GB/s",
               [lambda i=i: B.ptdp_bias_dropout_add_bwd(B.BF16, xs[i].data_ptr(), us[i].data_ptr(), db.data_ptr(),
                                                        scratch.data_ptr(), T, h, 0.1, 0, 0, 0, 0, sh) for i in range(n)])
        del xs, us
        n = sets(fp, 2)
        zs = [rnd(T, fp) for _ in range(n)]; gs = [torch.empty(T, fp, dtype=bf, device=dev) for _ in range(n)]
        b1 = torch.zeros(fp, dtype=bf, device=dev); db1 = torch.zeros(fp, device=dev)
        report("bias_gelu_fwd", T * fp * 4, "GB/s",
               [lambda i=i: B.ptdp_bias_gelu_fwd(B.BF16, B.GELU_ERF, zs[i].data_ptr(), b1.data_ptr(), gs[i].data_ptr(), T, fp, sh)
                for i in range(n)])
        report("bias_gelu_bwd", T * fp * 6, "GB/s",
               [lambda i=i: B.ptdp_bias_gelu_bwd(B.BF16, B.GELU_ERF, gs[i].data_ptr(), zs[i].data_ptr(), b1.data_ptr(),
                                                 gs[i].data_ptr(), db1.data_ptr(), scratch.data_ptr(), T, fp, sh) for i in range(n)])
        del zs, gs

    if args.only == "all":
        # ---- GEMMs of one layer ----------------------------------------------------------------------------
        ws = torch.empty(B.ptdp_gemm_workspace_bytes(), dtype=torch.uint8, device=dev)
        fwd = [("qkv", 3 * hp, h), ("attention output", h, hp), ("mlp h->4h/t", fp, h), ("mlp 4h/t->h", h, fp)]
        for name, N, K in fwd:
            a = rnd(T, K); wgt = rnd(K, N, scale=0.02); c = torch.empty(T, N, dtype=bf, device=dev)
            report("gemm forward %s [%d x %d x %d]" % (name, T, N, K), 2.0 * T * N * K, "TFLOP/s",
                   [lambda: B.ptdp_gemm(B.BF16, B.GEMM_NN, a.data_ptr(), wgt.data_ptr(), c.data_ptr(), None, T, N, K, 0, 0,
                                        ws.data_ptr(), ws.numel(), sh)])
            dy = rnd(T, N); dx = torch.empty(T, K, dtype=bf, device=dev)
            report("gemm data gradient %s [%d x %d x %d]" % (name, T, K, N), 2.0 * T * N * K, "TFLOP/s",
                   [lambda: B.ptdp_gemm(B.BF16, B.GEMM_NT, dy.data_ptr(), wgt.data_ptr(), dx.data_ptr(), None, T, K, N, 0, 0,
                                        ws.data_ptr(), ws.numel(), sh)])
            dw = torch.zeros(K, N, device=dev)
            report("gemm weight gradient %s [%d x %d x %d]" % (name, K, N, T), 2.0 * T * N * K, "TFLOP/s",
                   [lambda: B.ptdp_gemm(B.BF16, B.GEMM_TN, a.data_ptr(), dy.data_ptr(), dw.data_ptr(), None, K, N, T, 1, 1,
                                        ws.data_ptr(), ws.numel(), sh)])
            del a, wgt, c, dy, dx, dw

    if args.only == "elementwise":
        return

    # ---- attention -------------------------------------------------------------------------------------
    qkv = rnd(w["s"], w["b"], 3 * hp); ctx = torch.empty(w["s"], w["b"], hp, dtype=bf, device=dev)
    lse = torch.empty(w["b"], heads, w["s"], device=dev); delta = torch.empty_like(lse)
    dctx = rnd(w["s"], w["b"], hp); dqkv = torch.empty_like(qkv)
    fl = 4.0 * w["b"] * heads * w["s"] * w["s"] * dh
    report("attention forward (full-square FLOP count)", fl, "TFLOP/s",
           [lambda: B.ptdp_attn_fwd(B.BF16, qkv.data_ptr(), ctx.data_ptr(), lse.data_ptr(), w["s"], w["b"], heads, dh, sh)])
    report("attention backward (full-square FLOP count)", 2 * fl, "TFLOP/s",
           [lambda: B.ptdp_attn_bwd(B.BF16, qkv.data_ptr(), ctx.data_ptr(), lse.data_ptr(), dctx.data_ptr(), dqkv.data_ptr(),
                                    delta.data_ptr(), w["s"], w["b"], heads, dh, sh)])


if __name__ == "__main__":
    main()
