"""GPU parity of the GEMM and attention kernels against their plain definitions (oracle side)."""
import numpy as np
import pytest
import torch

from oracle import gpt_layer as L
from paper_2104_04473_amd import binding as B
from gpu_util import assert_close, np64, randn, stream, sync, tdt

pytestmark = pytest.mark.gpu

SHAPES = [(8, 8, 8), (136, 264, 72), (256, 256, 64), (520, 776, 200), (1032, 264, 1096), (264, 1032, 520),
          (264, 136, 128), (72, 520, 136), (136, 72, 192)]     # 1, 2, 3 and more k-steps, whole and ragged


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
@pytest.mark.parametrize("mode", [B.GEMM_NN, B.GEMM_NT, B.GEMM_TN])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm(dtype, mode, M, N, K):
    a = randn((M, K), dtype, 1)
    b = randn((K, N), dtype, 2)
    bias = randn((N,), dtype, 3)
    want = np64(a) @ np64(b)
    A = a.t().contiguous() if mode == B.GEMM_TN else a            # [K, M]
    Bm = b.t().contiguous() if mode == B.GEMM_NT else b           # [N, K]
    # storage-dtype output with bias
    c = torch.full((M, N), 9.0, dtype=tdt(dtype), device="cuda")
    B.check(B.ptdp_gemm(dtype, mode, A.data_ptr(), Bm.data_ptr(), c.data_ptr(), bias.data_ptr(), M, N, K,
                        1 if dtype == B.F32 else 0, 0, None, 0, stream()), "gemm")
    sync()
    assert_close(np64(c), want + np64(bias), dtype, "C")
    # fp32 accumulate (+=), twice
    acc = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    for _ in range(2):
        B.check(B.ptdp_gemm(dtype, mode, A.data_ptr(), Bm.data_ptr(), acc.data_ptr(), None, M, N, K, 1, 1, None, 0, stream()), "gemm")
    sync()
    assert_close(np64(acc) - 0.5, 2 * want, dtype, "C +=")


@pytest.mark.parametrize("mode", [B.GEMM_NN, B.GEMM_NT, B.GEMM_TN])
@pytest.mark.parametrize("K,Kpad", [(192, 256), (200, 256), (4096, 4104), (520, 576)])
def test_gemm_zero_padding_along_k_changes_no_bit(mode, K, Kpad):
    """The same product with the reduction index padded by zeros.  K = 192 -> 256 moves a k-contiguous operand from
    rows shorter than 256 elements (every operand request in the general form, with per-lane checks) to rows of 256
    (whole k-tiles requested in the lean form); 4096 -> 4104 and 520 -> 576 add or remove a partial last k-tile.
    Every output element adds the same products in the same order plus exact zeros: the results agree bit for bit."""
    M, N = 520, 264
    a = randn((M, K), B.BF16, 1)
    b = randn((K, N), B.BF16, 2)
    ap = torch.zeros((M, Kpad), dtype=torch.bfloat16, device="cuda"); ap[:, :K] = a
    bp = torch.zeros((Kpad, N), dtype=torch.bfloat16, device="cuda"); bp[:K] = b
    outs = []
    for (x, y, k) in ((a, b, K), (ap, bp, Kpad)):
        A = x.t().contiguous() if mode == B.GEMM_TN else x.contiguous()
        Bm = y.t().contiguous() if mode == B.GEMM_NT else y.contiguous()
        c = torch.full((M, N), 9.0, dtype=torch.bfloat16, device="cuda")
        acc = torch.full((M, N), 0.25, dtype=torch.float32, device="cuda")
        B.check(B.ptdp_gemm(B.BF16, mode, A.data_ptr(), Bm.data_ptr(), c.data_ptr(), None, M, N, k, 0, 0, None, 0, stream()), "gemm")
        B.check(B.ptdp_gemm(B.BF16, mode, A.data_ptr(), Bm.data_ptr(), acc.data_ptr(), None, M, N, k, 1, 1, None, 0, stream()), "gemm")
        sync()
        outs.append((c, acc))
    assert torch.equal(outs[0][0], outs[1][0])
    assert torch.equal(outs[0][1], outs[1][1])
    assert_close(np64(outs[0][1]) - 0.25, np64(a) @ np64(b), B.BF16, "C +=")


@pytest.mark.parametrize("mode", [B.GEMM_NN, B.GEMM_NT, B.GEMM_TN])
@pytest.mark.parametrize("M,N,K", [(520, 776, 4168), (264, 4104, 4096), (2048, 1288, 4160), (2048, 10248, 4096),
                                   (14336, 1792, 4096)])   # 56 row tiles: do not divide the compute-unit count
def test_gemm_split_along_k(mode, M, N, K):
    """Tile counts that do not fill the compute units: the remaining tiles are split along k through the
    workspace and reduced in a fixed order (bf16 output, or += into the fp32 accumulator)."""
    dtype = B.BF16
    a = randn((M, K), dtype, 1)
    b = randn((K, N), dtype, 2)
    bias = randn((N,), dtype, 3)
    want = np64(a) @ np64(b)
    A = a.t().contiguous() if mode == B.GEMM_TN else a
    Bm = b.t().contiguous() if mode == B.GEMM_NT else b
    ws = torch.full((B.ptdp_gemm_workspace_bytes() // 4,), 7.0, dtype=torch.float32, device="cuda")   # garbage on entry
    c = torch.full((M, N), 9.0, dtype=torch.bfloat16, device="cuda")
    B.check(B.ptdp_gemm(dtype, mode, A.data_ptr(), Bm.data_ptr(), c.data_ptr(), bias.data_ptr(), M, N, K, 0, 0,
                        ws.data_ptr(), ws.numel() * 4, stream()), "gemm")
    sync()
    assert_close(np64(c), want + np64(bias), dtype, "C")
    # bit-reproducible: the partial tiles are summed in a fixed order
    c1 = torch.empty_like(c)
    B.check(B.ptdp_gemm(dtype, mode, A.data_ptr(), Bm.data_ptr(), c1.data_ptr(), bias.data_ptr(), M, N, K, 0, 0,
                        ws.data_ptr(), ws.numel() * 4, stream()), "gemm")
    sync()
    assert torch.equal(c, c1)
    # same result as the unsplit path up to bf16 rounding of an fp32 sum taken in another order
    c2 = torch.empty_like(c)
    B.check(B.ptdp_gemm(dtype, mode, A.data_ptr(), Bm.data_ptr(), c2.data_ptr(), bias.data_ptr(), M, N, K, 0, 0,
                        None, 0, stream()), "gemm")
    sync()
    assert_close(np64(c), np64(c2), dtype, "split vs unsplit", 0.2)
    # too small a workspace falls back to the unsplit path
    B.check(B.ptdp_gemm(dtype, mode, A.data_ptr(), Bm.data_ptr(), c2.data_ptr(), bias.data_ptr(), M, N, K, 0, 0,
                        ws.data_ptr(), 1024, stream()), "gemm")
    acc = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    for _ in range(2):
        B.check(B.ptdp_gemm(dtype, mode, A.data_ptr(), Bm.data_ptr(), acc.data_ptr(), None, M, N, K, 1, 1,
                            ws.data_ptr(), ws.numel() * 4, stream()), "gemm")
    sync()
    assert_close(np64(acc) - 0.5, 2 * want, dtype, "C +=")


def run_attn(dtype, s, b, heads, dh, seed=0, scale=1.0):
    hp = heads * dh
    qkv = randn((s, b, 3 * hp), dtype, seed, scale)
    ctx = torch.zeros((s, b, hp), dtype=tdt(dtype), device="cuda")
    lse = torch.zeros((b, heads, s), device="cuda")
    B.check(B.ptdp_attn_fwd(dtype, qkv.data_ptr(), ctx.data_ptr(), lse.data_ptr(), s, b, heads, dh, stream()), "attn_fwd")
    sync()
    return qkv, ctx, lse


ATTN_CASES = [(B.F32, 128, 2, 4, 64), (B.F32, 77, 1, 2, 32), (B.F32, 1, 2, 1, 64), (B.F32, 40, 1, 1, 160),
              (B.BF16, 128, 2, 2, 64), (B.BF16, 300, 2, 3, 128), (B.BF16, 333, 1, 2, 160), (B.BF16, 1, 1, 1, 128),
              (B.BF16, 64, 1, 1, 128), (B.BF16, 129, 1, 1, 64), (B.BF16, 520, 1, 1, 128),
              (B.BF16, 200, 2, 3, 32), (B.BF16, 333, 1, 2, 96), (B.BF16, 65, 2, 1, 96),
              # more than 512 (query block, sample, head) triples: the backward kernels take their one-pair form
              # (fewer: two pairs of waves per workgroup, as in every case above)
              (B.BF16, 130, 8, 24, 32), (B.BF16, 200, 5, 27, 160), (B.BF16, 257, 3, 36, 128)]


@pytest.mark.parametrize("dtype,s,b,heads,dh", ATTN_CASES)
def test_attention_forward_backward(dtype, s, b, heads, dh):
    hp = heads * dh
    qkv, ctx, lse = run_attn(dtype, s, b, heads, dh)
    cfg = L.LayerConfig(h=hp, a=heads, t=1, s=s, b=b)
    wctx, probs, wlse = L.attention_core(np64(qkv), cfg)
    assert_close(np64(ctx), wctx, dtype, "ctx")
    assert_close(np64(lse), wlse, B.F32, "lse")
    dctx = randn((s, b, hp), dtype, 7)
    dqkv = torch.zeros_like(qkv)
    delta = torch.zeros((b, heads, s), device="cuda")
    B.check(B.ptdp_attn_bwd(dtype, qkv.data_ptr(), ctx.data_ptr(), lse.data_ptr(), dctx.data_ptr(), dqkv.data_ptr(),
                            delta.data_ptr(), s, b, heads, dh, stream()), "attn_bwd")
    sync()
    want = L.attention_core_backward(np64(dctx), np64(qkv), probs, cfg)
    got = np64(dqkv)
    for name, lo in (("dq", 0), ("dk", hp), ("dv", 2 * hp)):
        assert_close(got[..., lo:lo + hp], want[..., lo:lo + hp], dtype, name)


def test_attention_sharp_softmax_bf16():
    # logits with standard deviation ~10, as N(0, 0.02) weights give at h = 25600
    s, b, heads, dh = 256, 1, 2, 160
    qkv, ctx, lse = run_attn(B.BF16, s, b, heads, dh, seed=3, scale=3.2)
    cfg = L.LayerConfig(h=heads * dh, a=heads, t=1, s=s, b=b)
    wctx, _, wlse = L.attention_core(np64(qkv), cfg)
    assert_close(np64(ctx), wctx, B.BF16, "ctx")


def test_attention_causal_invariance_on_gpu():
    s, b, heads, dh = 200, 1, 2, 128
    qkv, ctx, _ = run_attn(B.BF16, s, b, heads, dh)
    q2 = qkv.clone()
    q2[131:] = randn((s - 131, b, 3 * heads * dh), B.BF16, 9)
    ctx2 = torch.zeros_like(ctx); lse2 = torch.zeros((b, heads, s), device="cuda")
    B.check(B.ptdp_attn_fwd(B.BF16, q2.data_ptr(), ctx2.data_ptr(), lse2.data_ptr(), s, b, heads, dh, stream()), "attn")
    sync()
    assert torch.equal(ctx[:131], ctx2[:131])
