"""GPU parity of the bandwidth-bound kernels against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import dropout_hash
from oracle import gpt_layer as L
from paper_2104_04473_amd import binding as B
from gpu_util import assert_close, dev_bytes, np64, randn, stream, sync, tdt

pytestmark = pytest.mark.gpu
DTYPES = [B.F32, B.BF16]


@pytest.mark.parametrize("n", [0, 1, 3, 4, 1000003])
def test_dropout_mask_bit_exact(n):
    for (p, seed, layer, site, mb) in [(0.1, 0, 0, 0, 0), (0.5, 12345678901234567, 95, 1, 7), (0.0, 3, 1, 1, 1)]:
        keep = torch.full((max(n, 1),), 7, dtype=torch.uint8, device="cuda")
        B.check(B.ptdp_dropout_mask(keep.data_ptr(), n, p, seed, layer, site, mb, stream()), "mask")
        sync()
        want = dropout_hash.keep_mask(seed, layer, site, mb, n, p)
        assert np.array_equal(keep.cpu().numpy()[:n].astype(bool), want)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("rows,width", [(1, 8), (7, 264), (300, 256), (33, 2048), (5, 12288), (3, 25600), (2, 1000)])
def test_layernorm_forward_backward(dtype, rows, width):
    if dtype == B.F32 and width > 16384:
        pytest.skip("fp32 LayerNorm keeps at most 16384 columns in registers")
    x = randn((rows, width), dtype, 1, 2.0) + 0.5
    gain = randn((width,), dtype, 2, 0.2) + 1.0
    bias = randn((width,), dtype, 3, 0.3)
    du = randn((rows, width), dtype, 4)
    resid = randn((rows, width), dtype, 5)
    u = torch.empty_like(x); xc = torch.empty_like(x)
    mu = torch.empty(rows, device="cuda"); rstd = torch.empty(rows, device="cuda")
    B.check(B.ptdp_layernorm_fwd(dtype, x.data_ptr(), gain.data_ptr(), bias.data_ptr(), u.data_ptr(), mu.data_ptr(),
                                 rstd.data_ptr(), xc.data_ptr(), rows, width, 1e-5, stream()), "ln_fwd")
    sync()
    wu, wmu, wrstd = L.layernorm(np64(x), np64(gain), np64(bias), float(np.float32(1e-5)))
    assert_close(np64(u), wu, dtype, "u")
    assert_close(np64(mu), wmu[:, 0], B.F32, "mu")
    assert_close(np64(rstd), wrstd[:, 0], B.F32, "rstd")
    assert torch.equal(xc, x)

    dg = torch.full((width,), 1.0, device="cuda"); db = torch.full((width,), -2.0, device="cuda")   # += semantics
    scratch = dev_bytes(B.ptdp_layernorm_bwd_scratch_bytes(rows, width))
    dx = torch.empty_like(x)
    B.check(B.ptdp_layernorm_bwd(dtype, du.data_ptr(), x.data_ptr(), gain.data_ptr(), mu.data_ptr(), rstd.data_ptr(),
                                 resid.data_ptr(), dx.data_ptr(), dg.data_ptr(), db.data_ptr(), scratch.data_ptr(),
                                 rows, width, stream()), "ln_bwd")
    sync()
    wdx, wdg, wdb = L.layernorm_backward(np64(du), np64(x), np64(gain), wmu, wrstd)
    assert_close(np64(dx), wdx + np64(resid), dtype, "dx")
    assert_close(np64(dg) - 1.0, wdg, dtype, "dgain")
    assert_close(np64(db) + 2.0, wdb, dtype, "dbias")
    # without residual, in place over du
    du2 = du.clone()
    B.check(B.ptdp_layernorm_bwd(dtype, du2.data_ptr(), x.data_ptr(), gain.data_ptr(), mu.data_ptr(), rstd.data_ptr(),
                                 None, du2.data_ptr(), dg.data_ptr(), db.data_ptr(), scratch.data_ptr(),
                                 rows, width, stream()), "ln_bwd")
    sync()
    assert_close(np64(du2), wdx, dtype, "dx in place")


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("mode", [B.GELU_ERF, B.GELU_TANH])
@pytest.mark.parametrize("rows,width", [(1, 8), (70, 264), (257, 1024), (33, 12800), (3, 1032), (35, 520)])
def test_bias_gelu(dtype, mode, rows, width):
    z = randn((rows, width), dtype, 1, 2.0)
    bias = randn((width,), dtype, 2, 0.5)
    dg = randn((rows, width), dtype, 3)
    g = torch.empty_like(z)
    B.check(B.ptdp_bias_gelu_fwd(dtype, mode, z.data_ptr(), bias.data_ptr(), g.data_ptr(), rows, width, stream()), "gelu")
    sync()
    zz = np64(z) + np64(bias)
    assert_close(np64(g), L.gelu(zz, mode == B.GELU_TANH), dtype, "g")
    db = torch.full((width,), 3.0, device="cuda")
    scratch = dev_bytes(B.ptdp_colsum_scratch_bytes(rows, width))
    dz = torch.empty_like(z)
    B.check(B.ptdp_bias_gelu_bwd(dtype, mode, dg.data_ptr(), z.data_ptr(), bias.data_ptr(), dz.data_ptr(), db.data_ptr(),
                                 scratch.data_ptr(), rows, width, stream()), "gelu_bwd")
    sync()
    want = np64(dg) * L.gelu_grad(zz, mode == B.GELU_TANH)
    assert_close(np64(dz), want, dtype, "dz")
    # the bias gradient sums what the kernel produced before rounding to storage; compare to the oracle's
    assert_close(np64(db) - 3.0, want.sum(axis=0), dtype, "db1")


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("p", [0.0, 0.1, 0.5])
@pytest.mark.parametrize("rows,width", [(1, 8), (70, 264), (256, 256), (19, 12288), (3, 1032), (35, 520)])
def test_bias_dropout_add(dtype, p, rows, width):
    seed, layer, site, mb = 42, 3, 1, 5
    a = randn((rows, width), dtype, 1)
    bias = randn((width,), dtype, 2, 0.5)
    resid = randn((rows, width), dtype, 3)
    out = torch.empty_like(a)
    B.check(B.ptdp_bias_dropout_add_fwd(dtype, a.data_ptr(), bias.data_ptr(), resid.data_ptr(), out.data_ptr(), rows,
                                        width, p, seed, layer, site, mb, stream()), "bda")
    sync()
    keep = dropout_hash.keep_mask(seed, layer, site, mb, rows * width, p).reshape(rows, width)
    scale = dropout_hash.keep_scale(p)
    want = np64(resid) + (np64(a) + np64(bias)) * keep * scale
    assert_close(np64(out), want, dtype, "out")
    # dropped positions pass the residual through untouched: the mask itself is bit-exact
    assert np.array_equal(np64(out)[~keep], np64(resid)[~keep])
    dout = randn((rows, width), dtype, 4)
    din = torch.empty_like(dout)
    db = torch.zeros(width, device="cuda")
    scratch = dev_bytes(B.ptdp_colsum_scratch_bytes(rows, width))
    B.check(B.ptdp_bias_dropout_add_bwd(dtype, dout.data_ptr(), din.data_ptr(), db.data_ptr(), scratch.data_ptr(), rows,
                                        width, p, seed, layer, site, mb, stream()), "bda_bwd")
    sync()
    wdin = np64(dout) * keep * scale
    assert_close(np64(din), wdin, dtype, "din")
    assert np.array_equal(np64(din) == 0, ~keep | (np64(dout) == 0))
    assert_close(np64(db), wdin.sum(axis=0), dtype, "dbias")
