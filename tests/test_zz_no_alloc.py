"""The entry point that allocates nothing (column-sum partials in a static device array) against the entry
point that takes caller scratch: same bits, on two calls in a row, the second on a smaller input."""
import numpy as np
import pytest
import torch

from oracle import dropout_hash
from paper_2104_04473_amd import binding as B
from gpu_util import assert_close, dev_bytes, np64, randn, stream, sync

pytestmark = pytest.mark.gpu


def both(dtype, rows, width, p, seed, layer, site, mb):
    dout = randn((rows, width), dtype, 4 + rows)
    outs = []
    for static in (False, True):
        din = torch.full_like(dout, 7.0)
        db = torch.full((width,), 0.25, device="cuda")                     # += semantics
        if static:
            before = torch.cuda.memory_allocated()
            B.check(B.ptdp_bias_dropout_add_bwd_noalloc(dtype, dout.data_ptr(), din.data_ptr(), db.data_ptr(), rows, width,
                                                        p, seed, layer, site, mb, stream()), "bda_bwd_noalloc")
            assert torch.cuda.memory_allocated() == before
        else:
            scratch = dev_bytes(B.ptdp_colsum_scratch_bytes(rows, width))
            B.check(B.ptdp_bias_dropout_add_bwd(dtype, dout.data_ptr(), din.data_ptr(), db.data_ptr(), scratch.data_ptr(),
                                                rows, width, p, seed, layer, site, mb, stream()), "bda_bwd")
        sync()
        outs.append((din, db))
    (din0, db0), (din1, db1) = outs
    assert torch.equal(din0, din1) and torch.equal(db0, db1), (rows, width)
    # and against the definition
    keep = dropout_hash.keep_mask(seed, layer, site, mb, rows * width, p).reshape(rows, width)
    want = np64(dout) * keep * dropout_hash.keep_scale(p)
    assert_close(np64(din1), want, dtype, "din")
    assert_close(np64(db1) - 0.25, want.sum(axis=0), dtype, "dbias")


@pytest.mark.parametrize("dtype", [B.BF16, B.F32])
def test_no_alloc_entry_point_matches_the_scratch_taking_one(dtype):
    assert B.ptdp_noalloc_scratch_bytes() == 8 << 20
    both(dtype, 2048, 12288 if dtype == B.BF16 else 4096, 0.1, 42, 3, 1, 5)   # several row tiles, many column blocks
    both(dtype, 70, 264, 0.1, 42, 3, 0, 6)                                    # smaller, ragged: stale partials lie beyond
    both(dtype, 1, 8, 0.0, 1, 0, 0, 0)


def test_no_alloc_entry_point_rejects_what_does_not_fit():
    rows, width = 4096, 25600                                                  # 128 row tiles x 25600 floats = 12.5 MiB
    assert B.ptdp_colsum_scratch_bytes(rows, width) > B.ptdp_noalloc_scratch_bytes()
    a = torch.zeros(8, device="cuda")
    rc = B.ptdp_bias_dropout_add_bwd_noalloc(B.BF16, a.data_ptr(), a.data_ptr() + 16, a.data_ptr(), rows, width, 0.1, 0, 0, 0, 0,
                                             stream())
    assert rc == B.E_TOO_SMALL
    assert B.ptdp_bias_dropout_add_bwd_noalloc(B.BF16, None, a.data_ptr(), a.data_ptr(), 8, 8, 0.1, 0, 0, 0, 0, stream()) == B.E_NULL_PTR
    B.ptdp_prof_enable(1)
    try:
        x = torch.zeros((8, 8), dtype=torch.bfloat16, device="cuda"); y = torch.zeros_like(x)
        assert B.ptdp_bias_dropout_add_bwd_noalloc(B.BF16, x.data_ptr(), y.data_ptr(), a.data_ptr(), 8, 8, 0.1, 0, 0, 0, 0,
                                                   stream()) == B.E_STATE
    finally:
        B.ptdp_prof_enable(0)
