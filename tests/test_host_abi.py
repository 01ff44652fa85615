"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host
logic (validation, sizes, hash, schedule) agrees with the oracle.  No kernels are launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import dropout_hash, flops, schedule
from paper_2104_04473_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ptdp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ptdp_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_functions()
    assert len(names) >= 30
    for n in names:
        assert hasattr(B.lib, n), n
        assert n in B.SIGNATURES, "binding lacks " + n
    assert set(B.SIGNATURES) == set(names)


def test_status_strings():
    for code in range(0, -7, -1):
        assert B.status_string(code) not in ("", "unknown status")
    assert B.status_string(-99) == "unknown status"


def cfg(**kw):
    base = dict(h=256, a=4, t=1, s=128, b=2, dtype=B.F32, p_hidden=0.1)
    base.update(kw)
    return B.make_cfg(**base)


def test_cfg_validation():
    ok = lambda c: B.ptdp_cfg_validate(C.byref(c))
    assert ok(cfg()) == B.OK
    assert ok(cfg(h=250)) == B.E_INVALID_ARG            # h % a
    assert ok(cfg(a=4, t=3)) == B.E_INVALID_ARG         # a % t
    assert ok(cfg(p_hidden=1.0)) == B.E_INVALID_ARG
    assert ok(cfg(p_hidden=-0.1)) == B.E_INVALID_ARG
    assert ok(cfg(ln_eps=0.0)) == B.E_INVALID_ARG
    assert ok(cfg(s=0)) == B.E_INVALID_ARG
    assert ok(cfg(dtype=7)) == B.E_INVALID_ARG
    assert ok(cfg(causal=0)) == B.OK            # general mask
    assert ok(cfg(causal=2)) == B.E_INVALID_ARG
    assert ok(cfg(h=96, a=4, dtype=B.BF16)) == B.E_UNSUPPORTED      # dh = 24: no MFMA attention
    assert ok(cfg(h=100, a=5)) == B.E_INVALID_ARG                   # dh = 20 not a multiple of 8
    bad = cfg(); bad.struct_size = 12
    assert ok(bad) == B.E_INVALID_ARG
    assert B.ptdp_cfg_validate(None) == B.E_NULL_PTR
    for shape in (dict(h=2048, a=16, s=2048, b=4), dict(h=12288, a=96, t=8, s=2048, b=1),
                  dict(h=25600, a=160, t=8, s=2048, b=1)):
        assert ok(cfg(dtype=B.BF16, **shape)) == B.OK


def test_flops_match_paper_closed_form():
    for shape in (dict(h=256, a=4, t=1, s=128, b=2), dict(h=12288, a=96, t=8, s=2048, b=1),
                  dict(h=25600, a=160, t=8, s=2048, b=1)):
        c = cfg(dtype=B.BF16 if shape["h"] > 256 else B.F32, **shape)
        want = flops.layer_forward_flops(shape["b"], shape["s"], shape["h"]) // shape["t"]
        assert B.ptdp_layer_flops_fwd(C.byref(c)) == want
    assert B.ptdp_layer_flops_fwd(C.byref(cfg(h=250))) == -1


def test_stash_layout():
    c = cfg(h=64, a=4, t=2, s=16, b=3, dtype=B.BF16 if False else B.F32)
    offs = B.stash_offsets(c)
    total = B.ptdp_layer_stash_bytes(C.byref(c))
    T, h, hp, fp = 48, 64, 32, 128
    sizes = dict(X=T * h * 4, U=T * h * 4, QKV=T * 3 * hp * 4, CTX=T * hp * 4, X1=T * h * 4, U2=T * h * 4,
                 Z=T * fp * 4, G=T * fp * 4, MU1=T * 4, RSTD1=T * 4, MU2=T * 4, RSTD2=T * 4, LSE=3 * 2 * 16 * 4)
    order = list(B.STASH_FIELDS)
    for i, name in enumerate(order):
        assert offs[name] % 256 == 0
        end = offs[order[i + 1]] if i + 1 < len(order) else total
        assert end - offs[name] >= sizes[name]
    assert B.ptdp_stash_offset(C.byref(c), 99) == 2 ** 64 - 1
    assert B.ptdp_workspace_bytes(C.byref(c)) > 0
    assert B.ptdp_layer_stash_bytes(C.byref(cfg(h=250))) == 0


def test_hash_matches_oracle_bit_for_bit():
    rng = np.random.default_rng(0)
    for _ in range(200):
        seed = int(rng.integers(0, 2 ** 63)); layer = int(rng.integers(0, 200)); site = int(rng.integers(0, 2))
        mb = int(rng.integers(0, 1000)); group = int(rng.integers(0, 2 ** 40))
        assert B.ptdp_hash(seed, layer, site, mb, group) == int(dropout_hash.hash_word(seed, layer, site, mb, np.uint64(group)))
    assert B.ptdp_hash(2 ** 64 - 1, 0, 0, 0, 0) == int(dropout_hash.hash_word(2 ** 64 - 1, 0, 0, 0, np.uint64(0)))


@pytest.mark.parametrize("p,v,m", [(4, 1, 8), (4, 2, 8), (4, 2, 4), (8, 4, 8), (2, 2, 4), (4, 3, 12), (1, 1, 3),
                                   (1, 2, 3), (5, 1, 3), (3, 2, 6)])
def test_schedule_matches_oracle(p, v, m):
    for r in range(p):
        steps = B.schedule_build(p, v, m, r)
        got = [(s.kind, s.chunk, s.microbatch) for s in steps]
        want = schedule.device_order(p, v, m, r)
        assert got == want
        assert B.ptdp_schedule_peak_inflight(p, v, m, r) == schedule.peak_in_flight(want)


def test_schedule_errors():
    n = C.c_int(0)
    assert B.ptdp_schedule_build(4, 2, 6, 0, None, 0, C.byref(n)) == B.E_INVALID_ARG     # m % p
    assert B.ptdp_schedule_build(4, 1, 6, 4, None, 0, C.byref(n)) == B.E_INVALID_ARG     # rank
    assert B.ptdp_schedule_build(4, 1, 6, 0, None, 0, None) == B.E_NULL_PTR
    assert B.ptdp_schedule_build(4, 1, 6, 0, None, 0, C.byref(n)) == B.OK and n.value == 12
    buf = (B.Step * 5)()
    assert B.ptdp_schedule_build(4, 1, 6, 0, buf, 5, C.byref(n)) == B.E_TOO_SMALL
    assert B.ptdp_schedule_peak_inflight(0, 1, 1, 0) == B.E_INVALID_ARG


def test_chunk_object_errors_without_device_work():
    h = C.c_void_p()
    assert B.ptdp_chunk_create(C.byref(cfg(h=250)), 1, 0, C.byref(h)) == B.E_INVALID_ARG
    assert B.ptdp_chunk_create(C.byref(cfg()), 0, 0, C.byref(h)) == B.E_INVALID_ARG
    assert B.ptdp_chunk_create(C.byref(cfg()), 1, 0, None) == B.E_NULL_PTR
    assert B.ptdp_chunk_create(C.byref(cfg()), 2, 4, C.byref(h)) == B.OK
    assert B.ptdp_chunk_n_layers(h) == 2
    P = B.LayerParams()          # all NULL
    assert B.ptdp_chunk_bind_params(h, 0, C.byref(P)) == B.E_NULL_PTR
    assert B.ptdp_chunk_bind_params(h, 2, C.byref(P)) == B.E_INVALID_ARG
    # forward before parameters are bound: refused on the host (fake non-null pointers are never touched)
    assert B.ptdp_layer_forward(h, 0, 0, 256, 512, 768, 1024, None) == B.E_STATE
    assert B.ptdp_layer_forward(h, 0, 0, None, 512, 768, 1024, None) == B.E_NULL_PTR
    assert B.ptdp_layer_forward(h, 5, 0, 256, 512, 768, 1024, None) == B.E_INVALID_ARG
    assert B.ptdp_layer_backward(h, 0, 0, 256, 512, 768, 1024, None) == B.E_STATE
    assert B.ptdp_chunk_forward(h, 0, 256, 512, 768, 1024, None) == B.E_STATE
    B.ptdp_chunk_destroy(h)


def test_single_kernel_argument_checks():
    assert B.ptdp_gemm(B.BF16, B.GEMM_NN, 256, 256, 256, None, 8, 8, 12, 0, 0, None, 0, None) == B.E_INVALID_ARG   # K % 8
    assert B.ptdp_gemm(B.BF16, 5, 256, 256, 256, None, 8, 8, 8, 0, 0, None, 0, None) == B.E_INVALID_ARG
    assert B.ptdp_gemm(B.BF16, B.GEMM_NN, None, 256, 256, None, 8, 8, 8, 0, 0, None, 0, None) == B.E_NULL_PTR
    assert B.ptdp_layernorm_fwd(B.F32, 256, 256, 256, 256, 256, 256, None, 4, 12, 1e-5, None) == B.E_INVALID_ARG
    assert B.ptdp_layernorm_fwd(B.F32, 256, 256, 256, 256, 256, 256, None, 4, 32768, 1e-5, None) == B.E_UNSUPPORTED
    assert B.ptdp_bias_dropout_add_fwd(B.F32, 256, 256, 256, 256, 4, 16, 1.5, 0, 0, 0, 0, None) == B.E_INVALID_ARG
    assert B.ptdp_attn_fwd(B.BF16, 256, 256, 256, 16, 1, 1, 24, None) == B.E_UNSUPPORTED
    assert B.ptdp_attn_fwd(B.F32, None, 256, 256, 16, 1, 1, 64, None) == B.E_NULL_PTR
    assert B.ptdp_dropout_mask(None, 16, 0.1, 0, 0, 0, 0, None) == B.E_NULL_PTR
    assert B.ptdp_colsum_scratch_bytes(2048, 25600) >= 64 * 25600 * 4


def test_batch_time_matches_oracle_and_rejects_bad_input():
    import math
    from oracle import flops as F
    for bp, b, p, tf, tb in [(128, 4, 8, 0.013, 0.027), (512, 1, 8, 1.0, 2.0), (12, 3, 1, 0.5, 1.5), (8, 8, 64, 2.0, 0.0)]:
        assert B.ptdp_batch_time(bp, b, p, tf, tb) == F.batch_time(bp, b, p, tf, tb)
    for bad in [(0, 1, 1, 1.0, 1.0), (8, 3, 2, 1.0, 1.0), (8, 2, 0, 1.0, 1.0), (8, 2, 2, -1.0, 1.0),
                (8, 2, 2, float("nan"), 1.0), (8, 2, 2, 1.0, float("inf"))]:
        assert math.isnan(B.ptdp_batch_time(*bad))


def _plan(M, N, K, out_f32=0, accumulate=0, has_bias=0, ws=None):
    ws = B.ptdp_gemm_workspace_bytes() if ws is None else ws
    d, n = C.c_int(0), C.c_int(0)
    tiles, parts = (C.c_int * 2)(), (C.c_int * 2)()
    assert B.ptdp_gemm_plan(M, N, K, out_f32, accumulate, has_bias, ws, C.byref(d), C.byref(n), tiles, parts) == B.OK
    return d.value, [(tiles[j], parts[j]) for j in range(n.value)]


def test_gemm_remainder_split_covers_every_tile_and_k_step_once():
    """Tiles beyond the whole rounds go to at most two groups; every tile of a group is shared by `parts`
    workgroups with contiguous, disjoint k-ranges: replay that arithmetic on the host, also for shapes whose
    row-tile count does not divide the number of compute units, and count how often each k-step is taken."""
    ncu = B.ptdp_gemm_workspace_bytes() // (2 * 256 * 256 * 4)
    shapes = [(14336, 12800, 51200), (26624, 11264, 33792), (2048, 9600, 25600), (2048, 25600, 12800), (2048, 12800, 25600),
              (2048, 3200, 25600), (2048, 4608, 12288), (8192, 6144, 2048), (14336, 1792, 4096), (7 * 256, 37 * 256, 8192),
              (56 * 256, 5 * 256, 16384), (3 * 256, 87 * 256, 6400), (8, 264 * 256, 4096), (2048 + 8, 9600 + 8, 25600 + 8),
              (2048, 6400, 25600), (264, 4104, 4096), (2048, 10248, 4096), (256, 256, 64), (256, 512, 128)]
    n_split = 0
    for (M, N, K) in shapes:
        for out_f32, acc in ((0, 0), (1, 1)):
            dp_cols, groups = _plan(M, N, K, out_f32, acc)
            tiles_m, tiles_n, nk = -(-M // 256), -(-N // 256), -(-K // 64)
            assert dp_cols == N or dp_cols % 256 == 0
            rem = tiles_m * (tiles_n - dp_cols // 256) if dp_cols < N else 0
            if not groups:
                assert dp_cols == N
                continue
            n_split += 1
            assert 0 < rem < ncu and sum(t for t, _ in groups) == rem, (M, N, K, groups)
            assert any(p > 1 for _, p in groups)
            seen = np.zeros((rem, nk), dtype=np.int32)
            tile0 = 0
            for (t, p) in groups:
                assert t >= 1 and 1 <= p <= nk and t * p <= ncu, (M, N, K, groups)
                for tile in range(t):
                    for part in range(p):
                        seen[tile0 + tile, nk * part // p: nk * (part + 1) // p] += 1
                tile0 += t
            assert (seen == 1).all(), (M, N, K)
    assert n_split >= 8
    assert _plan(14336, 12800, 51200, ws=0) == (12800, [])            # no workspace: never split
    # the layer shapes of the 1T-shaped shard: 144 remainder tiles -> 128 tiles on 2 workgroups each + 16 tiles on 16
    assert _plan(2048, 12800, 25600) == (8192, [(128, 2), (16, 16)])
    assert _plan(2048, 9600, 25600) == (8192, [(48, 5)])
    assert _plan(2048, 3200, 25600) == (0, [(64, 4), (40, 6)])


def test_cfg_refuses_operands_beyond_the_gemm_offset_range():
    big = B.make_cfg(h=25600, a=160, t=1, s=2048, b=1, dtype=B.BF16)    # w_1 is 5.2 GB
    assert B.ptdp_cfg_validate(C.byref(big)) == B.E_UNSUPPORTED
    assert B.ptdp_layer_stash_bytes(C.byref(big)) == 0
    assert B.ptdp_cfg_validate(C.byref(B.make_cfg(h=25600, a=160, t=8, s=2048, b=1, dtype=B.BF16))) == B.OK
