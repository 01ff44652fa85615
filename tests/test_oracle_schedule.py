"""Pins for oracle/schedule.py: p-device simulation against the paper's bubble
formulas and stash bound (section 2.2).  CPU only."""
import pytest

from oracle import schedule as S

CASES = [(4, 1, 8), (4, 2, 8), (4, 2, 4), (4, 2, 16), (8, 2, 16), (8, 4, 8), (2, 2, 4),
         (4, 3, 12), (3, 2, 6), (4, 2, 12), (1, 1, 3), (1, 2, 3), (2, 1, 1), (5, 1, 3), (6, 1, 20)]


@pytest.mark.parametrize("p,v,m", CASES)
def test_bubble_matches_closed_form(p, v, m):
    for tf, tb in ((1.0, 2.0), (1.0, 1.0), (3.0, 4.0)):
        makespan, _ = S.simulate(p, v, m, tf, tb)
        bubble = makespan - m * (tf + tb)
        assert bubble == pytest.approx((p - 1) * (tf + tb) / v, abs=1e-9)
        # as a fraction of the ideal time: (1/v)(p-1)/m
        assert bubble / (m * (tf + tb)) == pytest.approx((p - 1) / (v * m), abs=1e-9)


@pytest.mark.parametrize("p,v,m", CASES)
def test_every_pass_once_and_backward_after_forward(p, v, m):
    for r in range(p):
        steps = S.device_order(p, v, m, r)
        assert len(steps) == 2 * m * v
        seen_f, seen_b = set(), set()
        for kind, c, mb in steps:
            assert 0 <= c < v and 0 <= mb < m
            if kind == 0:
                assert (c, mb) not in seen_f
                seen_f.add((c, mb))
            else:
                assert (c, mb) in seen_f and (c, mb) not in seen_b
                seen_b.add((c, mb))
        assert len(seen_f) == len(seen_b) == m * v


def test_non_interleaved_stash_bound():
    for p, m in ((4, 8), (4, 2), (8, 32), (3, 3)):
        for r in range(p):
            peak = S.peak_in_flight(S.device_order(p, 1, m, r))
            assert peak == min(m, p - r) <= p


def test_figure_example_rank0():
    # 4 devices, 2 chunks, 8 microbatches: device 1 starts with 4 forwards of its
    # first chunk, then 4 of its second chunk (the paper's interleaved figure).
    steps = S.device_order(4, 2, 8, 0)
    assert steps[:8] == [(0, 0, i) for i in range(4)] + [(0, 1, i) for i in range(4)]
    assert S.peak_in_flight(steps) == 11
    first_b = next(i for i, st in enumerate(steps) if st[0] == 1)
    assert steps[first_b] == (1, 1, 0)        # last chunk's backward comes first


def test_argument_checks():
    with pytest.raises(ValueError):
        S.device_order(4, 2, 6, 0)            # m % p != 0 with interleaving
    with pytest.raises(ValueError):
        S.device_order(4, 1, 8, 4)
    S.device_order(4, 1, 6, 0)                # fine without interleaving


def test_simulator_detects_a_wrong_order():
    # a planted mistake: too few warm-up forwards on device 0 must deadlock or
    # lengthen the bubble
    real = S.warmup_count
    try:
        S.warmup_count = lambda p, v, m, rank: max(0, real(p, v, m, rank) - 2) if rank == 0 else real(p, v, m, rank)
        try:
            makespan, _ = S.simulate(4, 2, 8)
            assert makespan - 24.0 > 4.5 + 1e-9
        except RuntimeError:
            pass
    finally:
        S.warmup_count = real
