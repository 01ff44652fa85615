"""Pins for oracle/flops.py against the paper's printed arithmetic (CPU only)."""
import os

from oracle import flops as F

HERE = os.path.dirname(__file__)


def printed():
    out = {}
    for line in open(os.path.join(HERE, "golden", "paper_printed_numbers.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def test_layer_flops_closed_form():
    for (B, s, h) in [(1, 2048, 12288), (4, 2048, 2048), (2, 128, 256), (3, 7, 10)]:
        assert F.layer_forward_flops(B, s, h) == 24 * B * s * h * h + 4 * B * s * s * h


def test_iteration_flops_is_eq3():
    B, s, l, h, V = 1536, 2048, 96, 12288, 51200
    eq3 = 96 * B * s * l * h * h * (1 + s / (6 * h) + V / (16 * l * h))
    assert abs(F.iteration_flops(B, s, l, h, V) - eq3) / eq3 < 1e-12


def test_parameters_is_eq2_and_gives_gpt3():
    g = printed()
    l, h, V, s = int(g["gpt3_layers"]), int(g["gpt3_hidden"]), int(g["vocab"]), int(g["seq"])
    eq2 = 12 * l * h * h * (1 + 13 / (12 * h) + (V + s) / (12 * l * h))
    assert abs(F.parameters(l, h, V, s) - eq2) / eq2 < 1e-12
    assert round(F.parameters(l, h, V, s) / 1e9) == g["gpt3_params_billion"]


def test_training_time_estimates():
    g = printed()
    P175 = F.parameters(96, 12288, 51200, 2048)
    d = F.training_days(g["gpt3_tokens_billion"] * 1e9, P175, g["gpt3_gpus"], g["gpt3_tflops_per_gpu"] * 1e12)
    assert round(d) == g["gpt3_days"]
    # the 1T model: h = 25600, 128 layers reproduces ~1e12 parameters
    P1T = F.parameters(128, 25600, 51200, 2048)
    assert abs(P1T / 1e12 - 1.0) < 0.02
    d = F.training_days(g["t1_tokens_billion"] * 1e9, P1T, g["t1_gpus"], g["t1_tflops_per_gpu"] * 1e12)
    assert round(d) == g["t1_days"]
    assert round(100 * g["t1_tflops_per_gpu"] / g["a100_peak_tflops"]) == g["t1_percent_of_peak"]
    assert abs(g["t1_gpus"] * g["t1_tflops_per_gpu"] / 1000 - g["t1_aggregate_pflops"]) < 2


def test_shard_flops():
    assert F.shard_layer_flops(1, 2048, 25600, 8) == 3 * 4080218931200
    assert F.shard_layer_flops(1, 2048, 12288, 8) == 3 * 953482739712
    assert F.shard_layer_flops(2, 128, 256, 1) == 1308622848
    assert F.shard_layer_flops(1, 2048, 12288, 8, recompute=True) == 4 * 953482739712


def test_eq1_is_the_makespan_of_the_simulated_pipeline():
    """Eq. (1) against the p-device simulation of the non-interleaved schedule (an independent
    computation: event-driven dependencies, no closed form)."""
    from oracle import schedule as S
    for p, m, tf, tb in [(4, 8, 1.0, 2.0), (8, 16, 0.7, 1.9), (1, 5, 1.0, 1.0), (3, 3, 2.0, 3.5)]:
        makespan, _ = S.simulate(p, 1, m, t_f=tf, t_b=tb)
        assert abs(makespan - F.batch_time(m * 4, 4, p, tf, tb)) < 1e-9


def test_eq1_limits():
    # cost proportional to b (no fixed overhead): the smallest microbatch wins (fewest bubble samples)
    times = {b: F.batch_time(64, b, 8, 1.0 * b, 2.0 * b) for b in (1, 2, 4, 8)}
    assert min(times, key=times.get) == 1
    assert times[1] == (64 + 7) * 3.0
    # cost independent of b (pure overhead): the largest microbatch wins
    times = {b: F.batch_time(64, b, 8, 1.0, 2.0) for b in (1, 2, 4, 8)}
    assert min(times, key=times.get) == 8
    # p = 1: no bubble, time = (b'/b) (t_f + t_b)
    assert F.batch_time(12, 3, 1, 0.5, 1.5) == 4 * 2.0
