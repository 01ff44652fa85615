"""Closed forms of the paper (oracle side; test infrastructure).

* appendix: a transformer layer's forward pass costs 24 B s h^2 + 4 B s^2 h
  FLOPs (GEMMs only, full s x s attention matrix, multiply and add counted
  separately); the backward pass costs twice that; activation recomputation
  adds one more forward;
* eq. (2): parameter count of an l-layer GPT model;
* eq. (3): FLOPs per iteration including recomputation and the logit layer;
* section 5.1: end-to-end training time ~ 8 T P / (n X).
"""


def matmul_flops(m, k, n):
    return 2 * m * k * n


def layer_forward_flops(B, s, h):
    """Sum of the six matrix products of one layer's forward pass, unsharded."""
    qkv = matmul_flops(B * s, h, 3 * h)            # 6 B s h^2
    scores = B * matmul_flops(s, h, s)             # per sample, all heads: 2 B s^2 h
    over_values = B * matmul_flops(s, s, h)        # 2 B s^2 h
    proj = matmul_flops(B * s, h, h)               # 2 B s h^2
    mlp = matmul_flops(B * s, h, 4 * h) + matmul_flops(B * s, 4 * h, h)   # 16 B s h^2
    return qkv + scores + over_values + proj + mlp


def shard_layer_flops(b, s, h, t, recompute=False):
    """Model FLOPs of forward + backward of one layer for one microbatch on one
    of t tensor-parallel shards (x3, or x4 when a recompute forward runs)."""
    fwd = layer_forward_flops(b, s, h)
    assert fwd % t == 0
    return (4 if recompute else 3) * fwd // t


def parameters(l, h, V, s):
    """Eq. (2), written as the sum it abbreviates."""
    per_layer = 12 * h * h + 13 * h
    return l * per_layer + (V + s) * h


def iteration_flops(B, s, l, h, V):
    """Eq. (3): 4 x layer forward per layer + 6 B s h V for the logit layer."""
    return 4 * l * layer_forward_flops(B, s, h) + 6 * B * s * h * V


def training_days(T_tokens, P, n, X):
    return 8.0 * T_tokens * P / (n * X) / 86400.0


def batch_time(b_prime, b, p, t_f, t_b):
    """Eq. (1), section 3.4: b_prime/b microbatches through p stages cost
    (b_prime/b + p - 1) slots of one forward plus one backward each."""
    assert b_prime % b == 0
    return (b_prime // b + p - 1) * (t_f + t_b)
