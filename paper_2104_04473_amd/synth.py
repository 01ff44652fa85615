"""Seeded synthetic inputs with the shapes and value distributions of the paper's workloads.

Holds none of the method's arithmetic: only random draws and dtype casts.  Both the HIP path and
the tests' oracle calls are fed from here (the oracle receives the very same bits, upcast to fp64).

Recipe (paper section 5: GPT models, s = 2048; values are synthetic because throughput does not
depend on the data): weight matrices N(0, 0.02), biases small N(0, 0.02) by default (so that a
dropped bias is visible to parity tests; `zero_bias=True` gives the usual zero initialisation),
LayerNorm gain 1 (+ optional jitter) and bias 0 (+ jitter), activations and output gradients N(0, 1).
"""
import torch

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


def param_shapes(h, a, t):
    hp, fp = h // t, 4 * h // t
    return {"ln1_g": (h,), "ln1_b": (h,), "w_qkv": (h, 3 * hp), "b_qkv": (3 * hp,), "w_o": (hp, h), "b_o": (h,),
            "ln2_g": (h,), "ln2_b": (h,), "w_1": (h, fp), "b_1": (fp,), "w_2": (fp, h), "b_2": (h,)}


def torch_dtype(dtype_code):
    return torch.bfloat16 if dtype_code == 1 else torch.float32


def layer_params(h, a, t, dtype_code, seed, device="cpu", zero_bias=False, ln_jitter=0.1, std=0.02):
    """One layer's parameter dict in the storage dtype, drawn on `device` from a seeded generator."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    dt = torch_dtype(dtype_code)
    out = {}
    for name, shape in param_shapes(h, a, t).items():
        if name in ("ln1_g", "ln2_g"):
            v = 1.0 + ln_jitter * torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        elif name in ("ln1_b", "ln2_b"):
            v = ln_jitter * torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        elif name.startswith("b_"):
            v = torch.zeros(shape, device=device) if zero_bias else std * torch.randn(
                shape, generator=g, device=device, dtype=torch.float32)
        else:
            v = std * torch.randn(shape, generator=g, device=device, dtype=torch.float32)
        out[name] = v.to(dt).contiguous()
    return out


def activations(s, b, h, dtype_code, seed, device="cpu"):
    """N(0,1) tensor [s, b, h] in the storage dtype."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return torch.randn((s, b, h), generator=g, device=device, dtype=torch.float32).to(torch_dtype(dtype_code)).contiguous()


def zero_grads(h, a, t, device):
    return {n: torch.zeros(shp, device=device, dtype=torch.float32) for n, shp in param_shapes(h, a, t).items()}
