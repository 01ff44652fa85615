"""Activation recomputation (section 3.5), oracle side; test infrastructure only.

With c checkpoints over l layers only the c segment inputs stay alive per
in-flight microbatch; the backward pass reruns a segment's forward from its
checkpoint just before that segment's backward.  The paper's memory model is

    kept(c) = c * A_input + (l / c) * A_intermediate,

minimised at c = sqrt(l * A_intermediate / A_input).  The gradients are by
construction those of the plain forward + backward: the dropout masks are a
function of (seed, layer, site, microbatch, element) and so repeat exactly.

Pins (tests/test_oracle_recompute.py): the closed-form optimum against a brute
force scan and against the stationarity condition; the ledger of live arrays
of `chunk_backward_recompute` against kept(c); its gradients against
`gpt_layer.chunk_backward` (equal bit for bit in fp64, same operation order).
"""
import math

from . import gpt_layer as L


def kept_bytes(c, l, a_input, a_intermediate):
    """Activation bytes alive per in-flight microbatch with c checkpoints over l layers."""
    return c * a_input + (l / c) * a_intermediate


def optimal_checkpoints(l, a_input, a_intermediate):
    """The real-valued c minimising kept_bytes."""
    return math.sqrt(l * a_intermediate / a_input)


def segments(n_layers, seg_layers):
    """[l0, l1) ranges: consecutive groups of seg_layers layers, the last possibly shorter."""
    return [(l0, min(l0 + seg_layers, n_layers)) for l0 in range(0, n_layers, seg_layers)]


def chunk_forward_checkpoints(x, params_list, cfg, seg_layers, first_layer=0, microbatch=0):
    """Forward that keeps only every segment's input.  Returns (y, checkpoints)."""
    ckpts = []
    for l0, l1 in segments(len(params_list), seg_layers):
        ckpts.append(x)
        x, _ = L.chunk_forward(x, params_list[l0:l1], cfg, first_layer + l0, microbatch)
    return x, ckpts


def chunk_backward_recompute(dy, params_list, cfg, ckpts, seg_layers, first_layer=0, microbatch=0, ledger=None):
    """Backward from checkpoints: last segment first, each rerun and then differentiated.

    ledger (optional list) receives, per segment, the pair (checkpoints alive,
    layer caches alive) at the moment that segment's backward runs."""
    grads = [None] * len(params_list)
    segs = segments(len(params_list), seg_layers)
    for sg in reversed(range(len(segs))):
        l0, l1 = segs[sg]
        _, caches = L.chunk_forward(ckpts[sg], params_list[l0:l1], cfg, first_layer + l0, microbatch)
        if ledger is not None:
            ledger.append((sg + 1, len(caches)))
        dy, g = L.chunk_backward(dy, params_list[l0:l1], cfg, caches)
        grads[l0:l1] = g
    return dy, grads
