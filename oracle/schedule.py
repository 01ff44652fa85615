"""Order in which ONE pipeline device runs its forward and backward passes
(oracle side; test infrastructure).

Section 2.2 of the paper: the PipeDream-Flush (1F1B) schedule has a warm-up
phase of forward passes whose length depends on the device's position, a steady
state of one-forward-one-backward, and a cool-down of the remaining backward
passes; at most p microbatches are in flight.  The interleaved variant gives
each device v model chunks (device r holds stages r, r+p, r+2p, ...), needs
m % p == 0, and shrinks the bubble to (1/v)(p-1)/m of the ideal time.

The step order itself is only drawn in a figure of the paper; the reading used
here is written out below and is pinned by the p-device simulation in
``simulate`` (no deadlock, bubble equal to the closed form, bounded stash).

A step is (kind, chunk, microbatch), kind 0 = forward, 1 = backward.
"""


def forward_slot(k, p, v):
    """k-th forward pass of a device: microbatches advance in groups of p, each
    group visiting chunk 0, 1, ..., v-1 before the next group starts."""
    group, within = divmod(k, p * v)
    return (within // p, group * p + within % p)


def backward_slot(k, p, v):
    group, within = divmod(k, p * v)
    return (v - 1 - within // p, group * p + within % p)


def warmup_count(p, v, m, rank):
    total = m * v
    if v == 1:
        return min(total, p - rank - 1)
    return min(total, (v - 1) * p + 2 * (p - rank - 1))


def device_order(p, v, m, rank):
    """List of (kind, chunk, microbatch) for device ``rank`` of ``p``."""
    if p < 1 or v < 1 or m < 1 or not 0 <= rank < p:
        raise ValueError("bad schedule arguments")
    if v > 1 and m % p != 0:
        raise ValueError("interleaved schedule needs m % p == 0")
    total = m * v
    w = warmup_count(p, v, m, rank)
    steps = [(0,) + forward_slot(k, p, v) for k in range(w)]
    for k in range(total - w):
        steps.append((0,) + forward_slot(w + k, p, v))
        steps.append((1,) + backward_slot(k, p, v))
    steps += [(1,) + backward_slot(k, p, v) for k in range(total - w, total)]
    return steps


def peak_in_flight(steps):
    """Largest number of (chunk, microbatch) activations stashed at once."""
    live = peak = 0
    for kind, _, _ in steps:
        live += 1 if kind == 0 else -1
        peak = max(peak, live)
    return peak


def simulate(p, v, m, t_f=1.0, t_b=2.0):
    """Event simulation of all p devices with zero-latency links.

    Virtual stage of (device r, chunk c) is c*p + r.  The forward of a
    microbatch at virtual stage q needs its forward at stage q-1; the backward
    at stage q needs the backward at stage q+1 (and, at the last stage, its own
    forward).  Each device runs its list in order.  Returns (makespan, per-device
    busy time); raises RuntimeError on deadlock."""
    orders = [device_order(p, v, m, r) for r in range(p)]
    pos = [0] * p
    clock = [0.0] * p
    done = {}
    n_stage = p * v
    cf, cb = t_f / v, t_b / v
    remaining = sum(len(o) for o in orders)
    while remaining:
        progressed = False
        for r in range(p):
            while pos[r] < len(orders[r]):
                kind, c, mb = orders[r][pos[r]]
                q = c * p + r
                if kind == 0:
                    dep = None if q == 0 else (0, q - 1, mb)
                else:
                    dep = (0, q, mb) if q == n_stage - 1 else (1, q + 1, mb)
                if dep is not None and dep not in done:
                    break
                start = max(clock[r], done[dep] if dep is not None else 0.0)
                clock[r] = start + (cf if kind == 0 else cb)
                done[(kind, q, mb)] = clock[r]
                pos[r] += 1
                remaining -= 1
                progressed = True
        if not progressed:
            raise RuntimeError("schedule deadlocks")
    return max(clock), [m * (t_f + t_b)] * p
