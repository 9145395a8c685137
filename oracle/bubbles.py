"""Pipeline bubbles and their filling with the frozen part, plain Python (test infrastructure only).

Sec. 5: the idle time of the FIFO-1F1B pipeline is cut along the time line into bubbles
(start, end, idle devices); the bubbles are filled in chronological order with layers of the ready
non-trainable components, run data-parallel on the idle devices: Algorithm 2 (FFC) lists every way of
packing whole-batch layers of the ready components into the bubble, Algorithm 1 adds to each of them at
most one partial-batch layer (component, layer, samples) with the largest "regular" sample count that
still fits, and keeps the candidate that runs longest.  A layer started on part of the batch is the first
ready layer of its component afterwards and counts as a whole-batch layer on the remaining samples.

The paper obtains the bubbles "by simulating the pipeline schedule with the profiled results" without
printing the simulator; `simulate_1f1b` is this build's reading of it (listed in the design notes):
stage s of S runs min(S - 1 - s, M) warm-up forwards, then alternates one forward and one backward, then
drains its backwards, micro-batches in order; an operation starts when its stage is free and its input
has arrived (previous stage's forward, or next stage's backward, plus the transfer time).  Other
readings: a layer on n samples over d idle devices runs at local batch ceil(n / d); a local batch size
between two profiled ones is interpolated linearly (below the smallest: that one's time); valid sample
counts are d times the regular local sizes 4, 8, 12, 16, 24, 32, 48, 64, 96 and smaller than what is left of
the layer; readiness is judged at the start of a bubble; what does not fit any bubble runs after the
pipeline on all devices.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

REGULAR_LOCAL_BATCHES = (4, 8, 12, 16, 24, 32, 48, 64, 96)


# ------------------------------------------------------------------ schedule simulation
def order_1f1b(s: int, S: int, M: int):
    """Operation order of stage s: ('F' | 'B', micro-batch)."""
    warm = min(S - 1 - s, M)
    ops = [("F", m) for m in range(warm)]
    for i in range(M - warm):
        ops.append(("F", warm + i))
        ops.append(("B", i))
    ops += [("B", m) for m in range(M - warm, M)]
    return ops


def simulate_1f1b(fwd_ms, bwd_ms, M, comm_fwd_ms=None, comm_bwd_ms=None, tail_ms=None):
    """Per-stage busy intervals [(start, end, kind, micro-batch)] and the iteration time.
    comm_fwd_ms[s] / comm_bwd_ms[s]: transfer between stages s and s + 1; tail_ms[s]: busy time
    appended after the stage's last backward (gradient synchronisation that is not overlapped)."""
    S = len(fwd_ms)
    cf = comm_fwd_ms or [0.0] * (S - 1)
    cb = comm_bwd_ms or [0.0] * (S - 1)
    orders = [order_1f1b(s, S, M) for s in range(S)]
    pos = [0] * S
    free = [0.0] * S
    done = {}
    busy = [[] for _ in range(S)]
    progress = True
    while progress:
        progress = False
        for s in range(S):
            while pos[s] < len(orders[s]):
                kind, m = orders[s][pos[s]]
                if kind == "F":
                    ready = 0.0 if s == 0 else (done[("F", s - 1, m)] + cf[s - 1] if ("F", s - 1, m) in done else None)
                else:
                    if s == S - 1:
                        ready = done.get(("F", s, m))
                    else:
                        ready = done[("B", s + 1, m)] + cb[s] if ("B", s + 1, m) in done else None
                if ready is None:
                    break
                start = max(free[s], ready)
                end = start + (fwd_ms[s] if kind == "F" else bwd_ms[s])
                busy[s].append((start, end, kind, m))
                done[(kind, s, m)] = end
                free[s] = end
                pos[s] += 1
                progress = True
    assert all(pos[s] == len(orders[s]) for s in range(S)), "schedule deadlocked"
    if tail_ms:
        for s in range(S):
            if tail_ms[s] > 0:
                busy[s].append((free[s], free[s] + tail_ms[s], "S", -1))
                free[s] += tail_ms[s]
    return busy, max(free)


@dataclass
class Bubble:
    start: float
    end: float
    stages: tuple          # idle stages
    devices: int           # sum of their replicas


def find_bubbles(busy, t_end, replicas, min_ms=0.0):
    """Maximal time spans over which the set of idle stages is constant and non-empty, in
    chronological order; spans shorter than min_ms are dropped (Sec. 5 uses 10 ms)."""
    S = len(busy)
    cuts = {0.0, t_end}
    for s in range(S):
        for a, b, _, _ in busy[s]:
            cuts.add(a); cuts.add(b)
    cuts = sorted(cuts)
    out = []
    for a, b in zip(cuts, cuts[1:]):
        if b <= a:
            continue
        mid = 0.5 * (a + b)
        idle = tuple(s for s in range(S) if not any(x <= mid < y for x, y, _, _ in busy[s]))
        if not idle:
            continue
        if out and out[-1].stages == idle and out[-1].end == a:
            out[-1].end = b
        else:
            out.append(Bubble(a, b, idle, sum(replicas[s] for s in idle)))
    return [x for x in out if x.end - x.start >= min_ms]


# ------------------------------------------------------------------ bubble filling
@dataclass
class Component:
    n_layers: int
    fwd_ms: dict                       # local batch -> [time of each layer]
    deps: tuple = ()                   # components that must be complete before this one starts


def layer_time(c: Component, layer: int, local_batch: int) -> float:
    """P^f_{i,l}(b): profiled value, or the linear interpolation between the neighbouring profiled sizes."""
    sizes = sorted(c.fwd_ms)
    if local_batch in c.fwd_ms:
        return c.fwd_ms[local_batch][layer]
    if local_batch <= sizes[0]:
        return c.fwd_ms[sizes[0]][layer]
    if local_batch >= sizes[-1]:
        return c.fwd_ms[sizes[-1]][layer] * local_batch / sizes[-1]
    hi = next(x for x in sizes if x > local_batch)
    lo = sizes[sizes.index(hi) - 1]
    w = (local_batch - lo) / (hi - lo)
    return c.fwd_ms[lo][layer] * (1 - w) + c.fwd_ms[hi][layer] * w


def valid_num_samples(remaining: int, d: int):
    """getValidNumSamples: sample counts whose local size b / d is regular, smaller than what is left."""
    return [r * d for r in REGULAR_LOCAL_BATCHES if r * d < remaining]


@dataclass
class FillState:
    batch: int                                   # training batch size (bold B)
    u: list                                      # first unfinished layer of every component
    rem: list                                    # samples still to process of layer u[i]


def _full_time(comps, st: FillState, i: int, j: int, d: int) -> float:
    """Time of the j-th not yet finished layer of component i as a whole-batch layer on d devices."""
    n = st.rem[i] if j == 0 else st.batch
    return layer_time(comps[i], st.u[i] + j, math.ceil(n / d))


def ffc(comps, st: FillState, ready, t_b: float, d: int, pos: int):
    """Algorithm 2: every list (k_i for the ready components from position pos on) of whole-batch layer
    counts that fits into t_b, the component at `pos` varied from its maximum down to zero."""
    i = ready[pos]
    t, k0 = 0.0, 0
    while st.u[i] + k0 < comps[i].n_layers and t + _full_time(comps, st, i, k0, d) <= t_b:
        t += _full_time(comps, st, i, k0, d)
        k0 += 1
    if pos == len(ready) - 1:
        return [[k0]]
    out = []
    for k in range(k0, -1, -1):
        left = t_b - sum(_full_time(comps, st, i, h, d) for h in range(k))
        out += [[k] + rest for rest in ffc(comps, st, ready, left, d, pos + 1)]
    return out


def fill_one(comps, st: FillState, ready, t_b: float, d: int):
    """Algorithm 1: (k, partial, time) with partial = (component, layer, samples) or None."""
    best = None
    for k in ffc(comps, st, ready, t_b, d, 0):
        t_full = sum(_full_time(comps, st, i, j, d) for i, ki in zip(ready, k) for j in range(ki))
        cands = [(k, None, t_full)]
        for h, kh in zip(ready, k):
            layer = st.u[h] + kh
            if layer >= comps[h].n_layers:
                continue
            left = st.rem[h] if kh == 0 else st.batch
            fits = [b for b in valid_num_samples(left, d) if t_full + layer_time(comps[h], layer, b // d) <= t_b]
            if fits:
                b = max(fits)
                cands.append((k, (h, layer, b), t_full + layer_time(comps[h], layer, b // d)))
        for c in cands:
            if best is None or c[2] > best[2]:
                best = c
    return best


@dataclass
class Fill:
    bubble: int
    full: list            # (component, first layer, number of layers, samples of the first layer)
    partial: object       # (component, layer, samples) or None
    time_ms: float


@dataclass
class FillResult:
    fills: list = field(default_factory=list)
    filled_device_ms: float = 0.0
    bubble_device_ms: float = 0.0
    leftover_ms: float = 0.0          # frozen work that fits no bubble, run after the pipeline on all devices


def fill_all(bubbles, comps, batch: int, n_devices: int) -> FillResult:
    """Fills the bubbles in chronological order and accounts for what is left."""
    st = FillState(batch, [0] * len(comps), [batch] * len(comps))
    res = FillResult()
    for bi, bub in enumerate(bubbles):
        res.bubble_device_ms += (bub.end - bub.start) * bub.devices
        ready = [i for i, c in enumerate(comps) if st.u[i] < c.n_layers and all(st.u[j] >= comps[j].n_layers for j in c.deps)]
        if not ready:
            continue
        k, partial, t = fill_one(comps, st, ready, bub.end - bub.start, bub.devices)
        if t <= 0.0:
            continue
        full = []
        for i, ki in zip(ready, k):
            if ki:
                full.append((i, st.u[i], ki, st.rem[i]))
                st.u[i] += ki
                st.rem[i] = batch
        if partial:
            h, layer, b = partial
            assert st.u[h] == layer
            st.rem[h] -= b
        res.fills.append(Fill(bi, full, partial, t))
        res.filled_device_ms += t * bub.devices
    for i, c in enumerate(comps):
        for j in range(c.n_layers - st.u[i]):
            res.leftover_ms += _full_time(comps, st, i, j, n_devices)
    return res
