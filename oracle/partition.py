"""Backbone partitioning by dynamic programming, plain Python (test infrastructure only).

Sec. 4.1 (single backbone): the FIFO-1F1B pipeline time is bounded by
T_max = T_0 (M + 2S - 2) + T_0^{S-C} (Eq. 1), and a dynamic programme over
W(L, S, r, D) = T_0 and Y(L, S, r, D) = T_0^{S-C} of "the first L layers in S
stages on devices 1..D with the last stage replicated on the last r devices"
(Eq. 2-9) picks the partition and the replication of every stage.  Sec. 4.3 adds
self-conditioning: one more forward per stage (Eq. 17), a feedback transfer T_F,
and the objective becomes the expectation over the activation probability p
(Eq. 18).  The steps below are taken in the paper's order and notation; the
programme is a heuristic for its own objective (a state keeps one (W, Y) pair, the
objective is a weighted sum of two maxima), so `brute_force` -- every partition
and every replication vector scored by the definitions -- is its pin: equal where
the objective decomposes, never better than the programme's answer otherwise.

Readings where the text is silent (the same in the product, listed in the design
notes): a stage replicated r times runs at local batch B / r and r must divide B,
with the profile holding that batch size, otherwise the state is infeasible; the
first stage has no incoming transfer, so its communication term is zero; the gap
T_S - T_C is clamped at zero (a synchronisation that ends inside the compensation
window adds nothing to the bound); ties are broken towards the earlier candidate in
the loop order (fewer stages, smaller r, smaller l, smaller r').

Units: times in ms, sizes in bytes, bandwidths in GB/s (1e9 bytes per second).
"""
from __future__ import annotations

import itertools
import math
from dataclasses import dataclass, field


@dataclass
class Profile:
    """Cost profile of a backbone (Table "Notations"): per local batch size b,
    fwd_ms[b][l] = P^f_l(b), bwd_ms[b][l] = P^b_l(b), cf_bytes[b][l] = C^f_{l,l+1}(b),
    cb_bytes[b][l] = C^b_{l+1,l}(b), out_bytes[b] = O_L(b); grad_bytes[l] = G_l."""
    n_layers: int
    fwd_ms: dict
    bwd_ms: dict
    cf_bytes: dict
    cb_bytes: dict
    grad_bytes: list
    out_bytes: dict


@dataclass
class Options:
    micro_batch: int                 # B
    n_micro_batches: int             # M
    n_devices: int                   # D, the pipeline-parallel group
    p2p_gbps: float = 50.0           # R_p2p
    p2p_latency_ms: float = 0.01     # L_p2p
    ar_gbps: float = 100.0           # R_ar
    ar_latency_ms: float = 0.05      # L_ar
    self_cond_prob: float = 0.0      # p of Sec. 4.3 (0: Eq. 1 alone)
    max_stages: int = 0              # 0: up to min(L, D)
    uniform_replication: bool = False  # every stage on the same number of devices (the paper's evaluation setting)
    exact_stages: int = 0            # S fixed (one point of the hyper-parameter search of Sec. 3); 0: best S up to max_stages


@dataclass
class Plan:
    n_stages: int = 0
    first_layer: list = field(default_factory=list)
    n_layers: list = field(default_factory=list)
    replicas: list = field(default_factory=list)
    t0_ms: float = math.inf          # W
    t0_sc_ms: float = math.inf       # W under self-conditioning (Eq. 17)
    gap_ms: float = math.inf         # Y
    tf_ms: float = 0.0               # T_F
    t_max_ms: float = math.inf       # Eq. 1 / Eq. 18 in expectation


def _ms(nbytes, gbps):
    return nbytes / (gbps * 1e9) * 1e3


def stage_terms(prof: Profile, o: Options, lo: int, hi: int, r: int):
    """(T_0(s), T_0,SC(s), T_0^{S-C}(s)) of the stage holding layers lo..hi-1 (0-based) on r
    devices (Eq. 3-6 and Eq. 17), or None when B / r is not a profiled batch size."""
    if o.micro_batch % r:
        return None
    b = o.micro_batch // r
    if b not in prof.fwd_ms:
        return None
    pf = sum(prof.fwd_ms[b][lo:hi])
    pb = sum(prof.bwd_ms[b][lo:hi])
    if lo == 0:
        comm = comm_sc = 0.0
    else:
        cf, cb = prof.cf_bytes[b][lo - 1], prof.cb_bytes[b][lo - 1]
        comm = _ms(cf + cb, o.p2p_gbps) + 2 * o.p2p_latency_ms
        comm_sc = _ms(2 * cf + cb, o.p2p_gbps) + 3 * o.p2p_latency_ms
    t0 = max(pf + pb, comm)                                            # Eq. 3
    t0_sc = max(2 * pf + pb, comm_sc)                                  # Eq. 17
    ts = _ms(sum(prof.grad_bytes[lo:hi]), o.ar_gbps) + o.ar_latency_ms  # Eq. 4
    tc = pb                                                            # Eq. 5
    return t0, t0_sc, max(ts - tc, 0.0)                                # Eq. 6


def objective(o: Options, n_stages: int, w: float, w_sc: float, y: float) -> float:
    """Eq. 1 and Eq. 18 combined in expectation over p, without the constant p T_F."""
    p = o.self_cond_prob
    return (o.n_micro_batches + 2 * n_stages - 2) * (p * w_sc + (1.0 - p) * w) + y


def feedback_ms(prof: Profile, o: Options) -> float:
    """T_F = O_L(B) / R_p2p + L_p2p (Sec. 4.3); zero without self-conditioning."""
    if o.self_cond_prob <= 0.0:
        return 0.0
    return _ms(prof.out_bytes[o.micro_batch], o.p2p_gbps) + o.p2p_latency_ms


def solve(prof: Profile, o: Options) -> Plan:
    """The dynamic programme of Eq. 2-9, run once per total stage count S."""
    L, D = prof.n_layers, o.n_devices
    s_max = min(L, D) if o.max_stages <= 0 else min(L, D, o.max_stages)
    tf = feedback_ms(prof, o)
    best = Plan()
    for S in ([o.exact_stages] if o.exact_stages > 0 else range(1, s_max + 1)):
        if S > s_max:
            break
        # table[(l, s, r, d)] = (W, W_sc, Y, parent key or None)
        table = {}
        for d in range(1, D + 1):
            for l in range(1, L + 1):
                t = stage_terms(prof, o, 0, l, d)
                if t is not None:
                    table[(l, 1, d, d)] = (t[0], t[1], t[2], None)
        for s in range(2, S + 1):
            for d in range(s, D + 1):
                for r in range(1, d - (s - 1) + 1):
                    for l_end in range(s, L + 1):
                        pick = None
                        for l in range(s - 1, l_end):                # Eq. 9: the cut before the last stage
                            t = stage_terms(prof, o, l, l_end, r)
                            if t is None:
                                continue
                            for rp in range(1, d - r + 1):           # Eq. 9: replication of the stage before
                                if o.uniform_replication and rp != r:
                                    continue
                                sub = table.get((l, s - 1, rp, d - r))
                                if sub is None:
                                    continue
                                w, w_sc, y = max(sub[0], t[0]), max(sub[1], t[1]), max(sub[2], t[2])   # Eq. 7, 8
                                val = objective(o, S, w, w_sc, y)
                                if pick is None or val < pick[0]:
                                    pick = (val, w, w_sc, y, (l, s - 1, rp, d - r))
                        if pick is not None:
                            table[(l_end, s, r, d)] = pick[1:]
        for r in range(1, D + 1):                                    # Eq. 2
            st = table.get((L, S, r, D))
            if st is None:
                continue
            val = objective(o, S, st[0], st[1], st[2]) + o.self_cond_prob * tf
            if val < best.t_max_ms:
                plan = Plan(n_stages=S, t0_ms=st[0], t0_sc_ms=st[1], gap_ms=st[2], tf_ms=tf, t_max_ms=val)
                key, hi, stages = (L, S, r, D), L, []
                while key is not None:
                    parent = table[key][3]
                    lo = parent[0] if parent is not None else 0
                    stages.append((lo, hi - lo, key[2]))
                    hi, key = lo, parent
                stages.reverse()
                plan.first_layer = [a for a, _, _ in stages]
                plan.n_layers = [n for _, n, _ in stages]
                plan.replicas = [c for _, _, c in stages]
                best = plan
    return best


def score(prof: Profile, o: Options, cuts, replicas):
    """(W, W_sc, Y, T_max) of an explicit partition straight from the definitions (Eq. 1, 3-6, 17,
    18): cuts = first layer of every stage, replicas = devices per stage."""
    S = len(cuts)
    bounds = list(cuts) + [prof.n_layers]
    w = w_sc = y = 0.0
    for i in range(S):
        t = stage_terms(prof, o, bounds[i], bounds[i + 1], replicas[i])
        if t is None:
            return None
        w, w_sc, y = max(w, t[0]), max(w_sc, t[1]), max(y, t[2])
    return w, w_sc, y, objective(o, S, w, w_sc, y) + o.self_cond_prob * feedback_ms(prof, o)


def brute_force(prof: Profile, o: Options):
    """Minimum of `score` over every partition into 1..S_max contiguous stages and every way of
    dealing the D devices to them (small L and D only)."""
    L, D = prof.n_layers, o.n_devices
    s_max = min(L, D) if o.max_stages <= 0 else min(L, D, o.max_stages)
    best = (math.inf, None, None)
    for S in ([o.exact_stages] if o.exact_stages > 0 else range(1, s_max + 1)):
        if S > s_max:
            break
        for inner in itertools.combinations(range(1, L), S - 1):
            cuts = (0,) + inner
            for reps in itertools.product(range(1, D + 1), repeat=S):
                if sum(reps) != D or (o.uniform_replication and len(set(reps)) != 1):
                    continue
                sc = score(prof, o, cuts, reps)
                if sc is not None and sc[3] < best[0]:
                    best = (sc[3], cuts, reps)
    return best
