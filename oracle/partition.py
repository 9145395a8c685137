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

Sec. 4.2 (two backbones of a cascaded model, pipelined in opposite directions over the same devices):
`solve_bidirectional`, Eq. 10-16.  Readings: the text names the sub-problem's layers "the last L_d and the
first L_u"; with the down pipeline entering the device chain at rank 1 (its definition of "down"), the
devices 1..d hold the FIRST layers of the down backbone and the LAST layers of the up backbone, which is
what the state below holds (the two labelings are mirror images of one another).  M_CDM ("the number of
paired forward and backward stages between the down and up pipelines") is given no formula: it is an input
(n_micro_batches).  Both backbones are cut into the same number of stages; a chain position holds one
stage of each, replicated on the same r devices; self-conditioning is not combined with it.

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


# ------------------------------------------------------------------ two backbones, bidirectional pipelining (Sec. 4.2)
@dataclass
class BidirPlan:
    n_stages: int = 0
    first_layer_down: list = field(default_factory=list)   # per position along the device chain, low rank first
    n_layers_down: list = field(default_factory=list)
    first_layer_up: list = field(default_factory=list)     # in the up backbone's own layer numbering
    n_layers_up: list = field(default_factory=list)
    replicas: list = field(default_factory=list)
    t0_ms: float = math.inf          # W = T_0,CDM (Eq. 10)
    gap_ms: float = math.inf         # Y = T_0,CDM^{S-C} (Eq. 11)
    t_max_ms: float = math.inf       # Eq. 12


def bidir_stage_terms(prof: Profile, o: Options, lo: int, hi: int, r: int, incoming):
    """(T_0(s), T_0^{S-C}(s)) of one backbone's stage [lo, hi) on r devices as in Eq. 3-6, with the
    communication time doubled (Sec. 4.2: the two directions compete for the links).  `incoming` is the
    index of the layer boundary the stage receives its input over, or None for the backbone's first stage."""
    if o.micro_batch % r:
        return None
    b = o.micro_batch // r
    if b not in prof.fwd_ms:
        return None
    pf, pb = sum(prof.fwd_ms[b][lo:hi]), sum(prof.bwd_ms[b][lo:hi])
    comm = 0.0
    if incoming is not None:
        comm = 2.0 * (_ms(prof.cf_bytes[b][incoming] + prof.cb_bytes[b][incoming], o.p2p_gbps) + 2 * o.p2p_latency_ms)
    ts = _ms(sum(prof.grad_bytes[lo:hi]), o.ar_gbps) + o.ar_latency_ms
    return max(pf + pb, comm), max(ts - pb, 0.0)


def _bidir_pair(down: Profile, up: Profile, o: Options, ld0: int, ld1: int, lu0: int, lu1: int, r: int):
    """Terms of the device group that holds down layers [ld0, ld1) and, counted from the END of the up
    backbone, its layers [lu0, lu1) (the up pipeline enters the chain at the other end, so the low-rank
    devices hold its last layers): (max T_0, max T_0^{S-C}) over the two stages."""
    td = bidir_stage_terms(down, o, ld0, ld1, r, ld0 - 1 if ld0 > 0 else None)
    Lu = up.n_layers
    a, b = Lu - lu1, Lu - lu0                       # the same stage in the up backbone's own numbering
    tu = bidir_stage_terms(up, o, a, b, r, a - 1 if a > 0 else None)
    if td is None or tu is None:
        return None
    return max(td[0], tu[0]), max(td[1], tu[1])


def solve_bidirectional(down: Profile, up: Profile, o: Options) -> BidirPlan:
    """Eq. 13-16: state (l_d, l_u, s, r, d) = the first l_d layers of the down backbone and the last l_u
    layers of the up backbone in s stages on devices 1..d, the stage pair at the high-rank end on r devices.
    o.n_micro_batches is M_CDM.  One run per total stage count S; a state keeps the (W, Y) of the candidate
    with the least (M_CDM + 2S - 2) W + Y."""
    Ld, Lu, D = down.n_layers, up.n_layers, o.n_devices
    s_cap = min(Ld, Lu, D) if o.max_stages <= 0 else min(Ld, Lu, D, o.max_stages)
    best = BidirPlan()
    for S in ([o.exact_stages] if o.exact_stages > 0 else range(1, s_cap + 1)):
        if S > s_cap:
            break
        obj = lambda w, y: (o.n_micro_batches + 2 * S - 2) * w + y
        table = {}
        for d in range(1, D + 1):
            for ld in range(1, Ld + 1):
                for lu in range(1, Lu + 1):
                    t = _bidir_pair(down, up, o, 0, ld, 0, lu, d)
                    if t is not None:
                        table[(ld, lu, 1, d, d)] = (t[0], t[1], None)
        for s in range(2, S + 1):
            for d in range(s, D + 1):
                for r in range(1, d - (s - 1) + 1):
                    for ld in range(s, Ld + 1):
                        for lu in range(s, Lu + 1):
                            pick = None
                            for pd in range(s - 1, ld):              # Eq. 16: l_d, l_u, r'
                                for pu in range(s - 1, lu):
                                    t = _bidir_pair(down, up, o, pd, ld, pu, lu, r)
                                    if t is None:
                                        continue
                                    for rp in range(1, d - r + 1):
                                        if o.uniform_replication and rp != r:
                                            continue
                                        sub = table.get((pd, pu, s - 1, rp, d - r))
                                        if sub is None:
                                            continue
                                        w, y = max(sub[0], t[0]), max(sub[1], t[1])      # Eq. 14, 15
                                        if pick is None or obj(w, y) < pick[0]:
                                            pick = (obj(w, y), w, y, (pd, pu, s - 1, rp, d - r))
                            if pick is not None:
                                table[(ld, lu, s, r, d)] = pick[1:]
        for r in range(1, D + 1):                                    # Eq. 13
            st = table.get((Ld, Lu, S, r, D))
            if st is None or obj(st[0], st[1]) >= best.t_max_ms:
                continue
            plan = BidirPlan(n_stages=S, t0_ms=st[0], gap_ms=st[1], t_max_ms=obj(st[0], st[1]))
            key, stages = (Ld, Lu, S, r, D), []
            while key is not None:
                parent = table[key][2]
                pd, pu = (parent[0], parent[1]) if parent is not None else (0, 0)
                stages.append((pd, key[0] - pd, Lu - key[1], key[1] - pu, key[3]))
                key = parent
            stages.reverse()
            plan.first_layer_down = [x[0] for x in stages]; plan.n_layers_down = [x[1] for x in stages]
            plan.first_layer_up = [x[2] for x in stages]; plan.n_layers_up = [x[3] for x in stages]
            plan.replicas = [x[4] for x in stages]
            best = plan
    return best


def score_bidirectional(down: Profile, up: Profile, o: Options, cuts_down, cuts_up_from_end, replicas):
    """(W, Y, T_max) of an explicit pair of partitions from the definitions (Eq. 10-12): cuts_down = first
    down layer of every chain position, cuts_up_from_end = the same for the up backbone counted from its end."""
    S = len(replicas)
    bd, bu = list(cuts_down) + [down.n_layers], list(cuts_up_from_end) + [up.n_layers]
    w = y = 0.0
    for i in range(S):
        t = _bidir_pair(down, up, o, bd[i], bd[i + 1], bu[i], bu[i + 1], replicas[i])
        if t is None:
            return None
        w, y = max(w, t[0]), max(y, t[1])
    return w, y, (o.n_micro_batches + 2 * S - 2) * w + y


def brute_force_bidirectional(down: Profile, up: Profile, o: Options):
    Ld, Lu, D = down.n_layers, up.n_layers, o.n_devices
    s_cap = min(Ld, Lu, D) if o.max_stages <= 0 else min(Ld, Lu, D, o.max_stages)
    best = (math.inf, None, None, None)
    for S in ([o.exact_stages] if o.exact_stages > 0 else range(1, s_cap + 1)):
        if S > s_cap:
            break
        for cd in itertools.combinations(range(1, Ld), S - 1):
            for cu in itertools.combinations(range(1, Lu), S - 1):
                for reps in itertools.product(range(1, D + 1), repeat=S):
                    if sum(reps) != D or (o.uniform_replication and len(set(reps)) != 1):
                        continue
                    sc = score_bidirectional(down, up, o, (0,) + cd, (0,) + cu, reps)
                    if sc is not None and sc[2] < best[0]:
                        best = (sc[2], (0,) + cd, (0,) + cu, reps)
    return best
