"""Search over the pipeline hyper-parameters (S, M, D), plain Python (test infrastructure only).

Sec. 3 ("Workflow", steps 2-5, Table "Pipeline training hyper-parameters"): for every feasible
combination of the number of stages S, the number of micro-batches M and the pipeline-parallel group
size D (world size = D x data-parallel degree), partition the backbone (step 2, Sec. 4), derive the
FIFO-1F1B schedule of that partition (step 3), fill its bubbles with the non-trainable part (step 4,
Sec. 5), and keep the combination whose overall schedule has the least iteration time (step 5).

The steps are composed from the oracle's own partitioner and bubble filler; this module only walks the
combinations.  Readings where the text is silent (the same in the product):
  * a pipeline group trains training_batch * D / world_size samples per iteration, cut into M micro-batches
    of B samples; combinations where these are not integers, or where no partition into exactly S stages is
    feasible, are skipped;
  * a stage's forward time in the simulated schedule is (1 + p) sum P^f (the expected cost of the extra
    self-conditioning forward), its backward time sum P^b; the transfer between stages s and s + 1 takes
    C / R_p2p + L_p2p at the receiving stage's local batch; the gradient synchronisation T_S(s) of Eq. 4
    follows the stage's last backward;
  * iteration time = length of the simulated pipeline iteration + the time of the non-trainable layers that
    fit no bubble, run afterwards on the D devices of the group (with cross-iteration pipelining, Sec. 3.2,
    the bubbles of one iteration hold the frozen part of the next);
  * candidates are walked in the order of the D list, then the M list, then S ascending; ties keep the
    earlier one.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

from . import bubbles as Bu
from . import partition as P


@dataclass
class SearchOptions:
    world_size: int
    training_batch: int
    group_sizes: tuple                 # candidate D
    micro_batch_counts: tuple          # candidate M
    max_stages: int = 0
    uniform_replication: bool = True
    p2p_gbps: float = 50.0
    p2p_latency_ms: float = 0.01
    ar_gbps: float = 100.0
    ar_latency_ms: float = 0.05
    self_cond_prob: float = 0.0
    min_bubble_ms: float = 0.0


@dataclass
class Candidate:
    n_stages: int
    n_micro_batches: int
    group_size: int
    micro_batch: int
    plan: P.Plan
    pipeline_ms: float
    leftover_ms: float
    iteration_ms: float
    bubble_ratio: float               # idle device-time / (D x pipeline time), before filling
    bubble_ratio_filled: float        # after filling, over D x iteration time


def stage_times(prof: P.Profile, plan: P.Plan, o: SearchOptions, micro_batch: int):
    """Per-stage (fwd, bwd, tail) and per-boundary (comm_fwd, comm_bwd) of a plan, in ms."""
    f, b, tail, cf, cb = [], [], [], [], []
    for s in range(plan.n_stages):
        lo, hi = plan.first_layer[s], plan.first_layer[s] + plan.n_layers[s]
        lb = micro_batch // plan.replicas[s]
        f.append((1.0 + o.self_cond_prob) * sum(prof.fwd_ms[lb][lo:hi]))
        b.append(sum(prof.bwd_ms[lb][lo:hi]))
        tail.append(sum(prof.grad_bytes[lo:hi]) / (o.ar_gbps * 1e9) * 1e3 + o.ar_latency_ms)
        if s:
            cf.append(prof.cf_bytes[lb][lo - 1] / (o.p2p_gbps * 1e9) * 1e3 + o.p2p_latency_ms)
            cb.append(prof.cb_bytes[lb][lo - 1] / (o.p2p_gbps * 1e9) * 1e3 + o.p2p_latency_ms)
    return f, b, tail, cf, cb


def evaluate(prof: P.Profile, comps, o: SearchOptions, S: int, M: int, D: int):
    """One combination (steps 2-4), or None when it is infeasible."""
    if D <= 0 or o.world_size % D or (o.training_batch * D) % o.world_size:
        return None
    group_batch = o.training_batch * D // o.world_size
    if M <= 0 or group_batch % M or group_batch // M == 0:
        return None
    B = group_batch // M
    po = P.Options(micro_batch=B, n_micro_batches=M, n_devices=D, p2p_gbps=o.p2p_gbps, p2p_latency_ms=o.p2p_latency_ms,
                   ar_gbps=o.ar_gbps, ar_latency_ms=o.ar_latency_ms, self_cond_prob=o.self_cond_prob, max_stages=o.max_stages,
                   uniform_replication=o.uniform_replication, exact_stages=S)
    if o.self_cond_prob > 0.0 and B not in prof.out_bytes:
        return None
    plan = P.solve(prof, po)
    if plan.n_stages != S:
        return None
    f, b, tail, cf, cb = stage_times(prof, plan, o, B)
    busy, t_pipe = Bu.simulate_1f1b(f, b, M, cf or None, cb or None, tail)
    bubs = Bu.find_bubbles(busy, t_pipe, plan.replicas, o.min_bubble_ms)
    fill = Bu.fill_all(bubs, comps, group_batch, D)
    t_iter = t_pipe + fill.leftover_ms
    return Candidate(S, M, D, B, plan, t_pipe, fill.leftover_ms, t_iter, fill.bubble_device_ms / (D * t_pipe),
                     (fill.bubble_device_ms - fill.filled_device_ms) / (D * t_iter))


def search(prof: P.Profile, comps, o: SearchOptions):
    """All feasible candidates in walking order and the index of the one with the least iteration time (step 5)."""
    cands, best = [], -1
    for D in o.group_sizes:
        for M in o.micro_batch_counts:
            s_max = min(prof.n_layers, D) if o.max_stages <= 0 else min(prof.n_layers, D, o.max_stages)
            for S in range(1, s_max + 1):
                c = evaluate(prof, comps, o, S, M, D)
                if c is None:
                    continue
                cands.append(c)
                if best < 0 or c.iteration_ms < cands[best].iteration_ms:
                    best = len(cands) - 1
    return cands, best
