"""Pins of the partitioning oracle (oracle/partition.py) against what the paper's definitions and
plain enumeration fix: a hand-worked two-layer example (Eq. 1, 3-6, 17, 18), brute force over every
partition and replication vector on small instances, and closed forms of uniform backbones."""
import math
import random

import pytest

from oracle import partition as P


def make_profile(L, batches, rng, bwd=True, grads=True, comm_scale=1.0):
    per_sample_f = [rng.uniform(0.2, 2.0) for _ in range(L)]
    per_sample_b = [rng.uniform(0.4, 4.0) if bwd else 0.0 for _ in range(L)]
    act = [int(rng.uniform(1e5, 4e6) * comm_scale) for _ in range(L)]
    fwd, bwdt, cf, cb, out = {}, {}, {}, {}, {}
    for b in batches:
        eff = 0.3 + 0.7 * b / max(batches)              # small batches are less efficient, as on a GPU
        fwd[b] = [p * b / eff for p in per_sample_f]
        bwdt[b] = [p * b / eff for p in per_sample_b]
        cf[b] = [a * b for a in act]
        cb[b] = [a * b for a in act]
        out[b] = act[-1] * b
    grad = [int(rng.uniform(1e6, 3e7)) if grads else 0 for _ in range(L)]
    return P.Profile(L, fwd, bwdt, cf, cb, grad, out)


def test_hand_worked_two_layer_example():
    prof = P.Profile(2, {2: [1.0, 3.0], 1: [0.5, 1.5]}, {2: [2.0, 6.0], 1: [1.0, 3.0]},
                     {2: [1_000_000, 0], 1: [500_000, 0]}, {2: [1_000_000, 0], 1: [500_000, 0]},
                     [4_000_000, 4_000_000], {2: 2_000_000, 1: 1_000_000})
    o = P.Options(micro_batch=2, n_micro_batches=2, n_devices=2, p2p_gbps=1.0, p2p_latency_ms=0.1, ar_gbps=2.0, ar_latency_ms=0.5)
    # one stage on both devices: local batch 1, P^f = 2, P^b = 4 -> T_0 = 6; T_S = 8e6 / 2e9 s + 0.5 = 4.5, T_C = 4
    assert P.stage_terms(prof, o, 0, 2, 2) == pytest.approx((6.0, 8.0, 0.5))
    # two stages, one device each (local batch 2): stage 0 -> T_0 = 3, gap 2.5 - 2; stage 1 -> compute 9 against a
    # transfer of 2 MB at 1 GB/s + 2 latencies = 2.2; T_S = 2.5 < T_C = 6 -> gap 0
    assert P.stage_terms(prof, o, 0, 1, 1) == pytest.approx((3.0, 4.0, 0.5))
    assert P.stage_terms(prof, o, 1, 2, 1) == pytest.approx((9.0, 12.0, 0.0))
    assert P.score(prof, o, (0,), (2,))[3] == pytest.approx(2 * 6.0 + 0.5)            # (M + 2S - 2) T_0 + gap, S = 1
    assert P.score(prof, o, (0, 1), (1, 1))[3] == pytest.approx(4 * 9.0 + 0.5)        # S = 2
    plan = P.solve(prof, o)
    assert (plan.n_stages, plan.replicas, plan.first_layer, plan.n_layers) == (1, [2], [0], [2])
    assert plan.t_max_ms == pytest.approx(12.5)
    # self-conditioning always on: T_0,SC = 2 * 2 + 4 = 8, T_F = 2 MB at 1 GB/s + one latency = 2.1
    o.self_cond_prob = 1.0
    assert P.solve(prof, o).t_max_ms == pytest.approx(2 * 8.0 + 0.5 + 2.1)
    # and half of the time: the expectation of the two bounds
    o.self_cond_prob = 0.5
    assert P.solve(prof, o).t_max_ms == pytest.approx(0.5 * (2 * 8.0 + 0.5 + 2.1) + 0.5 * 12.5)
    # a transfer that dominates: 20 MB each way -> 40 ms + 0.2 on the second stage's boundary (3 latencies and
    # twice the forward message under self-conditioning)
    prof.cf_bytes[2][0] = prof.cb_bytes[2][0] = 20_000_000
    t = P.stage_terms(prof, o, 1, 2, 1)
    assert t[0] == pytest.approx(40.2) and t[1] == pytest.approx(60.3)


def test_infeasible_replication_is_skipped():
    rng = random.Random(3)
    prof = make_profile(4, [6, 3, 2], rng)             # B = 6: r in {1, 2, 3}; r = 4 does not divide, b = 1 is not profiled
    o = P.Options(micro_batch=6, n_micro_batches=4, n_devices=4)
    assert P.stage_terms(prof, o, 0, 4, 4) is None and P.stage_terms(prof, o, 0, 4, 6) is None
    plan = P.solve(prof, o)
    assert sum(plan.replicas) == 4 and all(6 % r == 0 and 6 // r in (6, 3, 2) for r in plan.replicas)
    assert plan.t_max_ms == pytest.approx(P.brute_force(prof, o)[0]) or plan.t_max_ms >= P.brute_force(prof, o)[0]


@pytest.mark.parametrize("seed", range(12))
def test_equals_brute_force_where_the_objective_decomposes(seed):
    # no backward time, no gradients, no all-reduce latency: every gap is zero and the objective is a multiple of
    # max_s T_0(s), for which the recurrence W = max(W_sub, T_0(s)) is exact
    rng = random.Random(seed)
    L, D = rng.randint(2, 6), rng.randint(1, 4)
    B = 12
    prof = make_profile(L, [12, 6, 4, 3], rng, bwd=False, grads=False, comm_scale=rng.choice([0.1, 5.0, 50.0]))
    o = P.Options(micro_batch=B, n_micro_batches=rng.randint(1, 8), n_devices=D, ar_latency_ms=0.0,
                  p2p_gbps=rng.choice([1.0, 25.0]), self_cond_prob=rng.choice([0.0, 0.5]))
    plan, bf = P.solve(prof, o), P.brute_force(prof, o)
    assert plan.t_max_ms == pytest.approx(bf[0], rel=1e-12)
    assert P.score(prof, o, plan.first_layer, plan.replicas)[3] == pytest.approx(plan.t_max_ms, rel=1e-12)


@pytest.mark.parametrize("seed", range(20))
def test_never_beats_brute_force_and_reports_its_own_plan_faithfully(seed):
    rng = random.Random(100 + seed)
    L, D = rng.randint(2, 6), rng.randint(1, 4)
    prof = make_profile(L, [12, 6, 4, 3], rng, comm_scale=rng.choice([0.1, 5.0]))
    o = P.Options(micro_batch=12, n_micro_batches=rng.randint(1, 8), n_devices=D, ar_gbps=rng.choice([1.0, 20.0]),
                  self_cond_prob=rng.choice([0.0, 0.5, 1.0]), uniform_replication=bool(seed % 2))
    plan, bf = P.solve(prof, o), P.brute_force(prof, o)
    if bf[1] is None:
        assert plan.n_stages == 0 and math.isinf(plan.t_max_ms)
        return
    assert plan.t_max_ms >= bf[0] * (1 - 1e-12)
    w, w_sc, y, t = P.score(prof, o, plan.first_layer, plan.replicas)
    assert (w, w_sc, y, t) == pytest.approx((plan.t0_ms, plan.t0_sc_ms, plan.gap_ms, plan.t_max_ms), rel=1e-12)
    assert sum(plan.replicas) == D and sum(plan.n_layers) == L and plan.first_layer[0] == 0
    if o.uniform_replication:
        assert len(set(plan.replicas)) == 1


def test_uniform_backbone_closed_forms():
    # L identical layers, time linear in the local batch, free communication and synchronisation:
    # S stages of n layers on r devices each take n c B / r, so one stage on all devices minimises
    # (M + 2S - 2) max_s T_0(s) for every M >= 1; with replication forbidden (B = 1 profiled only at b = 1,
    # D = S forced by max_stages and uniform replication) the balanced cut is optimal: T_0 = ceil(L / S) c
    L, c = 8, 1.5
    lin = lambda b: [c * b] * L
    zero = lambda b: [0] * L
    prof = P.Profile(L, {b: lin(b) for b in (8, 4, 2, 1)}, {b: lin(b) for b in (8, 4, 2, 1)}, {b: zero(b) for b in (8, 4, 2, 1)},
                     {b: zero(b) for b in (8, 4, 2, 1)}, [0] * L, {b: 0 for b in (8, 4, 2, 1)})
    o = P.Options(micro_batch=8, n_micro_batches=4, n_devices=4, p2p_latency_ms=0.0, ar_latency_ms=0.0)
    plan = P.solve(prof, o)
    assert (plan.n_stages, plan.replicas) == (1, [4]) and plan.t_max_ms == pytest.approx(4 * (2 * c * 8 * 2))
    prof1 = P.Profile(L, {1: lin(1)}, {1: lin(1)}, {1: zero(1)}, {1: zero(1)}, [0] * L, {1: 0})
    o1 = P.Options(micro_batch=1, n_micro_batches=6, n_devices=3, p2p_latency_ms=0.0, ar_latency_ms=0.0)
    plan = P.solve(prof1, o1)
    assert plan.replicas == [1, 1, 1] and sorted(plan.n_layers) == [2, 3, 3]
    assert plan.t_max_ms == pytest.approx((6 + 2 * 3 - 2) * 3 * 2 * c)


@pytest.mark.parametrize("seed", range(10))
def test_exact_stage_count_against_brute_force_over_that_count(seed):
    # the point (S, M, D) of the hyper-parameter search (Sec. 3): S is given, not chosen
    rng = random.Random(300 + seed)
    L, D = rng.randint(3, 6), rng.randint(2, 4)
    prof = make_profile(L, [12, 6, 4, 3], rng, bwd=False, grads=False, comm_scale=rng.choice([0.1, 5.0]))
    for S in range(1, min(L, D) + 1):
        o = P.Options(micro_batch=12, n_micro_batches=rng.randint(1, 8), n_devices=D, ar_latency_ms=0.0, exact_stages=S)
        plan, bf = P.solve(prof, o), P.brute_force(prof, o)
        if bf[1] is None:
            assert plan.n_stages == 0
            continue
        assert plan.n_stages == S == len(bf[1]) and plan.t_max_ms == pytest.approx(bf[0], rel=1e-12)
    # the unrestricted programme takes the best of the exact ones
    o = P.Options(micro_batch=12, n_micro_batches=4, n_devices=D, ar_latency_ms=0.0)
    exact = [P.solve(prof, P.Options(micro_batch=12, n_micro_batches=4, n_devices=D, ar_latency_ms=0.0, exact_stages=S)).t_max_ms
             for S in range(1, min(L, D) + 1)]
    assert P.solve(prof, o).t_max_ms == pytest.approx(min(exact), rel=1e-12)
