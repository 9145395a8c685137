"""Hyper-parameter search over (S, M, D) (Sec. 3, workflow steps 2-5): the oracle against a hand-worked
example and against its own parts called one by one, and the library's dp_schedule_search (host code) against
the oracle on seeded random profiles.  Runs without a GPU."""
import random

import numpy as np
import pytest

from oracle import bubbles as Bu
from oracle import partition as P
from oracle import search as S


@pytest.fixture(scope="module")
def B():
    from paper_2405_01248_amd import binding
    binding.load_library()
    return binding


# ------------------------------------------------------------------ hand-worked example
def _two_layer_profile():
    """Two identical layers: forward 1 ms and backward 2 ms per layer at local batch 2, half of that at local
    batch 1 (perfect scaling); no bytes anywhere, so transfers and synchronisation cost only their latencies."""
    f = {2: [1.0, 1.0], 1: [0.5, 0.5]}
    b = {2: [2.0, 2.0], 1: [1.0, 1.0]}
    z = {2: [0, 0], 1: [0, 0]}
    return P.Profile(2, f, b, z, z, [0, 0], {2: 0, 1: 0})


def test_hand_worked_two_layers_two_devices():
    # world = 2 devices, training batch 4, one frozen component of one layer that takes 0.25 ms at any local batch.
    prof = _two_layer_profile()
    comp = Bu.Component(1, {1: [0.25], 2: [0.25], 4: [0.25]})
    o = S.SearchOptions(world_size=2, training_batch=4, group_sizes=(1, 2), micro_batch_counts=(1, 2), p2p_latency_ms=0.0,
                        ar_latency_ms=0.0, uniform_replication=False)
    cands, best = S.search(prof, [comp], o)
    got = {(c.group_size, c.n_micro_batches, c.n_stages): c for c in cands}
    # D = 1 (pure data parallel): the group trains 2 samples.  M = 1: B = 2, one stage: 2 + 4 = 6 ms, no bubble,
    # the frozen layer runs afterwards: 6.25 ms.  M = 2: B = 1: two micro-batches of 1 + 2 ms: 6 ms + 0.25.
    assert got[(1, 1, 1)].iteration_ms == pytest.approx(6.25) and got[(1, 2, 1)].iteration_ms == pytest.approx(6.25)
    assert got[(1, 1, 1)].bubble_ratio == 0.0
    # D = 2, S = 1: one stage replicated on both devices: group batch 4, M = 2 -> B = 2 at local batch 1:
    # 2 x (1 + 2) = 6 ms, no bubble -> 6.25.  M = 1 -> B = 4, local batch 2: 6 ms -> 6.25.
    assert got[(2, 2, 1)].iteration_ms == pytest.approx(6.25) and got[(2, 1, 1)].iteration_ms == pytest.approx(6.25)
    # D = 2, S = 2, M = 2 (B = 2, one layer per stage, one device each): forward 1, backward 2 per micro-batch.
    #   stage 0: F0 [0,1] F1 [1,2] B0 [4,6] B1 [7,9];  stage 1: F0 [1,2] B0 [2,4] F1 [4,5] B1 [5,7]  -> 9 ms.
    #   idle: stage 1 in [0,1] and [7,9], stage 0 in [2,4] and [6,7]: 6 device-ms of 18; the frozen layer
    #   (0.25 ms on one device) fits the first bubble: nothing is left over.
    c = got[(2, 2, 2)]
    assert c.pipeline_ms == pytest.approx(9.0) and c.leftover_ms == 0.0 and c.iteration_ms == pytest.approx(9.0)
    assert c.bubble_ratio == pytest.approx(6.0 / 18.0) and c.bubble_ratio_filled == pytest.approx(5.75 / 18.0)
    assert c.plan.n_layers == [1, 1] and c.plan.replicas == [1, 1]
    # D = 2, S = 2, M = 1 (B = 4: local batch 4 is not profiled) is infeasible and absent
    assert (2, 1, 2) not in got
    # step 5: the least iteration time, the first one walked on ties
    assert cands[best].iteration_ms == pytest.approx(6.25) and (cands[best].group_size, cands[best].n_micro_batches) == (1, 1)


# ------------------------------------------------------------------ random problems
def random_search_problem(seed):
    rng = random.Random(seed)
    L = rng.randint(2, 7)
    world = rng.choice([2, 4, 8])
    Bt = world * rng.choice([4, 8, 16])
    f32 = lambda v: float(np.float32(v))
    batches = [1, 2, 4, 8, 16, 32, 64]
    prof = P.Profile(L, {}, {}, {}, {}, [int(rng.uniform(1e6, 4e7)) for _ in range(L)], {})
    per_f = [rng.uniform(0.1, 2.0) for _ in range(L)]
    per_b = [rng.uniform(0.2, 4.0) for _ in range(L)]
    act = [int(rng.uniform(1e5, 4e6)) for _ in range(L)]
    rows = []
    for b in batches:
        eff = 0.3 + 0.7 * min(b, 16) / 16
        prof.fwd_ms[b] = [f32(p * b / eff) for p in per_f]
        prof.bwd_ms[b] = [f32(p * b / eff) for p in per_b]
        prof.cf_bytes[b] = [a * b for a in act]
        prof.cb_bytes[b] = [a * b for a in act]
        prof.out_bytes[b] = act[-1] * b
        for l in range(L):
            rows.append({"component": 0, "layer": l, "batch": b, "fwd_ms": prof.fwd_ms[b][l], "bwd_ms": prof.bwd_ms[b][l], "out_bytes": act[l] * b,
                         "cf_bytes": prof.cf_bytes[b][l], "cb_bytes": prof.cb_bytes[b][l], "grad_bytes": prof.grad_bytes[l]})
    comps = []
    for cid in (1, 2)[: rng.randint(1, 2)]:
        nl = rng.randint(1, 5)
        per = [rng.uniform(0.05, 3.0) for _ in range(nl)]
        tab = {}
        for b in (4, 16, 64):
            tab[b] = [f32(p * (0.4 + 0.6 * b / 16)) for p in per]
            for l in range(nl):
                rows.append({"component": cid, "layer": l, "batch": b, "fwd_ms": tab[b][l], "bwd_ms": 0.0, "out_bytes": 0, "cf_bytes": 0,
                             "cb_bytes": 0, "grad_bytes": 0})
        comps.append(Bu.Component(nl, tab, deps=((0,) if cid == 2 and rng.random() < 0.5 else ())))
    rng.shuffle(rows)
    o = S.SearchOptions(world_size=world, training_batch=Bt, group_sizes=tuple(d for d in (1, 2, 4, 8, 3) if d <= world),
                        micro_batch_counts=(1, 2, 4, 8), max_stages=rng.choice([0, 0, 2]), uniform_replication=rng.random() < 0.6,
                        p2p_gbps=rng.choice([10.0, 150.0]), p2p_latency_ms=rng.choice([0.0, 0.02]), ar_gbps=rng.choice([20.0, 400.0]),
                        ar_latency_ms=rng.choice([0.0, 0.1]), self_cond_prob=rng.choice([0.0, 0.5]), min_bubble_ms=rng.choice([0.0, 0.5]))
    return rows, prof, comps, o


def lib_search(B, rows, comps, o):
    deps = [(i + 1, j + 1) for i, c in enumerate(comps) for j in c.deps]
    return B.schedule_search(rows, o.world_size, o.training_batch, o.group_sizes, o.micro_batch_counts, o.p2p_gbps, o.p2p_latency_ms,
                             o.ar_gbps, o.ar_latency_ms, o.self_cond_prob, o.max_stages, o.uniform_replication, o.min_bubble_ms, deps)


@pytest.mark.parametrize("seed", range(25))
def test_library_matches_oracle_on_random_problems(B, seed):
    rows, prof, comps, o = random_search_problem(seed)
    ref, ref_best = S.search(prof, comps, o)
    got, best = lib_search(B, rows, comps, o)
    assert [(c["group_size"], c["n_micro_batches"], c["n_stages"], c["micro_batch"]) for c in got] == \
           [(c.group_size, c.n_micro_batches, c.n_stages, c.micro_batch) for c in ref]
    for g, r in zip(got, ref):
        assert (g["first_layer"], g["replicas"]) == (r.plan.first_layer, r.plan.replicas)
        for k in ("pipeline_ms", "leftover_ms", "iteration_ms", "bubble_ratio", "bubble_ratio_filled"):
            assert g[k] == pytest.approx(getattr(r, k), rel=1e-9, abs=1e-12), k
    assert best == ref_best
    # step 5 is a minimum over what was walked
    assert all(got[best]["iteration_ms"] <= c["iteration_ms"] for c in got)


def test_oracle_search_is_its_parts_called_one_by_one():
    rows, prof, comps, o = random_search_problem(3)
    cands, _ = S.search(prof, comps, o)
    assert cands
    for c in cands[:: max(1, len(cands) // 6)]:
        po = P.Options(micro_batch=c.micro_batch, n_micro_batches=c.n_micro_batches, n_devices=c.group_size, p2p_gbps=o.p2p_gbps,
                       p2p_latency_ms=o.p2p_latency_ms, ar_gbps=o.ar_gbps, ar_latency_ms=o.ar_latency_ms, self_cond_prob=o.self_cond_prob,
                       max_stages=o.max_stages, uniform_replication=o.uniform_replication, exact_stages=c.n_stages)
        plan = P.solve(prof, po)
        assert (plan.first_layer, plan.replicas) == (c.plan.first_layer, c.plan.replicas)
        # an exact stage count is one of the candidates the unrestricted programme chooses from
        free = P.solve(prof, P.Options(**{**po.__dict__, "exact_stages": 0}))
        assert free.t_max_ms <= plan.t_max_ms * (1 + 1e-12)
        assert c.group_size * c.micro_batch * c.n_micro_batches * (o.world_size // c.group_size) == o.training_batch * c.group_size


def test_argument_checks(B):
    rows, prof, comps, o = random_search_problem(1)
    with pytest.raises(B.DpipeError) as ei:
        B.schedule_search([r for r in rows if r["component"] == 0], 4, 16, (1, 2), (1, 2), 50.0, 0.0, 100.0, 0.0)
    assert ei.value.code == -1                                   # no non-trainable component
    with pytest.raises(B.DpipeError) as ei:
        B.schedule_search(rows, 4, 16, (3,), (1, 2), 50.0, 0.0, 100.0, 0.0)
    assert ei.value.code == -2                                   # 3 does not divide the world size: nothing feasible
    with pytest.raises(B.DpipeError) as ei:
        B.schedule_search(rows, 0, 16, (1,), (1,), 50.0, 0.0, 100.0, 0.0)
    assert ei.value.code == -1
    with pytest.raises(B.DpipeError) as ei:
        B.schedule_search(rows, o.world_size, o.training_batch, o.group_sizes, o.micro_batch_counts, 50.0, 0.0, 100.0, 0.0, max_cands=1)
    assert ei.value.code == -3                                   # more candidates than rows to write them to
