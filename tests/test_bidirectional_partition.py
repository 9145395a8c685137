"""Bidirectional partitioning of two backbones (Sec. 4.2, Eq. 10-16): pins of the oracle (hand-worked
example, brute force over every pair of partitions, reduction to the single-backbone programme) and the
library's dp_partition_solve_bidirectional against the oracle.  Runs without a GPU."""
import math
import random

import numpy as np
import pytest

from oracle import partition as P
from test_oracle_partition import make_profile


@pytest.fixture(scope="module")
def B():
    from paper_2405_01248_amd import binding
    binding.load_library()
    return binding


def test_hand_worked_pair_of_two_layer_backbones():
    # down: layers of 1 + 2 and 3 + 6 ms (forward + backward) at local batch 2; up: 2 + 2 and 1 + 1 ms.
    # One message of 1 MB each way between the layers of either backbone; 1 GB/s, 0.1 ms latency.
    down = P.Profile(2, {2: [1.0, 3.0]}, {2: [2.0, 6.0]}, {2: [1_000_000, 0]}, {2: [1_000_000, 0]}, [0, 0], {2: 0})
    up = P.Profile(2, {2: [2.0, 1.0]}, {2: [2.0, 1.0]}, {2: [1_000_000, 0]}, {2: [1_000_000, 0]}, [0, 0], {2: 0})
    o = P.Options(micro_batch=2, n_micro_batches=6, n_devices=2, p2p_gbps=1.0, p2p_latency_ms=0.1, ar_gbps=1.0, ar_latency_ms=0.0)
    # two stages, one device each: position 0 holds down layer 0 (3 ms, no incoming transfer) and up layer 1
    # (2 ms against a doubled transfer of 2 (2 + 0.2) = 4.4 ms): T_0 = 4.4; position 1 holds down layer 1 (9 ms
    # against 4.4) and up layer 0 (4 ms, the up backbone's first stage): T_0 = 9.  No gradients: Y = 0.
    assert P.score_bidirectional(down, up, o, (0, 1), (0, 1), (1, 1)) == pytest.approx((9.0, 0.0, (6 + 2) * 9.0))
    # one stage on both devices would need local batch 1, which is not profiled
    assert P.score_bidirectional(down, up, o, (0,), (0,), (2,)) is None
    plan = P.solve_bidirectional(down, up, o)
    assert (plan.n_stages, plan.replicas) == (2, [1, 1]) and plan.t_max_ms == pytest.approx(72.0)
    assert (plan.first_layer_down, plan.n_layers_down, plan.first_layer_up, plan.n_layers_up) == ([0, 1], [1, 1], [1, 0], [1, 1])


@pytest.mark.parametrize("seed", range(10))
def test_equals_brute_force_where_the_objective_decomposes(seed):
    rng = random.Random(seed)
    Ld, Lu, D = rng.randint(2, 4), rng.randint(2, 4), rng.randint(1, 3)
    down = make_profile(Ld, [12, 6, 4], rng, bwd=False, grads=False, comm_scale=rng.choice([0.1, 5.0]))
    up = make_profile(Lu, [12, 6, 4], rng, bwd=False, grads=False, comm_scale=rng.choice([0.1, 5.0]))
    o = P.Options(micro_batch=12, n_micro_batches=rng.randint(2, 12), n_devices=D, ar_latency_ms=0.0, p2p_gbps=rng.choice([1.0, 25.0]))
    plan, bf = P.solve_bidirectional(down, up, o), P.brute_force_bidirectional(down, up, o)
    assert plan.t_max_ms == pytest.approx(bf[0], rel=1e-12)
    cuts_up_from_end = [Lu - (a + n) for a, n in zip(plan.first_layer_up, plan.n_layers_up)]
    assert P.score_bidirectional(down, up, o, plan.first_layer_down, cuts_up_from_end, plan.replicas)[2] == pytest.approx(plan.t_max_ms, rel=1e-12)
    assert sum(plan.n_layers_down) == Ld and sum(plan.n_layers_up) == Lu and sum(plan.replicas) == D


@pytest.mark.parametrize("seed", range(8))
def test_never_beats_brute_force_with_gaps(seed):
    rng = random.Random(50 + seed)
    Ld, Lu, D = rng.randint(2, 4), rng.randint(2, 4), rng.randint(1, 3)
    down, up = make_profile(Ld, [12, 6, 4], rng), make_profile(Lu, [12, 6, 4], rng)
    o = P.Options(micro_batch=12, n_micro_batches=rng.randint(2, 12), n_devices=D, ar_gbps=rng.choice([1.0, 20.0]), uniform_replication=bool(seed % 2))
    plan, bf = P.solve_bidirectional(down, up, o), P.brute_force_bidirectional(down, up, o)
    if bf[1] is None:
        assert plan.n_stages == 0
        return
    assert plan.t_max_ms >= bf[0] * (1 - 1e-12)


def test_a_free_up_backbone_reduces_to_the_single_backbone_programme_with_doubled_transfers():
    rng = random.Random(7)
    L = 5
    down = make_profile(L, [12, 6, 4, 3], rng, bwd=False, grads=False, comm_scale=5.0)
    z = lambda b: [0.0] * L
    zi = lambda b: [0] * L
    up = P.Profile(L, {b: z(b) for b in (12, 6, 4, 3)}, {b: z(b) for b in (12, 6, 4, 3)}, {b: zi(b) for b in (12, 6, 4, 3)},
                   {b: zi(b) for b in (12, 6, 4, 3)}, [0] * L, {b: 0 for b in (12, 6, 4, 3)})
    for D in (1, 2, 4):
        o = P.Options(micro_batch=12, n_micro_batches=5, n_devices=D, p2p_gbps=4.0, p2p_latency_ms=0.0, ar_latency_ms=0.0)
        single = P.solve(down, P.Options(micro_batch=12, n_micro_batches=5, n_devices=D, p2p_gbps=2.0, p2p_latency_ms=0.0, ar_latency_ms=0.0))
        both = P.solve_bidirectional(down, up, o)
        assert both.t_max_ms == pytest.approx(single.t_max_ms, rel=1e-12) and both.n_stages == single.n_stages
        assert both.first_layer_down == single.first_layer and both.replicas == single.replicas


def _rows(prof):
    f32 = lambda v: float(np.float32(v))
    rows = []
    for b in prof.fwd_ms:
        prof.fwd_ms[b] = [f32(v) for v in prof.fwd_ms[b]]
        prof.bwd_ms[b] = [f32(v) for v in prof.bwd_ms[b]]
        for l in range(prof.n_layers):
            rows.append({"component": 0, "layer": l, "batch": b, "fwd_ms": prof.fwd_ms[b][l], "bwd_ms": prof.bwd_ms[b][l], "out_bytes": 0,
                         "cf_bytes": prof.cf_bytes[b][l], "cb_bytes": prof.cb_bytes[b][l], "grad_bytes": prof.grad_bytes[l]})
    return rows


@pytest.mark.parametrize("seed", range(30))
def test_library_matches_oracle(B, seed):
    rng = random.Random(200 + seed)
    Ld, Lu, D = rng.randint(1, 6), rng.randint(1, 6), rng.randint(1, 5)
    down, up = make_profile(Ld, [12, 6, 4, 3], rng, comm_scale=rng.choice([0.1, 5.0])), make_profile(Lu, [12, 6, 4], rng)
    rd, ru = _rows(down), _rows(up)
    rng.shuffle(rd)
    o = P.Options(micro_batch=12, n_micro_batches=rng.randint(1, 16), n_devices=D, p2p_gbps=rng.choice([1.0, 50.0]), ar_gbps=rng.choice([1.0, 100.0]),
                  max_stages=rng.choice([0, 0, 2]), uniform_replication=rng.random() < 0.3, exact_stages=rng.choice([0, 0, 0, 2]))
    ref = P.solve_bidirectional(down, up, o)
    if ref.n_stages == 0:
        with pytest.raises(B.DpipeError) as ei:
            B.partition_solve_bidirectional(rd, ru, 12, o.n_micro_batches, D, o.p2p_gbps, o.p2p_latency_ms, o.ar_gbps, o.ar_latency_ms,
                                            o.max_stages, o.uniform_replication, o.exact_stages)
        assert ei.value.code == -2
        return
    got = B.partition_solve_bidirectional(rd, ru, 12, o.n_micro_batches, D, o.p2p_gbps, o.p2p_latency_ms, o.ar_gbps, o.ar_latency_ms,
                                          o.max_stages, o.uniform_replication, o.exact_stages)
    assert got["n_stages"] == ref.n_stages and got["replicas"] == ref.replicas
    assert (got["first_layer_down"], got["n_layers_down"], got["first_layer_up"], got["n_layers_up"]) == \
           (ref.first_layer_down, ref.n_layers_down, ref.first_layer_up, ref.n_layers_up)
    for k in ("t0_ms", "gap_ms", "t_max_ms"):
        assert got[k] == pytest.approx(getattr(ref, k), rel=1e-12)


def test_argument_checks(B):
    rng = random.Random(1)
    rd, ru = _rows(make_profile(3, [4, 2], rng)), _rows(make_profile(2, [4, 2], rng))
    ok = dict(micro_batch=4, n_paired_micro_batches=4, n_devices=2, p2p_gbps=10.0, p2p_latency_ms=0.0, ar_gbps=10.0, ar_latency_ms=0.0)
    assert B.partition_solve_bidirectional(rd, ru, **ok)["n_stages"] >= 1
    for bad, code in ((dict(n_devices=0), -1), (dict(p2p_gbps=0.0), -1), (dict(micro_batch=5), -2), (dict(n_devices=65), -1)):
        with pytest.raises(B.DpipeError) as ei:
            B.partition_solve_bidirectional(rd, ru, **{**ok, **bad})
        assert ei.value.code == code
    with pytest.raises(B.DpipeError) as ei:
        B.partition_solve_bidirectional(rd[:-1], ru, **ok)          # a missing (layer, batch) row
    assert ei.value.code == -1
