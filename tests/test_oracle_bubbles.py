"""Pins of the bubble oracle (oracle/bubbles.py): the 1F1B schedule against closed forms, a hand-worked
two-stage example and its dependency rules; Algorithm 2's candidate list against plain enumeration;
Algorithm 1 and the chronological filling against a worked example and conservation laws."""
import itertools
import math
import random

import pytest

from oracle import bubbles as Bu


def test_two_stage_two_microbatch_schedule_by_hand():
    # forward 1, backward 2 per stage, no transfer time.  Stage 1 (last): F0 [1,2] B0 [2,4] F1 [4,5] B1 [5,7];
    # stage 0: F0 [0,1] F1 [1,2] B0 [4,6] B1 [7,9].
    busy, t = Bu.simulate_1f1b([1.0, 1.0], [2.0, 2.0], 2)
    assert t == 9.0
    assert busy[0] == [(0.0, 1.0, "F", 0), (1.0, 2.0, "F", 1), (4.0, 6.0, "B", 0), (7.0, 9.0, "B", 1)]
    assert busy[1] == [(1.0, 2.0, "F", 0), (2.0, 4.0, "B", 0), (4.0, 5.0, "F", 1), (5.0, 7.0, "B", 1)]
    bub = Bu.find_bubbles(busy, t, [1, 3])
    assert [(b.start, b.end, b.stages, b.devices) for b in bub] == [(0.0, 1.0, (1,), 3), (2.0, 4.0, (0,), 1), (6.0, 7.0, (0,), 1), (7.0, 9.0, (1,), 3)]
    assert [b.start for b in Bu.find_bubbles(busy, t, [1, 3], min_ms=1.5)] == [2.0, 7.0]
    # the bound of Sec. 4.1 (T_0 (M + 2S - 2) with T_0 = 3) holds
    assert t <= 3.0 * (2 + 2 * 2 - 2)
    # transfers of 0.5 each way delay the second stage's input and the first stage's gradient
    busy, t = Bu.simulate_1f1b([1.0, 1.0], [2.0, 2.0], 2, [0.5], [0.5])
    assert busy[1][0][:2] == (1.5, 2.5) and busy[0][2][:2] == (5.0, 7.0)


@pytest.mark.parametrize("S,M", [(1, 3), (2, 1), (3, 2), (4, 4), (4, 9), (6, 3)])
def test_uniform_stages_closed_form(S, M):
    f, b = 1.25, 2.5
    busy, t = Bu.simulate_1f1b([f] * S, [b] * S, M)
    assert t == pytest.approx((M + S - 1) * (f + b))
    for s in range(S):
        assert sum(y - x for x, y, _, _ in busy[s]) == pytest.approx(M * (f + b))
    bub = Bu.find_bubbles(busy, t, [1] * S)
    idle = sum((x.end - x.start) * x.devices for x in bub)
    assert idle == pytest.approx(S * (S - 1) * (f + b))                      # bubble ratio (S - 1) / (M + S - 1)
    assert idle / (S * t) == pytest.approx((S - 1) / (M + S - 1))


@pytest.mark.parametrize("seed", range(10))
def test_schedule_respects_order_and_dependencies(seed):
    rng = random.Random(seed)
    S, M = rng.randint(1, 6), rng.randint(1, 8)
    f = [rng.uniform(0.5, 3) for _ in range(S)]
    b = [rng.uniform(0.5, 6) for _ in range(S)]
    cf = [rng.uniform(0, 1) for _ in range(S - 1)]
    cb = [rng.uniform(0, 1) for _ in range(S - 1)]
    tail = [rng.choice([0.0, 0.7]) for _ in range(S)]
    busy, t = Bu.simulate_1f1b(f, b, M, cf, cb, tail)
    end = {}
    for s in range(S):
        assert [(k, m) for _, _, k, m in busy[s] if k != "S"] == Bu.order_1f1b(s, S, M)
        for (x0, y0, _, _), (x1, y1, _, _) in zip(busy[s], busy[s][1:]):
            assert x1 >= y0 - 1e-12                                         # one operation at a time
        for x, y, k, m in busy[s]:
            end[(k, s, m)] = y
    for s in range(S):
        for x, y, k, m in busy[s]:
            if k == "F" and s > 0:
                assert x >= end[("F", s - 1, m)] + cf[s - 1] - 1e-12
            if k == "B":
                assert x >= (end[("B", s + 1, m)] + cb[s] if s < S - 1 else end[("F", s, m)]) - 1e-12
            # no operation could have started earlier: it starts at the later of "stage free" and "input there"
    rep = [rng.randint(1, 3) for _ in range(S)]
    bub = Bu.find_bubbles(busy, t, rep)
    busy_dev = sum((y - x) * rep[s] for s in range(S) for x, y, _, _ in busy[s])
    assert busy_dev + sum((x.end - x.start) * x.devices for x in bub) == pytest.approx(sum(rep) * t)
    for x, y in zip(bub, bub[1:]):
        assert y.start >= x.end - 1e-12 and (y.stages != x.stages or y.start > x.end)


def linear_component(n_layers, per_sample_ms, sizes=(4, 8, 12, 16, 24, 32, 48, 64, 96), deps=()):
    return Bu.Component(n_layers, {b: [p * b for p in per_sample_ms] for b in sizes}, tuple(deps))


def test_layer_time_lookup_and_interpolation():
    c = Bu.Component(1, {4: [1.0], 8: [1.5], 32: [4.5]})
    assert Bu.layer_time(c, 0, 8) == 1.5 and Bu.layer_time(c, 0, 2) == 1.0
    assert Bu.layer_time(c, 0, 6) == pytest.approx(1.25) and Bu.layer_time(c, 0, 20) == pytest.approx(3.0)
    assert Bu.layer_time(c, 0, 64) == pytest.approx(9.0)
    assert Bu.valid_num_samples(64, 2) == [8, 16, 24, 32, 48] and Bu.valid_num_samples(8, 2) == []


@pytest.mark.parametrize("seed", range(10))
def test_ffc_lists_exactly_the_candidates_of_its_definition(seed):
    # every vector of layer counts for all but the last ready component that fits, each completed by the
    # largest count of the last component that still fits
    rng = random.Random(seed)
    n = rng.randint(1, 3)
    comps = []
    for _ in range(n):
        L = rng.randint(1, 4)
        comps.append(linear_component(L, [rng.uniform(0.02, 0.2) for _ in range(L)]))
    st = Bu.FillState(64, [0] * n, [64] * n)
    d, t_b = rng.choice([1, 2, 4]), rng.uniform(1.0, 12.0)
    got = Bu.ffc(comps, st, list(range(n)), t_b, d, 0)
    tl = lambda i, j: Bu.layer_time(comps[i], j, math.ceil(64 / d))
    want = []
    for head in itertools.product(*[range(c.n_layers, -1, -1) for c in comps[:-1]]):
        # FFC only descends into counts that fit when taken alone after the earlier components
        used, ok = 0.0, True
        for i, k in enumerate(head):
            for j in range(k):
                used += tl(i, j)
            if used > t_b + 1e-12:
                ok = False
                break
        if not ok:
            continue
        k_last, t = 0, used
        while k_last < comps[-1].n_layers and t + tl(n - 1, k_last) <= t_b:
            t += tl(n - 1, k_last)
            k_last += 1
        want.append(list(head) + [k_last])
    assert sorted(got) == sorted(want)


def test_fill_one_worked_example():
    # one component, three layers of 4 ms at local batch 16 (0.25 ms per sample), batch 32 on 2 idle devices,
    # bubble 10 ms: two whole layers (8 ms) and, of layer 2, the largest regular slice that fits the remaining
    # 2 ms: 16 samples (local 8, 2 ms); 24 samples (3 ms) would overrun
    c = linear_component(3, [0.25, 0.25, 0.25])
    st = Bu.FillState(32, [0], [32])
    k, partial, t = Bu.fill_one([c], st, [0], 10.0, 2)
    assert (k, partial, t) == ([2], (0, 2, 16), pytest.approx(10.0))
    # with 9.9 ms only 8 samples fit; with 8.5 ms none does (the smallest regular slice takes 1 ms)
    assert Bu.fill_one([c], st, [0], 9.9, 2)[1] == (0, 2, 8)
    assert Bu.fill_one([c], st, [0], 8.5, 2)[1:] == (None, pytest.approx(8.0))


def test_fill_all_continues_partial_layers_and_respects_dependencies():
    enc = linear_component(3, [0.25, 0.25, 0.25])
    dep = linear_component(2, [0.1, 0.1], deps=(0,))
    bubbles = [Bu.Bubble(0, 10, (1,), 2), Bu.Bubble(20, 23, (0,), 2), Bu.Bubble(30, 40, (0, 1), 4)]
    res = Bu.fill_all(bubbles, [enc, dep], 32, 4)
    # bubble 0: layers 0, 1 whole + 16 samples of layer 2; bubble 1 (3 ms): the remaining 16 samples of layer 2 at
    # local batch 8 take 2 ms -> whole; the dependent component only becomes ready for bubble 2
    assert res.fills[0].full == [(0, 0, 2, 32)] and res.fills[0].partial == (0, 2, 16)
    assert res.fills[1].full == [(0, 2, 1, 16)] and res.fills[1].partial is None and res.fills[1].time_ms == pytest.approx(2.0)
    assert res.fills[2].full == [(1, 0, 2, 32)] and res.fills[2].time_ms == pytest.approx(2 * 0.1 * 8)
    assert res.leftover_ms == 0.0
    assert res.bubble_device_ms == pytest.approx(10 * 2 + 3 * 2 + 10 * 4)
    assert res.filled_device_ms == pytest.approx(10 * 2 + 2 * 2 + 1.6 * 4)


@pytest.mark.parametrize("seed", range(15))
def test_fill_all_conservation_and_limits(seed):
    rng = random.Random(seed)
    n = rng.randint(1, 3)
    comps = []
    for i in range(n):
        L = rng.randint(1, 5)
        comps.append(Bu.Component(L, {b: [rng.uniform(0.01, 0.08) * b + 0.05 for _ in range(L)] for b in (4, 8, 16, 32, 64, 96)},
                                  tuple(j for j in range(i) if rng.random() < 0.4)))
    batch = rng.choice([64, 96, 128])
    bubbles, t = [], 0.0
    for _ in range(rng.randint(1, 8)):
        t += rng.uniform(1, 5)
        ln = rng.uniform(0.5, 12)
        bubbles.append(Bu.Bubble(t, t + ln, (0,), rng.choice([1, 2, 4])))
        t += ln
    res = Bu.fill_all(bubbles, comps, batch, 4)
    seen = {(i, l): 0 for i, c in enumerate(comps) for l in range(c.n_layers)}
    finished_at = {}
    for f in res.fills:
        b = bubbles[f.bubble]
        assert f.time_ms <= (b.end - b.start) * (1 + 1e-12)
        for i, first, cnt, first_samples in f.full:
            for l in range(first, first + cnt):
                assert all(finished_at.get(j, 10**9) < f.bubble for j in comps[i].deps)        # dependencies complete in earlier bubbles
                assert all(seen[(i, q)] == batch for q in range(l))                             # layers in order
                seen[(i, l)] += first_samples if l == first else batch
            if first + cnt == comps[i].n_layers:
                finished_at[i] = f.bubble
        if f.partial:
            i, l, s = f.partial
            assert s % b.devices == 0 and s // b.devices in Bu.REGULAR_LOCAL_BATCHES and seen[(i, l)] + s < batch
            assert all(seen[(i, q)] == batch for q in range(l))
            seen[(i, l)] += s
    assert all(v <= batch for v in seen.values())
    # what was not placed is exactly what the leftover accounts for
    assert (res.leftover_ms == 0.0) == all(v == batch for v in seen.values())
    assert res.filled_device_ms <= res.bubble_device_ms * (1 + 1e-12)
