"""The library's bubble entry points (dp_bubbles_1f1b, dp_bubbles_fill; host code in libdpipe.so)
against the plain-Python oracle on seeded random pipelines and component profiles, plus their argument
checks.  Runs without a GPU: neither entry point makes a GPU call."""
import random

import numpy as np
import pytest

from oracle import bubbles as Bu


@pytest.fixture(scope="module")
def B():
    from paper_2405_01248_amd import binding
    binding.load_library()
    return binding


def random_pipeline(rng):
    S, M = rng.randint(1, 8), rng.randint(1, 12)
    f = [rng.uniform(0.5, 30) for _ in range(S)]
    b = [rng.uniform(0.5, 60) for _ in range(S)]
    cf = [rng.uniform(0, 3) for _ in range(S - 1)]
    cb = [rng.uniform(0, 3) for _ in range(S - 1)]
    tail = [rng.choice([0.0, 2.5]) for _ in range(S)]
    rep = [rng.randint(1, 4) for _ in range(S)]
    return f, b, M, cf, cb, tail, rep


@pytest.mark.parametrize("seed", range(40))
def test_schedule_and_bubbles_match_oracle(B, seed):
    rng = random.Random(seed)
    f, b, M, cf, cb, tail, rep = random_pipeline(rng)
    min_ms = rng.choice([0.0, 1.0, 10.0])
    busy, t = Bu.simulate_1f1b(f, b, M, cf, cb, tail)
    ref = Bu.find_bubbles(busy, t, rep, min_ms)
    got, t_lib = B.bubbles_1f1b(f, b, rep, M, cf or None, cb or None, tail, min_ms)
    assert t_lib == t
    assert [(x["start_ms"], x["end_ms"], x["stages"], x["n_devices"]) for x in got] == [(x.start, x.end, x.stages, x.devices) for x in ref]


def random_components(rng):
    f32 = lambda v: float(np.float32(v))
    n = rng.randint(1, 3)
    comps, rows, deps = [], [], []
    ids = sorted(rng.sample(range(1, 9), n))
    for i, cid in enumerate(ids):
        L = rng.randint(1, 6)
        sizes = sorted(rng.sample([1, 2, 4, 8, 12, 16, 24, 32, 48, 64, 96], rng.randint(2, 8)))
        per = [rng.uniform(0.01, 0.3) for _ in range(L)]
        base = [rng.uniform(0.02, 0.5) for _ in range(L)]
        ms = {s: [f32(base[l] + per[l] * s) for l in range(L)] for s in sizes}
        d = tuple(j for j in range(i) if rng.random() < 0.4)
        comps.append(Bu.Component(L, ms, d))
        deps += [(cid, ids[j]) for j in d]
        for s in sizes:
            for l in range(L):
                rows.append({"component": cid, "layer": l, "batch": s, "fwd_ms": ms[s][l], "bwd_ms": 0.0, "out_bytes": 0, "cf_bytes": 0,
                             "cb_bytes": 0, "grad_bytes": 0})
    rng.shuffle(rows)
    rows.append({"component": 0, "layer": 0, "batch": 8, "fwd_ms": 1.0, "bwd_ms": 2.0, "out_bytes": 0, "cf_bytes": 0, "cb_bytes": 0, "grad_bytes": 0})
    return ids, comps, rows, deps


def oracle_rows(res, ids):
    out = []
    for f in res.fills:
        for i, first, cnt, samples in f.full:
            out.append({"bubble": f.bubble, "component": ids[i], "first_layer": first, "n_layers": cnt, "samples": samples, "partial": 0, "fill_ms": f.time_ms})
        if f.partial:
            h, layer, b = f.partial
            out.append({"bubble": f.bubble, "component": ids[h], "first_layer": layer, "n_layers": 1, "samples": b, "partial": 1, "fill_ms": f.time_ms})
    return out


@pytest.mark.parametrize("seed", range(60))
def test_filling_matches_oracle(B, seed):
    rng = random.Random(1000 + seed)
    f, b, M, cf, cb, tail, rep = random_pipeline(rng)
    busy, t = Bu.simulate_1f1b(f, b, M, cf, cb, tail)
    bub = Bu.find_bubbles(busy, t, rep, rng.choice([0.0, 2.0]))
    ids, comps, rows, deps = random_components(rng)
    batch = rng.choice([32, 64, 96, 128, 256])
    ref = Bu.fill_all(bub, comps, batch, sum(rep))
    lib_bubbles = [{"start_ms": x.start, "end_ms": x.end, "n_devices": x.devices, "stages": x.stages} for x in bub]
    got, summ = B.bubbles_fill(lib_bubbles, rows, batch, sum(rep), deps)
    want = oracle_rows(ref, ids)
    assert [{k: v for k, v in r.items() if k != "fill_ms"} for r in got] == [{k: v for k, v in r.items() if k != "fill_ms"} for r in want]
    for g, w in zip(got, want):
        assert g["fill_ms"] == pytest.approx(w["fill_ms"], rel=1e-12)
    assert summ["bubble_device_ms"] == pytest.approx(ref.bubble_device_ms, rel=1e-12)
    assert summ["filled_device_ms"] == pytest.approx(ref.filled_device_ms, rel=1e-12, abs=1e-12)
    assert summ["leftover_ms"] == pytest.approx(ref.leftover_ms, rel=1e-12, abs=1e-12)


def test_worked_example_through_the_library(B):
    # three layers of 4 ms at local batch 16, batch 32, a 10 ms bubble on 2 devices: two whole layers and 16
    # samples of the third; the next (3 ms) bubble takes the remaining 16 samples
    rows = [{"component": 1, "layer": l, "batch": s, "fwd_ms": 0.25 * s, "bwd_ms": 0.0, "out_bytes": 0, "cf_bytes": 0, "cb_bytes": 0, "grad_bytes": 0}
            for l in range(3) for s in (4, 8, 12, 16)]
    bubbles = [{"start_ms": 0.0, "end_ms": 10.0, "n_devices": 2}, {"start_ms": 20.0, "end_ms": 23.0, "n_devices": 2}]
    got, summ = B.bubbles_fill(bubbles, rows, 32, 4)
    key = lambda r: (r["bubble"], r["first_layer"], r["n_layers"], r["samples"], r["partial"])
    assert [key(r) for r in got] == [(0, 0, 2, 32, 0), (0, 2, 1, 16, 1), (1, 2, 1, 16, 0)]
    assert got[0]["fill_ms"] == pytest.approx(10.0) and got[2]["fill_ms"] == pytest.approx(2.0) and summ["leftover_ms"] == 0.0


def test_bad_arguments_are_rejected(B):
    ok = dict(fwd_ms=[1.0, 1.0], bwd_ms=[2.0, 2.0], replicas=[1, 1], n_micro_batches=2)
    assert len(B.bubbles_1f1b(**ok)[0]) == 4
    for bad in (dict(n_micro_batches=0), dict(replicas=[1, 0]), dict(fwd_ms=[1.0, -1.0]), dict(min_ms=-1.0), dict(comm_fwd_ms=[-0.5]),
                dict(fwd_ms=[float("nan"), 1.0])):
        with pytest.raises(B.DpipeError) as ei:
            B.bubbles_1f1b(**{**ok, **bad})
        assert ei.value.code == -1, bad
    with pytest.raises(B.DpipeError) as ei:                 # too small an output array: count still reported
        B.bubbles_1f1b(**ok, max_out=2)
    assert ei.value.code == -3
    row = {"component": 1, "layer": 0, "batch": 4, "fwd_ms": 1.0, "bwd_ms": 0.0, "out_bytes": 0, "cf_bytes": 0, "cb_bytes": 0, "grad_bytes": 0}
    bub = [{"start_ms": 0.0, "end_ms": 5.0, "n_devices": 2}]
    B.bubbles_fill(bub, [row], 16, 2)
    for rows, kw in (([dict(row, component=0)], {}), ([row, row], {}), ([row, dict(row, layer=2)], {}), ([row], dict(deps=[(1, 2)])),
                     ([row], dict(deps=[(1, 1)])), ([dict(row, fwd_ms=float("nan"))], {})):
        with pytest.raises(B.DpipeError) as ei:
            B.bubbles_fill(bub, rows, 16, 2, **kw)
        assert ei.value.code == -1
    for b_, n_ in ((0, 2), (16, 0)):
        with pytest.raises(B.DpipeError):
            B.bubbles_fill(bub, [row], b_, n_)
    with pytest.raises(B.DpipeError):                       # bubbles out of order
        B.bubbles_fill([{"start_ms": 5.0, "end_ms": 6.0, "n_devices": 1}, {"start_ms": 1.0, "end_ms": 2.0, "n_devices": 1}], [row], 16, 2)
