"""Closest-variant mode of the GPU library (infaas_sel_select_closest) against the CPU oracle:
every element, both outputs.  The suggestion follows the last step of Section 4.1's Case I with
the distance stated in include/infaas_sel.h."""
import numpy as np
import pytest

import workloads
from gpu_util import gpu_select_closest, make_selector, query_args, table_args, to_dev
from test_gpu_parity import _random_queries, _random_table, _staircase_queries, _staircase_table, _table

pytestmark = pytest.mark.gpu

ENGINES = [0, 1, 2]       # auto, scan (suggestions by an exhaustive pass behind the selection), index
ENGINE_IDS = ["auto", "scan", "index"]


def _compare(oracle_lib, tb, queries, engine, label, queue=None, sel=None):
    print(f"closest case {label}: V={tb.V} T={tb.num_tasks} B={tb.B} N={len(queries[0])} engine={engine}", flush=True)
    own = sel is None
    if own:
        sel = make_selector(tb, engine=engine)
    got_sel, got_clo = gpu_select_closest(sel, *queries)
    want_sel, want_clo = oracle_lib.select_closest(*table_args(tb, queue), *queries)
    bad = np.flatnonzero(got_sel != want_sel)
    assert bad.size == 0, f"{label}: selection differs at {bad[:5]}: got {got_sel[bad[:5]]} want {want_sel[bad[:5]]}"
    bad = np.flatnonzero(got_clo != want_clo)
    assert bad.size == 0, (f"{label}: {bad.size} suggestions differ, first at {bad[:5]}: got {got_clo[bad[:5]]} "
                           f"want {want_clo[bad[:5]]} (selection {want_sel[bad[:5]]})")
    if own:
        sel.destroy()
    return want_sel, want_clo


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_closest_config0(oracle_lib, engine):
    tb = workloads.make_table(0)
    s, c = _compare(oracle_lib, tb, query_args(workloads.make_queries(0)), engine, "config0")
    assert (s < 0).mean() > 0.1 and (c >= 0).all()


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_closest_config1(oracle_lib, engine):
    """1M queries; a sixth of the slices lie outside LDS, so the suggestion is also searched in
    the index copy in global memory."""
    tb = workloads.make_table(1)
    _compare(oracle_lib, tb, query_args(workloads.make_queries(1)), engine, "config1")


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_closest_ties_and_invalid_queries(oracle_lib, engine):
    """Tiny value ranges: ties in every component of the order; queries outside the table; tasks
    without variants; negative bounds."""
    rng = np.random.default_rng(5)
    for span in (2, 3, 6, 40):
        sizes = rng.integers(0, 70, 12)
        sizes[3] = 0
        tb = _random_table(rng, 12, sizes, 3, span=span)
        qs = _random_queries(rng, 12, 3, 30_000, span=span)
        _compare(oracle_lib, tb, qs, engine, f"ties span={span}")


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
@pytest.mark.parametrize("steps", [1, 2, 31, 32, 33, 50, 62, 63, 300])
def test_closest_long_staircases(oracle_lib, engine, steps):
    """One body exactly full, two bodies (the offers of both are compared), and more steps than
    the index keeps (the wavefront scans the whole slice).  Queries aim above, inside and below
    the staircase in both dimensions, so all three kinds of suggestion occur."""
    rng = np.random.default_rng(100 + steps)
    tb = _staircase_table(4, steps)
    task, slo, acc, bidx = _staircase_queries(rng, tb, 30_000, steps)
    n = task.size
    slo = np.where(rng.random(n) < 0.3, rng.integers(-5, 200_000, n), slo).astype(np.int32)
    acc = np.where(rng.random(n) < 0.3, rng.integers(0, 3000, n), acc).astype(np.int32)
    s, c = _compare(oracle_lib, tb, (task, slo, acc, bidx), engine, f"staircase{steps}")
    assert (s < 0).mean() > 0.2


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_closest_equal_keys_across_bodies(oracle_lib, engine):
    """40 steps (two bodies) in which groups of steps share their accuracy or their latency, so
    that offers of the two bodies tie and the earlier rank must win."""
    rng = np.random.default_rng(41)
    n, T, B = 40, 3, 2
    task = np.repeat(np.arange(T, dtype=np.int32), n)
    i = np.tile(np.arange(n, dtype=np.int64), T)
    acc = 1000 + 10 * (i // 3)                       # plateaus of three
    lat = np.stack([100_000 - 100 * ((i + 1) // 3) + 7 * b for b in range(B)], axis=1)   # shifted plateaus
    cost = np.stack([10 + i + b for b in range(B)], axis=1)
    tb = _table(T, [1, 2], task, acc, lat, cost, np.zeros(T * n, np.int64))
    N = 40_000
    qs = (rng.integers(0, T, N), rng.integers(95_000, 101_000, N), rng.integers(990, 1150, N), rng.integers(0, B, N))
    qs = tuple(np.asarray(x, np.int32) for x in qs)
    _compare(oracle_lib, tb, qs, engine, "plateaus")


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_closest_after_load_update(oracle_lib, engine):
    tb = workloads.make_table(0)
    q = workloads.make_queries(0)
    sel = make_selector(tb, engine=engine)
    queue = tb.queue_us.copy()
    for chunk in (1, 2):
        up = workloads.make_load_update(4, tb.V, chunk, fraction=0.3) if tb.V >= 1000 else None
        rng = np.random.default_rng(chunk)
        idx = rng.choice(tb.V, tb.V // 3, replace=False).astype(np.int32)
        val = rng.integers(0, 400_000, idx.size).astype(np.int32)
        sel.update_load(to_dev(idx), to_dev(val))
        oracle_lib.update_load(queue, idx, val)
        _compare(oracle_lib, tb, query_args(q), engine, f"update{chunk}", queue=queue, sel=sel)
    sel.destroy()


def test_closest_extreme_values(oracle_lib):
    """Bounds and table values at the ends of int32: differences up to 2^32 must not wrap."""
    lo, hi = np.iinfo(np.int32).min, np.iinfo(np.int32).max
    rng = np.random.default_rng(9)
    n = 24
    task = np.zeros(n, np.int32)
    acc = rng.choice([lo + 1, -5, 0, 7000, hi - 1, hi], n)
    lat = rng.choice([0, 1, 1000, hi // 2, hi - 1, hi], (n, 1))
    queue = rng.choice([0, 5, hi // 2, hi], n)
    cost = rng.integers(0, 5, (n, 1))
    tb = _table(1, [1], task, acc, lat, cost, queue)
    N = 20_000
    qs = (np.zeros(N), rng.choice([lo, -1, 0, 999, hi // 2, hi - 1, hi], N),
          rng.choice([lo, -5, 0, 7001, hi - 1, hi], N), np.zeros(N))
    qs = tuple(np.asarray(x, np.int32) for x in qs)
    _compare(oracle_lib, tb, qs, 0, "extremes")


def test_closest_config2_every_query(oracle_lib):
    """Full 16M-query configuration in the launch shape bench.py times; selection and suggestion of
    every query against the oracle."""
    tb = workloads.make_table(2)
    q = workloads.make_queries(2)
    sel = make_selector(tb, engine=0)
    got_sel, got_clo = gpu_select_closest(sel, *query_args(q))
    print(f"closest config2: oracle over all {q.N} queries", flush=True)
    want_sel, want_clo = oracle_lib.select_closest(*table_args(tb), *query_args(q))
    assert np.array_equal(got_sel, want_sel)
    assert np.array_equal(got_clo, want_clo)
    assert int((want_sel < 0).sum()) > 100_000
    assert np.array_equal(got_clo[got_sel >= 0], got_sel[got_sel >= 0]) and (got_clo >= 0).all()
    sel.destroy()


def test_closest_without_the_index_on_a_wide_slice(oracle_lib):
    """A handle of the scan engine whose largest slice takes the device-wide path of the selection:
    the suggestions still come from the exhaustive pass; unaligned arrays and a ragged count."""
    import torch
    rng = np.random.default_rng(91)
    tb = _random_table(rng, 3, np.array([9000, 40, 700]), 2)
    qs = _random_queries(rng, 3, 2, 50_001)
    sel = make_selector(tb, engine=1, lds_segment_limit=4096)
    want_sel, want_clo = oracle_lib.select_closest(*table_args(tb), *qs)
    dev = [torch.from_numpy(np.concatenate([[0], x]).astype(np.int32)).cuda()[1:] for x in qs]
    out = torch.full((len(qs[0]) + 1,), -9, dtype=torch.int32, device="cuda")[1:]
    clo = torch.full((len(qs[0]) + 1,), -9, dtype=torch.int32, device="cuda")[1:]
    sel.select_closest(*dev, out, clo)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want_sel) and np.array_equal(clo.cpu().numpy(), want_clo)
    assert (want_sel < 0).sum() > 1000
    sel.destroy()
