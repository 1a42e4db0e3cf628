"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle.

All fields are integers, so the bar is bit-exact equality on every query, at every size: the
full-size configurations too are compared element by element (the oracle answers configuration
2's 16M queries in seconds on the host's cores), the streaming configuration on eight of its 64
chunks in full and on a sample of every other chunk.  Where the lookup kernel has slower paths
(second group of steps, slices outside LDS, rank-ordered scan, no feasible variant) the tests
also check, from the library's own counters, that the run reached them.
"""
import numpy as np
import pytest

import workloads
from gpu_util import gpu_select, make_selector, query_args, table_args, to_dev
from pins import check_invariants

pytestmark = pytest.mark.gpu

ENGINES = [0, 1, 2]  # auto (index if it fits in LDS, else scan), scan only, index always
ENGINE_IDS = ["auto", "scan", "index"]
I32MAX = 2**31 - 1


def _say(msg):
    print(msg, flush=True)


def _table(num_tasks, batch_sizes, task_id, acc, lat, cost, queue):
    return workloads.VariantTable(num_tasks=num_tasks, batch_sizes=np.asarray(batch_sizes, np.int32),
                                  task_id=np.asarray(task_id, np.int32), acc_bp=np.asarray(acc, np.int32),
                                  lat_us=np.asarray(lat, np.int32), cost=np.asarray(cost, np.int32),
                                  queue_us=np.asarray(queue, np.int32))


def _random_table(rng, T, sizes, B, span=None):
    """Table with given segment sizes; small `span` forces ties everywhere."""
    V = int(np.sum(sizes))
    task = np.repeat(np.arange(T, dtype=np.int32), sizes)
    if span is None:
        acc, lat, cost, queue = workloads.configs.make_variant_fields(
            rng, V, np.asarray([1, 2, 4, 8, 16, 32, 64, 128][:B], np.int32))
    else:
        acc = rng.integers(0, span, V); lat = rng.integers(0, span, (V, B))
        cost = rng.integers(0, span, (V, B)); queue = rng.integers(0, span, V)
    perm = rng.permutation(V)
    return _table(T, list(range(1, B + 1)), task[perm], acc, lat, cost, queue)


def _random_queries(rng, T, B, n, span=None, with_invalid=True):
    lo = -1 if with_invalid else 0
    task = rng.integers(lo, T + (1 if with_invalid else 0), n)
    bidx = rng.integers(lo, B + (1 if with_invalid else 0), n)
    if span is None:
        slo = np.clip(np.rint(rng.lognormal(np.log(20000.0), 1.0, n)), 1000, 2_000_000)
        acc = rng.integers(5000, 9501, n)
        if with_invalid:
            slo[rng.random(n) < 0.01] = -7
    else:
        slo = rng.integers(lo, 2 * span, n); acc = rng.integers(lo, span + 1, n)
    return tuple(np.asarray(x, np.int32) for x in (task, slo, acc, bidx))


def _compare(oracle_lib, tb, queries, engine, lds_limit=0, label=""):
    _say(f"case {label}: V={tb.V} T={tb.num_tasks} B={tb.B} N={len(queries[0])} engine={engine} "
         f"lds_limit={lds_limit}")
    sel = make_selector(tb, engine=engine, lds_segment_limit=lds_limit)
    got = gpu_select(sel, *queries)
    want = oracle_lib.select(*table_args(tb), *queries)
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, f"{label}: {bad.size} mismatches, first at {bad[:5]}: got {got[bad[:5]]} want {want[bad[:5]]}"
    sel.destroy()
    return got


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_config0_tiny_exact(oracle_lib, engine):
    tb = workloads.make_table(0)
    q = workloads.make_queries(0)
    _compare(oracle_lib, tb, query_args(q), engine, label="config0")


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_config1_medium_exact(oracle_lib, engine):
    """Config 1 at its full 1M queries: 200-variant segments, several tiles and a ragged tail."""
    tb = workloads.make_table(1)
    q = workloads.make_queries(1, n=1_000_003 if engine != 1 else 300_007)
    _compare(oracle_lib, tb, query_args(q), engine, label="config1")


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_ties_and_invalid_queries(oracle_lib, engine):
    """Small value ranges: many equal costs and latencies, so the row tie-break decides;
    queries include unknown tasks, bad batch indices and negative objectives."""
    rng = np.random.default_rng(11)
    for trial in range(6):
        T = int(rng.integers(1, 9)); B = int(rng.integers(1, 6))
        sizes = rng.integers(0, 70, T)
        span = int(rng.choice([2, 3, 7, 40]))
        tb = _random_table(rng, T, sizes, B, span=span)
        qs = _random_queries(rng, T, B, 5000, span=span)
        _compare(oracle_lib, tb, qs, engine, label=f"ties{trial}")


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
@pytest.mark.parametrize("lds_limit", [64, 128])
def test_wide_path_small_limit(oracle_lib, engine, lds_limit):
    """A low LDS limit sends config 1's 200-variant segments through the device-wide path
    (chunks of 64: three full chunks and a ragged one)."""
    tb = workloads.make_table(1)
    q = workloads.make_queries(1, n=100_000)
    _compare(oracle_lib, tb, query_args(q), engine, lds_limit=lds_limit, label="wide-small")


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_segment_sizes_around_the_limit_and_maximum(oracle_lib, engine):
    """Segments of 1, limit-1, limit, limit+1 variants and one of 20,000 (the largest a task
    may have in the skewed configuration), with an empty task in between."""
    rng = np.random.default_rng(5)
    sizes = np.array([1, 4095, 4096, 4097, 0, 20000, 3, 257], dtype=np.int64)
    tb = _random_table(rng, len(sizes), sizes, 8)
    qs = _random_queries(rng, len(sizes), 8, 60_000)
    got = _compare(oracle_lib, tb, qs, engine, label="limits")
    assert (got[qs[0] == 4] == -1).all()


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_degenerate_inputs(oracle_lib, engine):
    import torch
    import paper_1905_13348_amd as lib
    rng = np.random.default_rng(3)
    # all infeasible / all feasible / all ties
    tb = _random_table(rng, 3, np.array([50, 50, 50]), 2, span=5)
    n = 3000
    task = rng.integers(0, 3, n).astype(np.int32); bidx = rng.integers(0, 2, n).astype(np.int32)
    for slo, acc in ((np.full(n, 0), np.full(n, 100)), (np.full(n, I32MAX), np.full(n, -I32MAX - 1)),
                     (np.full(n, 4), np.full(n, 2))):
        _compare(oracle_lib, tb, (task, slo.astype(np.int32), acc.astype(np.int32), bidx), engine,
                 label="degenerate")
    # empty table and empty query batch
    sel = lib.Selector(4, [1, 2], engine=engine)
    e = np.zeros(0, np.int32)
    sel.load_variants(e, e, np.zeros((0, 2), np.int32), np.zeros((0, 2), np.int32), e)
    got = gpu_select(sel, task[:100] % 4, np.full(100, 5, np.int32), np.zeros(100, np.int32), bidx[:100])
    assert (got == -1).all()
    out = torch.zeros(1, dtype=torch.int32, device="cuda")
    sel.select(out, out, out, out, out, n=0)
    sel.destroy()
    # extreme values: the sum lat + queue must not wrap
    tb = _table(1, [1], [0, 0], [8000, 8000], [[I32MAX], [I32MAX]], [[1], [2]], [I32MAX, 0])
    qs = tuple(np.asarray(x, np.int32) for x in ([0, 0, 0], [I32MAX, I32MAX - 1, -5], [0, 0, 0], [0, 0, 0]))
    _compare(oracle_lib, tb, qs, engine, label="extremes")


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_update_load_then_select(oracle_lib, engine):
    """Load reports between batches: values land on the right rows, bad entries are skipped,
    and the next batch sees the new load (same stream ordering)."""
    import torch
    tb = workloads.make_table(1)
    sel = make_selector(tb, engine=engine)
    queue = tb.queue_us.copy()
    rng = np.random.default_rng(17)
    for step in range(4):
        q = workloads.make_queries(1, n=50_000, seed=900 + step)
        up = workloads.make_load_update(1, tb.V, chunk=step + 1, fraction=0.1)
        idx = up.variant_idx.copy(); val = up.queue_us.copy()
        if step == 2:  # bad entries: skipped by both sides
            idx[:3] = [-1, tb.V, tb.V + 5]; val[3:6] = -1
        _say(f"update step {step}: n={idx.size}")
        sel.update_load(to_dev(idx), to_dev(val))
        oracle_lib.update_load(queue, idx, val)
        got = gpu_select(sel, *query_args(q))
        want = oracle_lib.select(*table_args(tb, queue), *query_args(q))
        assert np.array_equal(got, want), f"step {step}"
        assert np.array_equal(sel.read_load(tb.V), queue)
    sel.destroy()


def _staircase_table(T, n, B=2, acc0=1000, acc_step=1, lat0=100_000):
    """Every variant of a task is a step: cost, accuracy rise and latency falls with the row, so no
    cheaper variant dominates a dearer one.  The staircase of a slice has n entries."""
    task = np.repeat(np.arange(T, dtype=np.int32), n)
    i = np.tile(np.arange(n, dtype=np.int64), T)
    acc = acc0 + acc_step * i
    lat = np.stack([lat0 - 100 * i + 7 * b for b in range(B)], axis=1)
    cost = np.stack([10 + i + b for b in range(B)], axis=1)
    queue = np.zeros(T * n, np.int64)
    return _table(T, list(range(1, B + 1)), task, acc, lat, cost, queue)


def _staircase_queries(rng, tb, n_queries, n, lat0=100_000):
    T, B = tb.num_tasks, tb.B
    task = rng.integers(0, T, n_queries)
    bidx = rng.integers(0, B, n_queries)
    want_row = rng.integers(-3, n + 3, n_queries)           # aim at a given depth of the staircase
    acc = tb.acc_bp.min() + (tb.acc_bp[1] - tb.acc_bp[0]) * want_row
    slo = rng.choice([lat0 + 50, lat0 * 6 // 10, lat0 // 5, lat0 * 99 // 100], n_queries) + rng.integers(-300, 300, n_queries)
    return tuple(np.asarray(x, np.int32) for x in (task, slo, acc, bidx))


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
@pytest.mark.parametrize("steps", [31, 32, 50, 62, 63, 300])
def test_long_staircases(oracle_lib, engine, steps):
    """Slices whose staircase fills one index body exactly (31), needs the second one (32..62), or
    exceeds the index capacity (63, 300: the in-kernel rank-ordered scan must finish the query)."""
    rng = np.random.default_rng(steps)
    tb = _staircase_table(5, steps)
    qs = _staircase_queries(rng, tb, 40_000, steps)
    _compare(oracle_lib, tb, qs, engine, label=f"staircase{steps}")
    if engine != 1:
        sel = make_selector(tb, engine=engine)
        info = sel.info()
        assert info["index_max_steps"] == min(steps, 62)
        assert (info["index_truncated"] > 0) == (steps > 62)
        if engine == 2 or steps <= 62:   # (auto hands a table of truncated slices to the scan engine)
            gpu_select(sel, *qs)
            info = sel.info()
            assert (info["lookup_second_body"] > 0) == (steps > 31)
            assert (info["lookup_scanned"] > 0) == (steps > 62)
        sel.destroy()


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_accuracy_range_too_wide_for_the_index(oracle_lib, engine):
    """Accuracies that span more than 16 bits inside a slice: those slices get no index body and
    every query of theirs is answered by the scan; the other task keeps its index."""
    rng = np.random.default_rng(8)
    wide = _staircase_table(1, 40, acc0=-50_000, acc_step=5_000)       # -50,000 .. 145,000
    narrow = _staircase_table(1, 40)
    tb = _table(2, [1, 2], np.concatenate([wide.task_id, narrow.task_id + 1]),
                np.concatenate([wide.acc_bp, narrow.acc_bp]), np.concatenate([wide.lat_us, narrow.lat_us]),
                np.concatenate([wide.cost, narrow.cost]), np.concatenate([wide.queue_us, narrow.queue_us]))
    n = 30_000
    task = rng.integers(0, 2, n)
    acc = np.where(task == 0, rng.integers(-60_000, 150_000, n), rng.integers(990, 1050, n))
    qs = tuple(np.asarray(x, np.int32) for x in (task, rng.integers(90_000, 101_000, n), acc, rng.integers(0, 2, n)))
    _compare(oracle_lib, tb, qs, engine, label="wide-acc")


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_extreme_accuracies(oracle_lib, engine):
    """The smallest and largest int32 as accuracies, in the table and in the queries: task 0 holds
    a variant at INT32_MIN (the index keeps no key for it, the scan answers its slices), task 1
    spans a narrow range just below INT32_MAX, task 2 a narrow range just above INT32_MIN + 1."""
    rng = np.random.default_rng(77)
    lo, hi = np.iinfo(np.int32).min, np.iinfo(np.int32).max
    a = _staircase_table(1, 20)
    acc0 = a.acc_bp.astype(np.int64).copy(); acc0[:] = lo + 1 + np.arange(20) * 3; acc0[0] = lo
    acc1 = hi - 3 * np.arange(20)[::-1].astype(np.int64)
    acc2 = lo + 1 + 5 * np.arange(20).astype(np.int64)
    tb = _table(3, [1, 2], np.concatenate([a.task_id, a.task_id + 1, a.task_id + 2]),
                np.concatenate([acc0, acc1, acc2]), np.concatenate([a.lat_us] * 3),
                np.concatenate([a.cost] * 3), np.concatenate([a.queue_us] * 3))
    n = 30_000
    task = rng.integers(0, 3, n)
    near_lo = lo + rng.integers(0, 120, n)
    near_hi = hi - rng.integers(0, 80, n)
    acc = np.where(task == 1, np.where(rng.random(n) < 0.8, near_hi, near_lo),
                   np.where(rng.random(n) < 0.8, near_lo, near_hi))
    qs = tuple(np.asarray(x, np.int32) for x in (task, rng.integers(90_000, 101_000, n), acc, rng.integers(0, 2, n)))
    _compare(oracle_lib, tb, qs, engine, label="extreme-acc")


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_rows_scattered_over_a_large_table(oracle_lib, engine):
    """300,000 variants.  Tasks 0-3 own rows spread over the first 200,000 (the first steps of a
    slice lie more than 65,536 rows apart, so the index cannot keep them as 16-bit offsets), tasks
    4-7 own contiguous blocks behind them, two of which start above row 2^18."""
    rng = np.random.default_rng(300)
    V, B = 300_000, 2
    acc, lat, cost, queue = workloads.configs.make_variant_fields(rng, V, np.asarray([1, 8], np.int32))
    task = np.empty(V, np.int32)
    task[:200_000] = rng.integers(0, 4, 200_000)
    task[200_000:] = 4 + np.arange(100_000) // 25_000
    tb = _table(8, [1, 8], task, acc, lat, cost, queue)
    qs = _random_queries(rng, 8, B, 6_000)
    got = _compare(oracle_lib, tb, qs, engine, label="scattered-rows")
    assert (got >= 262_144).any() and ((got >= 0) & (got < 200_000)).any()


def test_index_outgrows_lds_after_load_update(oracle_lib):
    """At load every slice has a one-step staircase (row 0 of each task dominates the rest), so the
    index fits in LDS.  A load report then pushes those rows out of reach: all staircases grow to
    62 steps, the index no longer fits, and the queries of the slices left outside LDS are
    finished from the index copy in global memory."""
    T, n = 700, 62
    tb = _staircase_table(T, n, B=1)
    first = np.arange(T) * n
    tb.acc_bp[first] = 5000          # most accurate ...
    tb.lat_us[first, 0] = 10         # ... and fastest, and it is the cheapest row of its task
    rng = np.random.default_rng(21)
    sel = make_selector(tb, engine=0)
    assert sel.info()["index_in_lds"] == 1 and sel.info()["index_max_steps"] == 1
    qs = _staircase_queries(rng, tb, 200_000, n)
    got = gpu_select(sel, *qs)
    assert np.array_equal(got, oracle_lib.select(*table_args(tb), *qs))
    queue = tb.queue_us.copy()
    idx = first.astype(np.int32); val = np.full(T, 2_000_000_000, np.int32)
    sel.update_load(to_dev(idx), to_dev(val))
    oracle_lib.update_load(queue, idx, val)
    got = gpu_select(sel, *qs)
    want = oracle_lib.select(*table_args(tb, queue), *qs)
    assert np.array_equal(got, want)
    assert (want >= 0).mean() > 0.3 and len(np.unique(want)) > 1000
    sel.destroy()


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_unaligned_query_arrays(oracle_lib, engine):
    """Query and result arrays that start 4 bytes into an allocation (not 16-byte aligned)."""
    import torch
    tb = workloads.make_table(1)
    q = workloads.make_queries(1, n=70_001)
    sel = make_selector(tb, engine=engine)
    dev = [torch.cat([torch.zeros(1, dtype=torch.int32), torch.from_numpy(x)]).cuda()[1:] for x in query_args(q)]
    out = torch.full((q.N + 1,), -7, dtype=torch.int32, device="cuda")[1:]
    assert dev[0].data_ptr() % 16 == 4
    sel.select(*dev, out, n=q.N)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle_lib.select(*table_args(tb), *query_args(q)))
    sel.destroy()


def test_error_codes():
    import torch
    import paper_1905_13348_amd as lib
    with pytest.raises(lib.InfaasSelError) as e:
        lib.Selector(0, [1])
    assert e.value.status == -1
    with pytest.raises(lib.InfaasSelError):
        lib.Selector(2, [1], lds_segment_limit=9)
    sel = lib.Selector(2, [1, 2])
    x = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(lib.InfaasSelError) as e:
        sel.select(x, x, x, x, x)
    assert e.value.status == -2
    one = np.ones(2, np.int32); two = np.ones((2, 2), np.int32)
    for bad in ("task_hi", "task_lo", "lat", "cost", "queue"):
        t, l, c, qu = np.array([0, 1], np.int32), two.copy(), two.copy(), one.copy()
        if bad == "task_hi": t[1] = 2
        if bad == "task_lo": t[0] = -1
        if bad == "lat": l[1, 1] = -1
        if bad == "cost": c[0, 0] = -3
        if bad == "queue": qu[1] = -1
        with pytest.raises(lib.InfaasSelError) as e:
            sel.load_variants(t, one, l, c, qu)
        assert e.value.status == -3, bad
    sel.load_variants(np.array([0, 1], np.int32), one, two, two, one)
    sel.select(x, x, x, x, x)
    torch.cuda.synchronize()
    sel.destroy()
    sel.destroy()


# ------------------------------------------------------------------ full-size configurations

def _sampled_parity(oracle_lib, tb, queue, q, got, sample, rng, label):
    table = table_args(tb, queue)
    check_invariants(table, query_args(q), got)
    pick = rng.choice(q.N, size=min(sample, q.N), replace=False)
    sub = tuple(np.ascontiguousarray(x[pick]) for x in query_args(q))
    want = oracle_lib.select(*table, *sub)
    bad = np.flatnonzero(got[pick] != want)
    assert bad.size == 0, f"{label}: {bad.size} of {pick.size} sampled queries differ"


_FULL = {}   # configuration -> (table, queries, the oracle's answer to every query): shared by the engines


def _full_reference(oracle_lib, cfg):
    if cfg not in _FULL:
        _FULL.clear()   # one configuration at a time (config 3 holds 1.3 GB)
        tb = workloads.make_table(cfg)
        q = workloads.make_queries(cfg)
        _say(f"config{cfg}: oracle over all {q.N} queries ...")
        _FULL[cfg] = (tb, q, oracle_lib.select(*table_args(tb), *query_args(q)))
        _say("... done")
    return _FULL[cfg]


def _assert_equal_everywhere(got, want, label):
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, f"{label}: {bad.size} of {want.size} queries differ, first at {bad[:5]}: " \
                          f"got {got[bad[:5]]} want {want[bad[:5]]}"


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_config2_full_size_every_query(oracle_lib, engine):
    """16M queries, 50 tasks x 2,000 variants, Zipf task popularity -- the benchmark's launch
    configuration.  Every answer is compared with the oracle's."""
    tb, q, want = _full_reference(oracle_lib, 2)
    _say(f"config2 engine={engine}: N={q.N}")
    sel = make_selector(tb, engine=engine)
    got = gpu_select(sel, *query_args(q))
    _assert_equal_everywhere(got, want, "config2")
    assert 0 < int((want < 0).sum()) < q.N // 10          # some queries have no feasible variant
    if engine != 1:
        info = sel.info()
        # staircases of more than 31 steps exist, and queries were decided by their second group
        assert info["index_max_steps"] > 31 and info["lookup_second_body"] > 1000
        assert info["lookup_parked"] >= info["lookup_second_body"] + info["lookup_unanswered"] > 0
        assert info["lookup_global_body"] == 0 and info["lookup_scanned"] == 0   # the whole index is in LDS
    sel.destroy()


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_config3_full_size_every_query(oracle_lib, engine):
    """64M queries over 1,000 tasks with lognormal segment sizes and a bimodal objective; the
    index does not fit in LDS, so most queries are answered from its copy in global memory."""
    tb, q, want = _full_reference(oracle_lib, 3)
    _say(f"config3 engine={engine}: N={q.N} V={tb.V}")
    sel = make_selector(tb, engine=engine)
    got = gpu_select(sel, *query_args(q))
    _assert_equal_everywhere(got, want, "config3")
    assert 0 < int((want < 0).sum()) < q.N
    if engine != 1:
        info = sel.info()
        # the tasks were dealt to groups; the few queries a group's LDS copy cannot decide (second
        # group of steps) were finished from global memory
        assert info["index_groups"] > 4 and info["lookup_parked"] > 0
        assert info["lookup_parked"] >= info["lookup_second_body"] + info["lookup_unanswered"] > 0
        # a batch too small for the group-by-group path takes the one-kernel lookup, where most
        # slices are answered from the copy of the index in global memory
        n = 900_000
        got = gpu_select(sel, *(x[:n] for x in query_args(q)))
        _assert_equal_everywhere(got, want[:n], "config3, one-kernel lookup")
        info = sel.info()
        assert info["lookup_parked"] > n // 2 and info["lookup_global_body"] > n // 10
    sel.destroy()
    if engine == ENGINES[-1]:
        _FULL.clear()


def test_config3_low_limit_forces_wide_path(oracle_lib):
    """Config 3's table with a 256-variant LDS limit: its large segments take the wide path."""
    tb = workloads.make_table(3)
    q = workloads.make_queries(3, n=2_000_000)
    want = None
    for engine in ENGINES:
        sel = make_selector(tb, engine=engine, lds_segment_limit=256)
        assert sel.info()["wide_segments"] > 10
        got = gpu_select(sel, *query_args(q))
        if want is None:
            want = oracle_lib.select(*table_args(tb), *query_args(q))
        _assert_equal_everywhere(got, want, "config3-wide")
        sel.destroy()


def test_config4_streaming_sampled(oracle_lib):
    """256M queries in 64 chunks of 4M; before every chunk after the first, 10% of the variants
    get a new load.  Eight chunks (the first, the last, six in between) are compared with the
    oracle on every query; the others on feasibility of every answer and 20k sampled queries.
    The oracle's copy of the load follows the same updates."""
    import torch
    tb = workloads.make_table(4)
    spec = workloads.config_spec(4)
    sel = make_selector(tb, engine=0)
    queue = tb.queue_us.copy()
    rng = np.random.default_rng(4)
    per_chunk = spec["num_queries"] // spec["chunks"]
    sel.reserve(per_chunk)
    for chunk in range(spec["chunks"]):
        if chunk > 0:
            up = workloads.make_load_update(4, tb.V, chunk)
            sel.update_load(to_dev(up.variant_idx), to_dev(up.queue_us))
            oracle_lib.update_load(queue, up.variant_idx, up.queue_us)
        q = workloads.make_queries(4, chunk=chunk)
        assert q.N == per_chunk
        if chunk % 8 == 0:
            _say(f"config4 chunk {chunk}")
        got = gpu_select(sel, *query_args(q))
        if chunk in (0, 1, 9, 18, 27, 36, 50, 63):
            want = oracle_lib.select(*table_args(tb, queue), *query_args(q))
            _assert_equal_everywhere(got, want, f"config4 chunk {chunk}")
            info = sel.info()
            assert info["lookup_second_body"] > 0 and info["lookup_parked"] > info["lookup_second_body"]
        else:
            _sampled_parity(oracle_lib, tb, queue, q, got, 20_000, rng, f"config4 chunk {chunk}")
    assert np.array_equal(sel.read_load(tb.V), queue)
    sel.destroy()


def test_results_do_not_depend_on_run(oracle_lib):
    """Two runs over the same input give the same bytes (bucket order is not deterministic,
    the answers are)."""
    tb = workloads.make_table(1)
    q = workloads.make_queries(1, n=400_000)
    for engine in ENGINES:
        sel = make_selector(tb, engine=engine)
        a = gpu_select(sel, *query_args(q))
        b = gpu_select(sel, *query_args(q))
        assert np.array_equal(a, b)
        sel.destroy()


def test_more_queries_than_one_pass(oracle_lib):
    """2^28 + 5000 queries in one call: the library splits the call into passes of 2^28.  Queries
    are drawn on the device; those around the seam, at both ends and a random sample are checked
    against the oracle, for the plain call and for the closest-variant call."""
    import torch
    tb = workloads.make_table(0)
    sel = make_selector(tb, engine=0)
    n = (1 << 28) + 5000
    g = torch.Generator(device="cuda"); g.manual_seed(28)
    task = torch.randint(0, tb.num_tasks, (n,), generator=g, device="cuda", dtype=torch.int32)
    slo = torch.randint(1000, 400_000, (n,), generator=g, device="cuda", dtype=torch.int32)
    acc = torch.randint(5000, 9501, (n,), generator=g, device="cuda", dtype=torch.int32)
    bidx = torch.randint(0, tb.B, (n,), generator=g, device="cuda", dtype=torch.int32)
    out = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    seam = 1 << 28
    pick = np.unique(np.concatenate([np.arange(2000), seam - 2000 + np.arange(4000), n - 2000 + np.arange(2000),
                                     np.random.default_rng(1).integers(0, n, 100_000)]))
    pick_d = torch.from_numpy(pick).cuda()
    qs = tuple(x[pick_d].cpu().numpy() for x in (task, slo, acc, bidx))
    want_sel, want_clo = oracle_lib.select_closest(*table_args(tb), *qs)
    sel.select(task, slo, acc, bidx, out)
    torch.cuda.synchronize()
    assert np.array_equal(out[pick_d].cpu().numpy(), want_sel)
    assert int((out == -7).sum()) == 0, "some results were never written"
    clo = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    out.fill_(-7)
    sel.select_closest(task, slo, acc, bidx, out, clo)
    torch.cuda.synchronize()
    assert np.array_equal(out[pick_d].cpu().numpy(), want_sel)
    assert np.array_equal(clo[pick_d].cpu().numpy(), want_clo)
    assert int((clo == -7).sum()) == 0 and int((out == -7).sum()) == 0
    sel.destroy()


def test_few_long_slices_with_reports(oracle_lib):
    """Few slices of thousands of variants each -- the index build that gives every slice a
    workgroup of its own and places the slices in the order of their numbers: segments of more than
    one 2048-entry chunk, one exactly at the chunk's edge, an empty task; the index rebuilt behind
    load reports, every query against the oracle each time."""
    rng = np.random.default_rng(77)
    sizes = np.array([5000, 0, 2500, 4100, 2048, 6000])
    tb = _random_table(rng, 6, sizes, 3)
    qs = _random_queries(rng, 6, 3, 60_000)
    sel = make_selector(tb, engine=2)
    queue = tb.queue_us.copy()
    for rnd in range(4):
        if rnd:
            idx = rng.choice(tb.V, tb.V // 5, replace=False).astype(np.int32)
            val = rng.integers(0, 150_000, idx.size).astype(np.int32)
            sel.update_load(to_dev(idx), to_dev(val))
            oracle_lib.update_load(queue, idx, val)
        got = gpu_select(sel, *qs)
        want = oracle_lib.select(tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, queue, *qs)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"round {rnd}: {bad.size} mismatches, first at {bad[:5]}"
    info = sel.info()
    assert info["index_truncated"] == 0 and 20 <= info["index_max_steps"] <= 62
    sel.destroy()


@pytest.mark.parametrize("engine", [0, 2], ids=["auto", "index"])
def test_few_slices_of_nothing_but_steps(oracle_lib, engine):
    """The same build on slices where every variant is a step (2100 of them, the index keeps 62):
    every slice truncated, the queries finished by the scan."""
    rng = np.random.default_rng(78)
    tb = _staircase_table(3, 2100, B=2, lat0=300_000)
    qs = _staircase_queries(rng, tb, 20_000, 2100, lat0=300_000)
    _compare(oracle_lib, tb, qs, engine, label="staircase2100")
    sel = make_selector(tb, engine=engine)
    info = sel.info()
    assert info["index_truncated"] == 6 and info["index_max_steps"] == 62
    sel.destroy()


def test_512_slices_in_groups(oracle_lib):
    """512 slices of 600 steps each: one workgroup per slice in the build, and bodies (62 steps kept
    per slice, 470 KB) that need groups; a call below and one above the size from which queries are
    binned by group."""
    rng = np.random.default_rng(79)
    tb = _staircase_table(64, 600, B=8)
    sel = make_selector(tb, engine=2)
    info = sel.info()
    assert info["index_groups"] > 1 and info["index_truncated"] == 512
    for n in (50_000, (1 << 20) + 3000):
        qs = _staircase_queries(rng, tb, n, 600)
        got = gpu_select(sel, *qs)
        want = oracle_lib.select(*table_args(tb), *qs)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, f"N={n}: {bad.size} mismatches, first at {bad[:5]}"
    sel.destroy()


@pytest.mark.parametrize("steps", [1, 2, 30, 31, 32, 33, 61, 62, 63])
def test_few_long_slices_with_exact_step_counts(oracle_lib, steps):
    """Slices of 640+ variants (the build with one workgroup per slice, the bodies shared by its four
    wavefronts) whose staircases have exactly `steps` steps: `steps` variants that are steps by
    construction and 640 fillers that the first of them dominates, shuffled through the ranks by
    their cost.  One step, the edges of the first body (31 | 32), of the index (62 | 63)."""
    rng = np.random.default_rng(400 + steps)
    T, B, fill = 2, 2, 640
    n = steps + fill
    task = np.repeat(np.arange(T, dtype=np.int32), n)
    i = np.arange(steps, dtype=np.int64)
    acc1 = np.concatenate([2000 + 10 * i, rng.integers(0, 2000, fill)])              # fillers: less accurate than step 0,
    lat1 = np.concatenate([200_000 - 1000 * i, rng.integers(200_001, 400_000, fill)])  # slower,
    cost1 = np.concatenate([1000 + 50 * i, rng.integers(1001, 1000 + 50 * steps + 500, fill)])  # and dearer than it
    acc = np.tile(acc1, T)
    lat = np.stack([np.tile(lat1, T) + 3 * b for b in range(B)], axis=1)
    cost = np.stack([np.tile(cost1, T) + b for b in range(B)], axis=1)
    tb = _table(T, [1, 2], task, acc, lat, cost, np.zeros(T * n, np.int64))
    nq = 30_000
    want_step = rng.integers(-2, steps + 2, nq)
    qs = (rng.integers(0, T, nq), rng.choice([250_000, 200_000 - 1000 * (steps // 2), 150_000, 199_999], nq) + rng.integers(-1500, 1500, nq),
          2000 + 10 * want_step - rng.integers(0, 2, nq), rng.integers(0, B, nq))
    qs = tuple(np.asarray(x, np.int32) for x in qs)
    for engine in (0, 2):
        _compare(oracle_lib, tb, qs, engine, label=f"{steps} steps among {n}")
    sel = make_selector(tb, engine=2)
    info = sel.info()
    assert info["index_max_steps"] == min(steps, 62) and info["index_truncated"] == (T * B if steps > 62 else 0)
    sel.destroy()
