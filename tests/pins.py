"""Pins of the CPU oracle: checks against what the paper prints and what the mathematics fixes.

Every function takes an ``oracle.Oracle`` and raises AssertionError when that oracle is
wrong.  They are run on the committed oracle (must pass) and on deliberately broken copies
of its source (each copy must be rejected by at least one pin).
"""
import os

import numpy as np

import workloads
from bruteforce_np import (case1_np, closest_key_np, closest_np, count_np, instances_np, select_np, tiered_np,
                           workers_np)

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
I32MAX = 2**31 - 1


def _both(o, *args):
    """Run the grouped and the literal form; they must agree; return the result."""
    a = o.select(*args)
    b = o.select_literal(*args)
    assert np.array_equal(a, b), "grouped and literal oracle disagree"
    return a


def _read_worked_example():
    names, lat_ms, cost, cases = [], [], [], []
    with open(os.path.join(GOLDEN, "tables_2_3_worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = line.split()
            if w[0] == "variant":
                names.append(w[1]); lat_ms.append(int(w[2])); cost.append(int(w[3]))
            elif w[0] == "case":
                cases.append((int(w[1]), w[2]))
    return names, lat_ms, cost, cases


def pin_worked_example(o):
    """Tables 2/3 of Section 2.2: SLO 300 ms -> variant A, SLO 50 ms -> variant B."""
    names, lat_ms, cost, cases = _read_worked_example()
    V = len(names)
    task = np.zeros(V, np.int32)
    acc = np.full(V, 7600, np.int32)             # same model, same accuracy
    lat = (np.array(lat_ms, np.int32) * 1000).reshape(V, 1)
    cst = np.array(cost, np.int32).reshape(V, 1)
    queue = np.zeros(V, np.int32)
    for slo_ms, want in cases:
        got = _both(o, task, acc, lat, cst, queue, [0], [slo_ms * 1000], [7000], [0])
        assert got[0] == names.index(want), (slo_ms, want, got)
    # the printed rows stay true whatever order the three variants are registered in
    for perm in ([2, 1, 0], [1, 2, 0], [2, 0, 1]):
        p = np.array(perm)
        for slo_ms, want in cases:
            got = _both(o, task, acc, lat[p], cst[p], queue, [0], [slo_ms * 1000], [7000], [0])
            assert p[got[0]] == names.index(want)


def pin_worked_example_consequences(o):
    """Consequences of the same rule on the same three variants (not printed values)."""
    names, lat_ms, cost, _ = _read_worked_example()
    V = len(names)
    task = np.zeros(V, np.int32)
    acc = np.full(V, 7600, np.int32)
    lat = (np.array(lat_ms, np.int32) * 1000).reshape(V, 1)
    cst = np.array(cost, np.int32).reshape(V, 1)
    zero = np.zeros(V, np.int32)
    assert _both(o, task, acc, lat, cst, zero, [0], [17000], [0], [0])[0] == 2     # only C fits
    assert _both(o, task, acc, lat, cst, zero, [0], [10000], [0], [0])[0] == -1    # nothing fits
    busy = np.array([150000, 0, 0], np.int32)   # A is queued behind 150 ms of work
    assert _both(o, task, acc, lat, cst, busy, [0], [300000], [0], [0])[0] == 1    # 350 ms > SLO
    busy = np.array([100000, 0, 0], np.int32)   # exactly 300 ms still fits
    assert _both(o, task, acc, lat, cst, busy, [0], [300000], [0], [0])[0] == 0
    assert _both(o, task, acc, lat, cst, zero, [0], [300000], [7601], [0])[0] == -1  # accuracy


def _tiny_random(rng, V, T, B, N, span):
    task = rng.integers(0, T, V).astype(np.int32)
    acc = rng.integers(0, span, V).astype(np.int32)
    lat = rng.integers(0, span, (V, B)).astype(np.int32)
    cost = rng.integers(0, span, (V, B)).astype(np.int32)
    queue = rng.integers(0, span, V).astype(np.int32)
    qt = rng.integers(-1, T + 1, N).astype(np.int32)
    qs = rng.integers(-1, 2 * span, N).astype(np.int32)
    qa = rng.integers(-1, span + 1, N).astype(np.int32)
    qb = rng.integers(-1, B + 1, N).astype(np.int32)
    return (task, acc, lat, cost, queue), (qt, qs, qa, qb)


def pin_numpy_enumerator(o):
    """Tiny tables with small value ranges (many ties) against the numpy enumerator."""
    rng = np.random.default_rng(7)
    for trial in range(40):
        V = int(rng.integers(1, 65)); T = int(rng.integers(1, 6)); B = int(rng.integers(1, 5))
        span = int(rng.choice([2, 3, 5, 9, 50]))
        tab, qry = _tiny_random(rng, V, T, B, 300, span)
        want = select_np(*tab, *qry)
        got = _both(o, *tab, *qry)
        assert np.array_equal(got, want), f"trial {trial}"
        cnt = o.count_feasible(tab[0], tab[1], tab[2], tab[4], *qry)
        assert np.array_equal(cnt, count_np(tab[0], tab[1], tab[2], tab[4], *qry))
        assert np.array_equal(cnt == 0, got == -1)


def check_invariants(table, queries, out):
    """Properties every correct answer has; usable at any size (vectorised)."""
    task_id = table[0].astype(np.int64); acc = table[1].astype(np.int64)
    lat = table[2].astype(np.int64); cost = table[3].astype(np.int64)
    queue = table[4].astype(np.int64)
    qt, qs, qa, qb = (np.asarray(x).astype(np.int64) for x in queries)
    out = np.asarray(out).astype(np.int64)
    V, B = lat.shape
    hit = out >= 0
    assert np.all(out[hit] < V)
    v = out[hit]; b = qb[hit]
    assert np.all((b >= 0) & (b < B))
    assert np.all(task_id[v] == qt[hit]), "answer from another task"
    assert np.all(acc[v] >= qa[hit]), "answer misses the accuracy minimum"
    assert np.all(lat[v, b] + queue[v] <= qs[hit]), "answer misses the latency objective"


def pin_invariants_tiny_config(o):
    """Config 0: feasibility of every answer; optimality and -1 <=> empty set via counting."""
    tb = workloads.make_table(0)
    q = workloads.make_queries(0)
    table = (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    queries = (q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
    out = _both(o, *table, *queries)
    check_invariants(table, queries, out)
    # no feasible variant of the task has a smaller key: full check, row by row
    lat = tb.lat_us.astype(np.int64); cost = tb.cost.astype(np.int64)
    tot = lat + tb.queue_us.astype(np.int64)[:, None]
    n_empty = 0
    for i in range(q.N):
        b = q.batch_idx[i]
        ok = (tb.task_id == q.task[i]) & (tb.acc_bp >= q.min_acc_bp[i]) & (tot[:, b] <= q.slo_us[i])
        if out[i] < 0:
            assert not ok.any()
            n_empty += 1
            continue
        assert ok[out[i]]
        w = out[i]
        rows = np.flatnonzero(ok)
        smaller = (cost[rows, b] < cost[w, b]) | \
                  ((cost[rows, b] == cost[w, b]) & (lat[rows, b] < lat[w, b])) | \
                  ((cost[rows, b] == cost[w, b]) & (lat[rows, b] == lat[w, b]) & (rows < w))
        assert not smaller.any()
    assert 0 < n_empty < q.N, "config 0 should have both outcomes"


def pin_all_feasible_is_lexsort(o):
    """With SLO = INT32_MAX and no accuracy floor the answer is the first row of a
    lexicographic sort of each (task, batch) slice: a library routine."""
    tb = workloads.make_table(0)
    T, B = tb.num_tasks, tb.B
    qt, qb = np.meshgrid(np.arange(T), np.arange(B), indexing="ij")
    qt = qt.ravel().astype(np.int32); qb = qb.ravel().astype(np.int32)
    n = qt.size
    queue = np.zeros(tb.V, np.int32)
    out = _both(o, tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, queue, qt,
                np.full(n, I32MAX, np.int32), np.full(n, -I32MAX, np.int32), qb)
    for i in range(n):
        rows = np.flatnonzero(tb.task_id == qt[i])
        order = np.lexsort((rows, tb.lat_us[rows, qb[i]], tb.cost[rows, qb[i]]))
        assert out[i] == rows[order[0]]


def pin_boundaries_and_ties(o):
    """Equality is feasible on both tests; tie order is cost, then profiled latency, then row."""
    task = np.zeros(4, np.int32)
    acc = np.array([7000, 7000, 7000, 7000], np.int32)
    lat = np.array([[100], [100], [100], [100]], np.int32)
    cost = np.array([[5], [5], [5], [5]], np.int32)
    queue = np.array([50, 50, 50, 50], np.int32)
    sel = lambda *a: _both(o, *a)
    # accuracy exactly at the minimum, latency exactly at the objective
    assert sel(task, acc, lat, cost, queue, [0], [150], [7000], [0])[0] == 0
    assert sel(task, acc, lat, cost, queue, [0], [149], [7000], [0])[0] == -1
    assert sel(task, acc, lat, cost, queue, [0], [150], [7001], [0])[0] == -1
    # all keys equal -> lowest row; make row 2 cheaper -> row 2
    c2 = cost.copy(); c2[2, 0] = 4
    assert sel(task, acc, lat, c2, queue, [0], [1000], [0], [0])[0] == 2
    # equal cost, row 3 has the lower PROFILED latency but the larger total (big queue):
    # the tie goes by profiled latency, not by latency plus queue
    l3 = lat.copy(); l3[3, 0] = 90
    q3 = queue.copy(); q3[3] = 500
    assert sel(task, acc, l3, cost, q3, [0], [1000], [0], [0])[0] == 3
    # cost dominates latency: a cheaper, slower variant wins over a dearer, faster one
    l4 = np.array([[900], [10], [10], [10]], np.int32)
    c4 = np.array([[1], [2], [2], [2]], np.int32)
    assert sel(task, acc, l4, c4, queue, [0], [1000], [0], [0])[0] == 0
    assert sel(task, acc, l4, c4, queue, [0], [100], [0], [0])[0] == 1
    # rows of a task need not be adjacent and the row tie-break is the caller's row number
    task2 = np.array([1, 0, 1, 0], np.int32)
    assert sel(task2, acc, lat, cost, queue, [0, 1], [1000, 1000], [0, 0], [0, 0]).tolist() == [1, 0]
    # the answer is the highest-accuracy-agnostic cheapest: accuracy above the floor does not matter
    acc5 = np.array([9000, 7000, 8000, 7500], np.int32)
    c5 = np.array([[9], [1], [3], [2]], np.int32)
    assert sel(task, acc5, lat, c5, queue, [0] * 4, [1000] * 4, [6000, 7001, 7501, 8001],
               [0] * 4).tolist() == [1, 3, 2, 0]


def pin_batch_column(o):
    """The batch index picks the column of BOTH profiles; latency and cost are not interchangeable."""
    task = np.zeros(2, np.int32)
    acc = np.full(2, 8000, np.int32)
    lat = np.array([[10, 500], [400, 20]], np.int32)
    cost = np.array([[7, 1], [2, 9]], np.int32)
    queue = np.zeros(2, np.int32)
    out = _both(o, task, acc, lat, cost, queue, [0, 0, 0, 0], [1000, 1000, 100, 100], [0] * 4,
                [0, 1, 0, 1])
    assert out.tolist() == [1, 0, 0, 1]
    out = _both(o, task, acc, lat, cost, queue, [0, 0, 0], [1000] * 3, [0] * 3, [-1, 2, 1])
    assert out.tolist() == [-1, -1, 0]
    # unknown task, negative task, task with no variants
    task3 = np.array([0, 2], np.int32)
    out = _both(o, task3, acc, lat, cost, queue, [1, 3, -1, 2], [1000] * 4, [0] * 4, [0] * 4)
    assert out.tolist() == [-1, -1, -1, 1]


def pin_no_wraparound(o):
    """lat + queue is an exact sum: two large int32 values must not wrap into feasibility."""
    task = np.zeros(2, np.int32)
    acc = np.full(2, 8000, np.int32)
    lat = np.array([[I32MAX], [I32MAX]], np.int32)
    cost = np.array([[1], [2]], np.int32)
    queue = np.array([I32MAX, 0], np.int32)
    out = _both(o, task, acc, lat, cost, queue, [0, 0, 0], [I32MAX, I32MAX - 1, -5], [0] * 3, [0] * 3)
    assert out.tolist() == [1, -1, -1]
    queue2 = np.array([1, 1], np.int32)
    assert _both(o, task, acc, lat, cost, queue2, [0], [I32MAX], [0], [0])[0] == -1


def pin_monotone_and_shift(o):
    """Relaxing a requirement never worsens the winning key; adding d to every queue and to
    the SLO changes nothing."""
    tb = workloads.make_table(0)
    q = workloads.make_queries(0, n=3000)
    table = (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    base = _both(o, *table, q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
    relaxed_slo = _both(o, *table, q.task, q.slo_us + 5000, q.min_acc_bp, q.batch_idx)
    relaxed_acc = _both(o, *table, q.task, q.slo_us, q.min_acc_bp - 300, q.batch_idx)

    def key(out):
        k = np.full((len(out), 3), np.iinfo(np.int64).max, dtype=np.int64)
        hit = out >= 0
        k[hit, 0] = tb.cost[out[hit], q.batch_idx[hit]]
        k[hit, 1] = tb.lat_us[out[hit], q.batch_idx[hit]]
        k[hit, 2] = out[hit]
        return k

    def leq(a, b):  # lexicographic a <= b, row-wise
        lt = np.zeros(len(a), bool); eq = np.ones(len(a), bool)
        for j in range(3):
            lt |= eq & (a[:, j] < b[:, j]); eq &= a[:, j] == b[:, j]
        return lt | eq

    assert leq(key(relaxed_slo), key(base)).all()
    assert leq(key(relaxed_acc), key(base)).all()
    assert (relaxed_slo != base).any() and (relaxed_acc != base).any()
    d = 12345
    shifted = _both(o, tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us + d, q.task,
                    q.slo_us + d, q.min_acc_bp, q.batch_idx)
    assert np.array_equal(shifted, base)


def pin_update_load(o):
    """Updates land on the named rows, in array order, skipping bad rows and negative values."""
    queue = np.array([10, 20, 30, 40], np.int32)
    o.update_load(queue, [2, 0, 2, 7, -1, 1], [300, 100, 301, 9, 9, -5])
    assert queue.tolist() == [100, 20, 301, 40]
    task = np.zeros(4, np.int32); acc = np.full(4, 8000, np.int32)
    lat = np.full((4, 1), 50, np.int32); cost = np.array([[1], [2], [3], [4]], np.int32)
    assert _both(o, task, acc, lat, cost, queue, [0], [100], [0], [0])[0] == 1
    o.update_load(queue, [1], [51])
    assert _both(o, task, acc, lat, cost, queue, [0], [100], [0], [0])[0] == 3
    assert _both(o, task, acc, lat, cost, queue, [0], [89], [0], [0])[0] == -1


ALL_PINS = [
    pin_worked_example,
    pin_worked_example_consequences,
    pin_numpy_enumerator,
    pin_invariants_tiny_config,
    pin_all_feasible_is_lexsort,
    pin_boundaries_and_ties,
    pin_batch_column,
    pin_no_wraparound,
    pin_monotone_and_shift,
    pin_update_load,
]


# ---------------------------------------------------------------- closest variant (Section 4.1, last step)

def _both_closest(o, *args):
    a = o.select_closest(*args)
    b = o.select_closest_literal(*args)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]), "grouped and literal oracle disagree"
    assert np.array_equal(a[0], o.select(*args)), "selection differs between the two entry points"
    return a


def pin_closest_worked_example(o):
    """The three variants of Tables 2/3 (A 200 ms, B 20 ms, C 15 ms; costs 1, 3, 16): consequences
    of the reading, not printed values.  SLO 10 ms: nothing fits, C overshoots least.  Accuracy
    floor above all three with a generous SLO: all miss only the accuracy, by the same amount, so
    the cheapest (A) is suggested.  Both missed by all: least overshoot first (C)."""
    names, lat_ms, cost, _ = _read_worked_example()
    V = len(names)
    task = np.zeros(V, np.int32)
    acc = np.full(V, 7600, np.int32)
    lat = (np.array(lat_ms, np.int32) * 1000).reshape(V, 1)
    cst = np.array(cost, np.int32).reshape(V, 1)
    zero = np.zeros(V, np.int32)
    sel, clo = _both_closest(o, task, acc, lat, cst, zero, [0, 0, 0, 0], [10000, 300000, 10000, 50000],
                             [0, 7700, 7700, 0], [0] * 4)
    assert sel.tolist() == [-1, -1, -1, 1]
    assert clo.tolist() == [2, 0, 2, 1]
    # a slightly more accurate B wins the accuracy-only case over the cheaper A
    acc2 = np.array([7600, 7650, 7600], np.int32)
    assert _both_closest(o, task, acc2, lat, cst, zero, [0], [300000], [7700], [0])[1][0] == 1
    # fitting the latency counts before accuracy shortfall: with SLO 17 ms only C fits, and it is
    # suggested although A and B are equally accurate and cheaper
    assert _both_closest(o, task, acc, lat, cst, zero, [0], [17000], [7700], [0])[1][0] == 2


def pin_closest_numpy(o):
    """Tiny tables with many ties against two numpy formulations (by cases, by sorted key)."""
    rng = np.random.default_rng(11)
    for trial in range(40):
        V = int(rng.integers(1, 65)); T = int(rng.integers(1, 6)); B = int(rng.integers(1, 5))
        span = int(rng.choice([2, 3, 5, 9, 50]))
        tab, qry = _tiny_random(rng, V, T, B, 300, span)
        sel, clo = _both_closest(o, *tab, *qry)
        assert np.array_equal(clo, closest_np(*tab, *qry)), f"trial {trial} (cases)"
        assert np.array_equal(clo, closest_key_np(*tab, *qry)), f"trial {trial} (key)"
        assert np.array_equal(sel, select_np(*tab, *qry))


def pin_closest_structure(o):
    """Config 0: the suggestion equals the selection wherever one exists; it is -1 exactly for
    queries outside the table; it belongs to the query's task; and when nothing is feasible it
    misses no more requirements than any other variant of the task."""
    tb = workloads.make_table(0)
    q = workloads.make_queries(0)
    table = (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    qt = q.task.copy(); qb = q.batch_idx.copy()
    qt[:50] = tb.num_tasks + 3; qb[50:100] = -1           # some queries outside the table
    sel, clo = _both_closest(o, *table, qt, q.slo_us, q.min_acc_bp, qb)
    hit = sel >= 0
    assert np.array_equal(clo[hit], sel[hit])
    outside = (qt < 0) | (qt >= tb.num_tasks) | (qb < 0) | (qb >= tb.B)
    assert np.array_equal(clo < 0, outside)
    inside = ~outside
    assert np.all(tb.task_id[clo[inside]] == qt[inside])
    tot = tb.lat_us.astype(np.int64) + tb.queue_us.astype(np.int64)[:, None]
    n_none = 0
    for i in np.flatnonzero(inside & ~hit)[:400]:
        rows = np.flatnonzero(tb.task_id == qt[i])
        missed = (tot[rows, qb[i]] > q.slo_us[i]).astype(int) + (tb.acc_bp[rows] < q.min_acc_bp[i])
        w = clo[i]
        mw = int(tot[w, qb[i]] > q.slo_us[i]) + int(tb.acc_bp[w] < q.min_acc_bp[i])
        assert mw == missed.min() and mw >= 1
        n_none += 1
    assert n_none > 50


def pin_closest_no_wraparound(o):
    """Overshoot and shortfall are exact differences: extreme int32 values must not wrap."""
    lo = -2**31
    task = np.zeros(3, np.int32)
    acc = np.array([lo, 0, I32MAX], np.int32)
    lat = np.array([[I32MAX], [I32MAX], [10]], np.int32)
    cost = np.array([[1], [1], [1]], np.int32)
    queue = np.array([I32MAX, 0, I32MAX], np.int32)
    # slo = INT32_MIN: overshoots are 2^32+2^31-2, 2^32-1 and 2^31+2^31+9: row 1 is closest
    sel, clo = _both_closest(o, task, acc, lat, cost, queue, [0], [lo], [lo], [0])
    assert sel[0] == -1 and clo[0] == 1
    # all fit (slo max is below two of the totals, so only row 1 fits): accuracy shortfall from INT32_MAX
    sel, clo = _both_closest(o, task, acc, lat, cost, queue, [0], [I32MAX], [I32MAX], [0])
    assert sel[0] == -1 and clo[0] == 1          # only row 1 fits the latency; it misses accuracy by 2^31-1
    # an overshoot of 2^32 + 4 must not look like 4: row 1 (overshoot 110) is closer
    lat3 = np.array([[I32MAX], [100], [I32MAX]], np.int32)
    queue3 = np.array([I32MAX - 4, 0, I32MAX], np.int32)
    sel, clo = _both_closest(o, task, np.zeros(3, np.int32), lat3, cost, queue3, [0], [-10], [0], [0])
    assert sel[0] == -1 and clo[0] == 1
    lat2 = np.array([[5], [6], [2000000000]], np.int32)
    zero = np.zeros(3, np.int32)
    sel, clo = _both_closest(o, task, acc, lat2, cost, zero, [0], [100], [I32MAX - 1], [0])
    assert sel[0] == -1 and clo[0] == 1          # rows 0, 1 fit; shortfalls 2^32-2 and 2^31-2
    sel, clo = _both_closest(o, task, acc, lat2, cost, zero, [0], [2], [I32MAX], [0])
    assert sel[0] == -1 and clo[0] == 2          # nothing fits, row 2 is accurate: it wins despite its overshoot


CLOSEST_PINS = [
    pin_closest_worked_example,
    pin_closest_numpy,
    pin_closest_structure,
    pin_closest_no_wraparound,
]


# ---------------------------------------------------------------- state-aware selection (Sections 4 and 4.1)

def _both_tiered(o, *args):
    a = o.select_tiered(*args)
    b = o.select_tiered(*args, literal=True)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]), "grouped and literal oracle disagree"
    return a


def pin_tiered_numpy(o):
    """Tiny tables with ties against the numpy enumerator."""
    rng = np.random.default_rng(13)
    for trial in range(40):
        V = int(rng.integers(1, 65)); T = int(rng.integers(1, 6)); B = int(rng.integers(1, 5))
        span = int(rng.choice([2, 3, 5, 9, 50]))
        tab, qry = _tiny_random(rng, V, T, B, 300, span)
        state = rng.integers(-1, 6, V).astype(np.int32)          # codes outside 0..3 are never selected
        load = rng.integers(0, span, V).astype(np.int32)
        got = _both_tiered(o, *tab, state, load, *qry)
        want = tiered_np(*tab, state, load, *qry)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]), f"trial {trial}"


def pin_tiered_reduces_to_plain(o):
    """Two special cases that reduce to the plain selection, which is pinned on its own:
    every variant Active -> exactly the plain selection; every variant Inactive -> the plain
    selection on the table with cost := load + lat, queue := load (same filter, same order)."""
    tb = workloads.make_table(0)
    q = workloads.make_queries(0, n=4000)
    st = workloads.make_states(0, tb.V)
    table = (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    queries = (q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
    got, tier = _both_tiered(o, *table, np.ones(tb.V, np.int32), st.load_us, *queries)
    plain = o.select(*table, *queries)
    assert np.array_equal(got, plain) and np.array_equal(tier, (plain >= 0).astype(np.int32))
    got, tier = _both_tiered(o, *table, np.zeros(tb.V, np.int32), st.load_us, *queries)
    combined = (tb.lat_us.astype(np.int64) + st.load_us.astype(np.int64)[:, None]).astype(np.int32)
    plain2 = o.select(tb.task_id, tb.acc_bp, tb.lat_us, combined, st.load_us, *queries)
    assert np.array_equal(got, plain2) and np.array_equal(tier, 2 * (plain2 >= 0).astype(np.int32))
    assert (plain2 >= 0).sum() > 100 and (plain2 < 0).sum() > 100


def pin_tiered_policy(o):
    """Hand-built cases: an Active match wins over a cheaper and faster Inactive one; Overloaded and
    Interfered variants are never chosen; the Inactive tier ignores the queue, charges the loading
    latency against the objective, and orders by load + latency, then latency, then row."""
    task = np.zeros(5, np.int32)
    acc = np.full(5, 8000, np.int32)
    lat = np.array([[100], [10], [10], [10], [50]], np.int32)
    cost = np.array([[9], [1], [1], [1], [1]], np.int32)
    queue = np.array([0, 0, 0, 0, 900], np.int32)
    load = np.array([0, 20, 0, 0, 40], np.int32)
    sel = lambda state, slo, amin=0: tuple(x[0] for x in _both_tiered(
        o, task, acc, lat, cost, queue, np.array(state, np.int32), load, [0], [slo], [amin], [0]))
    assert sel([1, 0, 2, 3, 0], 1000) == (0, 1)          # the Active one, although dearest and slowest
    assert sel([1, 0, 2, 3, 0], 99) == (1, 2)            # Active misses the bound: best Inactive (30 us combined)
    assert sel([2, 0, 2, 3, 0], 1000) == (1, 2)          # Overloaded / Interfered rows 0, 2, 3 are skipped
    assert sel([3, 2, 2, 3, 0], 1000) == (4, 2)          # row 4: queue 900 does not count, load 40 + lat 50 does
    assert sel([3, 2, 2, 3, 0], 89) == (-1, 0)           # 90 us combined misses an objective of 89
    assert sel([3, 2, 2, 3, 0], 90) == (4, 2)
    assert sel([0, 0, 0, 0, 0], 1000) == (2, 2)          # combined 100, 30, 10, 10, 90: rows 2, 3 tie -> lower row
    assert sel([0, 0, 2, 0, 0], 1000) == (3, 2)
    assert sel([0, 0, 0, 0, 0], 1000, 8001) == (-1, 0)   # accuracy applies to both tiers
    lat2 = np.array([[10], [20], [15], [15], [50]], np.int32)
    load2 = np.array([20, 10, 15, 15, 40], np.int32)     # all combine to 30: the lower inference latency first
    got = _both_tiered(o, task, acc, lat2, cost, queue, np.zeros(5, np.int32), load2, [0], [1000], [0], [0])
    assert (got[0][0], got[1][0]) == (0, 2)
    # no wrap in load + lat
    big = np.array([[I32MAX]] * 5, np.int32)
    got = _both_tiered(o, task, acc, big, cost, queue, np.zeros(5, np.int32), np.full(5, I32MAX, np.int32),
                       [0], [I32MAX], [0], [0])
    assert got[0][0] == -1


def pin_update_state(o):
    st = np.array([0, 1, 2, 3], np.int32)
    o.update_state(st, [3, 0, 9, -1, 1, 3], [1, 2, 1, 1, 7, 0])
    assert st.tolist() == [2, 1, 2, 0]


def _both_case1(o, *args):
    a = o.select_case1(*args)
    b = o.select_case1(*args, literal=True)
    assert all(np.array_equal(x, y) for x, y in zip(a, b)), "grouped and literal oracle disagree"
    return a


def pin_case1_numpy(o):
    """Tiny tables with ties and all state codes against the numpy enumerator."""
    rng = np.random.default_rng(29)
    for trial in range(40):
        V = int(rng.integers(1, 65)); T = int(rng.integers(1, 6)); B = int(rng.integers(1, 5))
        span = int(rng.choice([2, 3, 5, 9, 50]))
        tab, qry = _tiny_random(rng, V, T, B, 300, span)
        state = rng.integers(-1, 6, V).astype(np.int32)
        load = rng.integers(0, span, V).astype(np.int32)
        got = _both_case1(o, *tab, state, load, *qry)
        want = case1_np(*tab, state, load, *qry)
        for g, w, name in zip(got, want, ("variant", "tier", "suggestion")):
            assert np.array_equal(g, w), f"trial {trial}: {name}"


def pin_case1_reductions(o):
    """Reductions to routines that are pinned on their own: variant and tier are those of the
    state-aware selection; the suggestion equals the variant wherever one was selected; with
    every variant Active it is the plain closest-variant suggestion; with every variant Inactive
    it is that of the table with cost := load + lat and queue := load."""
    tb = workloads.make_table(0)
    q = workloads.make_queries(0, n=4000)
    st = workloads.make_states(0, tb.V)
    table = (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    queries = (q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
    var, tier, sug = _both_case1(o, *table, st.state, st.load_us, *queries)
    var2, tier2 = o.select_tiered(*table, st.state, st.load_us, *queries)
    assert np.array_equal(var, var2) and np.array_equal(tier, tier2)
    assert np.array_equal(sug[var >= 0], var[var >= 0]) and (var < 0).sum() > 100
    ok = (st.state == 0) | (st.state == 1)
    assert ok[sug[sug >= 0]].all() and (tb.task_id[sug[sug >= 0]] == q.task[sug >= 0]).all()
    _, _, sug_a = _both_case1(o, *table, np.ones(tb.V, np.int32), st.load_us, *queries)
    assert np.array_equal(sug_a, o.select_closest(*table, *queries)[1])
    _, _, sug_i = _both_case1(o, *table, np.zeros(tb.V, np.int32), st.load_us, *queries)
    combined = (tb.lat_us.astype(np.int64) + st.load_us.astype(np.int64)[:, None]).astype(np.int32)
    assert np.array_equal(sug_i, o.select_closest(tb.task_id, tb.acc_bp, tb.lat_us, combined, st.load_us, *queries)[1])


def pin_case1_policy(o):
    """Hand-built cases for the last step: Overloaded and Interfered variants are never suggested;
    an Active variant is measured with its queue (not its loading latency), an Inactive one with
    its loading latency (not its queue); fewer missed requirements first, then the smaller
    overshoot, then the smaller shortfall, then Active before Inactive, then the tier's own order;
    -1 only without an Active or Inactive variant; no 32-bit wrap in the differences."""
    task = np.zeros(6, np.int32)
    acc = np.array([9000, 7000, 9500, 7500, 9000, 9000], np.int32)
    lat = np.array([[100], [100], [10], [100], [100], [100]], np.int32)
    cost = np.array([[5], [1], [1], [9], [9], [1]], np.int32)
    queue = np.array([50, 999, 0, 999, 999, 50], np.int32)     # Active rows 0, 5 take 150 us; row 2 would fit anything
    load = np.array([999, 30, 0, 30, 50, 999], np.int32)       # Inactive rows 1, 3 take 130 us, row 4 150 us
    one = lambda state, slo, amin, bidx=0: tuple(int(x[0]) for x in _both_case1(
        o, task, acc, lat, cost, queue, np.array(state, np.int32), load, [0], [slo], [amin], [bidx]))
    X, Y = 2, 3
    assert one([1, 0, X, Y, Y, Y], 120, 9200) == (-1, 0, 1)   # rows 0 and 1 miss both: overshoot 10 (row 1) against 30
    assert one([1, 0, X, Y, Y, Y], 140, 9200) == (-1, 0, 1)   # row 1 misses one requirement, row 0 two
    assert one([1, 0, X, Y, Y, Y], 140, 8000) == (-1, 0, 1)   # one each: no overshoot (row 1) before no shortfall (row 0)
    assert one([X, 0, X, 0, Y, Y], 100, 8000) == (-1, 0, 3)   # equal overshoot: shortfall 500 (row 3) against 1000 (row 1)
    assert one([1, Y, X, Y, 0, Y], 100, 9500) == (-1, 0, 0)   # rows 0 and 4 equally far: the Active one
    assert one([1, Y, X, Y, 0, 1], 100, 9500) == (-1, 0, 5)   # two Active ones equally far: the cheaper
    assert one([0, Y, X, Y, 0, Y], 100, 9500) == (-1, 0, 4)   # row 0 Inactive: its loading latency counts now
    assert one([X, Y, X, Y, Y, X], 100, 9500) == (-1, 0, -1)  # nothing that may be selected at all
    assert one([1, 0, 1, 0, 0, 1], 100, 9500, bidx=1) == (-1, 0, -1)
    assert one([1, 0, 1, 0, 0, 1], 1000, 0) == (2, 1, 2)      # where a variant is selected it is the suggestion
    assert one([X, 0, X, 0, 0, Y], 1000, 7200) == (3, 2, 3)
    big = np.array([[I32MAX], [I32MAX]], np.int32)
    got = _both_case1(o, [0, 0], [5, 5], big, [[1], [1]], [0, 0], [0, 0], [I32MAX, 0], [0], [0], [0], [0])
    assert int(got[2][0]) == 1                                 # 2 * I32MAX must not wrap to a small overshoot
    got = _both_case1(o, [0, 0], [I32MAX, 0], [[1], [1]], [[1], [1]], [0, 0], [1, 1], [0, 0], [0], [5], [-I32MAX - 1], [0])
    assert int(got[0][0]) == 0                                 # an accuracy bound of INT32_MIN is met by everything


TIERED_PINS = [
    pin_tiered_numpy,
    pin_tiered_reduces_to_plain,
    pin_tiered_policy,
    pin_update_state,
]

CASE1_PINS = [
    pin_case1_numpy,
    pin_case1_reductions,
    pin_case1_policy,
]



# ---- worker selection (Section 4.1: the second output of Case I) ----------------------------------

def _both_workers(o, *args):
    a = o.select_workers(*args)
    b = o.select_workers(*args, literal=True)
    for x, y in zip(a, b):
        assert np.array_equal(x, y), "grouped and literal oracle disagree"
    return a


def _tiny_cluster(rng, V, span):
    W = int(rng.integers(1, 12)); H = int(rng.integers(1, 4)); I = int(rng.integers(0, 4 * V + 1))
    variant_hw = rng.integers(0, H + 1, V).astype(np.int32)      # class H: no worker has it
    worker_hw = rng.integers(0, H, W).astype(np.int32)
    worker_util = rng.integers(0, span, W).astype(np.int32)
    inst_variant = rng.integers(0, V, I).astype(np.int32)
    inst_worker = rng.integers(0, W, I).astype(np.int32)
    inst_load = rng.integers(0, span, I).astype(np.int32)
    return variant_hw, worker_hw, worker_util, inst_variant, inst_worker, inst_load


def pin_workers_numpy(o):
    """Tiny tables and clusters with ties everywhere against the numpy enumerators; variant and tier
    must be those of the state-aware selection."""
    rng = np.random.default_rng(17)
    for trial in range(40):
        V = int(rng.integers(1, 49)); T = int(rng.integers(1, 5)); B = int(rng.integers(1, 4))
        span = int(rng.choice([2, 3, 5, 50]))
        tab, qry = _tiny_random(rng, V, T, B, 300, span)
        state = rng.integers(0, 4, V).astype(np.int32)
        load = rng.integers(0, span, V).astype(np.int32)
        cl = _tiny_cluster(rng, V, span)
        got = _both_workers(o, *tab, state, load, *cl, *qry)
        want = tiered_np(*tab, state, load, *qry)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]), f"trial {trial}"
        assert np.array_equal(got[2], workers_np(want[0], want[1], *cl)), f"trial {trial}"


def pin_workers_policy(o):
    """Hand-built cases on one task with an Active row 0 (hardware 0), an Inactive row 1 (hardware
    1) and an Inactive row 2 (hardware 2, which no worker has)."""
    task = np.zeros(3, np.int32); acc = np.array([8000, 9000, 9500], np.int32)
    lat = np.array([[10], [10], [10]], np.int32); cost = np.array([[1], [1], [1]], np.int32)
    queue = np.zeros(3, np.int32); load = np.zeros(3, np.int32)
    state = np.array([1, 0, 0], np.int32)
    vhw = np.array([0, 1, 2], np.int32)
    whw = np.array([0, 0, 1, 1, 0, 1], np.int32)
    util = np.array([50, 10, 70, 30, 10, 30], np.int32)

    def run(min_acc, iv, iw, il, state=state, util=util, slo=1000):
        r = _both_workers(o, task, acc, lat, cost, queue, state, load, vhw, whw, util,
                          np.array(iv, np.int32), np.array(iw, np.int32), np.array(il, np.int32),
                          [0], [slo], [min_acc], [0])
        return tuple(int(x[0]) for x in r)

    inst = ([0, 0, 0], [0, 1, 4], [5, 3, 9])
    assert run(8000, *inst) == (0, 1, 1)                    # Active: instance load 3 on worker 1 is the least
    assert run(8000, [0], [4], [999]) == (0, 1, 4)          # a single instance: its worker, whatever its load
    assert run(8000, [0, 0, 0], [4, 0, 1], [3, 3, 3]) == (0, 1, 0)    # equal loads: the lowest worker number
    assert run(8000, [0, 0, 0], [1, 0, 4], [3, 3, 2]) == (0, 1, 4)    # ...but load comes first
    assert run(8000, [0, 0], [0, 1], [7, 2], util=np.array([0, 9999, 0, 0, 0, 0], np.int32)) == (0, 1, 1)  # utilisation is not looked at for an Active variant
    assert run(8000, [1, 2, 1], [0, 1, 4], [0, 0, 0]) == (0, 1, -1)   # instances of other variants only: no worker
    assert run(8000, [], [], []) == (0, 1, -1)
    # Inactive row 1 (hardware 1: workers 2, 3, 5 with utilisation 70, 30, 30): worker 3; instances do not matter
    assert run(8500, *inst) == (1, 2, 3)
    assert run(8500, [1, 1], [2, 5], [0, 0]) == (1, 2, 3)
    assert run(8500, *inst, util=np.array([0, 0, 20, 30, 0, 30], np.int32)) == (1, 2, 2)
    assert run(8500, *inst, util=np.array([0, 0, 31, 31, 0, 30], np.int32)) == (1, 2, 5)
    assert run(9200, *inst) == (2, 2, -1)                   # hardware 2: nobody has it; variant and tier stand
    assert run(9600, *inst) == (-1, 0, -1)
    assert run(8000, *inst, slo=5) == (-1, 0, -1)
    # instance arguments outside the tables are rejected
    for bad in (([3], [0], [0]), ([0], [6], [0]), ([-1], [0], [0]), ([0], [-1], [0])):
        try:
            run(8000, *bad)
        except ValueError:
            continue
        raise AssertionError("instance outside the tables accepted")


def pin_workers_structure(o):
    """Config 0 with its seeded cluster: the worker depends on (variant, tier) only; an Active
    answer's worker runs an instance of it and no instance of it has a smaller (load, worker); an
    Inactive answer's worker has the variant's hardware and no such worker is less utilised; the
    result does not change when the instance list is reordered or all loads are doubled."""
    tb = workloads.make_table(0); st = workloads.make_states(0, tb.V); wk = workloads.make_workers(0, st)
    q = workloads.make_queries(0, n=6000)
    table = (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us, st.state, st.load_us)
    queries = (q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
    cl = (wk.variant_hw, wk.worker_hw, wk.worker_util, wk.inst_variant, wk.inst_worker, wk.inst_load)
    v, t, w = _both_workers(o, *table, *cl, *queries)
    plain = o.select_tiered(*table, *queries)
    assert np.array_equal(v, plain[0]) and np.array_equal(t, plain[1])
    assert (t == 1).sum() > 500 and (t == 2).sum() > 500 and (t == 0).sum() > 100
    assert np.all(w[t == 0] == -1)
    seen = {}
    for i in range(len(v)):
        assert seen.setdefault((int(v[i]), int(t[i])), int(w[i])) == int(w[i])
    for i in np.flatnonzero(t == 1)[:400]:
        mine = np.flatnonzero(wk.inst_variant == v[i])
        assert mine.size and w[i] in wk.inst_worker[mine]
        best = min((int(wk.inst_load[j]), int(wk.inst_worker[j])) for j in mine)
        assert best[1] == w[i]
    for i in np.flatnonzero(t == 2)[:400]:
        hw = wk.variant_hw[v[i]]
        assert wk.worker_hw[w[i]] == hw
        cand = np.flatnonzero(wk.worker_hw == hw)
        assert (int(wk.worker_util[w[i]]), int(w[i])) == min((int(wk.worker_util[c]), int(c)) for c in cand)
    perm = np.random.default_rng(3).permutation(wk.I)
    again = _both_workers(o, *table, wk.variant_hw, wk.worker_hw, wk.worker_util, wk.inst_variant[perm],
                          wk.inst_worker[perm], wk.inst_load[perm], *queries)
    assert np.array_equal(again[2], w)
    again = _both_workers(o, *table, wk.variant_hw, wk.worker_hw, 2 * wk.worker_util, wk.inst_variant,
                          wk.inst_worker, 2 * wk.inst_load, *queries)
    assert np.array_equal(again[2], w)


def pin_worker_reports(o):
    util = np.array([5, 6, 7], np.int32)
    o.update_worker_util(util, [2, 0, 3, -1, 1, 2], [1, 9, 4, 4, -1, 8])
    assert util.tolist() == [9, 6, 8]
    load = np.array([5, 6, 7, 8], np.int32)
    o.update_instance_load(load, [3, 3, 4, 0, -2, 1], [1, 2, 9, -5, 3, 0])
    assert load.tolist() == [5, 0, 7, 2]


WORKER_PINS = [
    pin_workers_numpy,
    pin_workers_policy,
    pin_workers_structure,
    pin_worker_reports,
]


# ---- state per running instance (Section 4: the state machine is kept per variant instance) --------

def _both_instances(o, *args):
    a = o.select_instances(*args)
    b = o.select_instances(*args, literal=True)
    for x, y in zip(a, b):
        assert np.array_equal(x, y), "grouped and literal oracle disagree"
    return a


def pin_instances_numpy(o):
    """Tiny tables and clusters with ties everywhere and all three instance states against the numpy
    enumerator, which never forms a state per variant."""
    rng = np.random.default_rng(23)
    for trial in range(40):
        V = int(rng.integers(1, 33)); T = int(rng.integers(1, 5)); B = int(rng.integers(1, 4))
        span = int(rng.choice([2, 3, 5, 50]))
        tab, qry = _tiny_random(rng, V, T, B, 200, span)
        load = rng.integers(0, span, V).astype(np.int32)
        vhw, whw, util, iv, iw, il = _tiny_cluster(rng, V, span)
        ist = rng.choice([1, 2, 3], iv.size, p=[0.5, 0.3, 0.2]).astype(np.int32)
        got = _both_instances(o, *tab, load, vhw, whw, util, iv, iw, il, ist, *qry)
        want = instances_np(*tab, load, vhw, whw, util, iv, iw, il, ist, *qry)
        for g, w, name in zip(got, want, ("variant", "tier", "worker")):
            assert np.array_equal(g, w), f"trial {trial}: {name}"


def pin_instances_reduction(o):
    """Against the worker selection with a state per variant, which is pinned on its own: the same
    answers when that routine is given the states derived here by numpy and only the Active
    instances; and, with every instance Active, when it is given all of them."""
    tb = workloads.make_table(0); st = workloads.make_states(0, tb.V); wk = workloads.make_workers(0, st)
    q = workloads.make_queries(0, n=6000)
    rng = np.random.default_rng(5)
    ist = rng.choice([1, 2, 3], wk.I, p=[0.6, 0.25, 0.15]).astype(np.int32)
    table = (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    queries = (q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
    got = _both_instances(o, *table, st.load_us, wk.variant_hw, wk.worker_hw, wk.worker_util, wk.inst_variant,
                          wk.inst_worker, wk.inst_load, ist, *queries)
    running = np.bincount(wk.inst_variant, minlength=tb.V)
    serving = np.bincount(wk.inst_variant[ist == 1], minlength=tb.V)
    crowded = np.bincount(wk.inst_variant[ist == 2], minlength=tb.V)
    state = np.where(running == 0, 0, np.where(serving > 0, 1, np.where(crowded > 0, 2, 3))).astype(np.int32)
    assert np.array_equal(o.derive_states(tb.V, wk.inst_variant, ist), state)
    assert all((state == c).sum() > 3 for c in (0, 1, 2, 3))
    keep = ist == 1
    want = o.select_workers(*table, state, st.load_us, wk.variant_hw, wk.worker_hw, wk.worker_util,
                            wk.inst_variant[keep], wk.inst_worker[keep], wk.inst_load[keep], *queries)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
    assert (got[1] == 1).sum() > 300 and (got[1] == 2).sum() > 300
    ones = np.ones(wk.I, np.int32)
    got = _both_instances(o, *table, st.load_us, wk.variant_hw, wk.worker_hw, wk.worker_util, wk.inst_variant,
                          wk.inst_worker, wk.inst_load, ones, *queries)
    want = o.select_workers(*table, np.minimum(running, 1).astype(np.int32), st.load_us, wk.variant_hw, wk.worker_hw,
                            wk.worker_util, wk.inst_variant, wk.inst_worker, wk.inst_load, *queries)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)


def pin_instances_policy(o):
    """Hand-built cases: one task, rows 0..3 of rising accuracy and cost; hardware 0 for all; workers
    0..3 with utilisation 40, 10, 30, 20."""
    task = np.zeros(4, np.int32); acc = np.array([7000, 8000, 9000, 9500], np.int32)
    lat = np.array([[10], [10], [10], [10]], np.int32); cost = np.array([[1], [2], [3], [4]], np.int32)
    queue = np.zeros(4, np.int32); load = np.array([5, 5, 5, 5], np.int32)
    vhw = np.zeros(4, np.int32); whw = np.zeros(4, np.int32); util = np.array([40, 10, 30, 20], np.int32)

    def run(min_acc, iv, iw, il, ist, slo=1000):
        r = _both_instances(o, task, acc, lat, cost, queue, load, vhw, whw, util, np.array(iv, np.int32),
                            np.array(iw, np.int32), np.array(il, np.int32), np.array(ist, np.int32),
                            [0], [slo], [min_acc], [0])
        return tuple(int(x[0]) for x in r)

    # row 0 runs on workers 0 (load 1, Overloaded) and 2 (load 9, Active): selected, served by worker 2
    assert run(7000, [0, 0], [0, 2], [1, 9], [2, 1]) == (0, 1, 2)
    assert run(7000, [0, 0], [0, 2], [1, 9], [3, 1]) == (0, 1, 2)          # the same with an Interfered instance
    assert run(7000, [0, 0], [0, 2], [1, 9], [1, 1]) == (0, 1, 0)          # both Active: the smaller load
    assert run(7000, [0, 0, 0], [3, 2, 1], [4, 4, 4], [1, 1, 2]) == (0, 1, 2)   # equal loads: the lower Active worker
    # row 0's instances are all Overloaded / Interfered: it is not selected at all; rows 1..3 run
    # nowhere, so the second step takes row 1 and the least-utilised worker (1)
    assert run(7000, [0, 0], [0, 2], [1, 9], [2, 3]) == (1, 2, 1)
    assert run(7000, [0], [0], [1], [3]) == (1, 2, 1)
    # ... and when row 0 is the only row accurate enough for nothing else to match: no variant
    assert run(7000, [0, 1, 2, 3], [0, 1, 2, 3], [0, 0, 0, 0], [2, 3, 2, 3]) == (-1, 0, -1)
    # an Active instance of a dearer row beats an idle cheaper row (first step before second)
    assert run(7000, [2], [3], [7], [1]) == (2, 1, 3)
    # a row that runs somewhere is never taken in the second step, whatever the states
    assert run(9200, [3], [0], [0], [2]) == (-1, 0, -1)
    assert run(9200, [2], [0], [0], [2]) == (3, 2, 1)
    # the Active tier needs lat + queue <= slo, the second one load + lat <= slo
    assert run(7000, [0], [1], [0], [1], slo=12) == (0, 1, 1)
    assert run(8000, [0], [1], [0], [1], slo=12) == (-1, 0, -1)
    # states outside Active / Overloaded / Interfered are rejected: a loaded instance is not Inactive
    for bad in (0, 4, -1):
        try:
            run(7000, [0], [0], [0], [bad])
        except ValueError:
            continue
        raise AssertionError("instance state accepted")


def pin_instance_reports(o):
    ist = np.array([1, 1, 2, 3], np.int32)
    o.update_instance_state(ist, [0, 1, 1, 4, -1, 2, 3, 3], [2, 3, 1, 1, 1, 0, 4, 1])
    assert ist.tolist() == [2, 1, 2, 1]     # entry 1: 3 then 1; code 0 and code 4 skipped; indices 4, -1 skipped
    assert o.derive_states(5, [0, 0, 2, 3, 3, 4], [2, 1, 3, 3, 2, 1]).tolist() == [1, 0, 3, 2, 1]


INSTANCE_PINS = [
    pin_instances_numpy,
    pin_instances_reduction,
    pin_instances_policy,
    pin_instance_reports,
]


# ---- scaling decision on a change in load (Section 4.2) --------------------------------------------

def scale_py(arch_id, sat_qps, hw_cost, load_us, lat_us, lam, slack_pct, r_variant, r_instances, r_load,
             r_slo, r_bidx):
    """The decision in Python's unbounded integers, costs as exact fractions times 1,000,000."""
    V, B = np.asarray(lat_us).shape
    out = []
    for cur, n_cur, L, slo, b in zip(*(np.asarray(x).tolist() for x in (r_variant, r_instances, r_load, r_slo, r_bidx))):
        if not (0 <= cur < V and 0 <= b < B and 0 <= n_cur <= 10**6 and 0 <= L <= 10**9):
            out.append((0, -1, 0)); continue
        need = L * slack_pct
        if int(sat_qps[cur]) * n_cur * 100 >= need:
            out.append((0, -1, 0)); continue
        inst = lambda v: -((-need) // (100 * int(sat_qps[v])))
        unit = lambda v: int(hw_cost[v]) * (10**6 + lam * int(load_us[v]))
        options = []   # (cost, order, action, variant, instances); replication first among equals
        if int(lat_us[cur][b]) <= slo:
            d = inst(cur) - n_cur
            options.append((unit(cur) * d, -1, 1, cur, d))
        for u in range(V):
            if u != cur and arch_id[u] == arch_id[cur] and int(lat_us[u][b]) <= slo and sat_qps[u] > sat_qps[cur]:
                options.append((unit(u) * inst(u) - int(hw_cost[cur]) * n_cur * 10**6, u, 2, u, inst(u)))
        out.append(min(options)[2:] if options else (3, -1, 0))
    return tuple(np.array(x, dtype=np.int32) for x in zip(*out)) if out else (np.zeros(0, np.int32),) * 3


def _scaling_example():
    names, lat, qps, cost, alone, decide, down = [], [], [], [], [], [], []
    with open(os.path.join(GOLDEN, "tables_2_3_scaling_example.txt")) as f:
        for line in f:
            p = line.split()
            if not p or p[0].startswith("#"):
                continue
            if p[0] == "variant":
                names.append(p[1]); lat.append(int(p[2]) * 1000); qps.append(int(p[3])); cost.append(int(p[4]))
            elif p[0] == "alone":
                alone.append((int(p[1]), p[2], int(p[3]), int(p[4])))
            elif p[0] in ("decide", "down"):
                (decide if p[0] == "decide" else down).append(
                    (int(p[1]), int(p[2]) * 1000, p[3], int(p[4]), p[5], p[6], int(p[7])))
    return (names, np.array(lat, np.int32)[:, None], np.array(qps, np.int32), np.array(cost, np.int32), alone, decide,
            down)


def pin_scaling_paper_example(o):
    """Instance counts, costs and decisions of the printed example (Tables 2 and 3), in every
    registration order of the three variants.  An instance count is read off a replication from
    zero instances; a cost ratio off the decision between two variants."""
    import itertools
    names, lat, qps, cost, alone, decide, _ = _scaling_example()
    for perm in itertools.permutations(range(3)):
        perm = list(perm)
        row = {names[p]: i for i, p in enumerate(perm)}
        tab = (np.zeros(3, np.int32), qps[perm], cost[perm], np.zeros(3, np.int32), lat[perm])
        for load, name, inst, total in alone:
            a, v, n = o.scale(*tab, 0, 100, [row[name]], [0], [load], [10**9], [0])
            # from nothing, with every latency allowed: replicate unless a faster variant is cheaper
            alone_cost = inst * int(cost[names.index(name)])
            assert alone_cost == total, "fixture inconsistent"
            if a[0] == 1:
                assert (v[0], n[0]) == (row[name], inst), (name, load)
            else:   # an upgrade won: it must be strictly cheaper than the printed cost of replication
                u = perm[v[0]]
                assert a[0] == 2 and int(cost[u]) * int(n[0]) < total
        # the replication counts themselves, with upgrades ruled out by separate architectures
        solo = (np.arange(3, dtype=np.int32),) + tab[1:]
        for load, name, inst, total in alone:
            a, v, n = o.scale(*solo, 0, 100, [row[name]], [0], [load], [10**9], [0])
            assert (a[0], v[0], n[0]) == (1, row[name], inst), (name, load)
        for load, slo, name, running, action, target, inst in decide:
            a, v, n = o.scale(*tab, 0, 100, [row[name]], [running], [load], [slo], [0])
            assert (a[0], v[0], n[0]) == ({"replicate": 1, "upgrade": 2}[action], row[target], inst), (load, slo)


def pin_scaling_python(o):
    """Random small tables (ties in every field, invalid requests) against the enumerator in
    Python integers, with several lambdas and headrooms."""
    rng = np.random.default_rng(19)
    for trial in range(60):
        V = int(rng.integers(1, 40)); B = int(rng.integers(1, 4))
        span = int(rng.choice([2, 4, 9, 1000]))
        arch = rng.integers(0, max(1, V // 6) + 1, V).astype(np.int32)
        qps = rng.integers(1, span + 1, V).astype(np.int32)
        cost = rng.integers(0, span + 1, V).astype(np.int32)
        load = rng.integers(0, 50 * span, V).astype(np.int32)
        lat = rng.integers(1, span + 1, (V, B)).astype(np.int32)
        R = 200
        rv = rng.integers(-1, V + 1, R); rn = rng.integers(-1, 4, R); rl = rng.integers(-1, 12 * span, R)
        rs = rng.integers(0, span + 2, R); rb = rng.integers(-1, B + 1, R)
        lam = int(rng.choice([0, 1, 37, 1000])); slack = int(rng.choice([0, 100, 105, 200]))
        got = o.scale(arch, qps, cost, load, lat, lam, slack, rv, rn, rl, rs, rb)
        want = scale_py(arch, qps, cost, load, lat, lam, slack, rv, rn, rl, rs, rb)
        for g, w in zip(got, want):
            assert np.array_equal(g, w), f"trial {trial}"


def pin_scaling_closed_forms(o):
    """Hand-built cases and limits."""
    one = lambda *a: tuple(int(x[0]) for x in o.scale(*a))
    arch = np.zeros(3, np.int32); lat = np.array([[10], [10], [10]], np.int32)
    qps = np.array([10, 40, 40], np.int32); cost = np.array([5, 30, 30], np.int32); load = np.array([0, 0, 0], np.int32)
    tab = (arch, qps, cost, load, lat)
    req = lambda n, L, slo=100: ([0], [n], [L], [slo], [0])
    # headroom: 2 x 10 qps carry 20 qps at 100% but not at 105%
    assert one(*tab, 0, 100, *req(2, 20)) == (0, -1, 0)
    assert one(*tab, 0, 105, *req(2, 20))[0] != 0
    # lambda = 0: resulting hardware cost decides.  40 qps: 4 x row 0 = 20 against 1 x row 1 = 30 -> replicate 2
    assert one(*tab, 0, 100, *req(2, 40)) == (1, 0, 2)
    # 80 qps: 8 x 5 = 40 against 2 x 30 = 60 -> replicate 6; 41 qps: 5 x 5 = 25 against 2 x 30 = 60
    assert one(*tab, 0, 100, *req(2, 80)) == (1, 0, 6)
    assert one(*tab, 0, 100, *req(2, 41)) == (1, 0, 3)
    # dearer replicas: cost 31 each -> 4 x 31 = 124 against 30: upgrade to the lower of the equal rows 1, 2
    dear = (arch, qps, np.array([31, 30, 30], np.int32), load, lat)
    assert one(*dear, 0, 100, *req(2, 40)) == (2, 1, 1)
    # a tie between replication and upgrade goes to replication: 2 more x 15 = 30 = 30 + 2 x 15 - 2 x 15
    tie = (arch, qps, np.array([15, 60, 60], np.int32), load, lat)
    assert one(*tie, 0, 100, *req(2, 40)) == (1, 0, 2)
    # lambda: loading latency of 1 s doubles the cost of every loaded instance of that variant per unit of lambda
    slow = (arch, qps, np.array([31, 30, 30], np.int32), np.array([0, 10**6, 3 * 10**6], np.int32), lat)
    assert one(*slow, 0, 100, *req(2, 40)) == (2, 1, 1)        # 30 - 62 against 62
    assert one(*slow, 3, 100, *req(2, 40)) == (2, 1, 1)        # 30 x 4 - 62 = 58 against 62
    assert one(*slow, 4, 100, *req(2, 40)) == (1, 0, 2)        # 30 x 5 - 62 = 88 against 62
    # the latency objective binds new instances only: the running variant too slow -> no replication
    late = (arch, qps, cost, load, np.array([[200], [10], [300]], np.int32))
    assert one(*late, 0, 100, *req(2, 40, slo=100)) == (2, 1, 1)
    assert one(*late, 0, 100, *req(2, 40, slo=5)) == (3, -1, 0)
    assert one(*late, 0, 100, *req(2, 40, slo=250)) == (1, 0, 2)
    # upgrades need a strictly higher throughput and the same architecture
    flat = (arch, np.array([10, 10, 9], np.int32), np.array([99, 1, 1], np.int32), load, lat)
    assert one(*flat, 0, 100, *req(1, 40)) == (1, 0, 3)
    other = (np.array([0, 1, 1], np.int32), qps, np.array([99, 1, 1], np.int32), load, lat)
    assert one(*other, 0, 100, *req(1, 40)) == (1, 0, 3)
    # the largest values do not wrap: 10^9 qps on a 1 qps variant at 200% headroom, dearest hardware, lambda 1000
    big = (np.zeros(2, np.int32), np.array([1, 2], np.int32), np.array([2**20, 2**20], np.int32),
           np.array([I32MAX, I32MAX], np.int32), np.array([[1], [1]], np.int32))
    assert one(*big, 1000, 200, [0], [0], [10**9], [1], [0]) == (2, 1, 10**9)
    assert one(*big, 1000, 200, [1], [10**6], [10**9], [1], [0]) == (1, 1, 10**9 - 10**6)
    # an upgrade that costs 2.25 * 10^27 (its low 64 bits read as a negative number) against 2 * 10^15 for replicas
    wrap = (np.zeros(2, np.int32), np.array([1, 2], np.int32), np.array([1, 2**20], np.int32),
            np.array([0, 2147483641], np.int32), np.array([[1], [1]], np.int32))
    assert one(*wrap, 1000, 200, [0], [0], [10**9], [1], [0]) == (1, 0, 2 * 10**9)
    # and the other way round: replicas at 4.5 * 10^27 (low 64 bits negative) against an upgrade at 10^15
    wrap2 = (np.zeros(2, np.int32), np.array([1, 2], np.int32), np.array([2**20, 1], np.int32),
             np.array([2147483641, 0], np.int32), np.array([[1], [1]], np.int32))
    assert one(*wrap2, 1000, 200, [0], [0], [10**9], [1], [0]) == (2, 1, 10**9)
    # out-of-range parameters are rejected, out-of-range requests get no action
    for bad in ((1001, 100), (-1, 100), (0, 201), (0, -1)):
        try:
            o.scale(*tab, *bad, *req(2, 40))
        except ValueError:
            continue
        raise AssertionError("parameters outside their limits accepted")
    assert one(*tab, 0, 100, [0], [10**6 + 1], [40], [100], [0]) == (0, -1, 0)
    assert one(*tab, 0, 100, [0], [1], [10**9 + 1], [100], [0]) == (0, -1, 0)


# ---- scaling down (Section 4.2.2, second algorithm) ---------------------------------------------------

def scale_down_py(arch_id, sat_qps, hw_cost, load_us, lat_us, lam, slack_pct, r_variant, r_instances, r_load,
                  r_slo, r_bidx):
    """The scaling-down decision in Python's unbounded integers: every option with its objective
    (times 1,000,000), the least of them by (objective, keep < remove < downgrade by row)."""
    V, B = np.asarray(lat_us).shape
    out = []
    for cur, n_cur, L, slo, b in zip(*(np.asarray(x).tolist() for x in (r_variant, r_instances, r_load, r_slo, r_bidx))):
        if not (0 <= cur < V and 0 <= b < B and 0 <= n_cur <= 10**6 and 0 <= L <= 10**9):
            out.append((0, -1, 0)); continue
        need = L * slack_pct
        options = [(0, -2, 0, -1, 0)]   # (objective, order, action, variant, instances)
        if n_cur - 1 >= 1 and int(sat_qps[cur]) * (n_cur - 1) * 100 >= need:
            options.append((-int(hw_cost[cur]) * 10**6, -1, 1, cur, 1))
        for u in range(V):
            if u == cur or arch_id[u] != arch_id[cur] or int(lat_us[u][b]) > slo or not hw_cost[u] < hw_cost[cur]:
                continue
            inst = max(1, -((-need) // (100 * int(sat_qps[u]))))
            options.append((int(hw_cost[u]) * inst * (10**6 + lam * int(load_us[u])) - int(hw_cost[cur]) * n_cur * 10**6,
                            u, 2, u, inst))
        out.append(min(options)[2:])
    return tuple(np.array(x, dtype=np.int32) for x in zip(*out)) if out else (np.zeros(0, np.int32),) * 3


def pin_scale_down_paper_example(o):
    """The printed example read from the dear side: from one C at 10 QPS the cheapest configurations
    of Table 3's first two rows (2 x A, resp. 1 x B under 50 ms), in every registration order."""
    import itertools
    names, lat, qps, cost, _, _, down = _scaling_example()
    assert len(down) == 2
    for perm in itertools.permutations(range(3)):
        perm = list(perm)
        row = {names[p]: i for i, p in enumerate(perm)}
        tab = (np.zeros(3, np.int32), qps[perm], cost[perm], np.zeros(3, np.int32), lat[perm])
        for load, slo, name, running, action, target, inst in down:
            a, v, n = o.scale_down(*tab, 0, 100, [row[name]], [running], [load], [slo], [0])
            assert (a[0], v[0], n[0]) == ({"remove": 1, "downgrade": 2}[action], row[target], inst), (load, slo)


def pin_scale_down_python(o):
    """Random small tables (ties in every field, invalid requests) against the enumerator in Python
    integers, with several lambdas and headrooms."""
    rng = np.random.default_rng(23)
    seen = set()
    for trial in range(80):
        V = int(rng.integers(1, 40)); B = int(rng.integers(1, 4))
        span = int(rng.choice([2, 4, 9, 1000]))
        arch = rng.integers(0, max(1, V // 6) + 1, V).astype(np.int32)
        qps = rng.integers(1, span + 1, V).astype(np.int32)
        cost = rng.integers(0, span + 1, V).astype(np.int32)
        load = rng.integers(0, 50 * span, V).astype(np.int32)
        lat = rng.integers(1, span + 1, (V, B)).astype(np.int32)
        R = 200
        rv = rng.integers(-1, V + 1, R); rn = rng.integers(-1, 6, R); rl = rng.integers(-1, 6 * span, R)
        rs = rng.integers(0, span + 2, R); rb = rng.integers(-1, B + 1, R)
        lam = int(rng.choice([0, 1, 37, 1000])); slack = int(rng.choice([0, 100, 105, 200]))
        got = o.scale_down(arch, qps, cost, load, lat, lam, slack, rv, rn, rl, rs, rb)
        want = scale_down_py(arch, qps, cost, load, lat, lam, slack, rv, rn, rl, rs, rb)
        for g, w in zip(got, want):
            assert np.array_equal(g, w), f"trial {trial}"
        seen |= set(want[0].tolist())
    assert seen == {0, 1, 2}


def pin_scale_down_closed_forms(o):
    """Hand-built cases and limits."""
    one = lambda *a: tuple(int(x[0]) for x in o.scale_down(*a))
    arch = np.zeros(3, np.int32); lat = np.array([[10], [10], [10]], np.int32)
    qps = np.array([40, 10, 10], np.int32); cost = np.array([30, 5, 5], np.int32); load = np.array([0, 0, 0], np.int32)
    tab = (arch, qps, cost, load, lat)
    req = lambda n, L, slo=100, cur=0: ([cur], [n], [L], [slo], [0])
    # 3 x 40 qps at 90 = 3 x 30; 80 qps: two carry it at 100% (remove: -30) but 8 x 5 = 40 - 90 = -50: downgrade, lower row
    assert one(*tab, 0, 100, *req(3, 80)) == (2, 1, 8)
    # 120 qps: nothing can go (2 x 40 < 120), 12 x 5 = 60 < 90: downgrade; 121 qps: 13 x 5 = 65
    assert one(*tab, 0, 100, *req(3, 120)) == (2, 1, 12)
    assert one(*tab, 0, 100, *req(3, 121)) == (2, 1, 13)
    # without the cheap rows (other architecture): 80 qps -> remove one; 81 qps -> keep (2 x 40 < 81)
    solo = (np.array([0, 1, 1], np.int32), qps, cost, load, lat)
    assert one(*solo, 0, 100, *req(3, 80)) == (1, 0, 1)
    assert one(*solo, 0, 100, *req(3, 81)) == (0, -1, 0)
    # headroom: two carry 80 qps at 100% but not at 105%
    assert one(*solo, 0, 105, *req(3, 80)) == (0, -1, 0)
    assert one(*solo, 0, 105, *req(3, 76)) == (1, 0, 1)
    # the last instance stays, also without load; a downgrade keeps one instance serving
    assert one(*solo, 0, 100, *req(1, 0)) == (0, -1, 0)
    assert one(*solo, 0, 100, *req(2, 0)) == (1, 0, 1)
    assert one(*tab, 0, 100, *req(1, 0)) == (2, 1, 1)           # 5 - 30
    assert one(*tab, 0, 100, *req(0, 0)) == (0, -1, 0)          # nothing runs: nothing to gain
    # ties: a downgrade that saves exactly what a removal saves loses to it (2 x 30 -> 30 against 6 x 5 = 30)
    assert one(*tab, 0, 100, *req(2, 40)) == (2, 1, 4)          # 20 - 60 against -30
    tie = (arch, qps, np.array([30, 10, 10], np.int32), load, lat)
    assert one(*tie, 0, 100, *req(2, 30)) == (1, 0, 1)          # 3 x 10 - 60 = -30 = -30
    assert one(*tie, 0, 100, *req(2, 20)) == (2, 1, 2)          # 2 x 10 - 60 = -40
    # a switch that gains nothing is not made: 6 x 5 = 30 = 1 x 30
    assert one(*tab, 0, 100, *req(1, 60)) == (0, -1, 0)
    assert one(*tab, 0, 100, *req(1, 50)) == (2, 1, 5)
    # cheaper means a lower hardware cost per instance, not a lower total: equal cost is no downgrade
    same = (arch, np.array([10, 40, 40], np.int32), np.array([30, 30, 29], np.int32), load, lat)
    assert one(*same, 0, 100, *req(4, 40)) == (2, 2, 1)          # row 1 costs the same per instance: only row 2
    # lambda: a loading latency of 1 s adds one hardware cost per loaded instance and unit of lambda
    slow = (arch, qps, cost, np.array([0, 10**6, 3 * 10**6], np.int32), lat)
    assert one(*slow, 0, 100, *req(3, 120)) == (2, 1, 12)       # 60 - 90
    assert one(*slow, 1, 100, *req(3, 120)) == (0, -1, 0)       # 120 - 90 > 0 and 240 - 90 > 0
    assert one(*slow, 1, 100, *req(3, 80)) == (1, 0, 1)         # 80 - 90 = -10 against -30
    assert one(*slow, 1, 100, *req(3, 40)) == (2, 1, 4)         # 40 - 90 = -50 against -30
    # the latency objective binds the downgrade's instances, not the ones that stay
    late = (arch, qps, cost, load, np.array([[300], [200], [10]], np.int32))
    assert one(*late, 0, 100, *req(3, 80, slo=100)) == (2, 2, 8)
    assert one(*late, 0, 100, *req(3, 80, slo=5)) == (1, 0, 1)
    assert one(*late, 0, 100, *req(3, 120, slo=5)) == (0, -1, 0)
    # the batch-size column of the request
    two = (arch, qps, cost, load, np.array([[10, 10], [10, 500], [500, 10]], np.int32))
    assert tuple(int(x[0]) for x in o.scale_down(*two, 0, 100, [0], [3], [120], [100], [1])) == (2, 2, 12)
    # the largest values do not wrap: 10^9 qps at 200% on a 1 qps variant, lambda 1000, longest loading latency
    big = (np.zeros(2, np.int32), np.array([2, 1], np.int32), np.array([2**20, 2**20 - 1], np.int32),
           np.array([I32MAX, I32MAX], np.int32), np.array([[1], [1]], np.int32))
    assert one(*big, 0, 200, [0], [10**6], [10**9], [1], [0]) == (0, -1, 0)       # 2*10^9 dearer ones against 10^6
    assert one(*big, 0, 200, [0], [10**6], [10**5], [1], [0]) == (2, 1, 2 * 10**5)
    assert one(*big, 1000, 200, [0], [10**6], [10**5], [1], [0]) == (1, 0, 1)    # loading makes the switch dearer
    # an objective of 4.5 * 10^27 whose low 64 bits read as a negative number
    wrap = (np.zeros(2, np.int32), np.array([2, 1], np.int32), np.array([2**20, 2**20 - 1], np.int32),
            np.array([0, 2147483641], np.int32), np.array([[1], [1]], np.int32))
    assert one(*wrap, 1000, 200, [0], [1], [10**9], [1], [0]) == (0, -1, 0)
    for bad in ((1001, 100), (-1, 100), (0, 201), (0, -1)):
        try:
            o.scale_down(*tab, *bad, *req(2, 40))
        except ValueError:
            continue
        raise AssertionError("parameters outside their limits accepted")
    assert one(*tab, 0, 100, [0], [10**6 + 1], [40], [100], [0]) == (0, -1, 0)
    assert one(*tab, 0, 100, [0], [3], [10**9 + 1], [100], [0]) == (0, -1, 0)


SCALING_PINS = [
    pin_scaling_paper_example,
    pin_scaling_python,
    pin_scaling_closed_forms,
]

SCALE_DOWN_PINS = [
    pin_scale_down_paper_example,
    pin_scale_down_python,
    pin_scale_down_closed_forms,
]
