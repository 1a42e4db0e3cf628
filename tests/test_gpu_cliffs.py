"""Tables and load reports the staircase index handles badly: every variant a possible answer
(thousands of steps per slice, of which the index keeps 62 and scans for the rest), accuracies
beyond the index's 16-bit keys (no index at all), and an index that was fine when the table was
loaded and stops being so after a load report.  Answers never depend on any of this; which engine
a handle created with INFAAS_SEL_ENGINE_AUTO uses does."""
import numpy as np
import pytest

import workloads
from gpu_util import gpu_select, make_selector, query_args, table_args, to_dev
from test_gpu_parity import ENGINE_IDS, ENGINES, _assert_equal_everywhere, _table

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
@pytest.mark.parametrize("kind", ["long_staircases", "wide_accuracy"])
def test_cliff_tables(oracle_lib, engine, kind):
    tb = workloads.make_cliff_table(kind, cfg=1)
    q = workloads.make_queries(1, n=60_000)
    sel = make_selector(tb, engine=engine)
    got = gpu_select(sel, *query_args(q))
    want = oracle_lib.select(*table_args(tb), *query_args(q))
    _assert_equal_everywhere(got, want, f"{kind}, engine {engine}")
    assert (want >= 0).sum() > 1000 and len(np.unique(want)) > 500
    if engine != 1:
        assert sel.info()["index_truncated"] == tb.num_tasks * tb.B      # no slice has a complete index
    if engine == 2:
        assert sel.info()["lookup_scanned"] > 1000
    sel.destroy()


@pytest.mark.parametrize("engine", ENGINES, ids=ENGINE_IDS)
def test_index_degrades_after_a_load_report(oracle_lib, engine):
    """100 tasks of 200 equally accurate variants whose latency falls with the cost.  As loaded, the
    queues rise with the cost faster than the latencies fall: the cheapest variant of a task dominates
    the others and every staircase has one step.  A report then empties all queues -- 200 steps per
    slice, of which the index keeps 62 -- and a second one restores them.  Parity throughout; the AUTO
    handle turns to the exhaustive scan one call after the first report (the call that follows it
    still runs the index lookup, whose first kernel tells the host what the rebuild found) and back
    to the index one call after the second."""
    T, n, B = 100, 200, 8
    i = np.tile(np.arange(n, dtype=np.int64), T)
    b = np.arange(B, dtype=np.int64)[None, :]
    good = (600 * i).astype(np.int32)
    tb = _table(T, [1, 2, 4, 8, 16, 32, 64, 128], np.repeat(np.arange(T, dtype=np.int32), n), np.full(T * n, 8000),
                (60_000 - 295 * i)[:, None] + 10 * b, (100 + i)[:, None] + b, good)
    q = workloads.make_queries(1, n=120_000)
    sel = make_selector(tb, engine=engine)
    queue = tb.queue_us.copy()
    rows = np.arange(tb.V, dtype=np.int32)

    def used():   # kernels of the next call
        sel.set_timing(True)
        got = gpu_select(sel, *query_args(q))
        t = sel.get_timings()
        sel.set_timing(False)
        want = oracle_lib.select(*table_args(tb, queue), *query_args(q))
        _assert_equal_everywhere(got, want, "degrading table")
        assert (want >= 0).sum() > 10_000
        return "scan" if t["scan_lds"]["launches"] else "index"

    first = "scan" if engine == 1 else "index"
    assert used() == first
    if engine != 1:
        assert sel.info()["index_max_steps"] == 1
    for values, bad in ((np.zeros(tb.V, np.int32), True), (good, False)):
        sel.update_load(to_dev(rows), to_dev(values))
        oracle_lib.update_load(queue, rows, values)
        used()                                   # parity; its first kernel reports the rebuild's counters
        if engine != 1:
            info = sel.info()
            assert info["index_truncated"] == (T * B if bad else 0) and info["index_max_steps"] == (62 if bad else 1)
        assert used() == (("scan" if bad else "index") if engine == 0 else first)
    sel.destroy()
