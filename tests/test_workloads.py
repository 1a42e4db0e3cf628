"""The seeded input generators: determinism, ranges and shapes of the five configurations."""
import numpy as np

import workloads


def test_tables_are_deterministic_and_in_range():
    for cfg in (0, 1, 2):
        a = workloads.make_table(cfg); b = workloads.make_table(cfg)
        spec = workloads.config_spec(cfg)
        assert a.V == spec["num_tasks"] * spec["per_task"]
        for f in ("task_id", "acc_bp", "lat_us", "cost", "queue_us"):
            x, y = getattr(a, f), getattr(b, f)
            assert x.dtype == np.int32 and np.array_equal(x, y)
        assert a.acc_bp.min() >= 5000 and a.acc_bp.max() <= 9500
        assert a.queue_us.min() >= 0 and a.queue_us.max() <= 50000
        assert a.lat_us.min() >= 1 and a.lat_us[:, 0].max() <= 500000
        assert a.cost.min() >= 1
        assert np.all(np.bincount(a.task_id, minlength=spec["num_tasks"]) == spec["per_task"])
        # rows are not grouped by task
        assert np.any(np.diff(a.task_id) < 0)
        # cost = ceil(lat * price / b) for a price in {1, 4, 9}
        bs = a.batch_sizes.astype(np.int64)
        ok = np.zeros(a.V, bool)
        for price in (1, 4, 9):
            ok |= np.all(a.cost == (a.lat_us.astype(np.int64) * price + bs - 1) // bs, axis=1)
        assert ok.all()


def test_config3_segments_and_config4_table():
    t3 = workloads.make_table(3)
    sizes = np.bincount(t3.task_id, minlength=1000)
    assert sizes.min() >= 1 and sizes.max() <= 20000 and 60_000 <= t3.V <= 200_000
    t2 = workloads.make_table(2); t4 = workloads.make_table(4)
    assert np.array_equal(t2.lat_us, t4.lat_us) and np.array_equal(t2.task_id, t4.task_id)


def test_queries():
    q = workloads.make_queries(2, n=200_000)
    assert q.slo_us.min() >= 1000 and q.slo_us.max() <= 2_000_000
    assert q.min_acc_bp.min() >= 5000 and q.min_acc_bp.max() <= 9500
    assert q.batch_idx.min() == 0 and q.batch_idx.max() == 7
    share = np.bincount(q.task, minlength=50) / q.N
    assert 0.2 < share[0] < 0.32 and share[0] > share[1] > share[5] > share[40]
    q3 = workloads.make_queries(3, n=200_000)
    lg = np.log(q3.slo_us.astype(np.float64))
    assert (lg < np.log(30000)).mean() > 0.4 and (lg > np.log(30000)).mean() > 0.4  # two modes
    a = workloads.make_queries(4, chunk=3, n=1000); b = workloads.make_queries(4, chunk=3, n=1000)
    c = workloads.make_queries(4, chunk=4, n=1000)
    assert np.array_equal(a.slo_us, b.slo_us) and not np.array_equal(a.slo_us, c.slo_us)


def test_load_update():
    u = workloads.make_load_update(4, 100_000, chunk=1)
    assert u.variant_idx.size == 10_000 and np.unique(u.variant_idx).size == 10_000
    assert u.queue_us.min() >= 0 and u.queue_us.max() <= 200_000
