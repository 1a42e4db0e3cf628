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


def test_states_and_state_reports():
    tb = workloads.make_table(1)
    a, b = workloads.make_states(1, tb.V), workloads.make_states(1, tb.V)
    assert np.array_equal(a.state, b.state) and np.array_equal(a.load_us, b.load_us)
    assert a.state.dtype == np.int32 and a.state.shape == (tb.V,) and set(np.unique(a.state)) == {0, 1, 2, 3}
    frac = np.bincount(a.state) / tb.V
    assert abs(frac[0] - 0.5) < 0.02 and abs(frac[1] - 0.4) < 0.02
    assert a.load_us.min() >= 100 and a.load_us.max() <= 5_000_000
    assert (a.load_us.astype(np.int64)[:, None] + tb.lat_us <= np.iinfo(np.int32).max).all()
    u, v = workloads.make_state_update(1, tb.V, 1), workloads.make_state_update(1, tb.V, 2)
    assert np.unique(u.variant_idx).size == u.variant_idx.size == round(0.05 * tb.V)
    assert not np.array_equal(u.variant_idx, v.variant_idx)
    assert u.state.min() >= 0 and u.state.max() <= 3


def test_cluster_and_worker_reports():
    tb = workloads.make_table(1)
    st = workloads.make_states(1, tb.V)
    a, b = workloads.make_workers(1, st), workloads.make_workers(1, st)
    for x, y in zip((a.variant_hw, a.worker_hw, a.worker_util, a.inst_variant, a.inst_worker, a.inst_load),
                    (b.variant_hw, b.worker_hw, b.worker_util, b.inst_variant, b.inst_worker, b.inst_load)):
        assert x.dtype == np.int32 and np.array_equal(x, y)
    assert a.W == 256 and a.variant_hw.shape == (tb.V,)
    assert a.worker_util.min() >= 0 and a.worker_util.max() <= 10_000 and a.inst_load.min() >= 0
    # instances: only of loaded variants, on workers of the variant's hardware, at most 8 each, distinct workers
    assert (st.state[a.inst_variant] != 0).all()
    assert np.array_equal(a.worker_hw[a.inst_worker], a.variant_hw[a.inst_variant])
    per = np.bincount(a.inst_variant, minlength=tb.V)
    assert per.max() <= 8 and (per[st.state != 0] >= 1).all() and (per[st.state == 0] == 0).all()
    pairs = a.inst_variant.astype(np.int64) * a.W + a.inst_worker
    assert np.unique(pairs).size == pairs.size
    u = workloads.make_worker_update(1, a.W, a.I, 1)
    assert np.unique(u.worker_idx).size == u.worker_idx.size == round(0.1 * a.W)
    assert np.unique(u.inst_idx).size == u.inst_idx.size == round(0.1 * a.I)
    assert u.worker_util.max() <= 10_000 and u.inst_load.max() <= 1000 and u.inst_idx.max() < a.I


def test_scaling_profiles_and_requests():
    tb = workloads.make_table(1)
    a, b = workloads.make_scaling(1, tb), workloads.make_scaling(1, tb)
    for x, y in zip((a.arch_id, a.sat_qps, a.hw_cost, a.load_us), (b.arch_id, b.sat_qps, b.hw_cost, b.load_us)):
        assert x.dtype == np.int32 and x.shape == (tb.V,) and np.array_equal(x, y)
    assert a.sat_qps.min() >= 1 and a.hw_cost.min() >= 50 and a.hw_cost.max() <= 2000 and a.load_us.min() >= 100
    # an architecture belongs to one task; about 12 variants each
    task_of = {}
    for arch, task in zip(a.arch_id.tolist(), tb.task_id.tolist()):
        assert task_of.setdefault(arch, task) == task
    sizes = np.bincount(a.arch_id)
    assert 8 < sizes.mean() < 16
    r = workloads.make_scale_requests(1, tb, a, 50_000)
    assert r.R == 50_000 and r.variant.min() >= 0 and r.variant.max() < tb.V
    assert r.instances.min() >= 1 and r.load_qps.min() >= 0 and r.load_qps.max() <= 1_000_000_000
    assert r.batch_idx.min() >= 0 and r.batch_idx.max() < tb.B
    need = r.load_qps.astype(np.int64) * 105 > a.sat_qps[r.variant].astype(np.int64) * r.instances * 100
    assert 0.75 < need.mean() < 0.95     # most requests need scaling, some do not
    r2 = workloads.make_scale_requests(1, tb, a, 50_000, chunk=1)
    assert not np.array_equal(r.variant, r2.variant)
    d = workloads.make_scale_down_requests(1, tb, a, 50_000)
    assert d.R == 50_000 and d.instances.min() >= 1 and d.load_qps.min() >= 0
    spare = a.sat_qps[d.variant].astype(np.int64) * (d.instances - 1) * 100 >= d.load_qps.astype(np.int64) * 105
    assert 0.3 < (spare & (d.instances >= 2)).mean() < 0.8     # often an instance can go, often not
    assert not np.array_equal(d.variant, workloads.make_scale_down_requests(1, tb, a, 50_000, chunk=1).variant)
