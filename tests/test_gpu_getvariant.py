"""The whole of Case I in one call (infaas_sel_select_workers_closest: variant, tier, worker, and the
closest variant where neither tier answers) against the CPU oracle, every element of all four outputs
(Section 4.1), with the state kept per variant and per running instance."""
import numpy as np
import pytest

import workloads
from gpu_util import DeviceQueries, make_selector, query_args, table_args, to_dev
from test_gpu_parity import _random_queries, _random_table, _staircase_queries, _staircase_table
from test_gpu_workers import _random_cluster, cluster_args, load_cluster

pytestmark = pytest.mark.gpu


def gpu_get_variant(sel, task, slo, min_acc, bidx):
    import torch
    dq = DeviceQueries(task, slo, min_acc, bidx)
    extra = [torch.full_like(dq.out, -54321) for _ in range(3)]
    sel.select_workers_closest(dq.task, dq.slo, dq.min_acc, dq.bidx, dq.out, *extra, n=dq.n)
    torch.cuda.synchronize()
    return tuple(x[:dq.n].cpu().numpy() for x in [dq.out] + extra)


def _check(oracle_lib, sel, tb, state, load, cl, queries, label, queue=None, inst_state=None):
    print(f"getVariant case {label}: V={tb.V} T={tb.num_tasks} B={tb.B} W={len(cl[1])} I={len(cl[3])} "
          f"N={len(queries[0])} instance states: {inst_state is not None}", flush=True)
    got = gpu_get_variant(sel, *queries)
    want = oracle_lib.get_variant(*table_args(tb, queue), state, load, *cl, *queries, inst_state=inst_state)
    bad = np.flatnonzero((got[0] != want[0]) | (got[1] != want[1]) | (got[2] != want[2]) | (got[3] != want[3]))
    assert bad.size == 0, (f"{label}: {bad.size} differ, first at {bad[:5]}: got "
                           f"{[g[bad[:5]] for g in got]} want {[w[bad[:5]] for w in want]}")
    return want


def _properties(want):
    out, tier, worker, closest = want
    assert np.array_equal(closest[tier > 0], out[tier > 0]) and (out[tier == 0] == -1).all()
    assert (worker[tier == 0] == -1).all()


@pytest.mark.parametrize("cfg", [0, 1])
def test_getvariant_configs(oracle_lib, cfg):
    tb = workloads.make_table(cfg)
    st = workloads.make_states(cfg, tb.V)
    wk = workloads.make_workers(cfg, st)
    q = workloads.make_queries(cfg)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    load_cluster(sel, cluster_args(wk))
    want = _check(oracle_lib, sel, tb, st.state, st.load_us, cluster_args(wk), query_args(q), f"config{cfg}")
    _properties(want)
    tier, closest = want[1], want[3]
    assert all((tier == t).any() for t in (0, 1, 2)) and (closest[tier == 0] >= 0).any()
    # the same with the state kept per running instance
    ist = workloads.make_instance_states(cfg, wk.I)
    sel.load_instance_states(ist)
    want2 = _check(oracle_lib, sel, tb, None, st.load_us, cluster_args(wk), query_args(q), f"config{cfg}",
                   inst_state=ist)
    _properties(want2)
    assert (want2[0] != want[0]).sum() > 10
    sel.destroy()


def test_getvariant_ties_and_all_codes(oracle_lib):
    rng = np.random.default_rng(37)
    for span in (2, 3, 6, 40):
        sizes = rng.integers(0, 70, 12)
        sizes[3] = 0
        tb = _random_table(rng, 12, sizes, 3, span=span)
        state = rng.integers(0, 4, tb.V).astype(np.int32)
        load = rng.integers(0, span, tb.V).astype(np.int32)
        cl = _random_cluster(rng, tb.V, state, span)
        queries = _random_queries(rng, 12, 3, 30_000, span=span)
        sel = make_selector(tb, engine=0)
        sel.load_states(state, load)
        load_cluster(sel, cl)
        _properties(_check(oracle_lib, sel, tb, state, load, cl, queries, f"ties span={span}"))
        ist = rng.choice([1, 2, 3], len(cl[3]), p=[0.5, 0.3, 0.2]).astype(np.int32)
        sel.load_instance_states(ist)
        _properties(_check(oracle_lib, sel, tb, None, load, cl, queries, f"ties span={span}", inst_state=ist))
        sel.destroy()


def test_getvariant_long_staircases_and_reports(oracle_lib):
    """Slices with two bodies and truncated ones, state, load and worker reports between the calls."""
    rng = np.random.default_rng(41)
    tb = _staircase_table(3, 90)
    state = rng.choice([0, 1, 2, 3], tb.V, p=[0.4, 0.4, 0.1, 0.1]).astype(np.int32)
    load = rng.integers(0, 5000, tb.V).astype(np.int32)
    cl = _random_cluster(rng, tb.V, state, 50, W=17)
    queries = _staircase_queries(rng, tb, 60_000, 90)
    sel = make_selector(tb, engine=0)
    sel.load_states(state, load)
    load_cluster(sel, cl)
    _check(oracle_lib, sel, tb, state, load, cl, queries, "staircases")
    state = state.copy(); queue = tb.queue_us.copy(); util = cl[2].copy(); iload = cl[5].copy()
    for chunk in (1, 2):
        idx = rng.choice(tb.V, tb.V // 5, replace=False).astype(np.int32)
        val = rng.integers(0, 4, idx.size).astype(np.int32)
        sel.update_state(to_dev(idx), to_dev(val))
        oracle_lib.update_state(state, idx, val)
        qidx = rng.choice(tb.V, tb.V // 7, replace=False).astype(np.int32)
        qval = rng.integers(0, 20_000, qidx.size).astype(np.int32)
        sel.update_load(to_dev(qidx), to_dev(qval))
        oracle_lib.update_load(queue, qidx, qval)
        widx = rng.choice(len(util), 5, replace=False).astype(np.int32)
        wval = rng.integers(0, 50, 5).astype(np.int32)
        iidx = rng.integers(0, max(len(iload), 1), 9).astype(np.int32) if len(iload) else np.zeros(0, np.int32)
        ival = rng.integers(0, 50, iidx.size).astype(np.int32)
        sel.update_workers(to_dev(widx), to_dev(wval), to_dev(iidx), to_dev(ival))
        oracle_lib.update_worker_util(util, widx, wval)
        oracle_lib.update_instance_load(iload, iidx, ival)
        cl_now = (cl[0], cl[1], util, cl[3], cl[4], iload)
        _properties(_check(oracle_lib, sel, tb, state, load, cl_now, queries, f"staircases, reports {chunk}", queue=queue))
    sel.destroy()


def test_getvariant_config2_every_query(oracle_lib):
    """Configuration 2 at its full 16M queries: all four outputs of every query."""
    cfg = 2
    tb = workloads.make_table(cfg)
    st = workloads.make_states(cfg, tb.V)
    wk = workloads.make_workers(cfg, st)
    q = workloads.make_queries(cfg)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    load_cluster(sel, cluster_args(wk))
    want = _check(oracle_lib, sel, tb, st.state, st.load_us, cluster_args(wk), query_args(q), "config2")
    _properties(want)
    tier, closest = want[1], want[3]
    assert all(int((tier == t).sum()) > 10_000 for t in (0, 1, 2)) and int((closest[tier == 0] >= 0).sum()) > 10_000
    sel.destroy()


def test_getvariant_errors():
    import paper_1905_13348_amd as lib
    import torch
    tb = workloads.make_table(0)
    st = workloads.make_states(0, tb.V)
    wk = workloads.make_workers(0, st)
    z = torch.zeros(8, dtype=torch.int32, device="cuda")
    outs = [z.clone() for _ in range(4)]
    sel = make_selector(tb, engine=0)
    with pytest.raises(lib.InfaasSelError):                   # no states
        sel.select_workers_closest(z, z, z, z, *outs)
    sel.load_states(st.state, st.load_us)
    with pytest.raises(lib.InfaasSelError):                   # no workers
        sel.select_workers_closest(z, z, z, z, *outs)
    load_cluster(sel, cluster_args(wk))
    sel.select_workers_closest(z, z, z, z, *outs)
    sel.select_workers_closest(z, z, z, z, *outs, n=0)
    sel.destroy()
