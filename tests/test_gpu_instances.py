"""Case I with the state kept per running instance (infaas_sel_load_instance_states /
_update_instance_states, then _select_workers) against the CPU oracle: every element of all three
outputs (Section 4: the state machine is kept per variant instance)."""
import numpy as np
import pytest

import workloads
from gpu_util import make_selector, query_args, table_args, to_dev
from test_gpu_parity import _random_queries, _random_table
from test_gpu_workers import _random_cluster, cluster_args, gpu_select_workers, load_cluster

pytestmark = pytest.mark.gpu


def _check(oracle_lib, sel, tb, load, cl, ist, queries, label, queue=None):
    print(f"instance case {label}: V={tb.V} T={tb.num_tasks} B={tb.B} W={len(cl[1])} I={len(cl[3])} "
          f"N={len(queries[0])}", flush=True)
    got = gpu_select_workers(sel, *queries)
    want = oracle_lib.select_instances(*table_args(tb, queue), load, *cl, ist, *queries)
    bad = np.flatnonzero((got[0] != want[0]) | (got[1] != want[1]) | (got[2] != want[2]))
    assert bad.size == 0, (f"{label}: {bad.size} differ, first at {bad[:5]}: got "
                           f"{[g[bad[:5]] for g in got]} want {[w[bad[:5]] for w in want]}")
    return want


def _setup(cfg):
    tb = workloads.make_table(cfg)
    st = workloads.make_states(cfg, tb.V)
    wk = workloads.make_workers(cfg, st)
    ist = workloads.make_instance_states(cfg, wk.I)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    load_cluster(sel, cluster_args(wk))
    sel.load_instance_states(ist)
    return tb, st, wk, ist, sel


@pytest.mark.parametrize("cfg", [0, 1])
def test_instances_configs(oracle_lib, cfg):
    tb, st, wk, ist, sel = _setup(cfg)
    q = workloads.make_queries(cfg)
    want = _check(oracle_lib, sel, tb, st.load_us, cluster_args(wk), ist, query_args(q), f"config{cfg}")
    tier, worker = want[1], want[2]
    assert (tier == 1).any() and (tier == 2).any() and (tier == 0).any()
    assert (worker[tier > 0] >= 0).all() and (worker[tier == 0] == -1).all()
    # the instance states matter: a state per variant (loaded = Active) gives other answers
    running = np.bincount(wk.inst_variant, minlength=tb.V)
    as_variants = oracle_lib.select_workers(*table_args(tb), np.minimum(running, 1).astype(np.int32), st.load_us,
                                            *cluster_args(wk), *query_args(q))
    assert (as_variants[0] != want[0]).sum() > 10 and (as_variants[2] != want[2]).sum() > 10
    sel.destroy()


def test_instances_ties_and_all_codes(oracle_lib):
    rng = np.random.default_rng(31)
    for span in (2, 3, 6, 40):
        sizes = rng.integers(0, 70, 12)
        sizes[5] = 0
        tb = _random_table(rng, 12, sizes, 3, span=span)
        state = rng.integers(0, 4, tb.V).astype(np.int32)
        load = rng.integers(0, span, tb.V).astype(np.int32)
        cl = _random_cluster(rng, tb.V, state, span)
        ist = rng.choice([1, 2, 3], len(cl[3]), p=[0.5, 0.3, 0.2]).astype(np.int32)
        sel = make_selector(tb, engine=0)
        sel.load_states(state, load)
        load_cluster(sel, cl)
        sel.load_instance_states(ist)
        _check(oracle_lib, sel, tb, load, cl, ist, _random_queries(rng, 12, 3, 30_000, span=span), f"ties span={span}")
        sel.destroy()


def test_instance_state_reports_between_other_reports(oracle_lib):
    """Instance state, instance load, utilisation and queue reports in turn; entries that must be
    skipped in every one of them."""
    tb, st, wk, ist, sel = _setup(1)
    q = workloads.make_queries(1, n=200_000)
    ist = ist.copy(); queue = tb.queue_us.copy(); util = wk.worker_util.copy(); iload = wk.inst_load.copy()
    for chunk in (1, 2, 3):
        idx, val = workloads.make_instance_state_update(1, wk.I, chunk, fraction=0.2)
        idx = idx.copy(); val = val.copy()
        idx[:3] = [-1, wk.I, wk.I + 9]; val[3:6] = [0, 4, -2]              # entries that must be skipped
        sel.update_instance_states(to_dev(idx), to_dev(val))
        oracle_lib.update_instance_state(ist, idx, val)
        wu = workloads.make_worker_update(1, wk.W, wk.I, chunk)
        sel.update_workers(to_dev(wu.worker_idx), to_dev(wu.worker_util), to_dev(wu.inst_idx), to_dev(wu.inst_load))
        oracle_lib.update_worker_util(util, wu.worker_idx, wu.worker_util)
        oracle_lib.update_instance_load(iload, wu.inst_idx, wu.inst_load)
        lu = workloads.make_load_update(1, tb.V, chunk)
        sel.update_load(to_dev(lu.variant_idx), to_dev(lu.queue_us))
        oracle_lib.update_load(queue, lu.variant_idx, lu.queue_us)
        cl = (wk.variant_hw, wk.worker_hw, util, wk.inst_variant, wk.inst_worker, iload)
        _check(oracle_lib, sel, tb, st.load_us, cl, ist, query_args(q), f"reports {chunk}", queue=queue)
    sel.destroy()


def test_instances_all_one_state(oracle_lib):
    """Every instance Active: the worker selection with loaded = Active.  Every instance
    Overloaded: only the variants that run nowhere are left, all in the second step."""
    tb = workloads.make_table(0)
    st = workloads.make_states(0, tb.V)
    wk = workloads.make_workers(0, st)
    q = query_args(workloads.make_queries(0))
    for code in (1, 2, 3):
        ist = np.full(wk.I, code, np.int32)
        sel = make_selector(tb, engine=0)
        sel.load_states(st.state, st.load_us)
        load_cluster(sel, cluster_args(wk))
        sel.load_instance_states(ist)
        want = _check(oracle_lib, sel, tb, st.load_us, cluster_args(wk), ist, q, f"all instances {code}")
        if code == 1:
            running = np.bincount(wk.inst_variant, minlength=tb.V)
            same = oracle_lib.select_workers(*table_args(tb), np.minimum(running, 1).astype(np.int32), st.load_us,
                                             *cluster_args(wk), *q)
            assert all(np.array_equal(a, b) for a, b in zip(want, same))
        else:
            assert set(np.unique(want[1])) <= {0, 2} and (want[1] == 2).any()
        sel.destroy()


def test_instances_config2_every_query(oracle_lib):
    """Configuration 2 at its full 16M queries: variant, tier and worker of every query."""
    tb, st, wk, ist, sel = _setup(2)
    q = workloads.make_queries(2)
    want = _check(oracle_lib, sel, tb, st.load_us, cluster_args(wk), ist, query_args(q), "config2")
    assert all(int((want[1] == t).sum()) > 10_000 for t in (0, 1, 2))
    sel.destroy()


def test_instance_state_errors():
    import paper_1905_13348_amd as lib
    import torch
    tb = workloads.make_table(0)
    st = workloads.make_states(0, tb.V)
    wk = workloads.make_workers(0, st)
    ist = workloads.make_instance_states(0, wk.I)
    z = torch.zeros(4, dtype=torch.int32, device="cuda")
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    with pytest.raises(lib.InfaasSelError):                   # no workers yet
        sel.load_instance_states(ist)
    load_cluster(sel, cluster_args(wk))
    with pytest.raises(lib.InfaasSelError):                   # no instance states yet
        sel.update_instance_states(z, z)
    bad = ist.copy(); bad[2] = 0                              # a loaded instance is not Inactive
    with pytest.raises(lib.InfaasSelError):
        sel.load_instance_states(bad)
    sel.load_instance_states(ist)
    with pytest.raises(lib.InfaasSelError):                   # states per variant are derived from here on
        sel.update_state(z, z)
    load_cluster(sel, cluster_args(wk))                       # a new cluster drops the instance states
    sel.update_state(z, z)
    sel.destroy()
