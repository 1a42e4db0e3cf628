"""Worker selection of the GPU library (infaas_sel_load_workers / _update_workers / _select_workers)
against the CPU oracle: every element of all three outputs (Section 4.1: the policy returns the
variant and the worker that serves the query)."""
import numpy as np
import pytest

import workloads
from gpu_util import DeviceQueries, make_selector, query_args, table_args, to_dev
from test_gpu_parity import _random_queries, _random_table, _staircase_queries, _staircase_table

pytestmark = pytest.mark.gpu


def cluster_args(wk):
    return (wk.variant_hw, wk.worker_hw, wk.worker_util, wk.inst_variant, wk.inst_worker, wk.inst_load)


def load_cluster(sel, cl):
    variant_hw, worker_hw, worker_util, inst_variant, inst_worker, inst_load = cl
    sel.load_workers(worker_hw, worker_util, variant_hw, inst_variant, inst_worker, inst_load)


def gpu_select_workers(sel, task, slo, min_acc, bidx):
    import torch
    dq = DeviceQueries(task, slo, min_acc, bidx)
    tier = torch.full_like(dq.out, -54321)
    worker = torch.full_like(dq.out, -54321)
    sel.select_workers(dq.task, dq.slo, dq.min_acc, dq.bidx, dq.out, tier, worker, n=dq.n)
    torch.cuda.synchronize()
    return dq.out[:dq.n].cpu().numpy(), tier[:dq.n].cpu().numpy(), worker[:dq.n].cpu().numpy()


def _check(oracle_lib, sel, tb, state, load, cl, queries, label, queue=None):
    print(f"worker case {label}: V={tb.V} T={tb.num_tasks} B={tb.B} W={len(cl[1])} I={len(cl[3])} "
          f"N={len(queries[0])}", flush=True)
    got = gpu_select_workers(sel, *queries)
    want = oracle_lib.select_workers(*table_args(tb, queue), state, load, *cl, *queries)
    bad = np.flatnonzero((got[0] != want[0]) | (got[1] != want[1]) | (got[2] != want[2]))
    assert bad.size == 0, (f"{label}: {bad.size} differ, first at {bad[:5]}: got "
                           f"{[g[bad[:5]] for g in got]} want {[w[bad[:5]] for w in want]}")
    return want


def _random_cluster(rng, V, state, span, W=None):
    """Ties everywhere; one hardware code that no worker has; some loaded variants without instances."""
    W = int(rng.integers(1, 40)) if W is None else W
    H = int(rng.integers(1, 4))
    codes = rng.choice(np.array([-7, 0, 3, 1000, 2**31 - 1]), size=H + 1, replace=False)
    variant_hw = codes[rng.integers(0, H + 1, V)].astype(np.int32)     # codes[H]: no worker has it
    worker_hw = codes[rng.integers(0, H, W)].astype(np.int32)
    worker_util = rng.integers(0, span, W).astype(np.int32)
    I = int(rng.integers(0, 3 * V + 1))
    inst_variant = rng.integers(0, V, I).astype(np.int32)
    inst_worker = rng.integers(0, W, I).astype(np.int32)
    inst_load = rng.integers(0, span, I).astype(np.int32)
    return variant_hw, worker_hw, worker_util, inst_variant, inst_worker, inst_load


@pytest.mark.parametrize("cfg", [0, 1])
def test_workers_configs(oracle_lib, cfg):
    tb = workloads.make_table(cfg)
    st = workloads.make_states(cfg, tb.V)
    wk = workloads.make_workers(cfg, st)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    load_cluster(sel, cluster_args(wk))
    q = workloads.make_queries(cfg)
    want = _check(oracle_lib, sel, tb, st.state, st.load_us, cluster_args(wk), query_args(q), f"config{cfg}")
    tier, worker = want[1], want[2]
    assert (tier == 1).any() and (tier == 2).any() and (tier == 0).any()
    assert (worker[tier > 0] >= 0).all() and (worker[tier == 0] == -1).all()
    # the same call again (nothing to refresh), then the tiered call on the same handle
    _check(oracle_lib, sel, tb, st.state, st.load_us, cluster_args(wk), query_args(q), f"config{cfg} again")
    sel.destroy()


def test_workers_ties_and_missing_candidates(oracle_lib):
    rng = np.random.default_rng(23)
    for span in (2, 3, 6, 40):
        sizes = rng.integers(0, 70, 12)
        sizes[5] = 0
        tb = _random_table(rng, 12, sizes, 3, span=span)
        state = rng.integers(0, 4, tb.V).astype(np.int32)
        load = rng.integers(0, span, tb.V).astype(np.int32)
        cl = _random_cluster(rng, tb.V, state, span)
        sel = make_selector(tb, engine=0)
        sel.load_states(state, load)
        load_cluster(sel, cl)
        want = _check(oracle_lib, sel, tb, state, load, cl, _random_queries(rng, 12, 3, 30_000, span=span),
                      f"ties span={span}")
        assert ((want[1] > 0) & (want[2] < 0)).any(), "no answer without a worker in this case"
        sel.destroy()


@pytest.mark.parametrize("steps", [31, 63, 300])
def test_workers_long_staircases(oracle_lib, steps):
    """Slices whose staircase does not fit the index bodies: answers come from the second body and
    from the rank-ordered scan, whose workers are looked up by row."""
    rng = np.random.default_rng(300 + steps)
    tb = _staircase_table(4, steps)
    state = rng.choice(4, tb.V, p=[0.45, 0.45, 0.05, 0.05]).astype(np.int32)
    load = rng.integers(0, 60_000, tb.V).astype(np.int32)
    cl = _random_cluster(rng, tb.V, state, 50, W=64)
    sel = make_selector(tb, engine=0)
    sel.load_states(state, load)
    load_cluster(sel, cl)
    _check(oracle_lib, sel, tb, state, load, cl, _staircase_queries(rng, tb, 30_000, steps), f"staircase{steps}")
    sel.destroy()


def test_workers_more_than_16_bits(oracle_lib):
    """70,000 workers: worker numbers no longer fit the 16-bit copies the lookup keeps for the first
    steps of every slice, so every worker comes from the full-width tables."""
    rng = np.random.default_rng(29)
    tb = workloads.make_table(0)
    st = workloads.make_states(0, tb.V)
    cl = _random_cluster(rng, tb.V, st.state, 1000, W=70_000)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    load_cluster(sel, cl)
    want = _check(oracle_lib, sel, tb, st.state, st.load_us, cl, query_args(workloads.make_queries(0)), "70000 workers")
    assert want[2].max() > 65535
    sel.destroy()


def test_workers_empty_cluster(oracle_lib):
    """No workers and no instances at all: variant and tier as ever, worker -1 everywhere."""
    tb = workloads.make_table(0)
    st = workloads.make_states(0, tb.V)
    q = query_args(workloads.make_queries(0))
    e = np.zeros(0, np.int32)
    cl = (np.zeros(tb.V, np.int32), e, e, e, e, e)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    load_cluster(sel, cl)
    want = _check(oracle_lib, sel, tb, st.state, st.load_us, cl, q, "empty cluster")
    assert (want[2] == -1).all() and (want[1] > 0).any()
    sel.destroy()


def test_workers_reports(oracle_lib):
    """Worker reports, state reports and load reports interleaved; every call checked in full."""
    cfg = 1
    tb = workloads.make_table(cfg)
    st = workloads.make_states(cfg, tb.V)
    wk = workloads.make_workers(cfg, st)
    q = workloads.make_queries(cfg, n=200_000)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    load_cluster(sel, cluster_args(wk))
    state = st.state.copy(); queue = tb.queue_us.copy()
    util = wk.worker_util.copy(); iload = wk.inst_load.copy()
    cl = lambda: (wk.variant_hw, wk.worker_hw, util, wk.inst_variant, wk.inst_worker, iload)
    _check(oracle_lib, sel, tb, state, st.load_us, cl(), query_args(q), "before reports", queue=queue)
    for chunk in (1, 2, 3, 4):
        wu = workloads.make_worker_update(cfg, wk.W, wk.I, chunk, fraction=0.3)
        widx, wval, iidx, ival = (x.copy() for x in (wu.worker_idx, wu.worker_util, wu.inst_idx, wu.inst_load))
        widx[:3] = [-1, wk.W, wk.W + 5]; wval[3] = -1                  # entries that must be skipped
        iidx[:3] = [-4, wk.I, wk.I + 1]; ival[3] = -9
        if chunk == 2:      # utilisation only
            sel.update_workers(to_dev(widx), to_dev(wval))
            oracle_lib.update_worker_util(util, widx, wval)
        elif chunk == 3:    # instance loads only
            sel.update_workers(None, None, to_dev(iidx), to_dev(ival))
            oracle_lib.update_instance_load(iload, iidx, ival)
        else:
            sel.update_workers(to_dev(widx), to_dev(wval), to_dev(iidx), to_dev(ival))
            oracle_lib.update_worker_util(util, widx, wval)
            oracle_lib.update_instance_load(iload, iidx, ival)
        if chunk >= 2:      # the indexes are rebuilt under the workers: states, then loads
            su = workloads.make_state_update(cfg, tb.V, chunk, fraction=0.2)
            sel.update_state(to_dev(su.variant_idx), to_dev(su.state))
            oracle_lib.update_state(state, su.variant_idx, su.state)
        if chunk >= 3:
            lu = workloads.make_load_update(cfg, tb.V, chunk)
            sel.update_load(to_dev(lu.variant_idx), to_dev(lu.queue_us))
            oracle_lib.update_load(queue, lu.variant_idx, lu.queue_us)
        _check(oracle_lib, sel, tb, state, st.load_us, cl(), query_args(q), f"reports {chunk}", queue=queue)
    sel.destroy()


def test_workers_config2_every_query(oracle_lib):
    """Configuration 2 at its full 16M queries, the launch bench.py --workers times: variant, tier and
    worker of every query against the oracle."""
    cfg = 2
    tb = workloads.make_table(cfg)
    st = workloads.make_states(cfg, tb.V)
    wk = workloads.make_workers(cfg, st)
    q = workloads.make_queries(cfg)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    load_cluster(sel, cluster_args(wk))
    got = gpu_select_workers(sel, *query_args(q))
    print(f"workers config2: oracle over all {q.N} queries", flush=True)
    want = oracle_lib.select_workers(*table_args(tb), st.state, st.load_us, *cluster_args(wk), *query_args(q))
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
    # and by construction of the seeded cluster: a worker exactly where there is an answer (every loaded variant of the seeded
    # cluster has an instance, every hardware class a worker), and it depends on (variant, tier) only
    assert np.array_equal(got[0] >= 0, got[2] >= 0) and np.array_equal(got[0] >= 0, got[1] > 0)
    key = got[0].astype(np.int64) * 4 + got[1]
    order = np.argsort(key, kind="stable")
    same = key[order][1:] == key[order][:-1]
    assert np.array_equal(got[2][order][1:][same], got[2][order][:-1][same])
    sel.destroy()


def test_workers_config3_every_query(oracle_lib):
    """Config 3's table (1,000 tasks, 8,000 slices: only part of either index fits in LDS, so both
    tiers also answer from the copies in global memory) with 4M queries: variant, tier and worker of
    every query against the oracle."""
    cfg, n = 3, 4_000_000
    tb = workloads.make_table(cfg)
    st = workloads.make_states(cfg, tb.V)
    wk = workloads.make_workers(cfg, st)
    q = workloads.make_queries(cfg, n=n)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    load_cluster(sel, cluster_args(wk))
    print(f"worker case config3: V={tb.V} T={tb.num_tasks} W={wk.W} I={wk.I} N={n}", flush=True)
    got = gpu_select_workers(sel, *query_args(q))
    want = oracle_lib.select_workers(*table_args(tb), st.state, st.load_us, *cluster_args(wk), *query_args(q))
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
    assert sel.info()["lookup_global_body"] > 0
    assert all((want[1] == t).sum() > 1000 for t in (0, 1, 2))
    assert np.array_equal(got[0] >= 0, got[1] > 0) and np.array_equal(got[0] >= 0, got[2] >= 0)
    assert (tb.task_id[got[0][got[0] >= 0]] == q.task[got[0] >= 0]).all()
    sel.destroy()


def test_workers_errors():
    import paper_1905_13348_amd as lib
    import torch
    tb = workloads.make_table(0)
    st = workloads.make_states(0, tb.V)
    wk = workloads.make_workers(0, st)
    sel = make_selector(tb, engine=0)
    z = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(lib.InfaasSelError):      # no states yet
        load_cluster(sel, cluster_args(wk))
    sel.load_states(st.state, st.load_us)
    with pytest.raises(lib.InfaasSelError):      # no workers yet
        sel.select_workers(z, z, z, z, z.clone(), z.clone(), z.clone())
    with pytest.raises(lib.InfaasSelError):
        sel.update_workers(z, z)
    cl = list(cluster_args(wk))
    for pos, val in ((3, tb.V), (3, -1), (4, wk.W), (4, -1), (5, -1)):
        bad = [x.copy() for x in cl]
        bad[pos][0] = val
        with pytest.raises(lib.InfaasSelError):
            load_cluster(sel, bad)
    bad = [x.copy() for x in cl]
    bad[2][0] = -1                                # negative utilisation
    with pytest.raises(lib.InfaasSelError):
        load_cluster(sel, bad)
    load_cluster(sel, cl)
    sel.load_states(st.state, st.load_us)        # new states drop the cluster
    with pytest.raises(lib.InfaasSelError):
        sel.select_workers(z, z, z, z, z.clone(), z.clone(), z.clone())
    sel.destroy()
