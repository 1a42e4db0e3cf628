"""The complete Case I of Section 4.1 in one call (infaas_sel_select_tiered_closest): variant, tier
and, where neither tier answers, the closest Active or Inactive variant -- against the CPU oracle,
every element of all three outputs."""
import numpy as np
import pytest

import workloads
from gpu_util import DeviceQueries, make_selector, query_args, table_args, to_dev
from test_gpu_parity import _random_queries, _random_table, _staircase_queries, _staircase_table

pytestmark = pytest.mark.gpu
I32MAX = 2**31 - 1


def gpu_case1(sel, task, slo, min_acc, bidx):
    import torch
    dq = DeviceQueries(task, slo, min_acc, bidx)
    tier = torch.full_like(dq.out, -54321)
    closest = torch.full_like(dq.out, -98765)
    sel.select_tiered_closest(dq.task, dq.slo, dq.min_acc, dq.bidx, dq.out, tier, closest, n=dq.n)
    torch.cuda.synchronize()
    return tuple(x[:dq.n].cpu().numpy() for x in (dq.out, tier, closest))


def _check(oracle_lib, sel, tb, state, load, queries, label, queue=None):
    print(f"case1 {label}: V={tb.V} T={tb.num_tasks} B={tb.B} N={len(queries[0])}", flush=True)
    got = gpu_case1(sel, *queries)
    want = oracle_lib.select_case1(*table_args(tb, queue), state, load, *queries)
    for g, w, name in zip(got, want, ("variant", "tier", "suggestion")):
        bad = np.flatnonzero(g != w)
        assert bad.size == 0, f"{label}: {name}: {bad.size} differ, first at {bad[:5]}: got {g[bad[:5]]} want {w[bad[:5]]}"
    return want


@pytest.mark.parametrize("cfg", [0, 1])
def test_case1_configs(oracle_lib, cfg):
    tb = workloads.make_table(cfg)
    st = workloads.make_states(cfg, tb.V)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    q = workloads.make_queries(cfg)
    var, tier, sug = _check(oracle_lib, sel, tb, st.state, st.load_us, query_args(q), f"config{cfg}")
    assert all((tier == t).sum() > 50 for t in (0, 1, 2)) and ((var < 0) & (sug >= 0)).sum() > 50
    # suggestions come from both tiers
    assert {int(x) for x in np.unique(st.state[sug[(var < 0) & (sug >= 0)]])} == {0, 1}
    sel.destroy()


def test_case1_ties_and_invalid_queries(oracle_lib):
    rng = np.random.default_rng(19)
    for span in (2, 3, 6, 40):
        sizes = rng.integers(0, 70, 12)
        sizes[5] = 0
        tb = _random_table(rng, 12, sizes, 3, span=span)
        state = rng.integers(0, 4, tb.V).astype(np.int32)
        load = rng.integers(0, span, tb.V).astype(np.int32)
        sel = make_selector(tb, engine=0)
        sel.load_states(state, load)
        _check(oracle_lib, sel, tb, state, load, _random_queries(rng, 12, 3, 30_000, span=span), f"ties span={span}")
        sel.destroy()


@pytest.mark.parametrize("steps", [31, 50, 63, 300])
def test_case1_long_staircases(oracle_lib, steps):
    """Second groups of steps, and slices with more steps than the index keeps: their suggestions
    come from the scan of the whole slice."""
    rng = np.random.default_rng(300 + steps)
    tb = _staircase_table(4, steps)
    state = rng.choice(4, tb.V, p=[0.45, 0.45, 0.05, 0.05]).astype(np.int32)
    load = rng.integers(0, 60_000, tb.V).astype(np.int32)
    sel = make_selector(tb, engine=0)
    sel.load_states(state, load)
    qs = _staircase_queries(rng, tb, 30_000, steps)
    qs = (qs[0], (qs[1] - rng.choice([0, 0, 90_000], qs[1].size)).astype(np.int32), qs[2], qs[3])   # some bounds nothing meets
    _check(oracle_lib, sel, tb, state, load, qs, f"staircase{steps}")
    sel.destroy()


def test_case1_one_state_and_extremes(oracle_lib):
    tb = workloads.make_table(0)
    q = query_args(workloads.make_queries(0))
    st = workloads.make_states(0, tb.V)
    for code in (1, 2, 0, 3):
        state = np.full(tb.V, code, np.int32)
        sel = make_selector(tb, engine=0)
        sel.load_states(state, st.load_us)
        var, tier, sug = _check(oracle_lib, sel, tb, state, st.load_us, q, f"all state {code}")
        if code in (2, 3):
            assert (sug == -1).all()
        else:
            assert (sug >= 0).all()
        sel.destroy()
    # tasks in which only one tier, or neither, has variants; bounds at the ends of the int32 range
    rng = np.random.default_rng(23)
    tb = _random_table(rng, 6, np.array([40, 40, 40, 40, 3, 0]), 2)
    state = np.zeros(tb.V, np.int32)
    state[tb.task_id == 0] = 1
    state[tb.task_id == 1] = 0
    state[tb.task_id == 2] = rng.choice([2, 3], int((tb.task_id == 2).sum()))
    state[tb.task_id == 3] = rng.integers(0, 4, int((tb.task_id == 3).sum()))
    state[tb.task_id == 4] = [1, 2, 0]
    load = rng.integers(0, 300_000, tb.V).astype(np.int32)
    n = 40_000
    qs = (rng.integers(-1, 7, n), rng.choice([-I32MAX - 1, -5, 0, 1000, 20_000, 400_000, I32MAX], n),
          rng.choice([-I32MAX - 1, 0, 5000, 7000, 9000, 9500, 9501, I32MAX], n), rng.integers(-1, 3, n))
    qs = tuple(np.asarray(x, np.int32) for x in qs)
    sel = make_selector(tb, engine=0)
    sel.load_states(state, load)
    _check(oracle_lib, sel, tb, state, load, qs, "extremes")
    sel.destroy()


def test_case1_state_and_load_reports(oracle_lib):
    tb = workloads.make_table(1)
    st = workloads.make_states(1, tb.V)
    q = workloads.make_queries(1, n=200_000)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    state = st.state.copy(); queue = tb.queue_us.copy()
    for chunk in (1, 2):
        su = workloads.make_state_update(1, tb.V, chunk, fraction=0.2)
        sel.update_state(to_dev(su.variant_idx), to_dev(su.state))
        oracle_lib.update_state(state, su.variant_idx, su.state)
        lu = workloads.make_load_update(1, tb.V, chunk)
        sel.update_load(to_dev(lu.variant_idx), to_dev(lu.queue_us))
        oracle_lib.update_load(queue, lu.variant_idx, lu.queue_us)
        _check(oracle_lib, sel, tb, state, st.load_us, query_args(q), f"reports {chunk}", queue=queue)
    sel.destroy()


def test_case1_config3_and_config2(oracle_lib):
    """Configuration 3's table (most slices outside LDS: suggestions from the index copies in global
    memory) with 2M queries, and configuration 2 at its full 16M queries: every element."""
    for cfg, n in ((3, 2_000_000), (2, None)):
        tb = workloads.make_table(cfg)
        st = workloads.make_states(cfg, tb.V)
        q = workloads.make_queries(cfg, n=n)
        sel = make_selector(tb, engine=0)
        sel.load_states(st.state, st.load_us)
        var, tier, sug = _check(oracle_lib, sel, tb, st.state, st.load_us, query_args(q), f"config{cfg}")
        assert ((var < 0) & (sug >= 0)).sum() > 10_000
        sel.destroy()
