"""State-aware two-tier selection of the GPU library (infaas_sel_load_states / _update_state /
_select_tiered) against the CPU oracle: every element, both outputs (Sections 4 and 4.1)."""
import numpy as np
import pytest

import workloads
from gpu_util import DeviceQueries, gpu_select, make_selector, query_args, table_args, to_dev
from test_gpu_parity import _random_queries, _random_table, _staircase_queries, _staircase_table

pytestmark = pytest.mark.gpu


def gpu_select_tiered(sel, task, slo, min_acc, bidx):
    import torch
    dq = DeviceQueries(task, slo, min_acc, bidx)
    tier = torch.full_like(dq.out, -54321)
    sel.select_tiered(dq.task, dq.slo, dq.min_acc, dq.bidx, dq.out, tier, n=dq.n)
    torch.cuda.synchronize()
    return dq.out[:dq.n].cpu().numpy(), tier[:dq.n].cpu().numpy()


def _check(oracle_lib, sel, tb, state, load, queries, label, queue=None):
    print(f"tiered case {label}: V={tb.V} T={tb.num_tasks} B={tb.B} N={len(queries[0])}", flush=True)
    got, tier = gpu_select_tiered(sel, *queries)
    want, want_tier = oracle_lib.select_tiered(*table_args(tb, queue), state, load, *queries)
    bad = np.flatnonzero((got != want) | (tier != want_tier))
    assert bad.size == 0, (f"{label}: {bad.size} differ, first at {bad[:5]}: got {got[bad[:5]]}/{tier[bad[:5]]} "
                           f"want {want[bad[:5]]}/{want_tier[bad[:5]]}")
    return want, want_tier


@pytest.mark.parametrize("cfg", [0, 1])
def test_tiered_configs(oracle_lib, cfg):
    tb = workloads.make_table(cfg)
    st = workloads.make_states(cfg, tb.V)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    q = workloads.make_queries(cfg)
    want, tier = _check(oracle_lib, sel, tb, st.state, st.load_us, query_args(q), f"config{cfg}")
    assert (tier == 1).any() and (tier == 2).any() and (tier == 0).any()
    # the plain call now answers from the Active variants only
    got = gpu_select(sel, *query_args(q))
    assert np.array_equal(got, np.where(tier == 1, want, -1))
    sel.destroy()


def test_tiered_ties_and_invalid_queries(oracle_lib):
    rng = np.random.default_rng(17)
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
def test_tiered_long_staircases(oracle_lib, steps):
    rng = np.random.default_rng(200 + steps)
    tb = _staircase_table(4, steps)
    state = rng.choice(4, tb.V, p=[0.45, 0.45, 0.05, 0.05]).astype(np.int32)
    load = rng.integers(0, 60_000, tb.V).astype(np.int32)
    sel = make_selector(tb, engine=0)
    sel.load_states(state, load)
    _check(oracle_lib, sel, tb, state, load, _staircase_queries(rng, tb, 30_000, steps), f"staircase{steps}")
    sel.destroy()


def test_tiered_all_one_state(oracle_lib):
    """All Active: the plain selection.  All Overloaded: nothing.  All Inactive: second tier only."""
    tb = workloads.make_table(0)
    q = query_args(workloads.make_queries(0))
    st = workloads.make_states(0, tb.V)
    plain = oracle_lib.select(*table_args(tb), *q)
    for code in (1, 2, 0):
        state = np.full(tb.V, code, np.int32)
        sel = make_selector(tb, engine=0)
        sel.load_states(state, st.load_us)
        want, tier = _check(oracle_lib, sel, tb, state, st.load_us, q, f"all state {code}")
        if code == 1:
            assert np.array_equal(want, plain)
        if code == 2:
            assert (want == -1).all() and (tier == 0).all()
        if code == 0:
            assert set(np.unique(tier)) <= {0, 2} and (tier == 2).any()
        sel.destroy()


def test_tiered_state_and_load_reports(oracle_lib):
    tb = workloads.make_table(1)
    st = workloads.make_states(1, tb.V)
    q = workloads.make_queries(1, n=200_000)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    state = st.state.copy(); queue = tb.queue_us.copy()
    for chunk in (1, 2, 3):
        su = workloads.make_state_update(1, tb.V, chunk, fraction=0.2)
        idx = su.variant_idx.copy(); val = su.state.copy()
        idx[:3] = [-1, tb.V, tb.V + 7]; val[3:6] = [4, -1, 99]          # entries that must be skipped
        sel.update_state(to_dev(idx), to_dev(val))
        oracle_lib.update_state(state, idx, val)
        lu = workloads.make_load_update(1, tb.V, chunk)
        sel.update_load(to_dev(lu.variant_idx), to_dev(lu.queue_us))
        oracle_lib.update_load(queue, lu.variant_idx, lu.queue_us)
        _check(oracle_lib, sel, tb, state, st.load_us, query_args(q), f"reports {chunk}", queue=queue)
    sel.destroy()


def test_tiered_config2_every_query(oracle_lib):
    """Configuration 2 at its full 16M queries, the launch bench.py --tiered times: variant and tier
    of every query against the oracle."""
    tb = workloads.make_table(2)
    st = workloads.make_states(2, tb.V)
    q = workloads.make_queries(2)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    got, tier = gpu_select_tiered(sel, *query_args(q))
    print(f"tiered config2: oracle over all {q.N} queries", flush=True)
    want, want_tier = oracle_lib.select_tiered(*table_args(tb), st.state, st.load_us, *query_args(q))
    assert np.array_equal(got, want) and np.array_equal(tier, want_tier)
    assert all(int((want_tier == t).sum()) > 10_000 for t in (0, 1, 2))
    sel.destroy()


def test_tiered_more_queries_than_one_pass(oracle_lib):
    """2^26 + 5000 queries in one call (the state-aware call works in passes of 2^26), on a table
    where most queries reach the second tier: the seam, both ends and a random sample against the
    oracle; every element written; answer and tier consistent everywhere."""
    import torch
    tb = workloads.make_table(0)
    rng = np.random.default_rng(26)
    state = rng.choice(4, size=tb.V, p=(0.7, 0.1, 0.1, 0.1)).astype(np.int32)
    load = rng.integers(100, 100_000, tb.V).astype(np.int32)
    sel = make_selector(tb, engine=0)
    sel.load_states(state, load)
    n = (1 << 26) + 5000
    g = torch.Generator(device="cuda"); g.manual_seed(26)
    task = torch.randint(-1, tb.num_tasks + 1, (n,), generator=g, device="cuda", dtype=torch.int32)
    slo = torch.randint(-1000, 400_000, (n,), generator=g, device="cuda", dtype=torch.int32)
    acc = torch.randint(5000, 9501, (n,), generator=g, device="cuda", dtype=torch.int32)
    bidx = torch.randint(0, tb.B, (n,), generator=g, device="cuda", dtype=torch.int32)
    out = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    tier = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    seam = 1 << 26
    pick = np.unique(np.concatenate([np.arange(2000), seam - 2000 + np.arange(4000), n - 2000 + np.arange(2000),
                                     np.random.default_rng(1).integers(0, n, 100_000)]))
    pick_d = torch.from_numpy(pick).cuda()
    qs = tuple(x[pick_d].cpu().numpy() for x in (task, slo, acc, bidx))
    want, want_tier = oracle_lib.select_tiered(*table_args(tb), state, load, *qs)
    print(f"tiered case two passes: N={n}, tiers of the sample {np.bincount(want_tier, minlength=3)}", flush=True)
    sel.select_tiered(task, slo, acc, bidx, out, tier)
    torch.cuda.synchronize()
    assert np.array_equal(out[pick_d].cpu().numpy(), want)
    assert np.array_equal(tier[pick_d].cpu().numpy(), want_tier)
    assert int((out == -7).sum()) == 0 and int((tier == -7).sum()) == 0, "some results were never written"
    assert bool(((out >= 0) == (tier > 0)).all())
    sel.destroy()


def test_tiered_errors():
    import paper_1905_13348_amd as lib
    import torch
    tb = workloads.make_table(0)
    st = workloads.make_states(0, tb.V)
    z = torch.zeros(4, dtype=torch.int32, device="cuda")
    sel = make_selector(tb, engine=0)
    with pytest.raises(lib.InfaasSelError):                   # no states yet
        sel.select_tiered(z, z, z, z, z.clone(), z.clone())
    bad = st.state.copy(); bad[3] = 4
    with pytest.raises(lib.InfaasSelError):
        sel.load_states(bad, st.load_us)
    big = st.load_us.copy(); big[0] = 2**31 - 1
    with pytest.raises(lib.InfaasSelError):                   # load + latency would not fit int32
        sel.load_states(st.state, big)
    sel.load_states(st.state, st.load_us)
    with pytest.raises(lib.InfaasSelError):                   # the closest-variant call needs a stateless handle
        sel.select_closest(z, z, z, z, z.clone(), z.clone())
    sel.destroy()
    sel = make_selector(tb, engine=1)
    with pytest.raises(lib.InfaasSelError):                   # scan-only handle
        sel.load_states(st.state, st.load_us)
    sel.destroy()


def test_plain_select_honours_states_whatever_the_engine(oracle_lib):
    """A table whose staircases all exceed the index's capacity: a handle in automatic mode answers
    it with the exhaustive scan.  Once states are loaded the plain call answers from the Active
    variants only, as the header says -- also on such a handle."""
    rng = np.random.default_rng(41)
    tb = _staircase_table(4, 300)
    state = rng.choice(4, tb.V, p=[0.45, 0.45, 0.05, 0.05]).astype(np.int32)
    load = rng.integers(0, 60_000, tb.V).astype(np.int32)
    qs = _staircase_queries(rng, tb, 30_000, 300)
    sel = make_selector(tb, engine=0)
    assert sel.info()["index_truncated"] == 8
    plain = gpu_select(sel, *qs)
    assert np.array_equal(plain, oracle_lib.select(*table_args(tb), *qs))
    sel.load_states(state, load)
    want, tier = oracle_lib.select_tiered(*table_args(tb), state, load, *qs)
    got = gpu_select(sel, *qs)
    assert np.array_equal(got, np.where(tier == 1, want, -1)) and (tier == 1).sum() > 1000
    assert not np.array_equal(got, plain)
    sel.destroy()
