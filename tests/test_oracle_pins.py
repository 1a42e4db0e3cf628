"""The committed oracle against its pins (CPU only)."""
import numpy as np
import pytest

import pins
import workloads


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(oracle_lib, pin):
    pin(oracle_lib)


@pytest.mark.parametrize("pin", pins.CLOSEST_PINS, ids=lambda f: f.__name__)
def test_closest_pin(oracle_lib, pin):
    pin(oracle_lib)


@pytest.mark.parametrize("pin", pins.TIERED_PINS, ids=lambda f: f.__name__)
def test_tiered_pin(oracle_lib, pin):
    pin(oracle_lib)


@pytest.mark.parametrize("pin", pins.CASE1_PINS, ids=lambda f: f.__name__)
def test_case1_pin(oracle_lib, pin):
    pin(oracle_lib)


@pytest.mark.parametrize("pin", pins.WORKER_PINS, ids=lambda f: f.__name__)
def test_worker_pin(oracle_lib, pin):
    pin(oracle_lib)


@pytest.mark.parametrize("pin", pins.INSTANCE_PINS, ids=lambda f: f.__name__)
def test_instance_pin(oracle_lib, pin):
    pin(oracle_lib)


@pytest.mark.parametrize("pin", pins.SCALING_PINS, ids=lambda f: f.__name__)
def test_scaling_pin(oracle_lib, pin):
    pin(oracle_lib)


@pytest.mark.parametrize("pin", pins.SCALE_DOWN_PINS, ids=lambda f: f.__name__)
def test_scale_down_pin(oracle_lib, pin):
    pin(oracle_lib)


def test_get_variant_is_the_two_pinned_routines(oracle_lib):
    """Oracle.get_variant computes nothing of its own: its first three arrays are select_workers' (or
    select_instances'), its fourth select_case1's, in the literal forms as well; and the parts fit
    (a suggestion only where nothing was selected, a worker only where something was)."""
    tb = workloads.make_table(0)
    st = workloads.make_states(0, tb.V)
    wk = workloads.make_workers(0, st)
    ist = workloads.make_instance_states(0, wk.I)
    q = workloads.make_queries(0, n=4000)
    table = (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    cluster = (wk.worker_hw, wk.worker_util, wk.inst_variant, wk.inst_worker, wk.inst_load)
    queries = (q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
    for inst_state in (None, ist):
        got = oracle_lib.get_variant(*table, st.state, st.load_us, wk.variant_hw, *cluster, *queries, inst_state=inst_state)
        lit = oracle_lib.get_variant(*table, st.state, st.load_us, wk.variant_hw, *cluster, *queries, inst_state=inst_state,
                                     literal=True)
        assert all(np.array_equal(a, b) for a, b in zip(got, lit))
        if inst_state is None:
            three = oracle_lib.select_workers(*table, st.state, st.load_us, wk.variant_hw, *cluster, *queries)
            states = st.state
        else:
            three = oracle_lib.select_instances(*table, st.load_us, wk.variant_hw, *cluster, inst_state, *queries)
            states = oracle_lib.derive_states(tb.V, wk.inst_variant, inst_state)
        assert all(np.array_equal(a, b) for a, b in zip(got[:3], three))
        assert np.array_equal(got[3], oracle_lib.select_case1(*table, states, st.load_us, *queries)[2])
        out, tier, worker, closest = got
        assert np.array_equal(closest[tier > 0], out[tier > 0]) and (worker[tier == 0] == -1).all()
        assert (tier == 0).any() and (closest[tier == 0] >= 0).any() and (worker[tier > 0] >= 0).any()


def test_grouped_equals_literal_on_medium_sample(oracle_lib):
    tb = workloads.make_table(1)
    q = workloads.make_queries(1, n=2000)
    table = (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    queries = (q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
    a = oracle_lib.select(*table, *queries)
    b = oracle_lib.select_literal(*table, *queries)
    assert np.array_equal(a, b)
    pins.check_invariants(table, queries, a)
