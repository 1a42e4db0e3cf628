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


def test_grouped_equals_literal_on_medium_sample(oracle_lib):
    tb = workloads.make_table(1)
    q = workloads.make_queries(1, n=2000)
    table = (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)
    queries = (q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
    a = oracle_lib.select(*table, *queries)
    b = oracle_lib.select_literal(*table, *queries)
    assert np.array_equal(a, b)
    pins.check_invariants(table, queries, a)
