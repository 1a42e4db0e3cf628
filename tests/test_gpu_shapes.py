"""Many small tables of odd shapes (one task, one batch size, one variant, empty tasks, query counts
around the 256-query unit of the lookup kernel), every call of the library on each of them, every
element against the CPU oracle."""
import numpy as np
import pytest

from gpu_util import gpu_select, gpu_select_closest, make_selector, table_args
from test_gpu_parity import _random_queries, _random_table
from test_gpu_scale import gpu_scale
from test_gpu_tiered import gpu_select_tiered
from test_gpu_workers import _random_cluster, gpu_select_workers, load_cluster

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", range(24))
def test_every_call_on_a_small_odd_table(oracle_lib, seed):
    rng = np.random.default_rng(9000 + seed)
    T = int(rng.choice([1, 1, 2, 3, 7]))
    B = int(rng.choice([1, 1, 2, 3, 5, 8]))
    sizes = rng.choice([0, 1, 1, 2, 5, 40, 130], size=T)
    if sizes.sum() == 0:
        sizes[int(rng.integers(0, T))] = 1
    span = [None, 2, 3, 9][seed % 4]
    tb = _random_table(rng, T, sizes, B, span=span)
    n = int(rng.choice([1, 3, 255, 256, 257, 1023, 5000]))
    queries = _random_queries(rng, T, B, n, span=span)
    print(f"shape case {seed}: T={T} B={B} sizes={sizes.tolist()} V={tb.V} N={n} span={span}", flush=True)
    table = table_args(tb)

    sel = make_selector(tb, engine=0)
    want_sel, want_clo = oracle_lib.select_closest(*table, *queries)
    assert np.array_equal(gpu_select(sel, *queries), want_sel), "select"
    got = gpu_select_closest(sel, *queries)
    assert np.array_equal(got[0], want_sel) and np.array_equal(got[1], want_clo), "select_closest"

    vals = span if span else 50_000
    state = rng.integers(0, 4, tb.V).astype(np.int32)
    load = rng.integers(0, vals, tb.V).astype(np.int32)
    sel.load_states(state, load)
    want = oracle_lib.select_tiered(*table, state, load, *queries)
    got = gpu_select_tiered(sel, *queries)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1]), "select_tiered"

    cl = _random_cluster(rng, tb.V, state, vals)
    load_cluster(sel, cl)
    want = oracle_lib.select_workers(*table, state, load, *cl, *queries)
    got = gpu_select_workers(sel, *queries)
    for g, w, name in zip(got, want, ("variant", "tier", "worker")):
        assert np.array_equal(g, w), f"select_workers {name}"

    prof = (rng.integers(0, max(1, tb.V // 4) + 1, tb.V).astype(np.int32), rng.integers(1, vals + 1, tb.V).astype(np.int32),
            rng.integers(0, min(vals, 2**20) + 1, tb.V).astype(np.int32), rng.integers(0, vals, tb.V).astype(np.int32))
    lam, slack = int(rng.choice([0, 3, 1000])), int(rng.choice([0, 100, 105, 200]))
    sel.load_scaling(*prof, lam, slack)
    req = (rng.integers(-1, tb.V + 1, n).astype(np.int32), rng.integers(0, 4, n).astype(np.int32),
           rng.integers(0, 12 * vals, n).astype(np.int32), queries[1], queries[3])
    want = oracle_lib.scale(*prof, tb.lat_us, lam, slack, *req)
    got = gpu_scale(sel, req)
    for g, w, name in zip(got, want, ("action", "variant", "instances")):
        assert np.array_equal(g, w), f"scale {name}"
    sel.destroy()
