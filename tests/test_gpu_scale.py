"""Scaling decisions of the GPU library (infaas_sel_load_scaling / infaas_sel_scale / _scale_down)
against the CPU oracle: action, variant and instance count of every request (Section 4.2.2, scaling
up and scaling down)."""
import numpy as np
import pytest

import workloads
from gpu_util import make_selector, to_dev

pytestmark = pytest.mark.gpu


def profile_args(sc):
    return (sc.arch_id, sc.sat_qps, sc.hw_cost, sc.load_us)


def request_args(rq):
    return (rq.variant, rq.instances, rq.load_qps, rq.slo_us, rq.batch_idx)


def gpu_scale(sel, requests, down=False):
    import torch
    dev = [to_dev(np.ascontiguousarray(x, dtype=np.int32)) for x in requests]
    n = len(requests[0])
    outs = [torch.full((max(n, 1),), -54321, dtype=torch.int32, device="cuda") for _ in range(3)]
    sel.scale(*dev, *outs, n=n, down=down)
    torch.cuda.synchronize()
    return tuple(o[:n].cpu().numpy() for o in outs)


def _check(oracle_lib, sel, tb, prof, lam, slack, requests, label, down=False):
    print(f"scaling {'down' if down else 'up'} case {label}: V={tb.V} B={tb.B} R={len(requests[0])} lambda={lam} "
          f"slack={slack}", flush=True)
    got = gpu_scale(sel, requests, down)
    want = oracle_lib.scale(*prof, tb.lat_us, lam, slack, *requests, down=down)
    bad = np.flatnonzero((got[0] != want[0]) | (got[1] != want[1]) | (got[2] != want[2]))
    assert bad.size == 0, (f"{label}: {bad.size} differ, first at {bad[:5]}: got {[g[bad[:5]] for g in got]} "
                           f"want {[w[bad[:5]] for w in want]}")
    return want


@pytest.mark.parametrize("cfg,n", [(0, 100_000), (1, 300_000)])
def test_scale_configs(oracle_lib, cfg, n):
    tb = workloads.make_table(cfg)
    sc = workloads.make_scaling(cfg, tb)
    sel = make_selector(tb, engine=0)
    for lam, slack in ((50, 105), (0, 100), (1000, 200)):
        sel.load_scaling(*profile_args(sc), lam, slack)
        rq = workloads.make_scale_requests(cfg, tb, sc, n + 37, chunk=lam)       # a ragged tail
        want = _check(oracle_lib, sel, tb, profile_args(sc), lam, slack, request_args(rq), f"config{cfg}")
        if slack == 105:
            assert all((want[0] == a).any() for a in (0, 1, 2, 3))
    sel.destroy()


def test_scale_ties_and_invalid_requests(oracle_lib):
    """Tiny value ranges (equal costs, throughputs and latencies everywhere) and requests outside
    every limit."""
    rng = np.random.default_rng(41)
    for span in (2, 3, 6, 1000):
        V, B = int(rng.integers(20, 400)), int(rng.integers(1, 5))
        tb = workloads.VariantTable(num_tasks=1, batch_sizes=np.arange(1, B + 1, dtype=np.int32),
                                    task_id=np.zeros(V, np.int32), acc_bp=np.full(V, 8000, np.int32),
                                    lat_us=rng.integers(1, span + 1, (V, B)).astype(np.int32),
                                    cost=np.ones((V, B), np.int32), queue_us=np.zeros(V, np.int32))
        prof = (rng.integers(-3, max(1, V // 8), V).astype(np.int32), rng.integers(1, span + 1, V).astype(np.int32),
                rng.integers(0, span + 1, V).astype(np.int32), rng.integers(0, 40 * span, V).astype(np.int32))
        R = 50_000
        req = [rng.integers(-2, V + 2, R), rng.integers(-1, 5, R), rng.integers(-1, 14 * span, R),
               rng.integers(0, span + 2, R), rng.integers(-1, B + 1, R)]
        req[1][:4] = [1_000_000, 1_000_001, -1, 0]
        req[2][4:8] = [1_000_000_000, 1_000_000_001, -1, 0]
        req = tuple(np.asarray(x, dtype=np.int32) for x in req)
        sel = make_selector(tb, engine=0)
        for lam, slack in ((0, 100), (37, 105), (1000, 200), (5, 0)):
            sel.load_scaling(*prof, lam, slack)
            _check(oracle_lib, sel, tb, prof, lam, slack, req, f"ties span={span}")
            _check(oracle_lib, sel, tb, prof, lam, slack, req, f"ties span={span}", down=True)
        sel.destroy()


def test_scale_extreme_values(oracle_lib):
    """Costs near 2^100: largest load, headroom, hardware cost, loading latency and lambda at once."""
    rng = np.random.default_rng(43)
    V, B = 64, 2
    tb = workloads.VariantTable(num_tasks=1, batch_sizes=np.array([1, 2], np.int32), task_id=np.zeros(V, np.int32),
                                acc_bp=np.full(V, 8000, np.int32), lat_us=rng.integers(1, 3, (V, B)).astype(np.int32),
                                cost=np.ones((V, B), np.int32), queue_us=np.zeros(V, np.int32))
    prof = (rng.integers(0, 4, V).astype(np.int32), rng.integers(1, 4, V).astype(np.int32),
            (2**20 - rng.integers(0, 3, V)).astype(np.int32), (2**31 - 1 - rng.integers(0, 40, V)).astype(np.int32))
    R = 20_000
    req = (rng.integers(0, V, R).astype(np.int32), rng.choice([0, 1, 999_999, 1_000_000], R).astype(np.int32),
           (10**9 - rng.integers(0, 3, R)).astype(np.int32), rng.integers(1, 4, R).astype(np.int32),
           rng.integers(0, B, R).astype(np.int32))
    sel = make_selector(tb, engine=0)
    sel.load_scaling(*prof, 1000, 200)
    want = _check(oracle_lib, sel, tb, prof, 1000, 200, req, "extreme")
    assert want[2].max() > 5 * 10**8 and (want[0] == 1).any() and (want[0] == 2).any()
    low = (req[0], req[1], rng.choice([0, 1, 10**5, 10**9], R).astype(np.int32), req[3], req[4])
    for lam in (1000, 0):
        sel.load_scaling(*prof, lam, 200)
        want = _check(oracle_lib, sel, tb, prof, lam, 200, low, "extreme", down=True)
    assert all((want[0] == a).any() for a in (0, 1, 2)) and want[2].max() > 10**5
    sel.destroy()


def test_scale_large_architecture_and_empty(oracle_lib):
    """One architecture holding every variant of config 0 (a run of 256 candidates), every variant
    an architecture of its own (no upgrade possible), and an empty request list."""
    import torch
    tb = workloads.make_table(0)
    sc = workloads.make_scaling(0, tb)
    rq = workloads.make_scale_requests(0, tb, sc, 40_000)
    sel = make_selector(tb, engine=0)
    one = (np.zeros(tb.V, np.int32),) + profile_args(sc)[1:]
    sel.load_scaling(*one, 50, 105)
    _check(oracle_lib, sel, tb, one, 50, 105, request_args(rq), "one architecture")
    solo = (np.arange(tb.V, dtype=np.int32)[::-1].copy(),) + profile_args(sc)[1:]
    sel.load_scaling(*solo, 50, 105)
    want = _check(oracle_lib, sel, tb, solo, 50, 105, request_args(rq), "solo architectures")
    assert not (want[0] == 2).any()
    dn = request_args(workloads.make_scale_down_requests(0, tb, sc, 40_000))
    want = _check(oracle_lib, sel, tb, solo, 50, 105, dn, "solo architectures", down=True)
    assert not (want[0] == 2).any() and (want[0] == 1).any()
    sel.load_scaling(*one, 50, 105)
    want = _check(oracle_lib, sel, tb, one, 50, 105, dn, "one architecture", down=True)
    assert (want[0] == 2).mean() > 0.5
    z = torch.zeros(4, dtype=torch.int32, device="cuda")
    sel.scale(z, z, z, z, z, z.clone(), z.clone(), z.clone(), n=0)
    sel.destroy()


def test_scale_config2_every_request(oracle_lib):
    """4M requests on the 100,000-variant table (the benchmark's launch): action, variant and
    instance count of every request against the oracle, then the properties that need no oracle."""
    cfg = 2
    tb = workloads.make_table(cfg)
    sc = workloads.make_scaling(cfg, tb)
    rq = workloads.make_scale_requests(cfg, tb, sc, 4_000_000)
    sel = make_selector(tb, engine=0)
    sel.load_scaling(*profile_args(sc), 50, 105)
    got = gpu_scale(sel, request_args(rq))
    print(f"scale config2: oracle over all {rq.R} requests", flush=True)
    want = oracle_lib.scale(*profile_args(sc), tb.lat_us, 50, 105, *request_args(rq))
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
    assert all(int((want[0] == a).sum()) > 10_000 for a in (0, 1, 2, 3))
    act, var, inst = got
    assert np.array_equal(act == 1, var == rq.variant) and np.array_equal((act == 0) | (act == 3), var == -1)
    assert np.array_equal(var >= 0, inst > 0)
    up = act == 2
    assert (sc.arch_id[var[up]] == sc.arch_id[rq.variant[up]]).all()
    assert (sc.sat_qps[var[up]] > sc.sat_qps[rq.variant[up]]).all()
    assert (tb.lat_us[var[up], rq.batch_idx[up]] <= rq.slo_us[up]).all()
    carried = sc.sat_qps[var[up]].astype(np.int64) * inst[up] * 100
    assert (carried >= rq.load_qps[up].astype(np.int64) * 105).all()
    sel.destroy()


@pytest.mark.parametrize("cfg,n", [(0, 100_000), (1, 300_000)])
def test_scale_down_configs(oracle_lib, cfg, n):
    tb = workloads.make_table(cfg)
    sc = workloads.make_scaling(cfg, tb)
    sel = make_selector(tb, engine=0)
    for lam, slack in ((50, 105), (0, 100), (1000, 200)):
        sel.load_scaling(*profile_args(sc), lam, slack)
        rq = workloads.make_scale_down_requests(cfg, tb, sc, n + 37, chunk=lam)       # a ragged tail
        want = _check(oracle_lib, sel, tb, profile_args(sc), lam, slack, request_args(rq), f"config{cfg}", down=True)
        assert all((want[0] == a).any() for a in (0, 1, 2))
        # the requests of the scaling-up workload as well (mostly overloaded variants)
        up = workloads.make_scale_requests(cfg, tb, sc, 50_000, chunk=lam)
        _check(oracle_lib, sel, tb, profile_args(sc), lam, slack, request_args(up), f"config{cfg}, rising load", down=True)
    sel.destroy()


def test_scale_down_config2_every_request(oracle_lib):
    """4M scaling-down requests on the 100,000-variant table (the benchmark's launch): every request
    against the oracle, then the properties that need no oracle."""
    cfg = 2
    tb = workloads.make_table(cfg)
    sc = workloads.make_scaling(cfg, tb)
    rq = workloads.make_scale_down_requests(cfg, tb, sc, 4_000_000)
    sel = make_selector(tb, engine=0)
    sel.load_scaling(*profile_args(sc), 50, 105)
    got = gpu_scale(sel, request_args(rq), down=True)
    print(f"scale down config2: oracle over all {rq.R} requests", flush=True)
    want = oracle_lib.scale_down(*profile_args(sc), tb.lat_us, 50, 105, *request_args(rq))
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
    assert all(int((want[0] == a).sum()) > 10_000 for a in (0, 1, 2))
    act, var, inst = got
    assert np.array_equal(act == 0, var == -1) and np.array_equal(act == 0, inst == 0)
    rm = act == 1
    assert np.array_equal(var[rm], rq.variant[rm]) and (inst[rm] == 1).all() and (rq.instances[rm] >= 2).all()
    left = sc.sat_qps[rq.variant[rm]].astype(np.int64) * (rq.instances[rm] - 1) * 100
    assert (left >= rq.load_qps[rm].astype(np.int64) * 105).all()
    dn = act == 2
    assert (sc.arch_id[var[dn]] == sc.arch_id[rq.variant[dn]]).all()
    assert (sc.hw_cost[var[dn]] < sc.hw_cost[rq.variant[dn]]).all()
    assert (tb.lat_us[var[dn], rq.batch_idx[dn]] <= rq.slo_us[dn]).all() and (inst[dn] >= 1).all()
    carried = sc.sat_qps[var[dn]].astype(np.int64) * inst[dn] * 100
    assert (carried >= rq.load_qps[dn].astype(np.int64) * 105).all()
    sel.destroy()


def test_scale_errors():
    import paper_1905_13348_amd as lib
    import torch
    tb = workloads.make_table(0)
    sc = workloads.make_scaling(0, tb)
    sel = make_selector(tb, engine=0)
    z = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(lib.InfaasSelError):      # no profile yet
        sel.scale(z, z, z, z, z, z.clone(), z.clone(), z.clone())
    with pytest.raises(lib.InfaasSelError):
        sel.scale_down(z, z, z, z, z, z.clone(), z.clone(), z.clone())
    for lam, slack in ((-1, 100), (1001, 100), (0, -1), (0, 201)):
        with pytest.raises(lib.InfaasSelError):
            sel.load_scaling(*profile_args(sc), lam, slack)
    for pos, val in ((1, 0), (2, -1), (2, 2**20 + 1), (3, -1)):
        bad = [x.copy() for x in profile_args(sc)]
        bad[pos][5] = val
        with pytest.raises(lib.InfaasSelError):
            sel.load_scaling(*bad, 0, 100)
    sel.load_scaling(*profile_args(sc), 0, 100)
    sel.load_variants(tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us)     # a new table drops the profile
    with pytest.raises(lib.InfaasSelError):
        sel.scale(z, z, z, z, z, z.clone(), z.clone(), z.clone())
    sel.destroy()
