"""The calls that enqueue work allocate nothing and synchronise nothing once their scratch memory
exists, so a caller may capture them into a HIP graph.  Each graph is replayed several times with
new contents in its input buffers and eager work in between, and every replay is checked against
the CPU oracle."""
import numpy as np
import pytest

import workloads
from gpu_util import make_selector, table_args

pytestmark = pytest.mark.gpu


def _capture(fn):
    """Warm up on a side stream, then capture fn() into a graph."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g


def _fill(dst, src):
    import torch
    for d, x in zip(dst, src):
        d.copy_(torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)))


def test_graph_load_report_and_select(oracle_lib):
    import torch
    cfg, n = 1, 200_000
    tb = workloads.make_table(cfg)
    sel = make_selector(tb, engine=0)
    qs = [workloads.make_queries(cfg, n=n, chunk=c) for c in range(3)]
    ups = [workloads.make_load_update(cfg, tb.V, c + 1) for c in range(3)]
    dq = [torch.empty(n, dtype=torch.int32, device="cuda") for _ in range(4)]
    du = [torch.empty(ups[0].variant_idx.size, dtype=torch.int32, device="cuda") for _ in range(2)]
    out = torch.empty(n, dtype=torch.int32, device="cuda")
    clo = torch.empty_like(out)

    def step():
        sel.update_load(*du)
        sel.select_closest(*dq, out, clo)

    _fill(dq, (qs[0].task, qs[0].slo_us, qs[0].min_acc_bp, qs[0].batch_idx))
    _fill(du, (ups[0].variant_idx, ups[0].queue_us))
    graph = _capture(step)
    queue = tb.queue_us.copy()
    oracle_lib.update_load(queue, ups[0].variant_idx, ups[0].queue_us)       # applied by the warm-up and the capture run
    for rep in range(6):
        i = rep % 3
        q = qs[i]
        _fill(dq, (q.task, q.slo_us, q.min_acc_bp, q.batch_idx))
        _fill(du, (ups[i].variant_idx, ups[i].queue_us))
        out.fill_(-9); clo.fill_(-9)
        assert int((out + 1).sum().item()) == -8 * n                         # eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        oracle_lib.update_load(queue, ups[i].variant_idx, ups[i].queue_us)
        want = oracle_lib.select_closest(*table_args(tb, queue), q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
        print(f"graph replay {rep}", flush=True)
        assert np.array_equal(out.cpu().numpy(), want[0]) and np.array_equal(clo.cpu().numpy(), want[1]), f"replay {rep}"
    sel.destroy()


def test_graph_reports_workers_and_scaling(oracle_lib):
    """State report, worker report, the selection with workers and a batch of scaling decisions, up
    and down, in one graph."""
    import torch
    cfg, n, r = 1, 150_000, 50_000
    tb = workloads.make_table(cfg)
    st = workloads.make_states(cfg, tb.V)
    wk = workloads.make_workers(cfg, st)
    sc = workloads.make_scaling(cfg, tb)
    sel = make_selector(tb, engine=0)
    sel.load_states(st.state, st.load_us)
    sel.load_workers(wk.worker_hw, wk.worker_util, wk.variant_hw, wk.inst_variant, wk.inst_worker, wk.inst_load)
    sel.load_scaling(sc.arch_id, sc.sat_qps, sc.hw_cost, sc.load_us, 50, 105)
    sel.reserve(n)                                                            # the lists of open queries
    qs = [workloads.make_queries(cfg, n=n, chunk=c) for c in range(2)]
    sus = [workloads.make_state_update(cfg, tb.V, c + 1) for c in range(2)]
    wus = [workloads.make_worker_update(cfg, wk.W, wk.I, c + 1) for c in range(2)]
    rqs = [workloads.make_scale_requests(cfg, tb, sc, r, chunk=c) for c in range(2)]
    dq = [torch.empty(n, dtype=torch.int32, device="cuda") for _ in range(4)]
    ds = [torch.empty(sus[0].variant_idx.size, dtype=torch.int32, device="cuda") for _ in range(2)]
    dw = [torch.empty(x.size, dtype=torch.int32, device="cuda") for x in
          (wus[0].worker_idx, wus[0].worker_util, wus[0].inst_idx, wus[0].inst_load)]
    dr = [torch.empty(r, dtype=torch.int32, device="cuda") for _ in range(5)]
    res = [torch.empty(n, dtype=torch.int32, device="cuda") for _ in range(3)]
    dec = [torch.empty(r, dtype=torch.int32, device="cuda") for _ in range(3)]
    dec_down = [torch.empty(r, dtype=torch.int32, device="cuda") for _ in range(3)]

    def step():
        sel.update_state(*ds)
        sel.update_workers(*dw)
        sel.select_workers(*dq, *res)
        sel.scale(*dr, *dec)
        sel.scale_down(*dr, *dec_down)

    def stage(i):
        q, su, wu, rq = qs[i], sus[i], wus[i], rqs[i]
        _fill(dq, (q.task, q.slo_us, q.min_acc_bp, q.batch_idx))
        _fill(ds, (su.variant_idx, su.state))
        _fill(dw, (wu.worker_idx, wu.worker_util, wu.inst_idx, wu.inst_load))
        _fill(dr, (rq.variant, rq.instances, rq.load_qps, rq.slo_us, rq.batch_idx))

    state, util, iload = st.state.copy(), wk.worker_util.copy(), wk.inst_load.copy()

    def apply(i):
        oracle_lib.update_state(state, sus[i].variant_idx, sus[i].state)
        oracle_lib.update_worker_util(util, wus[i].worker_idx, wus[i].worker_util)
        oracle_lib.update_instance_load(iload, wus[i].inst_idx, wus[i].inst_load)

    stage(0)
    graph = _capture(step)
    apply(0)
    for rep in range(5):
        i = rep % 2
        stage(i)
        for t in res + dec + dec_down:
            t.fill_(-9)
        assert int((res[0] + 1).sum().item()) == -8 * n
        graph.replay()
        torch.cuda.synchronize()
        apply(i)
        q, rq = qs[i], rqs[i]
        want = oracle_lib.select_workers(*table_args(tb), state, st.load_us, wk.variant_hw, wk.worker_hw, util,
                                         wk.inst_variant, wk.inst_worker, iload, q.task, q.slo_us, q.min_acc_bp,
                                         q.batch_idx)
        want_dec = oracle_lib.scale(sc.arch_id, sc.sat_qps, sc.hw_cost, sc.load_us, tb.lat_us, 50, 105, rq.variant,
                                    rq.instances, rq.load_qps, rq.slo_us, rq.batch_idx)
        want_down = oracle_lib.scale_down(sc.arch_id, sc.sat_qps, sc.hw_cost, sc.load_us, tb.lat_us, 50, 105, rq.variant,
                                          rq.instances, rq.load_qps, rq.slo_us, rq.batch_idx)
        print(f"graph replay {rep}", flush=True)
        for g, w in zip(res + dec + dec_down, want + want_dec + want_down):
            assert np.array_equal(g.cpu().numpy(), w), f"replay {rep}"
    sel.destroy()
