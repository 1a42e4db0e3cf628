"""The group-by-group selection: tables whose staircase index does not fit one compute unit's LDS
have their tasks dealt to groups that do, and batches of a million queries or more are binned by
group, looked up with one group's index in LDS per workgroup, and put back into query order.  Every
answer is compared with the CPU oracle."""
import numpy as np
import pytest

import workloads
from gpu_util import gpu_select, make_selector, query_args, table_args, to_dev
from test_gpu_parity import _assert_equal_everywhere, _staircase_table, _table

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def test_groups_ragged_unaligned_and_invalid_queries(oracle_lib):
    """Configuration 3's table (8,000 slices, 11 groups), a batch that ends in the middle of a tile,
    query and result arrays that start 4 bytes into their allocations, and queries outside the table
    (unknown task, bad batch index, negative bound) mixed in."""
    import torch
    tb = workloads.make_table(3)
    n = 1_300_001
    q = workloads.make_queries(3, n=n)
    rng = np.random.default_rng(31)
    task, slo, acc, bidx = (x.copy() for x in query_args(q))
    bad = rng.random(n)
    task[bad < 0.01] = rng.choice([-1, tb.num_tasks, tb.num_tasks + 7, 2**31 - 1], int((bad < 0.01).sum()))
    bidx[(bad > 0.01) & (bad < 0.02)] = rng.choice([-1, tb.B, 99], int(((bad > 0.01) & (bad < 0.02)).sum()))
    slo[(bad > 0.02) & (bad < 0.03)] = -5
    acc[(bad > 0.03) & (bad < 0.04)] = rng.choice([-2**31, 2**31 - 1, 0], int(((bad > 0.03) & (bad < 0.04)).sum()))
    sel = make_selector(tb, engine=0)
    assert sel.info()["index_groups"] > 4
    want = oracle_lib.select(*table_args(tb), task, slo, acc, bidx)
    assert (want[bad < 0.03] == -1).all()
    for shift in (0, 1):
        dev = [torch.cat([torch.zeros(shift, dtype=torch.int32), torch.from_numpy(x)]).cuda()[shift:] for x in (task, slo, acc, bidx)]
        out = torch.full((n + shift,), -7, dtype=torch.int32, device="cuda")[shift:]
        _say(f"groups: N={n} shift={shift}")
        sel.select(*dev, out, n=n)
        torch.cuda.synchronize()
        _assert_equal_everywhere(out.cpu().numpy(), want, f"groups, arrays shifted by {shift}")
    # exactly one tile, one query more, one less than the threshold of the path (which then is not taken)
    for m in (1 << 20, (1 << 20) + 1, (1 << 20) - 1, 16384 * 65):
        got = gpu_select(sel, task[:m], slo[:m], acc[:m], bidx[:m])
        _assert_equal_everywhere(got, want[:m], f"groups, N={m}")
    sel.destroy()


def test_groups_follow_load_reports(oracle_lib):
    """Load reports rebuild the grouped index (every group's region is rewound and refilled); the
    next batch sees the new load."""
    tb = workloads.make_table(3)
    sel = make_selector(tb, engine=0)
    sel.reserve(1_500_000)
    queue = tb.queue_us.copy()
    for step in range(3):
        up = workloads.make_load_update(3, tb.V, chunk=step + 1, fraction=0.3)
        sel.update_load(to_dev(up.variant_idx), to_dev(up.queue_us))
        oracle_lib.update_load(queue, up.variant_idx, up.queue_us)
        q = workloads.make_queries(3, n=1_500_000, chunk=step + 1)
        _say(f"groups after report {step}")
        got = gpu_select(sel, *query_args(q))
        want = oracle_lib.select(*table_args(tb, queue), *query_args(q))
        _assert_equal_everywhere(got, want, f"groups after load report {step}")
    assert np.array_equal(sel.read_load(tb.V), queue)
    sel.destroy()


def test_groups_with_overflowing_regions_long_and_missing_staircases(oracle_lib):
    """12,000 one-batch-size tasks of 40 variants whose first row dominates the others when the table
    is loaded (one step per slice, so the tasks are dealt to few groups of many slices), 20 tasks
    with 300 steps (more than the index keeps: rank-ordered scan), one whose accuracies span more
    than 16 bits (no index at all) and two without variants.  A load report then slows the first
    rows down: every staircase grows to 40 steps, far more than the groups' regions hold, so most
    slices are stored behind the regions and answered from global memory; a second report restores
    half of the tasks."""
    rng = np.random.default_rng(77)
    T0, n0 = 12_000, 40
    i = np.tile(np.arange(n0, dtype=np.int64), T0)
    queue0 = (n0 - i) * 100
    queue0[i == 0] = 0                      # fastest and most accurate: dominates its task
    long_ = _staircase_table(20, 300, B=1)
    wide = _staircase_table(1, 40, B=1, acc0=-50_000, acc_step=5_000)
    T = T0 + 20 + 1 + 2
    task = np.concatenate([np.repeat(np.arange(T0, dtype=np.int32), n0), long_.task_id + T0, wide.task_id + T0 + 20])
    tb = _table(T, [1], task,
                np.concatenate([5000 - i, long_.acc_bp, wide.acc_bp]),
                np.concatenate([np.full((T0 * n0, 1), 1000), long_.lat_us, wide.lat_us]),
                np.concatenate([(10 + i)[:, None], long_.cost, wide.cost]),
                np.concatenate([queue0, long_.queue_us, wide.queue_us]))
    sel = make_selector(tb, engine=0)
    info = sel.info()
    _say(f"groups, staircases: groups={info['index_groups']} bytes={info['index_bytes']} truncated={info['index_truncated']}")
    assert info["index_groups"] >= 4 and info["index_truncated"] >= 21
    n = 1_200_000
    qt = rng.integers(0, T, n)
    special = rng.random(n) < 0.08
    qt[special] = T0 + rng.integers(0, 23, int(special.sum()))
    acc = np.where(qt < T0, 5000 - rng.integers(-3, n0 + 3, n), 1000 + rng.integers(-3, 310, n))
    acc[qt == T0 + 20] = rng.integers(-60_000, 150_000, int((qt == T0 + 20).sum()))
    slo = np.where(qt < T0, 1000 + rng.integers(-50, 4400, n),
                   rng.choice([100_000 + 50, 60_000, 97_000, 99_000, 70_000], n) + rng.integers(-300, 300, n))
    qs = tuple(np.asarray(x, np.int32) for x in (qt, slo, acc, np.zeros(n)))
    queue = tb.queue_us.copy()

    def check(label):
        got = gpu_select(sel, *qs)
        want = oracle_lib.select(*table_args(tb, queue), *qs)
        _assert_equal_everywhere(got, want, label)
        assert len(np.unique(want)) > 5000
        info = sel.info()
        _say(f"{label}: parked {info['lookup_parked']} second {info['lookup_second_body']} "
             f"memory {info['lookup_global_body']} scanned {info['lookup_scanned']} none {info['lookup_unanswered']}")
        return info

    def report(rows, value):
        vals = np.full(rows.size, value, np.int32)
        sel.update_load(to_dev(rows), to_dev(vals))
        oracle_lib.update_load(queue, rows, vals)

    info = check("groups, one-step staircases")
    assert info["lookup_scanned"] > 1000 and info["lookup_unanswered"] > 0 and info["lookup_global_body"] == 0
    first = (np.arange(T0) * n0).astype(np.int32)
    report(first, (n0 + 1) * 100)           # the first rows become the slowest: 40 steps everywhere
    info = check("groups, regions overflowing")
    assert info["lookup_global_body"] > n // 10 and info["lookup_second_body"] > 1000
    report(first[::2], 0)                   # every other task back to one step
    info = check("groups, half restored")
    assert info["lookup_global_body"] > 1000
    sel.destroy()


def test_groups_in_a_graph(oracle_lib):
    """The group-by-group call allocates nothing once its scratch exists: captured into a HIP graph
    with the load report in front of it and replayed with new inputs."""
    import torch
    from test_gpu_graph import _capture, _fill
    tb = workloads.make_table(3)
    n = 1_100_000
    sel = make_selector(tb, engine=0)
    sel.reserve(n)
    qs = [workloads.make_queries(3, n=n, chunk=c) for c in range(2)]
    ups = [workloads.make_load_update(3, tb.V, c + 1) for c in range(2)]
    dq = [torch.empty(n, dtype=torch.int32, device="cuda") for _ in range(4)]
    du = [torch.empty(ups[0].variant_idx.size, dtype=torch.int32, device="cuda") for _ in range(2)]
    out = torch.empty(n, dtype=torch.int32, device="cuda")

    def step():
        sel.update_load(*du)
        sel.select(*dq, out)

    _fill(dq, query_args(qs[0]))
    _fill(du, (ups[0].variant_idx, ups[0].queue_us))
    graph = _capture(step)
    queue = tb.queue_us.copy()
    oracle_lib.update_load(queue, ups[0].variant_idx, ups[0].queue_us)
    for rep in range(4):
        i = rep % 2
        _fill(dq, query_args(qs[i]))
        _fill(du, (ups[i].variant_idx, ups[i].queue_us))
        graph.replay()
        torch.cuda.synchronize()
        oracle_lib.update_load(queue, ups[i].variant_idx, ups[i].queue_us)
        want = oracle_lib.select(*table_args(tb, queue), *query_args(qs[i]))
        _assert_equal_everywhere(out.cpu().numpy(), want, f"graph replay {rep}")
        (out + 1).sum().item()   # eager work between the replays
    sel.destroy()
