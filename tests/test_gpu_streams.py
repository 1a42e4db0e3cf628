"""Two handles with different tables working at the same time on two streams: every answer against the
CPU oracle.  A handle owns its table, index and scratch memory, so handles do not have to be ordered
with each other (only infaas_sel_select_noalloc shares memory between handles)."""
import numpy as np
import pytest

import workloads
from gpu_util import make_selector, query_args, table_args, to_dev

pytestmark = pytest.mark.gpu


def test_two_handles_on_two_streams(oracle_lib):
    import torch
    cfgs, n, rounds = (1, 4), 600_000, 3
    tabs = [workloads.make_table(c) for c in cfgs]
    sels = [make_selector(tb, engine=0) for tb in tabs]
    for sel in sels:
        sel.reserve(n)
    streams = [torch.cuda.Stream() for _ in cfgs]
    queues = [tb.queue_us.copy() for tb in tabs]
    batches = [[workloads.make_queries(c, n=n, chunk=r) for r in range(rounds)] for c in cfgs]
    reports = [[workloads.make_load_update(c, tb.V, r + 1) for r in range(rounds)] for c, tb in zip(cfgs, tabs)]
    dev_q = [[[to_dev(x) for x in query_args(q)] for q in qs] for qs in batches]
    dev_r = [[(to_dev(u.variant_idx), to_dev(u.queue_us)) for u in us] for us in reports]
    outs = [[torch.full((n,), -777, dtype=torch.int32, device="cuda") for _ in range(rounds)] for _ in cfgs]
    torch.cuda.synchronize()
    # report, select, report, select ... on each handle's own stream, the two streams interleaved
    for r in range(rounds):
        for k in range(2):
            with torch.cuda.stream(streams[k]):
                sels[k].update_load(*dev_r[k][r])
                sels[k].select(*dev_q[k][r], outs[k][r])
    torch.cuda.synchronize()
    for k, (c, tb) in enumerate(zip(cfgs, tabs)):
        for r in range(rounds):
            oracle_lib.update_load(queues[k], reports[k][r].variant_idx, reports[k][r].queue_us)
            print(f"two streams: config {c} round {r}", flush=True)
            want = oracle_lib.select(*table_args(tb, queues[k]), *query_args(batches[k][r]))
            got = outs[k][r].cpu().numpy()
            bad = np.flatnonzero(got != want)
            assert bad.size == 0, f"config {c} round {r}: {bad.size} differ, first at {bad[:5]}"
    for sel in sels:
        sel.destroy()
