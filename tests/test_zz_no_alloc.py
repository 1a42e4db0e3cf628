"""infaas_sel_select_noalloc (the entry point that allocates nothing: its scratch is a static device
array of the library) against infaas_sel_select, through the C ABI, bit-exact."""
import ctypes

import numpy as np
import pytest

import workloads
from gpu_util import DeviceQueries, make_selector, query_args, table_args

pytestmark = pytest.mark.gpu


def _both(sel, q, n):
    """Answers of the two entry points for the first n queries of q."""
    import torch
    dq = DeviceQueries(q.task[:n], q.slo_us[:n], q.min_acc_bp[:n], q.batch_idx[:n])
    sel.select(dq.task, dq.slo, dq.min_acc, dq.bidx, dq.out, n=n)
    torch.cuda.synchronize()
    want = dq.out[:n].cpu().numpy().copy()
    dq.out.fill_(-777)
    sel.select_noalloc(dq.task, dq.slo, dq.min_acc, dq.bidx, dq.out, n=n)
    torch.cuda.synchronize()
    return dq.out[:n].cpu().numpy(), want


def test_noalloc_matches_select_on_two_calls_in_a_row(oracle_lib):
    """Configuration 2's table (staircases with second bodies: the parked-query queues, which are
    what lives in the static array, are used by every wavefront); a large call, then a smaller one
    that finds the array as the first call left it; then a call after a load report."""
    import torch
    tb = workloads.make_table(2)
    q = workloads.make_queries(2, n=3_000_000)
    sel = make_selector(tb)
    assert sel.info()["index_max_steps"] > 31       # second bodies exist, so queries get parked
    got, want = _both(sel, q, 3_000_000)
    assert np.array_equal(got, want)
    got2, want2 = _both(sel, q, 70_001)             # smaller, ragged
    assert np.array_equal(got2, want2)
    ref = oracle_lib.select(*table_args(tb), *(f[:70_001] for f in query_args(q)))
    assert np.array_equal(got2, ref)
    up = workloads.make_load_update(4, tb.V, chunk=1)
    sel.update_load(torch.from_numpy(up.variant_idx).cuda(), torch.from_numpy(up.queue_us).cuda())
    got3, want3 = _both(sel, q, 500_000)
    assert np.array_equal(got3, want3)
    assert not np.array_equal(got3, want[:500_000])   # the report changed answers
    sel.destroy()


def test_noalloc_small_tables_and_limits():
    import torch
    import paper_1905_13348_amd as lib
    tb = workloads.make_table(0)
    q = workloads.make_queries(0)
    sel = make_selector(tb)
    got, want = _both(sel, q, q.N)
    assert np.array_equal(got, want)
    got, want = _both(sel, q, 1)
    assert np.array_equal(got, want)
    dq = DeviceQueries(q.task, q.slo_us, q.min_acc_bp, q.batch_idx)
    sel.select_noalloc(dq.task, dq.slo, dq.min_acc, dq.bidx, dq.out, n=0)   # no-op
    # beyond the limit: refused with a clear message before any pointer is used
    raw = lib.load_library()
    rc = raw.infaas_sel_select_noalloc(sel._h, ctypes.c_int64((1 << 28) + 1), dq.task.data_ptr(), dq.slo.data_ptr(),
                                       dq.min_acc.data_ptr(), dq.bidx.data_ptr(), dq.out.data_ptr(), None)
    assert rc == -1 and b"exceed the limit" in raw.infaas_sel_last_error()
    sel.destroy()
    # a handle of the exhaustive-scan engine has no index: refused
    scan = make_selector(tb, engine=lib.ENGINE_SCAN)
    with pytest.raises(lib.InfaasSelError) as e:
        scan.select_noalloc(dq.task, dq.slo, dq.min_acc, dq.bidx, dq.out, n=q.N)
    assert e.value.status == -1
    scan.destroy()
    torch.cuda.synchronize()
