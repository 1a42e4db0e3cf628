"""Helpers of the GPU parity tests: move inputs to the device, call the library, bring results back."""
import numpy as np


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


class DeviceQueries:
    def __init__(self, task, slo, min_acc, bidx):
        import torch
        self.task, self.slo, self.min_acc, self.bidx = (to_dev(x) for x in (task, slo, min_acc, bidx))
        self.out = torch.full((max(self.task.numel(), 1),), -12345, dtype=torch.int32, device="cuda")
        self.n = int(self.task.numel())


def gpu_select(sel, task, slo, min_acc, bidx):
    """Run infaas_sel_select on host arrays; returns the host result."""
    import torch
    dq = DeviceQueries(task, slo, min_acc, bidx)
    sel.select(dq.task, dq.slo, dq.min_acc, dq.bidx, dq.out, n=dq.n)
    torch.cuda.synchronize()
    return dq.out[:dq.n].cpu().numpy()


def make_selector(table, engine=0, lds_segment_limit=0):
    import paper_1905_13348_amd as lib
    sel = lib.Selector(table.num_tasks, table.batch_sizes, device=0, engine=engine,
                       lds_segment_limit=lds_segment_limit)
    sel.load_variants(table.task_id, table.acc_bp, table.lat_us, table.cost, table.queue_us)
    return sel


def table_args(tb, queue=None):
    return (tb.task_id, tb.acc_bp, tb.lat_us, tb.cost, tb.queue_us if queue is None else queue)


def query_args(q):
    return (q.task, q.slo_us, q.min_acc_bp, q.batch_idx)


def gpu_select_closest(sel, task, slo, min_acc, bidx):
    """Run infaas_sel_select_closest on host arrays; returns (selection, suggestion) on the host."""
    import torch
    dq = DeviceQueries(task, slo, min_acc, bidx)
    closest = torch.full_like(dq.out, -54321)
    sel.select_closest(dq.task, dq.slo, dq.min_acc, dq.bidx, dq.out, closest, n=dq.n)
    torch.cuda.synchronize()
    return dq.out[:dq.n].cpu().numpy(), closest[:dq.n].cpu().numpy()
