"""Second, independently written enumerator of the selection rule (numpy).

Builds the whole feasibility mask of one query at a time and takes the first row of
a lexicographic sort.  Used only to pin the C oracle on small tables.
"""
import numpy as np


def select_np(task_id, acc_bp, lat_us, cost, queue_us, q_task, q_slo, q_min_acc, q_bidx):
    task_id = np.asarray(task_id, dtype=np.int64)
    acc_bp = np.asarray(acc_bp, dtype=np.int64)
    lat_us = np.asarray(lat_us, dtype=np.int64)
    cost = np.asarray(cost, dtype=np.int64)
    queue_us = np.asarray(queue_us, dtype=np.int64)
    V, B = lat_us.shape
    rows = np.arange(V, dtype=np.int64)
    out = np.full(len(q_task), -1, dtype=np.int32)
    for q in range(len(q_task)):
        b = int(q_bidx[q])
        if not 0 <= b < B:
            continue
        ok = (task_id == int(q_task[q]))
        ok &= acc_bp >= int(q_min_acc[q])
        ok &= (lat_us[:, b] + queue_us) <= int(q_slo[q])
        cand = rows[ok]
        if cand.size == 0:
            continue
        order = np.lexsort((cand, lat_us[cand, b], cost[cand, b]))  # last key is primary
        out[q] = cand[order[0]]
    return out


def count_np(task_id, acc_bp, lat_us, queue_us, q_task, q_slo, q_min_acc, q_bidx):
    task_id = np.asarray(task_id, dtype=np.int64)
    lat_us = np.asarray(lat_us, dtype=np.int64)
    V, B = lat_us.shape
    out = np.zeros(len(q_task), dtype=np.int32)
    for q in range(len(q_task)):
        b = int(q_bidx[q])
        if not 0 <= b < B:
            continue
        ok = (task_id == int(q_task[q])) & (np.asarray(acc_bp, dtype=np.int64) >= int(q_min_acc[q]))
        ok &= (lat_us[:, b] + np.asarray(queue_us, dtype=np.int64)) <= int(q_slo[q])
        out[q] = int(ok.sum())
    return out


def closest_np(task_id, acc_bp, lat_us, cost, queue_us, q_task, q_slo, q_min_acc, q_bidx):
    """Closest variant by CASES instead of one lexicographic key: if some variant of the task
    meets the latency objective, the most accurate of those; else if some variant meets the
    accuracy minimum, the fastest (latency + queue) of those; else the fastest of all, the most
    accurate among equally fast ones.  Remaining ties by (cost, lat, row).  A query with a
    feasible variant gets the selected variant.  -1 when the task has no row at that batch index."""
    task_id = np.asarray(task_id, dtype=np.int64)
    acc_bp = np.asarray(acc_bp, dtype=np.int64)
    lat_us = np.asarray(lat_us, dtype=np.int64)
    cost = np.asarray(cost, dtype=np.int64)
    queue_us = np.asarray(queue_us, dtype=np.int64)
    V, B = lat_us.shape
    out = np.full(len(q_task), -1, dtype=np.int32)

    def first_by_key(cand, b):
        return cand[np.lexsort((cand, lat_us[cand, b], cost[cand, b]))[0]]

    for q in range(len(q_task)):
        b = int(q_bidx[q])
        if not 0 <= b < B:
            continue
        rows = np.flatnonzero(task_id == int(q_task[q]))
        if rows.size == 0:
            continue
        tot = lat_us[rows, b] + queue_us[rows]
        fits = tot <= int(q_slo[q])
        accurate = acc_bp[rows] >= int(q_min_acc[q])
        if (fits & accurate).any():
            out[q] = first_by_key(rows[fits & accurate], b)
        elif fits.any():
            r = rows[fits]
            out[q] = first_by_key(r[acc_bp[r] == acc_bp[r].max()], b)
        elif accurate.any():
            r = rows[accurate]; t = tot[accurate]
            out[q] = first_by_key(r[t == t.min()], b)
        else:
            r = rows[tot == tot.min()]
            out[q] = first_by_key(r[acc_bp[r] == acc_bp[r].max()], b)
    return out


def closest_key_np(task_id, acc_bp, lat_us, cost, queue_us, q_task, q_slo, q_min_acc, q_bidx):
    """The same by sorting the task's rows on (missed, overshoot, shortfall, cost, lat, row)."""
    task_id = np.asarray(task_id, dtype=np.int64)
    acc_bp = np.asarray(acc_bp, dtype=np.int64)
    lat_us = np.asarray(lat_us, dtype=np.int64)
    cost = np.asarray(cost, dtype=np.int64)
    queue_us = np.asarray(queue_us, dtype=np.int64)
    V, B = lat_us.shape
    out = np.full(len(q_task), -1, dtype=np.int32)
    for q in range(len(q_task)):
        b = int(q_bidx[q])
        if not 0 <= b < B:
            continue
        rows = np.flatnonzero(task_id == int(q_task[q]))
        if rows.size == 0:
            continue
        over = np.maximum(lat_us[rows, b] + queue_us[rows] - int(q_slo[q]), 0)
        short = np.maximum(int(q_min_acc[q]) - acc_bp[rows], 0)
        missed = (over > 0).astype(np.int64) + (short > 0)
        out[q] = rows[np.lexsort((rows, lat_us[rows, b], cost[rows, b], short, over, missed))[0]]
    return out


def tiered_np(task_id, acc_bp, lat_us, cost, queue_us, state, load_us, q_task, q_slo, q_min_acc, q_bidx):
    """State-aware selection: cheapest matching Active variant, else the matching Inactive variant
    with the lowest load + inference latency; returns (variant, tier)."""
    task_id = np.asarray(task_id, dtype=np.int64)
    acc_bp = np.asarray(acc_bp, dtype=np.int64)
    lat_us = np.asarray(lat_us, dtype=np.int64)
    cost = np.asarray(cost, dtype=np.int64)
    queue_us = np.asarray(queue_us, dtype=np.int64)
    state = np.asarray(state, dtype=np.int64)
    load_us = np.asarray(load_us, dtype=np.int64)
    V, B = lat_us.shape
    rows = np.arange(V, dtype=np.int64)
    out = np.full(len(q_task), -1, dtype=np.int32)
    tier = np.zeros(len(q_task), dtype=np.int32)
    for q in range(len(q_task)):
        b = int(q_bidx[q])
        if not 0 <= b < B:
            continue
        mine = (task_id == int(q_task[q])) & (acc_bp >= int(q_min_acc[q]))
        act = rows[mine & (state == 1) & (lat_us[:, b] + queue_us <= int(q_slo[q]))]
        if act.size:
            out[q] = act[np.lexsort((act, lat_us[act, b], cost[act, b]))[0]]
            tier[q] = 1
            continue
        ina = rows[mine & (state == 0) & (load_us + lat_us[:, b] <= int(q_slo[q]))]
        if ina.size:
            out[q] = ina[np.lexsort((ina, lat_us[ina, b], load_us[ina] + lat_us[ina, b]))[0]]
            tier[q] = 2
    return out, tier


def case1_np(task_id, acc_bp, lat_us, cost, queue_us, state, load_us, q_task, q_slo, q_min_acc, q_bidx):
    """Complete Case I: tiered_np, and where that finds nothing the first Active or Inactive variant
    of the task under (requirements missed, latency beyond the objective, accuracy below the minimum,
    Active before Inactive, the tier's own order); latency = lat + queue (Active), load + lat (Inactive).
    Returns (variant, tier, suggestion)."""
    out, tier = tiered_np(task_id, acc_bp, lat_us, cost, queue_us, state, load_us, q_task, q_slo, q_min_acc, q_bidx)
    task_id = np.asarray(task_id, dtype=np.int64)
    acc_bp = np.asarray(acc_bp, dtype=np.int64)
    lat_us = np.asarray(lat_us, dtype=np.int64)
    cost = np.asarray(cost, dtype=np.int64)
    queue_us = np.asarray(queue_us, dtype=np.int64)
    state = np.asarray(state, dtype=np.int64)
    load_us = np.asarray(load_us, dtype=np.int64)
    V, B = lat_us.shape
    closest = out.copy()
    for q in np.flatnonzero(out < 0):
        b = int(q_bidx[q])
        if not 0 <= b < B:
            continue
        rows = np.flatnonzero((task_id == int(q_task[q])) & ((state == 0) | (state == 1)))
        if rows.size == 0:
            continue
        act = state[rows] == 1
        total = lat_us[rows, b] + np.where(act, queue_us[rows], load_us[rows])
        over = np.maximum(total - int(q_slo[q]), 0)
        short = np.maximum(int(q_min_acc[q]) - acc_bp[rows], 0)
        missed = (over > 0).astype(np.int64) + (short > 0)
        first_key = np.where(act, cost[rows, b], load_us[rows] + lat_us[rows, b])   # the tier's own order: its first part
        closest[q] = rows[np.lexsort((rows, lat_us[rows, b], first_key, ~act, short, over, missed))[0]]
    return out, tier, closest


def workers_np(variant, tier, variant_hw, worker_hw, worker_util, inst_variant, inst_worker, inst_load):
    """Worker for every (variant, tier) decision: tier 1 -> the worker of the variant's instance
    with the smallest (load, worker); tier 2 -> the worker of the variant's hardware class with the
    smallest (utilisation, worker); otherwise, or when there is no candidate, -1."""
    variant_hw = np.asarray(variant_hw, dtype=np.int64)
    worker_hw = np.asarray(worker_hw, dtype=np.int64)
    worker_util = np.asarray(worker_util, dtype=np.int64)
    inst_variant = np.asarray(inst_variant, dtype=np.int64)
    inst_worker = np.asarray(inst_worker, dtype=np.int64)
    inst_load = np.asarray(inst_load, dtype=np.int64)
    ids = np.arange(worker_hw.size, dtype=np.int64)
    out = np.full(len(variant), -1, dtype=np.int32)
    for q in range(len(variant)):
        v = int(variant[q])
        if tier[q] == 1:
            mine = np.flatnonzero(inst_variant == v)
            if mine.size:
                out[q] = inst_worker[mine[np.lexsort((inst_worker[mine], inst_load[mine]))[0]]]
        elif tier[q] == 2:
            cand = ids[worker_hw == variant_hw[v]]
            if cand.size:
                out[q] = cand[np.lexsort((cand, worker_util[cand]))[0]]
    return out


def instances_np(task_id, acc_bp, lat_us, cost, queue_us, load_us, variant_hw, worker_hw, worker_util,
                 inst_variant, inst_worker, inst_load, inst_state, q_task, q_slo, q_min_acc, q_bidx):
    """Case I with the state kept per running instance, written out per query and per variant: a
    variant with an Active instance (code 1) competes in the first step and is served by the Active
    instance with the smallest (load, worker); a variant that runs nowhere competes in the second
    step and is served by the least-utilised worker of its hardware; any other variant is skipped.
    Returns (variant, tier, worker)."""
    lat_us = np.asarray(lat_us, dtype=np.int64)
    cost = np.asarray(cost, dtype=np.int64)
    V, B = lat_us.shape
    inst_variant = np.asarray(inst_variant, dtype=np.int64)
    inst_state = np.asarray(inst_state, dtype=np.int64)
    out = np.full(len(q_task), -1, dtype=np.int32)
    tier = np.zeros(len(q_task), dtype=np.int32)
    worker = np.full(len(q_task), -1, dtype=np.int32)
    for q in range(len(q_task)):
        b = int(q_bidx[q])
        if not 0 <= b < B:
            continue
        best1 = best2 = None
        for v in range(V):
            if int(task_id[v]) != int(q_task[q]) or int(acc_bp[v]) < int(q_min_acc[q]):
                continue
            mine = np.flatnonzero(inst_variant == v)
            serving = [int(i) for i in mine if inst_state[i] == 1]
            if serving:
                if int(lat_us[v, b]) + int(queue_us[v]) <= int(q_slo[q]):
                    key = (int(cost[v, b]), int(lat_us[v, b]), v)
                    if best1 is None or key < best1[0]:
                        best1 = (key, min((int(inst_load[i]), int(inst_worker[i])) for i in serving)[1])
            elif mine.size == 0:
                if int(load_us[v]) + int(lat_us[v, b]) <= int(q_slo[q]):
                    key = (int(load_us[v]) + int(lat_us[v, b]), int(lat_us[v, b]), v)
                    if best2 is None or key < best2[0]:
                        cand = [(int(worker_util[w]), w) for w in range(len(worker_hw)) if int(worker_hw[w]) == int(variant_hw[v])]
                        best2 = (key, min(cand)[1] if cand else -1)
        if best1 is not None:
            out[q], tier[q], worker[q] = best1[0][2], 1, best1[1]
        elif best2 is not None:
            out[q], tier[q], worker[q] = best2[0][2], 2, best2[1]
    return out, tier, worker
