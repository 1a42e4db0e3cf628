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
