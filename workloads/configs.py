"""Synthetic workloads shaped like the paper's variant population and query mix.

The paper's own populations (its profiled variants, Section 6 / Appendix table of
model architectures; the production trace of Section 6.1) are not available, so
every table and query stream here is drawn from a seeded generator.  What is
taken from the paper is only the *shape*: accuracies spread over tens of
percent, single-query latencies spread over three to four orders of magnitude,
hardware prices spread over roughly one order of magnitude (Section 2.1),
per-batch-size latency profiles at power-of-two batch sizes (Section 5), Zipf
task popularity (Section 6.1) and "thousands of variants" per task (Section 1).

All fields are int32.  Generator: numpy ``Generator(PCG64(seed))``.  The draw
order inside each function is part of the recipe -- changing it changes every
stored expectation -- and is spelled out in the comments.

Five workload configurations:

  0 tiny       8 tasks x 32 variants,        4 batch sizes {1,4,16,64},   10,000 queries
  1 medium     100 tasks x 200 variants,     8 batch sizes {1..128},      1M queries
  2 thousands  50 tasks x 2,000 variants,    8 batch sizes,               16M queries, Zipf(1.1) tasks
  3 skewed     1,000 tasks, lognormal sizes, 8 batch sizes,               64M queries, bimodal SLO
  4 streaming  config 2's table,             256M queries in 64 chunks of 4M, 10% load redraw per chunk
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

CONFIG_NAMES = ("tiny", "medium", "thousands", "skewed", "streaming")

_SEED0 = 190513348  # one documented seed per configuration: _SEED0 + config id


def base_seed(cfg: int) -> int:
    """Seed of configuration ``cfg``'s variant table (config 4 shares config 2's)."""
    return _SEED0 + (2 if cfg == 4 else cfg)


@dataclass
class VariantTable:
    num_tasks: int
    batch_sizes: np.ndarray  # [B] int32
    task_id: np.ndarray      # [V] int32, caller order (NOT grouped by task)
    acc_bp: np.ndarray       # [V] int32, accuracy in basis points
    lat_us: np.ndarray       # [V, B] int32, profiled latency per batch size
    cost: np.ndarray         # [V, B] int32, per-query cost per batch size
    queue_us: np.ndarray     # [V] int32, current queueing delay

    @property
    def V(self) -> int:
        return int(self.task_id.shape[0])

    @property
    def B(self) -> int:
        return int(self.batch_sizes.shape[0])


@dataclass
class QueryBatch:
    task: np.ndarray        # [N] int32
    slo_us: np.ndarray      # [N] int32
    min_acc_bp: np.ndarray  # [N] int32
    batch_idx: np.ndarray   # [N] int32, index into VariantTable.batch_sizes

    @property
    def N(self) -> int:
        return int(self.task.shape[0])


@dataclass
class LoadUpdate:
    variant_idx: np.ndarray  # [n] int32, distinct caller-order variant rows
    queue_us: np.ndarray     # [n] int32, new queueing delay


def config_spec(cfg: int) -> dict:
    """Static description of one configuration (no random draws)."""
    if cfg == 0:
        return dict(name="tiny", num_tasks=8, per_task=32, batch_sizes=[1, 4, 16, 64],
                    num_queries=10_000, chunks=1, task_popularity="uniform", slo="unimodal")
    if cfg == 1:
        return dict(name="medium", num_tasks=100, per_task=200,
                    batch_sizes=[1, 2, 4, 8, 16, 32, 64, 128],
                    num_queries=1_000_000, chunks=1, task_popularity="uniform", slo="unimodal")
    if cfg == 2:
        return dict(name="thousands", num_tasks=50, per_task=2000,
                    batch_sizes=[1, 2, 4, 8, 16, 32, 64, 128],
                    num_queries=16_000_000, chunks=1, task_popularity="zipf1.1", slo="unimodal")
    if cfg == 3:
        return dict(name="skewed", num_tasks=1000, per_task=None,
                    batch_sizes=[1, 2, 4, 8, 16, 32, 64, 128],
                    num_queries=64_000_000, chunks=1, task_popularity="uniform", slo="bimodal")
    if cfg == 4:
        return dict(name="streaming", num_tasks=50, per_task=2000,
                    batch_sizes=[1, 2, 4, 8, 16, 32, 64, 128],
                    num_queries=256_000_000, chunks=64, task_popularity="zipf1.1", slo="unimodal",
                    update_fraction=0.10)
    raise ValueError(f"unknown configuration {cfg}")


def _segment_sizes(cfg: int, rng: np.random.Generator) -> np.ndarray:
    spec = config_spec(cfg)
    T = spec["num_tasks"]
    if spec["per_task"] is not None:
        return np.full(T, spec["per_task"], dtype=np.int64)
    # config 3: lognormal with ARITHMETIC mean 100 and sigma 1.5, clamped to 1..20000
    sigma = 1.5
    mu = np.log(100.0) - 0.5 * sigma * sigma
    sizes = np.rint(rng.lognormal(mu, sigma, size=T)).astype(np.int64)
    return np.clip(sizes, 1, 20000)


def make_variant_fields(rng: np.random.Generator, V: int, batch_sizes: np.ndarray):
    """Draw the per-variant fields.  Draw order: acc, hw class, base latency, alpha, queue."""
    acc_bp = rng.integers(5000, 9501, size=V, dtype=np.int64)
    hw = rng.integers(0, 3, size=V, dtype=np.int64)
    price = np.array([1, 4, 9], dtype=np.int64)[hw]
    base_us = np.clip(rng.lognormal(np.log(2000.0), 1.0, size=V), 100.0, 500000.0)
    alpha = rng.uniform(0.3, 1.0, size=V)
    queue_us = rng.integers(0, 50001, size=V, dtype=np.int64)
    b = batch_sizes.astype(np.float64)[None, :]
    lat = np.rint(base_us[:, None] * b ** alpha[:, None]).astype(np.int64)
    lat = np.maximum(lat, 1)
    bi = batch_sizes.astype(np.int64)[None, :]
    cost = (lat * price[:, None] + bi - 1) // bi          # ceil(lat * price / b)
    return (acc_bp.astype(np.int32), lat.astype(np.int32), cost.astype(np.int32),
            queue_us.astype(np.int32))


def make_table(cfg: int, seed: Optional[int] = None) -> VariantTable:
    """Variant table of configuration ``cfg``.

    Draw order: segment sizes (config 3 only), variant fields (see
    ``make_variant_fields``), then one permutation that shuffles the rows so that
    the caller's order is not grouped by task.
    """
    spec = config_spec(cfg)
    rng = np.random.default_rng(np.random.PCG64(base_seed(cfg) if seed is None else seed))
    sizes = _segment_sizes(cfg, rng)
    T = spec["num_tasks"]
    V = int(sizes.sum())
    batch_sizes = np.asarray(spec["batch_sizes"], dtype=np.int32)
    task_sorted = np.repeat(np.arange(T, dtype=np.int32), sizes)
    acc, lat, cost, queue = make_variant_fields(rng, V, batch_sizes)
    perm = rng.permutation(V)
    return VariantTable(num_tasks=T, batch_sizes=batch_sizes, task_id=task_sorted[perm].copy(),
                        acc_bp=acc, lat_us=lat, cost=cost, queue_us=queue)


def _task_probabilities(spec: dict) -> Optional[np.ndarray]:
    if spec["task_popularity"] == "uniform":
        return None
    T = spec["num_tasks"]
    w = (np.arange(T, dtype=np.float64) + 1.0) ** -1.1   # bounded Zipf over task ids 0..T-1
    return w / w.sum()


def make_queries(cfg: int, n: Optional[int] = None, chunk: int = 0,
                 seed: Optional[int] = None) -> QueryBatch:
    """Query stream of configuration ``cfg`` (``n`` queries; default: the configured size,
    or one chunk of it for the streaming configuration).

    Seed: base_seed(cfg) + 1000 + chunk for config 4's chunks, base_seed(cfg) + 1000 otherwise
    (config 4 uses its own stream: _SEED0 + 4 + 1000 + chunk).
    Draw order: task, SLO (for the bimodal mix: component selector, then both components),
    minimum accuracy, batch index.
    """
    spec = config_spec(cfg)
    if n is None:
        n = spec["num_queries"] // spec["chunks"]
    if seed is None:
        seed = _SEED0 + cfg + 1000 + chunk
    rng = np.random.default_rng(np.random.PCG64(seed))
    T = spec["num_tasks"]
    B = len(spec["batch_sizes"])
    p = _task_probabilities(spec)
    if p is None:
        task = rng.integers(0, T, size=n, dtype=np.int64)
    else:
        task = rng.choice(T, size=n, p=p)
    if spec["slo"] == "unimodal":
        slo = rng.lognormal(np.log(20000.0), 1.0, size=n)
    else:
        pick = rng.random(size=n) < 0.5
        lo = rng.lognormal(np.log(5000.0), 1.0, size=n)
        hi = rng.lognormal(np.log(200000.0), 1.0, size=n)
        slo = np.where(pick, lo, hi)
        del pick, lo, hi
    slo = np.clip(np.rint(slo), 1000, 2_000_000)
    min_acc = rng.integers(5000, 9501, size=n, dtype=np.int64)
    bidx = rng.integers(0, B, size=n, dtype=np.int64)
    return QueryBatch(task=task.astype(np.int32), slo_us=slo.astype(np.int32),
                      min_acc_bp=min_acc.astype(np.int32), batch_idx=bidx.astype(np.int32))


def make_load_update(cfg: int, V: int, chunk: int, fraction: float = 0.10,
                     seed: Optional[int] = None) -> LoadUpdate:
    """Load redraw applied before chunk ``chunk`` (>= 1) of the streaming configuration:
    ``fraction`` of the variants, chosen without replacement, get a new queueing delay
    uniform in 0..200000.  Seed: _SEED0 + cfg + 5000 + chunk.  Draw order: rows, values.
    """
    if seed is None:
        seed = _SEED0 + cfg + 5000 + chunk
    rng = np.random.default_rng(np.random.PCG64(seed))
    n = int(round(V * fraction))
    rows = rng.choice(V, size=n, replace=False)
    vals = rng.integers(0, 200001, size=n, dtype=np.int64)
    return LoadUpdate(variant_idx=rows.astype(np.int32), queue_us=vals.astype(np.int32))


# ---------------------------------------------------------------- tables and reports the index handles badly

def make_degrading_load_update(tb: VariantTable) -> LoadUpdate:
    """A load report over ALL rows under which the cheaper a variant of a task is (at the first batch
    size), the longer its queue: latency plus queue then falls along the cost order, so that (at the
    first batch size exactly, at the others mostly) no variant dominates a dearer one and every variant
    is a possible answer.  The worst case for an index of non-dominated variants; no randomness."""
    queue = np.zeros(tb.V, dtype=np.int64)
    for t in range(tb.num_tasks):
        rows = np.flatnonzero(tb.task_id == t)
        order = rows[np.argsort(tb.cost[rows, 0], kind="stable")]
        queue[order] = (order.size - np.arange(order.size)) * 600_000
    assert queue.max() < 2**31 - 1
    return LoadUpdate(variant_idx=np.arange(tb.V, dtype=np.int32), queue_us=queue.astype(np.int32))


def make_cliff_table(kind: str, cfg: int = 2) -> VariantTable:
    """Configuration ``cfg``'s table bent into a shape the staircase index cannot hold:
    'long_staircases': in every task accuracy rises and latency falls with the cost, so every variant
    is a possible answer (thousands of steps per slice, of which the index keeps 62);
    'wide_accuracy': accuracies spread over 200,001 values, more than the 16-bit keys of the index span."""
    tb = make_table(cfg)
    if kind == "wide_accuracy":
        rng = np.random.default_rng(np.random.PCG64(_SEED0 + cfg + 21000))
        tb.acc_bp = rng.integers(-100_000, 100_001, size=tb.V, dtype=np.int64).astype(np.int32)
        return tb
    if kind != "long_staircases":
        raise ValueError(f"unknown table kind {kind}")
    b = np.arange(tb.B, dtype=np.int64)[None, :]
    for t in range(tb.num_tasks):
        rows = np.flatnonzero(tb.task_id == t)
        i = np.arange(rows.size, dtype=np.int64)
        tb.acc_bp[rows] = 5000 + (4500 * i) // max(rows.size, 1)
        tb.lat_us[rows] = (60_000 - (59_000 * i) // max(rows.size, 1))[:, None] + 10 * b
        tb.cost[rows] = (100 + i)[:, None] + b
        tb.queue_us[rows] = 0
    return tb


# ---------------------------------------------------------------- variant states (state-aware selection)

@dataclass
class VariantStates:
    """Dynamic state and loading latency of every variant (Section 4: Inactive 0, Active 1,
    Overloaded 2, Interfered 3)."""
    state: np.ndarray     # [V] int32
    load_us: np.ndarray   # [V] int32


@dataclass
class StateUpdate:
    variant_idx: np.ndarray   # [n] int32, distinct rows
    state: np.ndarray         # [n] int32


_STATE_P = (0.50, 0.40, 0.05, 0.05)   # Inactive, Active, Overloaded, Interfered


def make_states(cfg: int, V: int, seed: Optional[int] = None) -> VariantStates:
    """Stand-in for the state the paper's monitoring daemons keep (it publishes no population):
    state drawn with probabilities (0.50, 0.40, 0.05, 0.05) for (Inactive, Active, Overloaded,
    Interfered); loading latency = clamp(lognormal(ln 20000, 1.5), 100, 5,000,000) microseconds,
    so that part of the unloaded variants can still meet the latency objectives of the query
    generator.  Seed: _SEED0 + cfg + 7000.  Draw order: states, loading latencies."""
    if seed is None:
        seed = _SEED0 + cfg + 7000
    rng = np.random.default_rng(np.random.PCG64(seed))
    state = rng.choice(4, size=V, p=_STATE_P).astype(np.int32)
    load = np.clip(np.rint(rng.lognormal(np.log(20000.0), 1.5, size=V)), 100, 5_000_000)
    return VariantStates(state=state, load_us=load.astype(np.int32))


def make_state_update(cfg: int, V: int, chunk: int, fraction: float = 0.05,
                      seed: Optional[int] = None) -> StateUpdate:
    """State report before chunk ``chunk``: ``fraction`` of the variants, chosen without
    replacement, get a new state drawn as in make_states.  Seed: _SEED0 + cfg + 9000 + chunk."""
    if seed is None:
        seed = _SEED0 + cfg + 9000 + chunk
    rng = np.random.default_rng(np.random.PCG64(seed))
    n = int(round(V * fraction))
    rows = rng.choice(V, size=n, replace=False)
    vals = rng.choice(4, size=n, p=_STATE_P)
    return StateUpdate(variant_idx=rows.astype(np.int32), state=vals.astype(np.int32))


@dataclass
class WorkerTables:
    """Workers and running instances (Sections 4.1 and 5: an instance is a {variant, worker} pair)."""
    variant_hw: np.ndarray    # [V] int32, target hardware class of every variant
    worker_hw: np.ndarray     # [W] int32, hardware class of every worker
    worker_util: np.ndarray   # [W] int32, utilisation in basis points
    inst_variant: np.ndarray  # [I] int32
    inst_worker: np.ndarray   # [I] int32
    inst_load: np.ndarray     # [I] int32, load figure of the instance (outstanding queries)

    @property
    def W(self) -> int:
        return int(self.worker_hw.shape[0])

    @property
    def I(self) -> int:
        return int(self.inst_variant.shape[0])


@dataclass
class WorkerUpdate:
    worker_idx: np.ndarray    # [n] int32, distinct workers
    worker_util: np.ndarray   # [n] int32
    inst_idx: np.ndarray      # [m] int32, distinct instances
    inst_load: np.ndarray     # [m] int32


_NUM_WORKERS = {0: 48, 1: 256, 2: 1024, 3: 2048, 4: 1024}
_NUM_HW = 3   # the paper's cluster has three kinds of hardware (CPU, GPU, Inferentia)


def make_workers(cfg: int, states: VariantStates, seed: Optional[int] = None) -> WorkerTables:
    """Stand-in for the cluster the paper's controller sees (it publishes no such table): W workers
    (48 / 256 / 1024 / 2048 / 1024 for configs 0..4) of hardware class U{0,1,2} with utilisation
    U{0..10000} basis points; every variant has a target class U{0,1,2}; every variant that is
    loaded (state Active, Overloaded or Interfered) runs min(1 + Poisson(1), 8) instances on
    distinct workers of its class, each with a load U{0..1000}; Inactive variants run none.  The
    instance list is shuffled.  Seed: _SEED0 + cfg + 11000.  Draw order: worker classes, worker
    utilisations, variant classes, instance counts, then per loaded variant its workers, then all
    loads, then the shuffle."""
    if seed is None:
        seed = _SEED0 + cfg + 11000
    rng = np.random.default_rng(np.random.PCG64(seed))
    V = int(states.state.shape[0])
    W = _NUM_WORKERS[cfg]
    worker_hw = rng.integers(0, _NUM_HW, size=W).astype(np.int32)
    worker_util = rng.integers(0, 10001, size=W).astype(np.int32)
    variant_hw = rng.integers(0, _NUM_HW, size=V).astype(np.int32)
    count = np.minimum(1 + rng.poisson(1.0, size=V), 8)
    by_class = [np.flatnonzero(worker_hw == c) for c in range(_NUM_HW)]
    iv, iw = [], []
    for v in np.flatnonzero(states.state != 0):
        pool = by_class[variant_hw[v]]
        k = min(int(count[v]), pool.size)
        if k:
            iw.append(rng.choice(pool, size=k, replace=False))
            iv.append(np.full(k, v))
    inst_variant = np.concatenate(iv) if iv else np.zeros(0, dtype=np.int64)
    inst_worker = np.concatenate(iw) if iw else np.zeros(0, dtype=np.int64)
    inst_load = rng.integers(0, 1001, size=inst_variant.size)
    order = rng.permutation(inst_variant.size)
    return WorkerTables(variant_hw=variant_hw, worker_hw=worker_hw, worker_util=worker_util,
                        inst_variant=inst_variant[order].astype(np.int32),
                        inst_worker=inst_worker[order].astype(np.int32),
                        inst_load=inst_load[order].astype(np.int32))


def make_worker_update(cfg: int, W: int, I: int, chunk: int, fraction: float = 0.10,
                       seed: Optional[int] = None) -> WorkerUpdate:
    """Report before chunk ``chunk``: ``fraction`` of the workers get a new utilisation
    U{0..10000} and ``fraction`` of the instances a new load U{0..1000}, both chosen without
    replacement.  Seed: _SEED0 + cfg + 13000 + chunk."""
    if seed is None:
        seed = _SEED0 + cfg + 13000 + chunk
    rng = np.random.default_rng(np.random.PCG64(seed))
    n, m = int(round(W * fraction)), int(round(I * fraction))
    widx = rng.choice(W, size=n, replace=False) if n else np.zeros(0, dtype=np.int64)
    util = rng.integers(0, 10001, size=n)
    iidx = rng.choice(I, size=m, replace=False) if m else np.zeros(0, dtype=np.int64)
    load = rng.integers(0, 1001, size=m)
    return WorkerUpdate(worker_idx=widx.astype(np.int32), worker_util=util.astype(np.int32),
                        inst_idx=iidx.astype(np.int32), inst_load=load.astype(np.int32))


def make_instance_states(cfg: int, I: int, seed: Optional[int] = None) -> np.ndarray:
    """State of every running instance (the paper publishes no population): Active, Overloaded,
    Interfered with probabilities (0.80, 0.12, 0.08), so that of the variants with 1 + Poisson(1)
    instances about one in eight has no Active instance left.  Seed: _SEED0 + cfg + 19000."""
    if seed is None:
        seed = _SEED0 + cfg + 19000
    rng = np.random.default_rng(np.random.PCG64(seed))
    return rng.choice(np.array([1, 2, 3], dtype=np.int32), size=I, p=(0.80, 0.12, 0.08)).astype(np.int32)


def make_instance_state_update(cfg: int, I: int, chunk: int, fraction: float = 0.05,
                               seed: Optional[int] = None):
    """Report before chunk ``chunk``: ``fraction`` of the instances, chosen without replacement,
    get a new state from the distribution of make_instance_states.  Returns (inst_idx, state).
    Seed: _SEED0 + cfg + 21000 + chunk."""
    if seed is None:
        seed = _SEED0 + cfg + 21000 + chunk
    rng = np.random.default_rng(np.random.PCG64(seed))
    n = int(round(I * fraction))
    idx = rng.choice(I, size=n, replace=False) if n else np.zeros(0, dtype=np.int64)
    val = rng.choice(np.array([1, 2, 3], dtype=np.int32), size=n, p=(0.80, 0.12, 0.08))
    return idx.astype(np.int32), val.astype(np.int32)


@dataclass
class ScalingProfile:
    """What the scaling decision of Section 4.2 reads per variant, besides the latency profile."""
    arch_id: np.ndarray   # [V] int32, model architecture (variants of one architecture share a task)
    sat_qps: np.ndarray   # [V] int32, saturation throughput in queries per second
    hw_cost: np.ndarray   # [V] int32, hardware cost per second
    load_us: np.ndarray   # [V] int32, loading latency


@dataclass
class ScaleRequests:
    variant: np.ndarray    # [R] int32, the running variant
    instances: np.ndarray  # [R] int32, its running instances
    load_qps: np.ndarray   # [R] int32, incoming load
    slo_us: np.ndarray     # [R] int32
    batch_idx: np.ndarray  # [R] int32

    @property
    def R(self) -> int:
        return int(self.variant.shape[0])


def make_scaling(cfg: int, tb: VariantTable, seed: Optional[int] = None) -> ScalingProfile:
    """Stand-in for the profiles behind the paper's autoscaler (not published): every task's
    variants are dealt uniformly to max(1, round(size / 12)) architectures (the paper's 175
    variants come from 22 architectures, 8 per architecture on average); saturation throughput
    clamp(lognormal(ln 200, 1.2), 1, 200000) queries per second; hardware cost U{50..2000}; loading
    latency clamp(lognormal(ln 20000, 1.5), 100, 5,000,000) microseconds.  Seed: _SEED0 + cfg +
    15000.  Draw order: architecture of every variant (tasks in ascending order), throughput,
    cost, loading latency."""
    if seed is None:
        seed = _SEED0 + cfg + 15000
    rng = np.random.default_rng(np.random.PCG64(seed))
    V = tb.V
    arch = np.zeros(V, dtype=np.int64)
    nxt = 0
    for t in range(tb.num_tasks):
        rows = np.flatnonzero(tb.task_id == t)
        k = max(1, int(round(rows.size / 12.0)))
        arch[rows] = nxt + rng.integers(0, k, size=rows.size)
        nxt += k
    qps = np.clip(np.rint(rng.lognormal(np.log(200.0), 1.2, size=V)), 1, 200_000)
    cost = rng.integers(50, 2001, size=V)
    load = np.clip(np.rint(rng.lognormal(np.log(20000.0), 1.5, size=V)), 100, 5_000_000)
    return ScalingProfile(arch_id=arch.astype(np.int32), sat_qps=qps.astype(np.int32),
                          hw_cost=cost.astype(np.int32), load_us=load.astype(np.int32))


def make_scale_requests(cfg: int, tb: VariantTable, sc: ScalingProfile, n: int, chunk: int = 0,
                        seed: Optional[int] = None) -> ScaleRequests:
    """``n`` scaling requests: running variant uniform over the table, 1 + Poisson(1) running
    instances, incoming load = their combined saturation throughput times U(0.5, 4) (so about a
    sixth of the requests need no scaling at a slack of 105%), latency objective and batch index
    as in the query generator (unimodal).  Seed: _SEED0 + cfg + 17000 + chunk."""
    if seed is None:
        seed = _SEED0 + cfg + 17000 + chunk
    rng = np.random.default_rng(np.random.PCG64(seed))
    variant = rng.integers(0, tb.V, size=n)
    inst = 1 + rng.poisson(1.0, size=n)
    load = np.rint(sc.sat_qps[variant].astype(np.float64) * inst * rng.uniform(0.5, 4.0, size=n))
    slo = np.clip(rng.lognormal(np.log(20000.0), 1.0, size=n), 1000.0, 2_000_000.0)
    bidx = rng.integers(0, tb.B, size=n)
    return ScaleRequests(variant=variant.astype(np.int32), instances=inst.astype(np.int32),
                         load_qps=np.minimum(load, 1_000_000_000).astype(np.int32),
                         slo_us=np.rint(slo).astype(np.int32), batch_idx=bidx.astype(np.int32))


def make_scale_down_requests(cfg: int, tb: VariantTable, sc: ScalingProfile, n: int, chunk: int = 0,
                             seed: Optional[int] = None) -> ScaleRequests:
    """``n`` scaling-down requests (the regular check of Section 4.2.2): running variant uniform over
    the table, 1 + Poisson(2) running instances, incoming load = their combined saturation throughput
    times U(0, 1.2) (mostly below capacity, as when load has fallen; about a sixth above it), latency
    objective and batch index as in ``make_scale_requests``.  Seed: _SEED0 + cfg + 19000 + chunk."""
    if seed is None:
        seed = _SEED0 + cfg + 19000 + chunk
    rng = np.random.default_rng(np.random.PCG64(seed))
    variant = rng.integers(0, tb.V, size=n)
    inst = 1 + rng.poisson(2.0, size=n)
    load = np.rint(sc.sat_qps[variant].astype(np.float64) * inst * rng.uniform(0.0, 1.2, size=n))
    slo = np.clip(rng.lognormal(np.log(20000.0), 1.0, size=n), 1000.0, 2_000_000.0)
    bidx = rng.integers(0, tb.B, size=n)
    return ScaleRequests(variant=variant.astype(np.int32), instances=inst.astype(np.int32),
                         load_qps=np.minimum(load, 1_000_000_000).astype(np.int32),
                         slo_us=np.rint(slo).astype(np.int32), batch_idx=bidx.astype(np.int32))
