"""Seeded synthetic workloads (inputs only — none of the method's arithmetic lives here).

The paper trains on three proprietary click-through-rate datasets with a production
DLRM whose architecture is withheld (Section 4); what it does state is the shape of the
problem: a sparse part of ~200 GB held once, a dense part of ~50 MB replicated per
trainer, hundreds of tables with billions of rows.  The generators below stand in for
that data: dense features ~ N(0,1), multi-hot categorical features with Poisson bag
lengths and Zipf-distributed row popularity, labels drawn from a fixed random logistic
teacher.  Everything is a pure function of (config, seed, step).

Both the CPU oracle's tests and the HIP library's callers draw their inputs from here;
the initial table values h0 come from a counter-based hash so that a 51 GB table can be
filled on the device (the library implements the same hash on its own) while the tests
materialise only the rows a batch touches.
"""

from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Dict, List, Sequence, Tuple

import numpy as np

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_STREAM_MUL = _U64(0xD1B54A32D192ED03)


# --------------------------------------------------------------------------- hashing
def mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on uint64 arrays (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z + _GOLDEN).astype(_U64)
        z = ((z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)).astype(_U64)
        z = ((z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)).astype(_U64)
        return z ^ (z >> _U64(31))


def hash_u24(seed: int, stream: int, index: np.ndarray) -> np.ndarray:
    """24 random bits per counter value: mix64(mix64(seed ^ stream*C) + index*golden) >> 40."""
    with np.errstate(over="ignore"):
        key = mix64(np.asarray([seed], dtype=_U64) ^ (_U64(stream) * _STREAM_MUL))
        z = mix64(key + np.asarray(index, dtype=_U64) * _GOLDEN)
    return (z >> _U64(40)).astype(np.int64)


TABLE_STREAM0 = 1000  # table t uses hash stream TABLE_STREAM0 + t
TABLE_INIT_RANGE = np.float32(0.05)


def table_rows_h0(seed: int, table: int, rows: np.ndarray, d: int) -> np.ndarray:
    """Initial values h0 of the given rows of one table, float32 (len(rows), d):
    (u24 - 2^23) * (0.05 * 2^-23), uniform in [-0.05, 0.05), one rounding per value.
    The counter of element (row, col) is row*d + col."""
    rows = np.asarray(rows, dtype=np.int64)
    idx = (rows[:, None] * d + np.arange(d, dtype=np.int64)[None, :]).astype(_U64)
    k = hash_u24(seed, TABLE_STREAM0 + table, idx) - (1 << 23)
    scale = np.float32(TABLE_INIT_RANGE * np.float32(2.0 ** -23))
    return k.astype(np.float32) * scale


# --------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    batch: int
    rows: Tuple[int, ...]          # rows per table
    emb_dim: int
    bag_lambda: float              # bag length = Poisson(bag_lambda) + 1
    zipf_s: float
    bot_dims: Tuple[int, ...]
    top_dims: Tuple[int, ...]
    bf16: bool
    num_replicas: int
    algo: str                      # "easgd" | "ma" | "bmuf"
    alpha: float
    eta: float = 1.0
    mu: float = 0.0
    sync_gap: int = 1              # trainer steps per replica between rounds
    num_dense: int = 13
    lr_dense: float = 0.01
    lr_emb: float = 0.01
    adagrad_eps: float = 1e-8
    pooling: str = "sum"           # "sum" | "mean"
    emb_optimizer: str = "rowwise_adagrad"   # | "adam"
    adam_betas: Tuple[float, float] = (0.9, 0.999)
    emb_row_shards: int = 1        # > 1: every table split into that many row ranges

    @property
    def num_tables(self) -> int:
        return len(self.rows)

    @property
    def row_base(self) -> np.ndarray:
        return np.concatenate(([0], np.cumsum(np.asarray(self.rows, dtype=np.int64))))

    @property
    def mean_ids(self) -> float:
        return self.batch * self.num_tables * (self.bag_lambda + 1)

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


def _large_rows(seed: int) -> Tuple[int, ...]:
    """26 row counts log-uniform in [1e3, 4e7], rescaled to total ~2e8 and clamped
    (the config states both; plain log-uniform averages half that total)."""
    rng = np.random.default_rng([seed, 77])
    r = np.exp(rng.uniform(math.log(1e3), math.log(4e7), size=26))
    for _ in range(2):
        r = np.clip(r * (2e8 / r.sum()), 1e3, 4e7)
    return tuple(int(v) for v in r)


def tiny() -> Workload:
    return Workload("tiny", 1, 128, (1000,) * 4, 16, 3.0, 1.05, (13, 64, 16),
                    (26, 64, 1), False, 2, "ma", 1.0, sync_gap=1)


def mid() -> Workload:
    return Workload("mid", 2, 2048, (1_000_000,) * 8, 64, 20.0, 1.05,
                    (13, 256, 128, 64), (100, 512, 256, 1), True, 4, "easgd", 0.1,
                    sync_gap=5)


def large() -> Workload:
    return Workload("large", 3, 8192, _large_rows(3), 64, 30.0, 1.1,
                    (13, 512, 256, 64), (415, 1024, 1024, 512, 256, 1), True, 4, "bmuf",
                    0.5, eta=1.0, mu=0.9, sync_gap=1)


def hogwild() -> Workload:
    return replace(mid(), name="hogwild", seed=5, batch=1024, zipf_s=1.3, algo="ma",
                   alpha=0.5, sync_gap=1)


WORKLOADS = {"tiny": tiny, "mid": mid, "large": large, "hogwild": hogwild}


# --------------------------------------------------------------------------- Zipf ids
class ZipfRows:
    """Bounded Zipf over N rows, P(rank k) ∝ (k+1)^-s for k = 0..N-1 (inverse CDF), with
    ranks scattered over the table by the bijection row = (rank*A + C) mod N."""

    _cdf_cache: Dict[Tuple[int, float], np.ndarray] = {}

    def __init__(self, n_rows: int, s: float, seed: int, table: int):
        self.n = int(n_rows)
        key = (self.n, float(s))
        if key not in ZipfRows._cdf_cache:
            p = np.arange(1, self.n + 1, dtype=np.float64) ** (-s)
            cdf = np.cumsum(p)
            ZipfRows._cdf_cache[key] = cdf / cdf[-1]
        self.cdf = ZipfRows._cdf_cache[key]
        a = max(1, int(0.6180339887 * self.n))
        while math.gcd(a, self.n) != 1:
            a += 1
        self.a = a
        self.c = int(hash_u24(seed, 500 + table, np.asarray([0]))[0]) % self.n

    def ranks(self, u: np.ndarray) -> np.ndarray:
        return np.minimum(np.searchsorted(self.cdf, u, side="right"), self.n - 1)

    def rows_of_ranks(self, ranks: np.ndarray) -> np.ndarray:
        return (ranks.astype(np.int64) * self.a + self.c) % self.n

    def sample(self, rng: np.random.Generator, size: int) -> np.ndarray:
        return self.rows_of_ranks(self.ranks(rng.random(size)))


# --------------------------------------------------------------------------- batches
@dataclass
class Batch:
    dense: np.ndarray      # (B, num_dense) float32
    labels: np.ndarray     # (B,) float32 in {0, 1}
    indices: np.ndarray    # (n,) int32, row within its table
    offsets: np.ndarray    # (T*B+1,) int32, table-major CSR over (t, b)

    def as_tuple(self):
        return self.dense, self.labels, self.indices, self.offsets


class BatchGenerator:
    def __init__(self, wl: Workload):
        self.wl = wl
        self.zipf = [ZipfRows(n, wl.zipf_s, wl.seed, t) for t, n in enumerate(wl.rows)]
        rng = np.random.default_rng([wl.seed, 11])
        self.teacher_a = rng.standard_normal(wl.num_dense)
        self.teacher_b0 = math.log(0.2 / 0.8)

    def _teacher_c(self, table: int, rows: np.ndarray) -> np.ndarray:
        u = hash_u24(self.wl.seed, 700 + table, rows.astype(np.int64)) / float(1 << 24)
        return (u - 0.5) * math.sqrt(12.0) * 0.5

    def batch(self, step: int) -> Batch:
        wl = self.wl
        B, T = wl.batch, wl.num_tables
        rng = np.random.default_rng([wl.seed, 13, step])
        x = rng.standard_normal((B, wl.num_dense)).astype(np.float32)
        lengths = rng.poisson(wl.bag_lambda, size=(T, B)).astype(np.int64) + 1
        offsets = np.concatenate(([0], np.cumsum(lengths.ravel())))
        n = int(offsets[-1])
        indices = np.empty(n, dtype=np.int32)
        logit = x.astype(np.float64) @ self.teacher_a / math.sqrt(wl.num_dense)
        logit += self.teacher_b0
        for t in range(T):
            lo, hi = int(offsets[t * B]), int(offsets[(t + 1) * B])
            rows = self.zipf[t].sample(rng, hi - lo)
            indices[lo:hi] = rows
            c = self._teacher_c(t, rows)
            seg = offsets[t * B : (t + 1) * B] - lo
            logit += np.add.reduceat(c, seg) / lengths[t]
        p = 1.0 / (1.0 + np.exp(-logit))
        y = (rng.random(B) < p).astype(np.float32)
        return Batch(x, y, indices, offsets.astype(np.int32))


def dense_w0(wl: Workload) -> np.ndarray:
    """Initial dense vector w0: W ~ U(+-sqrt(6/(in+out))), b = 0; bottom layers then top
    layers, each W[out][in] row-major followed by b[out]."""
    rng = np.random.default_rng([wl.seed, 17])
    parts = []
    for dims in (wl.bot_dims, wl.top_dims):
        for i in range(len(dims) - 1):
            fan_in, fan_out = dims[i], dims[i + 1]
            lim = math.sqrt(6.0 / (fan_in + fan_out))
            parts.append(rng.uniform(-lim, lim, size=fan_out * fan_in).astype(np.float32))
            parts.append(np.zeros(fan_out, dtype=np.float32))
    return np.concatenate(parts)


def full_tables_h0(wl: Workload) -> np.ndarray:
    """All rows of all tables stacked, float32 (sum rows, d).  Small workloads only."""
    out = []
    for t, n in enumerate(wl.rows):
        out.append(table_rows_h0(wl.seed, t, np.arange(n), wl.emb_dim))
    return np.concatenate(out, axis=0)


# --------------------------------------------------------------------------- compaction
@dataclass
class CompactProblem:
    """The sub-problem spanned by the rows a set of batches touches: row ids relabelled
    by their rank among the touched rows of their table (an order-preserving map, so a
    stable sort by row gives the same permutation as on the original ids)."""
    rows: Tuple[int, ...]                 # touched rows per table
    touched: List[np.ndarray]             # original row ids, ascending, per table
    h0: np.ndarray                        # (sum touched, d) float32
    batches: List[Batch]                  # indices remapped to compact ids


def compact_problem(wl: Workload, batches: Sequence[Batch]) -> CompactProblem:
    B, T = wl.batch, wl.num_tables
    touched = []
    for t in range(T):
        ids = [b.indices[b.offsets[t * B] : b.offsets[(t + 1) * B]] for b in batches]
        touched.append(np.unique(np.concatenate(ids)).astype(np.int64))
    h0 = np.concatenate(
        [table_rows_h0(wl.seed, t, touched[t], wl.emb_dim) for t in range(T)], axis=0)
    out = []
    for b in batches:
        idx = np.empty_like(b.indices)
        for t in range(T):
            lo, hi = b.offsets[t * B], b.offsets[(t + 1) * B]
            idx[lo:hi] = np.searchsorted(touched[t], b.indices[lo:hi])
        out.append(Batch(b.dense, b.labels, idx, b.offsets))
    return CompactProblem(tuple(len(t) for t in touched), touched, h0, out)
