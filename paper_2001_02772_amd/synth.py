"""Seeded synthetic inputs for DLRM-style inference workloads.

This module only produces *inputs* (dense features, bag lengths, lookup
indices, embedding tables, FC weights, query sizes).  It holds none of the
model's arithmetic and is the one piece shared by the CPU oracle's tests and
the GPU path's tests / benchmark.

Random numbers come from a counter-based generator, so any element of any
stream can be produced without producing the ones before it (a single table
row of a 5 GB model, say):

    key(seed, stream)      = mix(seed + GAMMA * (stream + 1))
    draw(seed, stream, i)  = mix(key + GAMMA * (i + 1))

where ``mix`` is the SplitMix64 output function (Steele, Lea, Flood 2014:
xor-shift 30, multiply, xor-shift 27, multiply, xor-shift 31) and GAMMA the
64-bit golden-ratio increment 0x9E3779B97F4A7C15.  ``draw(., ., i)`` is
therefore the i-th output of a SplitMix64 generator started at ``key``.

The workloads follow the model shapes of Table I of the DeepRecSys paper
(RMC1/RMC2/RMC3: Dense-FC and Predict-FC stacks, up to 10/40/10 tables, about
80/80/20 lookups per table, sum pooling) with the concrete dimensions listed
in ``CONFIGS`` below.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

MASTER_SEED = 20200102

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# stream kinds (stream id = kind * 2**20 + index)
K_DENSE, K_LENGTHS, K_INDICES, K_TABLE, K_PERM, K_WEIGHT, K_BIAS, K_QUERY, K_ARRIVAL = range(9)


def stream_id(kind: int, index: int = 0) -> int:
    return (kind << 20) + index


def _mix(x: np.ndarray) -> np.ndarray:
    x = (x ^ (x >> np.uint64(30))) * _M1
    x = (x ^ (x >> np.uint64(27))) * _M2
    return x ^ (x >> np.uint64(31))


def stream_key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        s = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + _GAMMA * np.uint64(stream + 1)
        return _mix(np.asarray(s, dtype=np.uint64))[()]


def draws_at(seed: int, stream: int, counters: np.ndarray) -> np.ndarray:
    """uint64 draws at arbitrary counter positions."""
    c = np.asarray(counters).astype(np.uint64)
    with np.errstate(over="ignore"):
        return _mix(stream_key(seed, stream) + _GAMMA * (c + np.uint64(1)))


def draws(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    return draws_at(seed, stream, np.arange(start, start + count, dtype=np.uint64))


def _u24(u: np.ndarray) -> np.ndarray:
    """uniform float32 on [0,1) with 24 random bits (exact in fp32)."""
    return (u >> np.uint64(40)).astype(np.float32) * np.float32(2.0 ** -24)


def _u53(u: np.ndarray) -> np.ndarray:
    return (u >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


def uniform_f32_at(seed, stream, counters, lo, hi) -> np.ndarray:
    """lo + (hi-lo)*u evaluated in fp32 (one multiply, one add, each rounded)."""
    u = _u24(draws_at(seed, stream, counters))
    return (np.float32(lo) + np.float32(hi - lo) * u).astype(np.float32)


def uniform_f32(seed, stream, start, count, lo, hi) -> np.ndarray:
    return uniform_f32_at(seed, stream, np.arange(start, start + count, dtype=np.uint64), lo, hi)


def normal_f32(seed, stream, start, count) -> np.ndarray:
    """Standard normals by Box-Muller in float64 (draws 2i and 2i+1), rounded to fp32."""
    c = np.arange(start, start + count, dtype=np.uint64)
    u1 = _u53(draws_at(seed, stream, c * np.uint64(2)))
    u2 = _u53(draws_at(seed, stream, c * np.uint64(2) + np.uint64(1)))
    r = np.sqrt(-2.0 * np.log(1.0 - u1))  # 1-u1 in (0,1]
    return (r * np.cos(2.0 * math.pi * u2)).astype(np.float32)


def randint(seed, stream, start, count, lo, hi) -> np.ndarray:
    """Integers uniform on {lo..hi} inclusive: lo + floor(u32 * span / 2**32)."""
    u = draws(seed, stream, start, count) >> np.uint64(32)
    span = np.uint64(hi - lo + 1)
    return (lo + ((u * span) >> np.uint64(32)).astype(np.int64)).astype(np.int64)


def permutation(seed, stream, n) -> np.ndarray:
    """A permutation of 0..n-1: stable argsort of n random 64-bit keys."""
    return np.argsort(draws(seed, stream, 0, n), kind="stable").astype(np.int64)


def zipf_cdf(n: int, alpha: float) -> np.ndarray:
    """CDF of the finite Zipf law P(rank r) = r^-alpha / H(n, alpha), r = 1..n."""
    w = np.arange(1, n + 1, dtype=np.float64) ** (-alpha)
    c = np.cumsum(w)
    return c / c[-1]


def zipf_ranks(seed, stream, start, count, cdf: np.ndarray) -> np.ndarray:
    """0-based ranks by inverse CDF: smallest r with cdf[r] > u."""
    u = _u53(draws(seed, stream, start, count))
    return np.minimum(np.searchsorted(cdf, u, side="right"), len(cdf) - 1).astype(np.int64)


def lognormal_query_sizes(seed, count, mu=4.5, sigma=1.0, lo=1, hi=1000) -> np.ndarray:
    """Query sizes n = clip(round_half_even(exp(mu + sigma z)), lo, hi), z ~ N(0,1)."""
    c = np.arange(count, dtype=np.uint64)
    st = stream_id(K_QUERY)
    u1 = _u53(draws_at(seed, st, c * np.uint64(2)))
    u2 = _u53(draws_at(seed, st, c * np.uint64(2) + np.uint64(1)))
    z = np.sqrt(-2.0 * np.log(1.0 - u1)) * np.cos(2.0 * math.pi * u2)
    return np.clip(np.rint(np.exp(mu + sigma * z)), lo, hi).astype(np.int64)


def unit_poisson_arrivals(seed, count) -> np.ndarray:
    """Arrival times (float64, increasing) of a rate-1 Poisson process: cumulative sums of
    unit-mean exponential gaps -ln(1-u).  Divide by a rate to get arrivals at that rate."""
    u = _u53(draws(seed, stream_id(K_ARRIVAL), 0, count))
    return np.cumsum(-np.log(1.0 - u))


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class Config:
    name: str
    B: int                 # batch size
    F: int                 # dense features per sample
    T: int                 # embedding tables
    R: int                 # rows per table
    D: int                 # embedding dimension (= bottom-MLP output width)
    len_lo: int            # bag length ~ Uniform{len_lo..len_hi}
    len_hi: int
    index_dist: str        # "uniform" | "zipf"
    dense_dist: str        # "uniform01" | "normal"
    bottom: tuple          # layer widths, bottom[0] == F, bottom[-1] == D
    top: tuple             # layer widths, top[0] == D + V(V-1)/2, top[-1] == 1
    bf16: bool = False     # MLP operands rounded to bf16 (fp32 accumulate)
    zipf_alpha: float = 1.05
    interaction: str = "dot"   # "dot": pairwise dots (DLRM); "concat": top input = [bottom output | embeddings]

    @property
    def V(self) -> int:
        return self.T + 1

    @property
    def P(self) -> int:
        return self.V * (self.V - 1) // 2

    def replace(self, **kw) -> "Config":
        d = dict(self.__dict__)
        d.update(kw)
        return Config(**d)


CONFIGS = {
    "tiny": Config("tiny", 64, 13, 8, 10_000, 32, 20, 20, "uniform", "uniform01",
                   (13, 64, 32), (68, 64, 1)),
    "rmc1": Config("rmc1", 256, 13, 10, 1_000_000, 32, 60, 100, "uniform", "uniform01",
                   (13, 256, 128, 32), (87, 256, 64, 1)),
    "rmc2": Config("rmc2", 1024, 13, 40, 500_000, 64, 60, 100, "zipf", "uniform01",
                   (13, 256, 128, 64), (884, 512, 128, 1)),
    "rmc2-uniform": Config("rmc2-uniform", 1024, 13, 40, 500_000, 64, 60, 100, "uniform",
                           "uniform01", (13, 256, 128, 64), (884, 512, 128, 1)),
    "rmc3": Config("rmc3", 1024, 2560, 10, 1_000_000, 32, 10, 30, "uniform", "normal",
                   (2560, 1024, 256, 32), (87, 512, 256, 1), bf16=True),
    # Wide&Deep-shaped (Table I): no dense stack, ~1000 dense features joined with one lookup from each of
    # tens of tables, predictor 1024-512-256 and a 1-wide output
    "wnd": Config("wnd", 1024, 1024, 32, 500_000, 32, 1, 1, "zipf", "normal",
                  (1024,), (2048, 1024, 512, 256, 1), bf16=True, interaction="concat"),
    "wnd-tiny": Config("wnd-tiny", 48, 16, 5, 5_000, 8, 1, 1, "uniform", "normal",
                       (16,), (56, 32, 16, 1), interaction="concat"),
}

# the query-size sweep runs on the rmc2 model
SWEEP_BATCH_SIZES = (16, 64, 256, 1024)
SWEEP_QUERIES = 2000


def check_config(c: Config) -> None:
    assert c.bottom[0] == c.F and c.top[-1] == 1
    if c.interaction == "concat":
        assert c.top[0] == c.bottom[-1] + c.T * c.D
    else:
        assert c.interaction == "dot" and c.bottom[-1] == c.D and c.top[0] == c.D + c.P


for _c in CONFIGS.values():
    check_config(_c)


# --------------------------------------------------------------------------
# model parameters
# --------------------------------------------------------------------------

TABLE_LO, TABLE_HI = -0.05, 0.05


def table_rows(cfg: Config, t: int, rows: np.ndarray, seed: int = MASTER_SEED) -> np.ndarray:
    """Rows ``rows`` of table t as fp32 [len(rows)][D]; element (r, d) is draw r*D+d."""
    rows = np.asarray(rows, dtype=np.uint64)
    c = rows[:, None] * np.uint64(cfg.D) + np.arange(cfg.D, dtype=np.uint64)[None, :]
    return uniform_f32_at(seed, stream_id(K_TABLE, t), c, TABLE_LO, TABLE_HI)


def table_full(cfg: Config, t: int, seed: int = MASTER_SEED, chunk_rows: int = 1 << 17) -> np.ndarray:
    out = np.empty((cfg.R, cfg.D), dtype=np.float32)
    for r0 in range(0, cfg.R, chunk_rows):
        r1 = min(cfg.R, r0 + chunk_rows)
        out[r0:r1] = uniform_f32(seed, stream_id(K_TABLE, t), r0 * cfg.D, (r1 - r0) * cfg.D,
                                 TABLE_LO, TABLE_HI).reshape(r1 - r0, cfg.D)
    return out


def table_full_torch(cfg: Config, t: int, device, seed: int = MASTER_SEED, chunk_rows: int = 1 << 20):
    """Same values as ``table_full`` computed with torch integer ops on ``device``.

    int64 arithmetic wraps like uint64; logical right shifts are emulated by
    masking the sign-extended bits.  Bit-equality with the NumPy version is
    covered by a test.
    """
    import torch

    def s64(v: int) -> int:  # reinterpret a uint64 constant as int64
        v &= 0xFFFFFFFFFFFFFFFF
        return v - (1 << 64) if v >= (1 << 63) else v

    def lsr(x, s):
        return (x >> s) & ((1 << (64 - s)) - 1)

    key = s64(int(stream_key(seed, stream_id(K_TABLE, t))))
    gamma, m1, m2 = s64(int(_GAMMA)), s64(int(_M1)), s64(int(_M2))
    out = torch.empty((cfg.R, cfg.D), dtype=torch.float32, device=device)
    flat = out.view(-1)
    lo = torch.tensor(TABLE_LO, dtype=torch.float32, device=device)
    scale = torch.tensor(np.float32(TABLE_HI - TABLE_LO), dtype=torch.float32, device=device)
    for r0 in range(0, cfg.R, chunk_rows):
        r1 = min(cfg.R, r0 + chunk_rows)
        c = torch.arange(r0 * cfg.D + 1, r1 * cfg.D + 1, dtype=torch.int64, device=device)
        x = c * gamma + key
        x = (x ^ lsr(x, 30)) * m1
        x = (x ^ lsr(x, 27)) * m2
        x = x ^ lsr(x, 31)
        u = lsr(x, 40).to(torch.float32) * (2.0 ** -24)
        flat[r0 * cfg.D:r1 * cfg.D] = lo + scale * u
    return out


@dataclass
class MLPParams:
    widths: tuple
    W: list = field(default_factory=list)     # fp32 [out][in] row-major
    b: list = field(default_factory=list)     # fp32 [out]


def mlp_params(widths, stack: int, seed: int = MASTER_SEED) -> MLPParams:
    """W ~ U(-a, a), a = sqrt(6/(in+out)); b ~ U(-1/sqrt(in), 1/sqrt(in))."""
    p = MLPParams(tuple(widths))
    for l in range(len(widths) - 1):
        n_in, n_out = widths[l], widths[l + 1]
        a = math.sqrt(6.0 / (n_in + n_out))
        c = 1.0 / math.sqrt(n_in)
        p.W.append(uniform_f32(seed, stream_id(K_WEIGHT, stack * 64 + l), 0, n_in * n_out, -a, a)
                   .reshape(n_out, n_in))
        p.b.append(uniform_f32(seed, stream_id(K_BIAS, stack * 64 + l), 0, n_out, -c, c))
    return p


# --------------------------------------------------------------------------
# per-batch inputs
# --------------------------------------------------------------------------

@dataclass
class Batch:
    B: int
    dense: np.ndarray      # fp32 [B][F]
    lengths: np.ndarray    # int32 [T*B], bag order table-major (bag = t*B + b)
    indices: np.ndarray    # int32 [sum(lengths)], concatenated in bag order


class BatchGenerator:
    """Draws batches of a config; batch ``k`` is a pure function of (seed, k)."""

    def __init__(self, cfg: Config, seed: int = MASTER_SEED):
        self.cfg, self.seed = cfg, seed
        self._cdf = zipf_cdf(cfg.R, cfg.zipf_alpha) if cfg.index_dist == "zipf" else None
        self._perm = {}

    def perm(self, t: int) -> np.ndarray:
        if t not in self._perm:
            self._perm[t] = permutation(self.seed, stream_id(K_PERM, t), self.cfg.R)
        return self._perm[t]

    def batch(self, k: int, B: int | None = None) -> Batch:
        cfg = self.cfg
        B = cfg.B if B is None else B
        # every batch owns a disjoint counter range of each stream
        span = 1 << 40
        base = k * span
        if cfg.dense_dist == "uniform01":
            dense = uniform_f32(self.seed, stream_id(K_DENSE), base, B * cfg.F, 0.0, 1.0)
        else:
            dense = normal_f32(self.seed, stream_id(K_DENSE), base, B * cfg.F)
        dense = dense.reshape(B, cfg.F)
        lengths = randint(self.seed, stream_id(K_LENGTHS), base, cfg.T * B, cfg.len_lo, cfg.len_hi)
        per_table = lengths.reshape(cfg.T, B).sum(axis=1)
        parts = []
        for t in range(cfg.T):
            n = int(per_table[t])
            st = stream_id(K_INDICES, t)
            if cfg.index_dist == "zipf":
                r = zipf_ranks(self.seed, st, base, n, self._cdf)
                parts.append(self.perm(t)[r])
            else:
                parts.append(randint(self.seed, st, base, n, 0, cfg.R - 1))
        indices = np.concatenate(parts) if parts else np.zeros(0, np.int64)
        return Batch(B, dense, lengths.astype(np.int32), indices.astype(np.int32))


def compact_tables(cfg: Config, batch: Batch, seed: int = MASTER_SEED):
    """Only the table rows a batch touches, as small per-table arrays, plus the batch's
    indices renumbered into them.  Lets a CPU run of a full-size batch do without the
    multi-GB tables: pooled sums over the compact tables equal those over the full ones."""
    off = np.concatenate([[0], np.cumsum(batch.lengths, dtype=np.int64)])
    tables, idx = [], np.empty_like(batch.indices)
    for t in range(cfg.T):
        lo, hi = off[t * batch.B], off[(t + 1) * batch.B]
        used = np.unique(batch.indices[lo:hi])
        if used.size == 0:
            used = np.zeros(1, dtype=batch.indices.dtype)
        tables.append(table_rows(cfg, t, used, seed))
        idx[lo:hi] = np.searchsorted(used, batch.indices[lo:hi])
    return tables, idx
