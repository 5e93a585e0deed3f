"""Seeded synthetic inputs for the K-hop precompute: edge lists and feature matrices.

This module only draws random graphs and random features.  It holds none of the
method's arithmetic (no degrees, no normalisation, no aggregation, no block
planning), so both the CPU oracle's tests and the HIP library's tests may feed
from it without sharing any code of the method.

All randomness comes from numpy's Philox generator (counter based, so the same
(seed, stream) pair gives the same numbers on every host).  The five workloads
mirror the shapes of the public graphs the paper measures on (Table 1: an
arxiv-sized citation graph, a Reddit-sized dense community graph, a
papers100M-sized graph) plus a tiny case and a mid-sized power-law case; the
graphs themselves are synthetic stand-ins, no dataset record is reproduced.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 220712000

# plan flags / aggregation kinds: plain integers of the C boundary, repeated
# here only so a workload description can be handed to either side.
SYMMETRISE = 1
ADD_SELF_LOOPS = 2
AGG_SYM, AGG_MEAN, AGG_SUM = 0, 1, 2
F32, BF16 = 0, 1


def rng_for(seed: int, stream: int) -> np.random.Generator:
    """Philox generator keyed by (seed, stream)."""
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


# --------------------------------------------------------------------------
# graph generators: each returns (src, dst) int32 arrays of directed pairs
# --------------------------------------------------------------------------

def _first_distinct(keys: np.ndarray, want: int) -> np.ndarray:
    """Keep the first `want` distinct keys in draw order (fewer if not enough)."""
    _, first = np.unique(keys, return_index=True)
    first.sort()
    return keys[first[:want]]


def gnm_pairs(n: int, M: int, rng: np.random.Generator):
    """G(n, M): exactly M distinct unordered non-loop pairs, by rejection."""
    if n < 2 or M > n * (n - 1) // 2:
        raise ValueError("too many pairs for n")
    keys = np.empty(0, dtype=np.int64)
    while keys.size < M:
        need = M - keys.size
        k = int(need * 1.2) + 64
        u = rng.integers(0, n, size=k, dtype=np.int64)
        v = rng.integers(0, n, size=k, dtype=np.int64)
        ok = u != v
        lo = np.minimum(u, v)[ok]
        hi = np.maximum(u, v)[ok]
        keys = _first_distinct(np.concatenate([keys, lo * n + hi]), M)
    return (keys // n).astype(np.int32), (keys % n).astype(np.int32)


def _powerlaw_inverse_cdf(u: np.ndarray, n: int, a: float, i0: float) -> np.ndarray:
    """Node index drawn with probability proportional to the integral of
    (x + i0)^(-a) over [i, i+1): closed-form inverse of that CDF at u in [0,1)."""
    if abs(a - 1.0) < 1e-12:
        x = i0 * np.exp(u * np.log((n + i0) / i0)) - i0
    else:
        p = 1.0 - a
        lo = i0 ** p
        hi = (n + i0) ** p
        x = (lo + u * (hi - lo)) ** (1.0 / p) - i0
    idx = np.floor(x).astype(np.int64)
    np.clip(idx, 0, n - 1, out=idx)
    return idx


def _powerlaw_mass_of_node0(n: int, a: float, i0: float) -> float:
    if abs(a - 1.0) < 1e-12:
        return float(np.log((1 + i0) / i0) / np.log((n + i0) / i0))
    p = 1.0 - a
    return float(((1 + i0) ** p - i0 ** p) / ((n + i0) ** p - i0 ** p))


def chung_lu_offset(n: int, draws: int, gamma: float, max_expected_degree: float) -> float:
    """Offset i0 of the weight sequence w_i ~ (i + i0)^(-1/(gamma-1)) for which
    the heaviest node's expected number of endpoint hits over `draws` endpoint
    draws equals max_expected_degree (bisection; the mass is monotone in i0)."""
    a = 1.0 / (gamma - 1.0)
    lo, hi = 1e-9, float(n) * 1e3
    for _ in range(200):
        mid = np.sqrt(lo * hi)
        if draws * _powerlaw_mass_of_node0(n, a, mid) > max_expected_degree:
            lo = mid
        else:
            hi = mid
    return float(np.sqrt(lo * hi))


def chung_lu_pairs(n: int, M: int, gamma: float, max_expected_degree: float,
                   rng: np.random.Generator, chunk: int = 1 << 24, progress=None):
    """Chung-Lu style power-law graph: M pairs whose two endpoints are drawn
    independently with probability proportional to w_i; self pairs are kept
    (the planner drops them) and duplicates may occur (the planner collapses
    them), so the stored non-zero count is a little below 2M."""
    a = 1.0 / (gamma - 1.0)
    i0 = chung_lu_offset(n, 2 * M, gamma, max_expected_degree)
    perm = rng.permutation(n).astype(np.int32)      # ids carry no locality
    src = np.empty(M, dtype=np.int32)
    dst = np.empty(M, dtype=np.int32)
    for s in range(0, M, chunk):
        e = min(M, s + chunk)
        src[s:e] = perm[_powerlaw_inverse_cdf(rng.random(e - s), n, a, i0)]
        dst[s:e] = perm[_powerlaw_inverse_cdf(rng.random(e - s), n, a, i0)]
        if progress:
            progress("pairs drawn", e, M)
    return src, dst


def sbm_pairs(n_comm: int, comm_size: int, M: int, intra_frac: float,
              rng: np.random.Generator, contiguous_ids: bool = False):
    """Stochastic block model with equal communities: M distinct unordered
    non-loop pairs, a fraction intra_frac of the draws inside one community and
    the rest between two different ones, by rejection until M are distinct."""
    n = n_comm * comm_size
    keys = np.empty(0, dtype=np.int64)
    while keys.size < M:
        need = M - keys.size
        k = int(need * 1.15) + 64
        intra = rng.random(k) < intra_frac
        cu = rng.integers(0, n_comm, size=k, dtype=np.int64)
        shift = rng.integers(1, max(n_comm, 2), size=k, dtype=np.int64)
        cv = np.where(intra, cu, (cu + shift) % n_comm)
        u = cu * comm_size + rng.integers(0, comm_size, size=k, dtype=np.int64)
        v = cv * comm_size + rng.integers(0, comm_size, size=k, dtype=np.int64)
        ok = u != v
        lo = np.minimum(u, v)[ok]
        hi = np.maximum(u, v)[ok]
        keys = _first_distinct(np.concatenate([keys, lo * n + hi]), M)
    u = keys // n
    v = keys % n
    if not contiguous_ids:
        perm = rng.permutation(n)
        u, v = perm[u], perm[v]
    return u.astype(np.int32), v.astype(np.int32)


# --------------------------------------------------------------------------
# features
# --------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even narrowing of float32 values to bfloat16 bit
    patterns (uint16).  Input preparation only; finite inputs assumed."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def features(n: int, d: int, dist: str, rng: np.random.Generator) -> np.ndarray:
    if dist == "normal":
        return rng.standard_normal((n, d), dtype=np.float32)
    if dist == "uniform":
        x = rng.random((n, d), dtype=np.float32)
        x *= np.float32(2.0)
        x -= np.float32(1.0)
        return x
    raise ValueError(dist)


def fill_features(out: np.ndarray, dist: str, rng: np.random.Generator, chunk_rows: int = 1 << 18, progress=None) -> None:
    """Draws features() row chunk by row chunk into `out` (float32, or uint16 for
    bf16 bit patterns), so that a matrix too large to hold twice can be generated
    in place (e.g. into pinned host memory).  Same stream, same numbers."""
    n, d = out.shape
    for r0 in range(0, n, chunk_rows):
        x = features(min(chunk_rows, n - r0), d, dist, rng)
        out[r0:r0 + x.shape[0]] = f32_to_bf16_bits(x) if out.dtype == np.uint16 else x
        if progress:
            progress("feature rows drawn", r0 + x.shape[0], n)


# --------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    n: int
    d: int
    K: int
    agg: int
    dtype: int
    flags: int
    block_budget_edges: Optional[int]   # None: derived from n_blocks after planning
    n_blocks: Optional[int]
    src: np.ndarray = field(repr=False)
    dst: np.ndarray = field(repr=False)
    X: np.ndarray = field(repr=False)   # float32 (n,d), or uint16 bf16 bit patterns
    streamed: bool = False

    @property
    def m(self) -> int:
        return int(self.src.shape[0])


def _scaled(x: int, scale: float, lo: int = 1) -> int:
    return max(lo, int(round(x * scale)))


def make_workload(config: int, scale: float = 1.0, d: Optional[int] = None,
                  with_features: bool = True, contiguous_ids: bool = False, progress=None) -> Workload:
    """Workload `config` (1..5).  scale < 1 shrinks node and pair counts
    together (mean degree kept) for tests; scale = 1 is the full size.
    contiguous_ids (config 4 only) keeps every community's nodes on consecutive
    ids instead of permuting them: the same graph with its locality given.
    progress (config 5: minutes at full size): called as progress(what, done, total)
    after every chunk of generated pairs."""
    seed = BASE_SEED + config
    g = rng_for(seed, 0)
    xr = rng_for(seed, 1)
    if config == 1:
        n, M, dd, K = _scaled(10_000, scale, 8), _scaled(100_000, scale), d or 128, 2
        src, dst = gnm_pairs(n, M, g)
        w = Workload("tiny_gnm", n, dd, K, AGG_SYM, F32, SYMMETRISE | ADD_SELF_LOOPS,
                     None, 4, src, dst, None)
        dist = "normal"
    elif config == 2:
        n, M, dd, K = _scaled(169_343, scale, 8), _scaled(1_166_243, scale), d or 128, 3
        src, dst = chung_lu_pairs(n, M, 2.1, min(1.0e3, n / 4), g)
        w = Workload("chunglu_arxiv_like", n, dd, K, AGG_SYM, F32,
                     SYMMETRISE | ADD_SELF_LOOPS, 1 << 20, None, src, dst, None)
        dist = "normal"
    elif config == 3:
        n, M, dd, K = _scaled(2_450_000, scale, 8), _scaled(61_900_000, scale), d or 100, 3
        src, dst = chung_lu_pairs(n, M, 2.0, min(1.0e4, n / 4), g)
        w = Workload("chunglu_mean", n, dd, K, AGG_MEAN, F32, SYMMETRISE,
                     _scaled(8_000_000, scale, 16), None, src, dst, None)
        dist = "normal"
    elif config == 4:
        comm = _scaled(4_660, np.sqrt(scale), 4)
        n_comm = 50
        n = comm * n_comm
        M = min(_scaled(57_000_000, scale), n * (comm - 1) // 4)
        dd, K = d or 602, 2
        src, dst = sbm_pairs(n_comm, comm, M, 0.9, g, contiguous_ids=contiguous_ids)
        w = Workload("sbm_dense_sum", n, dd, K, AGG_SUM, F32, SYMMETRISE | ADD_SELF_LOOPS,
                     _scaled(8_000_000, scale, 16), None, src, dst, None)
        dist = "uniform"
    elif config == 5:
        n, M, dd, K = _scaled(111_059_956, scale, 8), _scaled(1_615_685_872, scale), d or 128, 3
        src, dst = chung_lu_pairs(n, M, 2.1, min(1.0e5, n / 4), g, progress=progress)
        w = Workload("chunglu_papers_like_streamed", n, dd, K, AGG_SYM, BF16,
                     SYMMETRISE | ADD_SELF_LOOPS, _scaled(1 << 28, scale, 16), None,
                     src, dst, None, streamed=True)
        dist = "normal"
    else:
        raise ValueError("config must be 1..5")
    if with_features:
        x = features(w.n, w.d, dist, xr)
        w.X = f32_to_bf16_bits(x) if w.dtype == BF16 else x
    return w


def stored_nonzeros_upper_bound(n: int, m_pairs: int, flags: int) -> int:
    """Upper bound of the stored non-zero count before duplicates collapse:
    both orientations of every pair when symmetrising, plus the diagonal."""
    nz = m_pairs * (2 if flags & SYMMETRISE else 1)
    if flags & ADD_SELF_LOOPS:
        nz += n
    return nz
