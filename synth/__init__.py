"""Seeded synthetic inputs for the GCN hot path (graphs, permutations, features, weights, labels).

This module is shared by the tests, the benchmark, the CPU oracle's callers and the HIP
path's callers.  It holds none of the method's arithmetic: no normalisation, no sparse
product, no layer maths.  Everything is a pure function of (seed, stream, element index)
through one counter-based 64-bit generator, written with torch integer ops so the same
code gives the same integers on the host and on the device.  Floating-point draws (normal
features) may differ in the last bit between devices; callers therefore generate a tensor
ONCE and hand the same bits to both sides.

The graphs stand in for the datasets of Table 4 of the paper (which are not available
here): same node counts, edge counts, feature widths and skew, no record of any dataset.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import torch

__all__ = [
    "mix64", "hash_u64", "uniform_int", "uniform01", "normal", "glorot", "labels",
    "permutation", "affine_bijection", "rmat_edges", "road_edges", "shard_block",
    "GraphConfig", "CONFIGS", "BASE_SEED",
]

BASE_SEED = 0x504C5800

_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

# streams (independent sequences under one seed)
S_EDGE, S_PERM_R, S_PERM_C, S_FEAT, S_WEIGHT, S_LABEL, S_AUX = 1, 2, 3, 4, 5, 6, 7


def _s64(c: int) -> int:
    """Python unsigned 64-bit constant -> the signed value torch.int64 stores for it."""
    c &= (1 << 64) - 1
    return c - (1 << 64) if c >= (1 << 63) else c


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right on int64 (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """The splitmix64 output function on wrapping int64 tensors."""
    z = x + _s64(_GOLDEN)
    z = (z ^ _lsr(z, 30)) * _s64(_M1)
    z = (z ^ _lsr(z, 27)) * _s64(_M2)
    return z ^ _lsr(z, 31)


def mix64_py(x: int) -> int:
    """Same function on a Python int (reference for the tests of the torch version)."""
    m = (1 << 64) - 1
    z = (x + _GOLDEN) & m
    z = ((z ^ (z >> 30)) * _M1) & m
    z = ((z ^ (z >> 27)) * _M2) & m
    return z ^ (z >> 31)


def _key(seed: int, stream: int) -> int:
    return _s64(mix64_py((seed & ((1 << 64) - 1)) ^ mix64_py(stream)))


def hash_u64(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """64 random bits per element of the int64 index tensor `idx` (returned as int64)."""
    return mix64(mix64(idx + _key(seed, stream)) ^ _s64(_M2 * (stream + 1)))


def uniform_int(seed: int, stream: int, idx: torch.Tensor, n: int) -> torch.Tensor:
    """Integers in [0, n): 63 hashed bits modulo n (bias < n / 2^63)."""
    return _lsr(hash_u64(seed, stream, idx), 1) % n


def uniform01(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """fp64 in [0,1) with 53 random bits; exact, hence identical on every device."""
    return _lsr(hash_u64(seed, stream, idx), 11).to(torch.float64) * (2.0 ** -53)


def _arange(n0: int, n1: int, device) -> torch.Tensor:
    return torch.arange(n0, n1, dtype=torch.int64, device=device)


def normal(seed: int, stream: int, rows: int, cols: int, device="cpu", dtype=torch.float32,
           chunk_rows: Optional[int] = None) -> torch.Tensor:
    """rows x cols standard-normal matrix (Box-Muller on two hashed uniforms per element).

    Element (i, j) depends only on (seed, stream, i*cols + j), so any row slice can be
    regenerated alone (used by the sampled parity checks at full size)."""
    out = torch.empty((rows, cols), dtype=dtype, device=device)
    if rows == 0 or cols == 0:
        return out
    if chunk_rows is None:
        chunk_rows = max(1, (1 << 25) // cols)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = normal_rows(seed, stream, r0, r1, cols, device, dtype)
    return out


def normal_rows(seed: int, stream: int, r0: int, r1: int, cols: int, device="cpu",
                dtype=torch.float32) -> torch.Tensor:
    idx = _arange(r0 * cols, r1 * cols, device)
    u1 = 1.0 - uniform01(seed, stream, idx * 2)          # (0, 1]
    u2 = uniform01(seed, stream, idx * 2 + 1)
    z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
    return z.reshape(r1 - r0, cols).to(dtype)


def glorot(seed: int, layer: int, d_in: int, d_out: int, device="cpu", dtype=torch.float32) -> torch.Tensor:
    """Glorot-uniform U(-a, a), a = sqrt(6 / (d_in + d_out)); one stream per layer."""
    a = math.sqrt(6.0 / (d_in + d_out))
    idx = _arange(0, d_in * d_out, device)
    u = uniform01(seed, S_WEIGHT + 16 * (layer + 1), idx)
    return ((2.0 * u - 1.0) * a).reshape(d_in, d_out).to(dtype)


def labels(seed: int, n: int, n_classes: int, device="cpu") -> torch.Tensor:
    """Uniform random class per node, int64."""
    return uniform_int(seed, S_LABEL, _arange(0, n, device), n_classes)


def permutation(seed: int, stream: int, n: int, device="cpu") -> torch.Tensor:
    """A random bijection perm[old] = new on [0, n): rank order of hashed keys.

    Ties between 64-bit keys are broken by index (stable sort), so the result is the same
    on every device."""
    keys = hash_u64(seed, stream, _arange(0, n, device))
    order = torch.sort(keys, stable=True).indices          # order[new] = old
    perm = torch.empty_like(order)
    perm[order] = _arange(0, n, device)
    return perm


def _coprime_multiplier(seed: int, stream: int, n: int) -> int:
    g = mix64_py(_key(seed, stream) & ((1 << 64) - 1)) % n
    g |= 1
    while math.gcd(g, n) != 1 or g < 2:
        g += 2
    return g % n if n > 2 else 1


def affine_bijection(seed: int, stream: int, n: int, x: torch.Tensor) -> torch.Tensor:
    """x -> (g*x + b) mod n with gcd(g, n) = 1: a cheap id scrambler for huge index ranges
    (no table).  n < 2^31 so g*x stays below 2^62."""
    assert n < (1 << 31)
    g = _coprime_multiplier(seed, stream, n)
    b = mix64_py(g ^ stream) % n
    return (x * g + b) % n


# ----------------------------------------------------------------------------------------
# graphs
# ----------------------------------------------------------------------------------------

def _rmat_bits(seed: int, stream: int, idx: torch.Tensor, scale_r: int, scale_c: int,
               abcd=(0.57, 0.19, 0.19, 0.05)) -> Tuple[torch.Tensor, torch.Tensor]:
    """Recursive-quadrant (R-MAT) sample per element of idx: at every level one hashed
    53-bit integer is compared with the integer thresholds of (a, a+b, a+b+c), so the
    result is exact.  With scale_r < scale_c the first (scale_c - scale_r) levels choose a
    column bit only (probability b+d of a one), which gives a rectangular power-law block."""
    a, b, c, d = abcd
    t_a = int(a * (1 << 53))
    t_ab = int((a + b) * (1 << 53))
    t_abc = int((a + b + c) * (1 << 53))
    t_col = int((a + c) * (1 << 53))
    levels = max(scale_r, scale_c)
    r = torch.zeros_like(idx)
    cidx = torch.zeros_like(idx)
    for lev in range(levels):
        h = _lsr(hash_u64(seed, stream + 64 * (lev + 1), idx), 11)
        both = (levels - lev) <= min(scale_r, scale_c)
        if both:
            rb = (h >= t_ab).to(torch.int64)
            cb = ((h >= t_a) & (h < t_ab) | (h >= t_abc)).to(torch.int64)
            r = (r << 1) | rb
            cidx = (cidx << 1) | cb
        elif scale_c > scale_r:
            cidx = (cidx << 1) | (h >= t_col).to(torch.int64)
        else:
            r = (r << 1) | (h >= t_ab).to(torch.int64)
    return r, cidx


def _first_unique(keys: torch.Tensor, limit: Optional[int]) -> torch.Tensor:
    """Distinct values of `keys`, ordered by first occurrence, at most `limit` of them."""
    if keys.numel() == 0:
        return keys
    srt = torch.sort(keys, stable=True)
    k, pos = srt.values, srt.indices
    first = torch.ones_like(k, dtype=torch.bool)
    first[1:] = k[1:] != k[:-1]
    fpos = torch.sort(pos[first]).values                  # sample positions of first occurrences
    if limit is not None:
        fpos = fpos[:limit]
    return keys[fpos]


def rmat_edges(seed: int, n: int, n_edges: int, device="cpu", abcd=(0.57, 0.19, 0.19, 0.05),
               batch: Optional[int] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Exactly `n_edges` distinct undirected non-loop R-MAT edges on n nodes.

    Scale = ceil(log2 n); endpoints >= n are rejected; samples are drawn in index order
    until enough distinct {u, v} pairs exist, then the first n_edges distinct pairs (by
    sample index) are kept.  Returned as (src, dst) with src < dst, int64, in first-
    occurrence order: one direction only -- symmetrising is the library's job."""
    scale = max(1, math.ceil(math.log2(max(n, 2))))
    max_pairs = n * (n - 1) // 2
    assert n_edges <= max_pairs
    if batch is None:
        batch = max(1 << 16, min(1 << 27, int(n_edges * 1.3) + 1024))
    kept = torch.empty(0, dtype=torch.int64, device=device)
    drawn = 0
    while kept.numel() < n_edges:
        idx = _arange(drawn, drawn + batch, device)
        drawn += batch
        u, v = _rmat_bits(seed, S_EDGE, idx, scale, scale, abcd)
        ok = (u < n) & (v < n) & (u != v)
        lo = torch.minimum(u, v)[ok]
        hi = torch.maximum(u, v)[ok]
        kept = _first_unique(torch.cat([kept, lo * n + hi]), n_edges)
        if drawn > 400 * max(n_edges, 1) + (1 << 22):
            raise RuntimeError("rmat_edges: cannot reach the requested number of distinct edges")
    return kept // n, kept % n


def road_edges(seed: int, gx: int, gy: int, keep_prob: float, long_range_frac: float,
               device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """Road-like graph on a gx x gy grid (node id = x*gy + y, row-major): every 4-neighbour
    grid edge is kept with probability keep_prob, plus round(long_range_frac * n) uniformly
    random long-range pairs.  May contain a few duplicate pairs (the library dedupes)."""
    n = gx * gy
    thr = int(keep_prob * (1 << 53))
    ids = _arange(0, n, device)
    x, y = ids // gy, ids % gy
    # edge to the next node in y, and to the next node in x
    keep_y = (y + 1 < gy) & (_lsr(hash_u64(seed, S_EDGE, ids * 2), 11) < thr)
    keep_x = (x + 1 < gx) & (_lsr(hash_u64(seed, S_EDGE, ids * 2 + 1), 11) < thr)
    n_long = int(round(long_range_frac * n))
    li = _arange(0, n_long, device)
    lu = uniform_int(seed, S_AUX, li * 2, n)
    lv = uniform_int(seed, S_AUX, li * 2 + 1, n)
    src = torch.cat([ids[keep_y], ids[keep_x], lu])
    dst = torch.cat([ids[keep_y] + 1, ids[keep_x] + gy, lv])
    return src, dst


def shard_block(seed: int, m: int, k: int, n_samples: int, device="cpu",
                abcd=(0.57, 0.19, 0.19, 0.05)) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """One GPU's rectangular block (m rows x k cols) of a double-permuted power-law
    adjacency, synthesised directly: rectangular R-MAT samples (row scale ceil(log2 m),
    column scale ceil(log2 k), out-of-range rejected), rows and columns scrambled by two
    different affine bijections (the double permutation leaves no locality), duplicates
    removed, sorted into canonical CSR.  Values are 1/sqrt((4*len_r+1)*(16*len_c+1)) --
    a degree-shaped positive weight, not the library's normalisation (the block is fed to
    the library as an already-built CSR).

    Returns (rowptr int64[m+1], col int32[nnz], val float32[nnz])."""
    sr = max(1, math.ceil(math.log2(max(m, 2))))
    sc = max(1, math.ceil(math.log2(max(k, 2))))
    parts: List[torch.Tensor] = []
    batch = 1 << 26
    for s0 in range(0, n_samples, batch):
        idx = _arange(s0, min(n_samples, s0 + batch), device)
        r, c = _rmat_bits(seed, S_EDGE, idx, sr, sc, abcd)
        ok = (r < m) & (c < k)
        r = affine_bijection(seed, S_PERM_R, m, r[ok])
        c = affine_bijection(seed, S_PERM_C, k, c[ok])
        parts.append(r * k + c)
        del idx, r, c, ok
    keys = torch.unique(torch.cat(parts)) if parts else torch.empty(0, dtype=torch.int64, device=device)
    del parts
    rows = keys // k
    cols = keys % k
    del keys
    rlen = torch.bincount(rows, minlength=m)
    clen = torch.bincount(cols, minlength=k)
    rowptr = torch.zeros(m + 1, dtype=torch.int64, device=device)
    rowptr[1:] = torch.cumsum(rlen, 0)
    val = torch.rsqrt(((4 * rlen + 1)[rows] * (16 * clen + 1)[cols]).to(torch.float64)).to(torch.float32)
    return rowptr, cols.to(torch.int32), val


# ----------------------------------------------------------------------------------------
# the five workloads
# ----------------------------------------------------------------------------------------

@dataclass
class GraphConfig:
    """One workload: graph recipe + network widths.  `dims` = [D0, D1, ..., DL]."""
    name: str
    cid: int
    kind: str                      # "rmat" | "road" | "shard"
    n: int = 0
    n_edges: int = 0               # distinct undirected edges (rmat)
    dims: List[int] = field(default_factory=list)
    n_classes: int = 0
    grid: Tuple[int, int] = (0, 0)
    keep_prob: float = 0.0
    long_frac: float = 0.0
    m: int = 0                     # shard block rows
    k: int = 0                     # shard block cols
    n_samples: int = 0             # shard R-MAT samples before dedupe

    @property
    def seed(self) -> int:
        return BASE_SEED + self.cid

    def edges(self, device="cpu"):
        if self.kind == "rmat":
            return rmat_edges(self.seed, self.n, self.n_edges, device)
        if self.kind == "road":
            return road_edges(self.seed, self.grid[0], self.grid[1], self.keep_prob, self.long_frac, device)
        raise ValueError(self.kind)

    def perms(self, device="cpu"):
        return (permutation(self.seed, S_PERM_R, self.n, device),
                permutation(self.seed, S_PERM_C, self.n, device))

    def features(self, device="cpu", dtype=torch.float32):
        return normal(self.seed, S_FEAT, self.n, self.dims[0], device, dtype)

    def weights(self, device="cpu", dtype=torch.float32):
        return [glorot(self.seed, l, self.dims[l], self.dims[l + 1], device, dtype)
                for l in range(len(self.dims) - 1)]

    def labels(self, device="cpu"):
        return labels(self.seed, self.n, self.n_classes, device)

    def scaled(self, factor: float, name: Optional[str] = None) -> "GraphConfig":
        """Same recipe shrunk by `factor` in nodes and edges (used by CPU-sized tests)."""
        c = GraphConfig(**self.__dict__)
        c.name = name or f"{self.name}_x{factor:g}"
        c.n = max(8, int(self.n * factor))
        c.n_edges = max(8, int(self.n_edges * factor))
        c.grid = (max(2, int(self.grid[0] * math.sqrt(factor))), max(2, int(self.grid[1] * math.sqrt(factor))))
        if self.kind == "road":
            c.n = c.grid[0] * c.grid[1]
        c.m = max(8, int(self.m * factor))
        c.k = max(8, int(self.k * factor))
        c.n_samples = max(8, int(self.n_samples * factor))
        return c


CONFIGS = {
    # configs[0]: tiny R-MAT, exactly 65,536 undirected edges => nnz = 2*65,536 + 4,096
    "tiny": GraphConfig("tiny", 1, "rmat", n=4096, n_edges=65536, dims=[128, 128, 128, 16], n_classes=16),
    # configs[1]: Reddit-shaped (Table 4 row 1)
    "social": GraphConfig("social", 2, "rmat", n=232_965, n_edges=57_300_000, dims=[602, 128, 128, 41], n_classes=41),
    # configs[2]: ogbn-products-shaped (Table 4 row 2)
    "copurchase": GraphConfig("copurchase", 3, "rmat", n=2_449_029, n_edges=61_860_000, dims=[100, 128, 128, 47], n_classes=47),
    # configs[3]: one GPU's block of a billion-edge graph; layer is 32 -> 128 on the block
    "shard": GraphConfig("shard", 4, "shard", m=7_000_000, k=28_000_000, n_samples=210_000_000, dims=[32, 128]),
    # configs[4]: europe_osm-shaped thinned grid (Table 4 row 5)
    "road": GraphConfig("road", 5, "road", n=50_000_000, grid=(10_000, 5_000), keep_prob=0.53, long_frac=0.02,
                        dims=[64, 128, 16], n_classes=16),
    # secondary rows: the shard block at the entry count a 1/16 x 1/4 block of a 3.2 B-entry matrix
    # would really hold (~50 M), and the road grid with every 4-neighbour edge kept (~250 M entries)
    "shard_sparse": GraphConfig("shard_sparse", 6, "shard", m=7_000_000, k=28_000_000, n_samples=51_000_000, dims=[32, 128]),
    "road_full": GraphConfig("road_full", 7, "road", n=50_000_000, grid=(10_000, 5_000), keep_prob=1.0, long_frac=0.02,
                             dims=[64, 128, 16], n_classes=16),
}
