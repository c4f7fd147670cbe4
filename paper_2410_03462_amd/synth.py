"""Seeded synthetic inputs: graphs in CSR, modulation vectors f, and Q/K/V tensors.

This module holds no arithmetic of the method itself (no walks, no features, no
attention).  It only builds the inputs that both the HIP path and the CPU checker
are fed with, so that the two can be compared on identical data.

Graphs are returned as ``Graph(n, row_ptr[int32, n+1], col[int32, nnz], w[float32, nnz])``
with strictly ascending columns inside each row, no self loops and no duplicates.

The five named workloads stand in for the paper's image-patch grids (Sec. 4, ViT
experiments: a square grid of patches) and its large point clouds (Sec. 4 and
App. C: up to 32768 particles with nearest-neighbour graphs); the paper's own
datasets are not used anywhere.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass
class Graph:
    n: int
    row_ptr: np.ndarray  # int32 [n+1]
    col: np.ndarray      # int32 [nnz]
    w: np.ndarray        # float32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.col.shape[0])

    def degrees(self) -> np.ndarray:
        return np.diff(self.row_ptr).astype(np.int64)

    def dense(self) -> np.ndarray:
        """Dense float64 weighted adjacency matrix W (small graphs only)."""
        W = np.zeros((self.n, self.n), dtype=np.float64)
        rows = np.repeat(np.arange(self.n), self.degrees())
        W[rows, self.col] = self.w.astype(np.float64)
        return W


# --------------------------------------------------------------------------- CSR helpers

def csr_from_edges(n: int, src: np.ndarray, dst: np.ndarray, w: Optional[np.ndarray] = None) -> Graph:
    """Directed edge list (src -> dst) to CSR with sorted, de-duplicated columns."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    keep = src != dst
    src, dst = src[keep], dst[keep]
    if w is not None:
        w = np.asarray(w, dtype=np.float64)[keep]
    key = src * n + dst
    key, first = np.unique(key, return_index=True)
    src, dst = key // n, key % n
    if w is not None:
        w = w[first]
    else:
        w = np.ones(src.shape[0], dtype=np.float64)
    counts = np.bincount(src, minlength=n)
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=row_ptr[1:])
    assert row_ptr[-1] < 2**31
    return Graph(n, row_ptr.astype(np.int32), dst.astype(np.int32), w.astype(np.float32))


def with_weights(g: Graph, scheme: str) -> Graph:
    """Replace edge weights of a pattern.

    ``inv_deg``      w_ij = 1/deg(i)                 (row-normalised, not symmetric in general)
    ``sym_norm``     w_ij = 1/sqrt(deg(i) deg(j))    (the symmetric choice named in Sec. 3.1)
    ``row_norm``     w_ij = w_ij / sum_j w_ij        (row-normalise existing weights)
    """
    deg = g.degrees()
    rows = np.repeat(np.arange(g.n), deg)
    if scheme == "inv_deg":
        w = 1.0 / deg[rows]
    elif scheme == "sym_norm":
        w = 1.0 / np.sqrt(deg[rows].astype(np.float64) * deg[g.col].astype(np.float64))
    elif scheme == "row_norm":
        s = np.bincount(rows, weights=g.w.astype(np.float64), minlength=g.n)
        w = g.w.astype(np.float64) / s[rows]
    else:
        raise ValueError(scheme)
    return Graph(g.n, g.row_ptr, g.col, w.astype(np.float32))


# --------------------------------------------------------------------------- graph families

def grid_graph(h: int, w: int, neighbours: int = 4, periodic: bool = False, weights: str = "inv_deg") -> Graph:
    """h x w grid, row-major node ids, 4- or 8-neighbour stencil."""
    if neighbours == 4:
        offs = [(-1, 0), (1, 0), (0, -1), (0, 1)]
    elif neighbours == 8:
        offs = [(dy, dx) for dy in (-1, 0, 1) for dx in (-1, 0, 1) if (dy, dx) != (0, 0)]
    else:
        raise ValueError("neighbours must be 4 or 8")
    ys, xs = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    ys, xs = ys.ravel(), xs.ravel()
    src, dst = [], []
    for dy, dx in offs:
        y2, x2 = ys + dy, xs + dx
        if periodic:
            y2, x2 = y2 % h, x2 % w
            ok = np.ones_like(ys, dtype=bool)
        else:
            ok = (y2 >= 0) & (y2 < h) & (x2 >= 0) & (x2 < w)
        src.append((ys * w + xs)[ok])
        dst.append((y2 * w + x2)[ok])
    g = csr_from_edges(h * w, np.concatenate(src), np.concatenate(dst))
    return with_weights(g, weights)


def path_graph(n: int, weights: str = "inv_deg") -> Graph:
    """1-D grid (the graph family of the paper's FLOP-count figure)."""
    return grid_graph(1, n, 4, weights=weights)


def ring_graph(n: int, weights: str = "inv_deg") -> Graph:
    i = np.arange(n)
    g = csr_from_edges(n, np.concatenate([i, i]), np.concatenate([(i + 1) % n, (i - 1) % n]))
    return with_weights(g, weights)


def star_graph(n: int, weights: str = "inv_deg") -> Graph:
    """Node 0 is the hub; leaves 1..n-1."""
    leaves = np.arange(1, n)
    g = csr_from_edges(n, np.concatenate([np.zeros(n - 1, dtype=np.int64), leaves]),
                       np.concatenate([leaves, np.zeros(n - 1, dtype=np.int64)]))
    return with_weights(g, weights)


def matching_graph(n_pairs: int, rng: np.random.Generator) -> Graph:
    """Perfect matching (every node has degree 1) with random symmetric weights in (0.25, 1)."""
    a = np.arange(0, 2 * n_pairs, 2)
    b = a + 1
    wt = rng.uniform(0.25, 1.0, size=n_pairs)
    return csr_from_edges(2 * n_pairs, np.concatenate([a, b]), np.concatenate([b, a]), np.concatenate([wt, wt]))


def random_graph(n: int, avg_deg: float, rng: np.random.Generator, weights: str = "sym_norm",
                 isolated: int = 0) -> Graph:
    """Undirected Erdos-Renyi-like graph; optionally the last ``isolated`` nodes get no edges."""
    m = int(n * avg_deg / 2)
    hi = n - isolated
    a = rng.integers(0, hi, size=m)
    b = rng.integers(0, hi, size=m)
    g = csr_from_edges(n, np.concatenate([a, b]), np.concatenate([b, a]))
    deg = g.degrees()
    if weights in ("inv_deg", "sym_norm"):
        rows = np.repeat(np.arange(n), deg)
        if weights == "inv_deg":
            w = 1.0 / deg[rows]
        else:
            w = 1.0 / np.sqrt(deg[rows].astype(np.float64) * deg[g.col].astype(np.float64))
        return Graph(n, g.row_ptr, g.col, w.astype(np.float32))
    return g


def knn_graph(points: np.ndarray, k: int, kernel: str) -> Graph:
    """Symmetrised exact k-nearest-neighbour graph with kernel weights, row-normalised.

    i ~ j if either lists the other among its k nearest.  ``kernel`` is ``"exp"``
    (w = exp(-dist/sigma)) or ``"gauss"`` (w = exp(-dist^2 / (2 sigma^2))); sigma is the
    median over all directed kNN edge lengths.
    """
    from scipy.spatial import cKDTree

    n = points.shape[0]
    tree = cKDTree(points)
    dist, idx = tree.query(points, k=k + 1)
    dist, idx = dist[:, 1:], idx[:, 1:]
    sigma = float(np.median(dist))
    src = np.repeat(np.arange(n), k)
    dst = idx.ravel()
    dd = dist.ravel()
    if kernel == "exp":
        wt = np.exp(-dd / sigma)
    elif kernel == "gauss":
        wt = np.exp(-(dd * dd) / (2.0 * sigma * sigma))
    else:
        raise ValueError(kernel)
    g = csr_from_edges(n, np.concatenate([src, dst]), np.concatenate([dst, src]), np.concatenate([wt, wt]))
    return with_weights(g, "row_norm")


def uniform_points(n: int, rng: np.random.Generator) -> np.ndarray:
    return rng.random((n, 3))


def cluster_points(n: int, n_clusters: int, std: float, rng: np.random.Generator) -> np.ndarray:
    """Equal-weight mixture of isotropic Gaussians with centres uniform in the unit cube."""
    centres = rng.random((n_clusters, 3))
    which = rng.integers(0, n_clusters, size=n)
    return centres[which] + std * rng.standard_normal((n, 3))


# --------------------------------------------------------------------------- tensors

def one_long_column(length, rng):
    """A hand-made feature matrix in CSR, for tests of list-length boundaries: n = length + 3 rows, a diagonal, and a
    column 0 of `length` entries (rows 0 .. length-1); values uniform in 0.2 .. 1.  Returns (n, row_ptr, col, val[1, nnz])."""
    n = length + 3
    rows = np.concatenate([np.arange(n), np.arange(1, length)])
    cols = np.concatenate([np.arange(n), np.zeros(length - 1, dtype=np.int64)])
    order = np.lexsort((cols, rows))
    rows, cols = rows[order], cols[order]
    rp = np.zeros(n + 1, dtype=np.int32)
    np.add.at(rp, rows + 1, 1)
    rp = np.cumsum(rp).astype(np.int32)
    val = rng.uniform(0.2, 1.0, size=(1, len(cols))).astype(np.float32)
    return n, rp, cols.astype(np.int32), val



def columns_of_lengths(lengths, rng):
    """A hand-made n x n feature matrix in CSR whose column l has exactly ``lengths[l]`` entries (n = len(lengths)), for
    tests of how column lists of given lengths sit next to each other: the rows are dealt out along a random permutation,
    so the entries of a column lie in distinct rows and, if the lengths sum to at least n, no row is empty; values uniform
    in 0.2 .. 1.  Returns (n, row_ptr, col, val[1, nnz])."""
    lengths = np.asarray(lengths, dtype=np.int64)
    n = int(lengths.shape[0])
    assert lengths.max() <= n
    perm = rng.permutation(n)
    cols = np.repeat(np.arange(n), lengths)
    rows = perm[np.arange(cols.shape[0]) % n]
    order = np.lexsort((cols, rows))
    rows, cols = rows[order], cols[order]
    rp = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rp, rows + 1, 1)
    rp = np.cumsum(rp).astype(np.int32)
    val = rng.uniform(0.2, 1.0, size=(1, len(cols))).astype(np.float32)
    return n, rp, cols.astype(np.int32), val


def modulation(f_len: int, rng: np.random.Generator, kind: str = "decay", n_f: int = 1, std: float = 1.0) -> np.ndarray:
    """f of shape [n_f, f_len], float32.  ``decay``: N(0,1)/(k+1); ``normal``: N(0, std)."""
    g = rng.standard_normal((n_f, f_len))
    if kind == "decay":
        g = g / (np.arange(f_len) + 1.0)
    elif kind == "normal":
        g = g * std
    else:
        raise ValueError(kind)
    return g.astype(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def qkv(B: int, H: int, n: int, d: int, rng: np.random.Generator, dtype: str = "f32"):
    """Q, K, V ~ N(0,1), shape [B,H,n,d].

    Returns float32 arrays.  For ``dtype == "bf16"`` the values are already rounded to
    bfloat16-representable numbers, so converting them to bf16 bit patterns is exact.
    """
    out = []
    for _ in range(3):
        x = rng.standard_normal((B, H, n, d), dtype=np.float32)
        if dtype == "bf16":
            x = bf16_bits_to_f32(f32_to_bf16_bits(x))
        elif dtype != "f32":
            raise ValueError(dtype)
        out.append(x)
    return out


# --------------------------------------------------------------------------- named workloads

@dataclass
class Workload:
    name: str
    graph: Graph
    f: np.ndarray          # [n_f, f_len] float32
    p_halt: float
    n_walks: int
    B: int
    H: int
    d: int
    dtype: str             # "f32" | "bf16"
    walk_seed: int = 0
    data_seed: int = 0
    notes: dict = field(default_factory=dict)

    @property
    def f_len(self) -> int:
        return int(self.f.shape[1])

    @property
    def n_f(self) -> int:
        return int(self.f.shape[0])

    def qkv(self):
        rng = np.random.default_rng([self.data_seed, 7])
        return qkv(self.B, self.H, self.graph.n, self.d, rng, self.dtype)


def workload(name: str, data_seed: int = 0, walk_seed: int = 0) -> Workload:
    """The five benchmark configurations, by name.

    ``tiny_grid``        16x16 4-neighbour grid, n=4, p=0.5, L=8, B=1, H=1, d=32, f32
    ``vit_grid``         32x32 8-neighbour grid, n=8, p=0.5, L=10, B=32, H=8, d=64, f32
    ``cloud_8k``         8192 uniform points, kNN k=8, exp kernel, n=16, p=0.25, L=12, B=8, H=8, d=64, f32
    ``cloud_32k``        32768 points in 16 Gaussian clusters, kNN k=16, Gaussian kernel,
                         n=32, p=0.2, L=16, B=1, H=8, d=64, f32   (the headline workload)
    ``cloud_128k``       131072 uniform points, kNN k=16, Gaussian kernel, n=32, p=0.2, L=16,
                         per-head f, B=1, H=16, d=64, bf16 inputs
    """
    rng = np.random.default_rng([data_seed, 1])
    if name == "tiny_grid":
        g = grid_graph(16, 16, 4)
        return Workload(name, g, modulation(8, rng, "decay"), 0.5, 4, 1, 1, 32, "f32", walk_seed, data_seed)
    if name == "vit_grid":
        g = grid_graph(32, 32, 8)
        return Workload(name, g, modulation(10, rng, "normal", std=0.5), 0.5, 8, 32, 8, 64, "f32", walk_seed, data_seed)
    if name == "cloud_8k":
        pts = uniform_points(8192, rng)
        g = knn_graph(pts, 8, "exp")
        return Workload(name, g, modulation(12, rng, "decay"), 0.25, 16, 8, 8, 64, "f32", walk_seed, data_seed,
                        {"points": pts, "k": 8, "kernel": "exp"})
    if name == "cloud_32k":
        pts = cluster_points(32768, 16, 0.05, rng)
        g = knn_graph(pts, 16, "gauss")
        return Workload(name, g, modulation(16, rng, "decay"), 0.2, 32, 1, 8, 64, "f32", walk_seed, data_seed,
                        {"points": pts, "k": 16, "kernel": "gauss"})
    if name == "cloud_128k":
        pts = uniform_points(131072, rng)
        g = knn_graph(pts, 16, "gauss")
        return Workload(name, g, modulation(16, rng, "decay", n_f=16), 0.2, 32, 1, 16, 64, "bf16", walk_seed, data_seed,
                        {"points": pts, "k": 16, "kernel": "gauss"})
    raise ValueError(name)


WORKLOADS = ("tiny_grid", "vit_grid", "cloud_8k", "cloud_32k", "cloud_128k")
