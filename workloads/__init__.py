"""Seeded synthetic inputs for the TT-embedding path.

This module holds no arithmetic of the method: it only draws shapes, node ids, core values and
upstream gradients.  The same arrays feed the CPU oracle and the GPU library.

The five workloads stand in for the graphs the paper trains on (ogbn-arxiv, ogbn-products,
ogbn-papers100M), which are not available here: table shapes are those graphs' node counts rounded
to near-cubes, embedding widths and TT ranks are the paper's, and the id streams imitate a sampled
minibatch (uniform with replacement), a degree-skewed minibatch (bounded Zipf over a random
relabelling) and a partition-ordered minibatch (draws clustered in contiguous id blocks).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    n: tuple          # node factors (n1, n2, n3)
    d: tuple          # embedding-dimension factors (d1, d2, d3)
    r: tuple          # inner TT ranks (r1, r2)
    batch: int        # rows per step, duplicates counted
    ids: str          # "uniform" | "zipf_perm" | "zipf_affine" | "clusters"
    zipf_s: float = 0.0
    init_std: float = 0.0
    lr: float = 0.01
    extra: dict = field(default_factory=dict)

    @property
    def N(self) -> int:
        return self.n[0] * self.n[1] * self.n[2]

    @property
    def D(self) -> int:
        return self.d[0] * self.d[1] * self.d[2]

    def core_shapes(self):
        (n1, n2, n3), (d1, d2, d3), (r1, r2) = self.n, self.d, self.r
        return (n1, d1, r1), (n2, r1, d2, r2), (n3, r2, d3)


CONFIGS = {
    1: Workload("c1_tiny_1k_r4", (10, 10, 10), (2, 2, 2), (4, 4), 256, "uniform", init_std=0.1),
    2: Workload("c2_175k_r16", (56, 56, 56), (4, 4, 4), (16, 16), 50_000, "uniform",
                init_std=1 / math.sqrt(16)),
    3: Workload("c3_2p5m_r32_zipf1.1", (136, 136, 136), (4, 4, 8), (32, 32), 200_000, "zipf_perm",
                zipf_s=1.1, init_std=1 / math.sqrt(32)),
    4: Workload("c4_111m_r16_zipf1.0", (480, 480, 482), (4, 4, 8), (16, 16), 500_000,
                "zipf_affine", zipf_s=1.0, init_std=1 / math.sqrt(16)),
    5: Workload("c5_111m_r64_clusters", (480, 480, 482), (4, 4, 8), (64, 64), 500_000, "clusters",
                init_std=1 / math.sqrt(64), extra={"blocks": 500, "block_len": 1000}),
    # The paper's own factorisations and dimension orders (Table "ogb-dim-tt"), with the id streams
    # of configs 2-4: not benchmark configurations, measured beside them.
    6: Workload("p_arxiv_55x55x56_d8x4x4_r16", (55, 55, 56), (8, 4, 4), (16, 16), 50_000, "uniform",
                init_std=1 / math.sqrt(16)),
    7: Workload("p_products_125x140x140_d4x5x5_r32", (125, 140, 140), (4, 5, 5), (32, 32), 200_000,
                "zipf_perm", zipf_s=1.1, init_std=1 / math.sqrt(32)),
    8: Workload("p_papers100m_480x500x500_d8x4x4_r16", (480, 500, 500), (8, 4, 4), (16, 16),
                500_000, "zipf_affine", zipf_s=1.0, init_std=1 / math.sqrt(16)),
}


def bounded_zipf_ranks(rng: np.random.Generator, N: int, s: float, size: int) -> np.ndarray:
    """Ranks in [0, N) with P(rank k) proportional to (k+1)^-s, by inverting the exact CDF."""
    w = np.arange(1, N + 1, dtype=np.float64)
    np.power(w, -s, out=w)
    np.cumsum(w, out=w)
    w /= w[-1]
    ranks = np.searchsorted(w, rng.random(size), side="left")
    return np.minimum(ranks, N - 1).astype(np.int64)


def make_ids(w: Workload, seed: int, batch: int | None = None) -> np.ndarray:
    """int64 node ids of one minibatch."""
    B = w.batch if batch is None else batch
    rng = np.random.default_rng(seed)
    N = w.N
    if w.ids == "uniform":
        return rng.integers(0, N, size=B, dtype=np.int64)
    if w.ids == "zipf_perm":
        ranks = bounded_zipf_ranks(rng, N, w.zipf_s, B)
        perm = rng.permutation(N)
        return perm[ranks].astype(np.int64)
    if w.ids == "zipf_affine":
        ranks = bounded_zipf_ranks(rng, N, w.zipf_s, B)
        # id = (a*rank + c) mod N with gcd(a, N) = 1: a bijection that scatters hot ranks
        a = int(rng.integers(N // 3, N // 2))
        while math.gcd(a, N) != 1:
            a += 1
        c = int(rng.integers(0, N))
        assert N < 2**31  # ranks*a stays far below 2^63
        return ((ranks * a + c) % N).astype(np.int64)
    if w.ids == "clusters":
        blocks, blen = w.extra["blocks"], w.extra["block_len"]
        per = B // blocks
        starts = rng.integers(0, N - blen + 1, size=blocks, dtype=np.int64)
        offs = rng.integers(0, blen, size=(blocks, per), dtype=np.int64)
        ids = (starts[:, None] + offs).reshape(-1)
        if ids.size < B:  # B not a multiple of the block count: top up from the last block
            extra = starts[-1] + rng.integers(0, blen, size=B - ids.size, dtype=np.int64)
            ids = np.concatenate([ids, extra])
        return ids.astype(np.int64)
    raise ValueError(w.ids)


def make_cores(w: Workload, seed: int):
    """fp32 cores g1[n1,d1,r1], g2[n2,r1,d2,r2], g3[n3,r2,d3], i.i.d. N(0, init_std^2)."""
    rng = np.random.default_rng(seed + 7919)
    return tuple((rng.standard_normal(cs, dtype=np.float32) * np.float32(w.init_std))
                 for cs in w.core_shapes())


def make_grads(w: Workload, seed: int, batch: int | None = None) -> np.ndarray:
    """fp32 upstream gradients grad[B, D], i.i.d. N(0, 1)."""
    B = w.batch if batch is None else batch
    rng = np.random.default_rng(seed + 104729)
    return rng.standard_normal((B, w.D), dtype=np.float32)


def batch_structure(w: Workload, ids: np.ndarray) -> dict:
    """Counts that describe a batch: unique ids U, unique (i1,i2) prefixes Q, hottest multiplicity."""
    ids = np.asarray(ids, dtype=np.int64)
    ok = ids[(ids >= 0) & (ids < w.N)]
    u, cnt = np.unique(ok, return_counts=True)
    q = np.unique(u // w.n[2])
    return {"B": int(ids.size), "U": int(u.size), "Q": int(q.size),
            "max_multiplicity": int(cnt.max()) if cnt.size else 0,
            "i1": int(np.unique(q // w.n[1]).size), "i2": int(np.unique(q % w.n[1]).size),
            "i3": int(np.unique(u % w.n[2]).size)}


def make_orthogonal_cores(n, d, r, seed: int):
    """Cores initialised as in the paper's Algorithm 2 ("Orthogonal Initialization of TT-cores"):
    for core i, n_i*R_{i-1} orthonormal vectors of length m_i*R_i (paper letters: m = node factor,
    n = dimension factor) fill the core so that its unfolding is semi-orthogonal; Claim 1 then
    makes the columns of the full table orthogonal.  Needs d_i*R_{i-1} <= n_i*R_i for every core
    (the paper's feasibility condition, Section 4.1).  Returns fp32 cores in slice-contiguous
    layout g1[n1,d1,r1], g2[n2,r1,d2,r2], g3[n3,r2,d3].  This is input generation for tests; it is
    not on the lookup path."""
    rng = np.random.default_rng(seed)
    ranks = (1, int(r[0]), int(r[1]), 1)
    cores = []
    for i in range(3):
        rows, cols = int(n[i]) * ranks[i + 1], int(d[i]) * ranks[i]
        if cols > rows:
            raise ValueError(f"core {i + 1}: {cols} orthogonal vectors of length {rows} do not exist")
        q, _ = np.linalg.qr(rng.standard_normal((rows, cols)))     # columns: orthonormal vectors v
        v = q.T.reshape(ranks[i], int(d[i]), int(n[i]), ranks[i + 1])  # v[r, j, i_k, s]
        # layout per Algorithm 2 (Section 4.1): vector number n_i*r + j fills the (r, j) fibre of
        # core i over (node index, outgoing rank); stored here as g[i_k][r][j][s]
        cores.append(np.ascontiguousarray(np.transpose(v, (2, 0, 1, 3))).astype(np.float32))
    g1 = cores[0].reshape(int(n[0]), int(d[0]), ranks[1])
    g2 = cores[1]
    g3 = cores[2].reshape(int(n[2]), ranks[2], int(d[2]))
    return g1, g2, g3


def make_ttsvd_cores(n, d, r, seed: int, matrix: np.ndarray | None = None, return_info: bool = False):
    """Cores from the paper's Algorithm 1 ("TTM Decomposition", Section 4.1): a TT-SVD of a given
    N x D matrix - by default a random matrix with orthonormal columns, which is the initialisation
    the paper calls decomp-ortho - in the TT-matrix format of Eq. "tt-matrix".  The matrix is viewed
    as a tensor over (i1, i2, i3, j1, j2, j3), its modes are paired as (i1 j1), (i2 j2), (i3 j3), and
    the cores are peeled off left to right: unfold with (incoming rank, i_k, j_k) as rows, take the
    leading R_k left singular vectors as core k, carry diag(singular values) times the right
    singular vectors on; what is left after the second step is the third core.  With ranks at
    least the unfoldings' ranks the product of the cores reproduces the matrix exactly; otherwise
    the Frobenius error is at most the root of the summed squares of the discarded singular values
    of both steps.  Host-side SVDs of dense unfoldings: for small tables only (the paper reports
    31 minutes for its largest one).  Returns fp32 cores in slice-contiguous layout
    g1[n1,d1,r1], g2[n2,r1,d2,r2], g3[n3,r2,d3]; with return_info also a dict holding the matrix
    and the discarded singular values.  This is input generation for tests; it is not on the lookup
    path."""
    n1, n2, n3 = (int(x) for x in n)
    d1, d2, d3 = (int(x) for x in d)
    r1, r2 = int(r[0]), int(r[1])
    N, D = n1 * n2 * n3, d1 * d2 * d3
    rng = np.random.default_rng(seed)
    if matrix is None:
        if D > N:
            raise ValueError("a matrix with orthonormal columns needs at least as many rows as columns")
        matrix, _ = np.linalg.qr(rng.standard_normal((N, D)))
    W = np.asarray(matrix, dtype=np.float64)
    if W.shape != (N, D):
        raise ValueError(f"matrix shape {W.shape} != {(N, D)}")
    Y = W.reshape(n1, n2, n3, d1, d2, d3).transpose(0, 3, 1, 4, 2, 5)      # (i1,j1,i2,j2,i3,j3)
    dropped = []
    # first core: rows (i1, j1)
    U, S, Vt = np.linalg.svd(Y.reshape(n1 * d1, -1), full_matrices=False)
    k1 = min(r1, S.size)
    dropped.append(S[k1:].copy())
    G1 = np.zeros((n1, d1, r1))
    G1[:, :, :k1] = U[:, :k1].reshape(n1, d1, k1)
    Y = np.zeros((r1, n2 * d2 * n3 * d3))
    Y[:k1] = S[:k1, None] * Vt[:k1]
    # second core: rows (incoming rank, i2, j2)
    U, S, Vt = np.linalg.svd(Y.reshape(r1 * n2 * d2, n3 * d3), full_matrices=False)
    k2 = min(r2, S.size)
    dropped.append(S[k2:].copy())
    G2 = np.zeros((r1, n2, d2, r2))
    G2[..., :k2] = U[:, :k2].reshape(r1, n2, d2, k2)
    G3 = np.zeros((r2, n3, d3))
    G3[:k2] = (S[:k2, None] * Vt[:k2]).reshape(k2, n3, d3)
    g1 = np.ascontiguousarray(G1, dtype=np.float32)
    g2 = np.ascontiguousarray(G2.transpose(1, 0, 2, 3), dtype=np.float32)
    g3 = np.ascontiguousarray(G3.transpose(1, 0, 2), dtype=np.float32)
    if return_info:
        return (g1, g2, g3), {"matrix": W, "dropped": dropped}
    return g1, g2, g3
