"""Pins for the CPU oracle: every check here is fixed by the paper or by mathematics, none by the
oracle's own formulas.  A dropped term, a wrong sign or index, or a transposed operand anywhere in
oracle/tt_emb_oracle.c fails at least one of them.

  index split      the paper's worked example (48 nodes, id 46), the 10x10x10 sharing pattern,
                   round trips                                        [Section 3; Section 4.2]
  forward          element-by-element dense reconstruction from Eq. "tt-embedding" (different loop
                   structure: scalar triple product per table entry), the Kronecker special case
                   at ranks (1,1,1,1) against numpy.kron, multilinearity, the rank bound on rows
                   that share an (i1,i2) prefix                       [Section 3; Section 4.2]
  sizes            parameter counts and memory reductions of Table "ogb-dim-tt"
  backward         central finite differences of L in fp64 (exact here, because L is affine in
                   every single core entry), Euler's identity <dGk, Gk> = L for each core
  update           lr = 0, untouched slices, G_new - G_old = -lr*dG, affinity in lr
"""
import itertools
import os

import numpy as np
import pytest

from oracle import tt_oracle as ora
from oracle.tt_oracle import Shape
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_cores(shape, rng, std=1.0):
    return tuple((rng.standard_normal(cs) * std).astype(np.float32) for cs in shape.core_shapes())


def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


# ----------------------------------------------------------------------------- index split

def test_worked_index_example_and_its_factorisation():
    (nodes, node_id, i1, i2, i3), = [[int(x) for x in r] for r in _golden_rows("index_example.txt")]
    # enumerate every ordered factorisation of 48 into three factors; exactly one reproduces the
    # printed coordinate, so the example pins both the formula and the (unprinted) factors
    hits = []
    for m1, m2 in itertools.product(range(1, nodes + 1), repeat=2):
        if nodes % (m1 * m2):
            continue
        m3 = nodes // (m1 * m2)
        got = ora.decompose(Shape((m1, m2, m3), (1, 1, 1), (1, 1)), node_id)
        if got == (i1, i2, i3):
            hits.append((m1, m2, m3))
    assert hits == [(3, 4, 4)]


def test_sharing_pattern_of_the_1000_node_figure():
    # Fig. "node-index": 10x10x10; ten consecutive ids share (i1,i2), a hundred share i1
    s = Shape((10, 10, 10), (2, 2, 2), (4, 4))
    coords = [ora.decompose(s, i) for i in range(1000)]
    for base in range(0, 1000, 10):
        assert len({c[:2] for c in coords[base:base + 10]}) == 1
        assert [c[2] for c in coords[base:base + 10]] == list(range(10))
    for base in range(0, 1000, 100):
        assert len({c[0] for c in coords[base:base + 100]}) == 1
    assert len({c[:2] for c in coords}) == 100


@pytest.mark.parametrize("n", [(3, 4, 4), (10, 10, 10), (7, 3, 5), (480, 480, 482)])
def test_index_round_trip_and_range(n):
    s = Shape(n, (1, 1, 1), (1, 1))
    N = s.N
    probe = list(range(min(N, 300))) + [N - 1, N // 2, N - n[2], N - n[2] - 1]
    for i in probe:
        i1, i2, i3 = ora.decompose(s, i)
        assert 0 <= i1 < n[0] and 0 <= i2 < n[1] and 0 <= i3 < n[2]
        assert (i1 * n[1] + i2) * n[2] + i3 == i          # Eq. "tt-embedding": i = sum i_p prod m_q
    assert ora.decompose(s, N) is None and ora.decompose(s, -1) is None


# ----------------------------------------------------------------------------- forward

def dense_table_elementwise(shape, g1, g2, g3):
    """W(i, j) = G1(:,i1,j1,:) G2(:,i2,j2,:) G3(:,i3,j3,:) entry by entry, in fp64, from cores put
    back into the paper's index order (R_{k-1}, m_k, n_k, R_k)."""
    (n1, n2, n3), (d1, d2, d3) = shape.n, shape.d
    G1 = g1.astype(np.float64)[None]                                               # (1,n1,d1,r1)
    G2 = np.transpose(g2.astype(np.float64), (1, 0, 2, 3))                          # (r1,n2,d2,r2)
    G3 = np.transpose(g3.astype(np.float64), (1, 0, 2))[..., None]                  # (r2,n3,d3,1)
    W = np.zeros((shape.N, shape.D))
    for i1 in range(n1):
        for i2 in range(n2):
            for i3 in range(n3):
                i = (i1 * n2 + i2) * n3 + i3
                for j1 in range(d1):
                    row = G1[:, i1, j1, :]                      # 1 x r1
                    for j2 in range(d2):
                        mat = G2[:, i2, j2, :]                  # r1 x r2
                        for j3 in range(d3):
                            col = G3[:, i3, j3, :]              # r2 x 1
                            j = (j1 * d2 + j2) * d3 + j3
                            W[i, j] = (row @ mat @ col)[0, 0]
    return W


@pytest.mark.parametrize("n,d,r", [((3, 4, 4), (2, 3, 2), (3, 5)), ((5, 2, 3), (1, 2, 4), (2, 2)),
                                   ((4, 4, 4), (2, 2, 2), (4, 4))])
def test_forward_equals_dense_table_small(n, d, r):
    s = Shape(n, d, r)
    rng = np.random.default_rng(1)
    g = _rand_cores(s, rng)
    W = dense_table_elementwise(s, *g)
    ids = rng.permutation(s.N)
    out = ora.forward_f64(s, *g, ids)
    np.testing.assert_allclose(out, W[ids], rtol=1e-12, atol=1e-13)
    out32 = ora.forward(s, *g, ids)
    np.testing.assert_array_equal(out32, W[ids].astype(np.float32))


def test_forward_equals_dense_table_config1_in_full():
    # the tiny benchmark configuration, all 1000 x 8 entries
    s = Shape((10, 10, 10), (2, 2, 2), (4, 4))
    rng = np.random.default_rng(2)
    g = _rand_cores(s, rng, 0.1)
    W = dense_table_elementwise(s, *g)
    out = ora.forward_f64(s, *g, np.arange(s.N))
    np.testing.assert_allclose(out, W, rtol=1e-12, atol=1e-15)


def test_kronecker_special_case():
    # ranks (1,1,1,1): W = G1 (x) G2 (x) G3 with Gk the n_k x d_k matrices
    s = Shape((4, 3, 5), (2, 3, 2), (1, 1))
    rng = np.random.default_rng(3)
    g1, g2, g3 = _rand_cores(s, rng)
    K = np.kron(np.kron(g1[:, :, 0].astype(np.float64), g2[:, 0, :, 0].astype(np.float64)),
                g3[:, 0, :].astype(np.float64))
    out = ora.forward_f64(s, g1, g2, g3, np.arange(s.N))
    np.testing.assert_allclose(out, K, rtol=1e-13, atol=0)


def test_forward_is_multilinear_in_the_cores():
    s = Shape((3, 4, 4), (2, 2, 3), (3, 2))
    rng = np.random.default_rng(4)
    g1, g2, g3 = _rand_cores(s, rng)
    ids = np.arange(s.N)
    base = ora.forward_f64(s, g1, g2, g3, ids)
    # powers of two scale fp32 inputs exactly
    np.testing.assert_allclose(ora.forward_f64(s, g1, g2 * np.float32(4), g3, ids), 4 * base, rtol=1e-14)
    np.testing.assert_allclose(ora.forward_f64(s, g1 * np.float32(.5), g2, g3 * np.float32(8), ids),
                               4 * base, rtol=1e-14)
    h1 = _rand_cores(s, rng)[0]
    summed = ora.forward_f64(s, g1, g2, g3, ids) + ora.forward_f64(s, h1, g2, g3, ids)
    both = ora.forward_f64(s, (g1.astype(np.float64) + h1).astype(np.float32), g2, g3, ids)
    np.testing.assert_allclose(both, summed, rtol=1e-5, atol=1e-6)   # g1+h1 is rounded to fp32


def test_rows_sharing_a_prefix_have_rank_at_most_r2():
    # Section 4.2: ids in [i - i3, i + m3 - i3) are one fixed (d1 d2 x r2) matrix times G3[i3]
    s = Shape((3, 3, 9), (2, 3, 4), (3, 2))
    rng = np.random.default_rng(5)
    g = _rand_cores(s, rng)
    out = ora.forward_f64(s, *g, np.arange(s.N))
    for q in range(s.n[0] * s.n[1]):
        block = out[q * s.n[2]:(q + 1) * s.n[2]]                      # n3 rows, D columns
        stacked = block.reshape(s.n[2], s.d[0] * s.d[1], s.d[2])
        stacked = np.transpose(stacked, (1, 0, 2)).reshape(s.d[0] * s.d[1], -1)
        sv = np.linalg.svd(stacked, compute_uv=False)
        assert (sv > 1e-10 * sv[0]).sum() <= s.r[1]


def test_duplicate_and_out_of_range_ids():
    s = Shape((3, 4, 4), (2, 2, 2), (2, 3))
    rng = np.random.default_rng(6)
    g = _rand_cores(s, rng)
    ids = np.array([5, 5, 47, -1, 48, 0, 5], dtype=np.int64)
    out = ora.forward(s, *g, ids)
    np.testing.assert_array_equal(out[0], out[1])
    np.testing.assert_array_equal(out[0], out[6])
    assert not out[3].any() and not out[4].any() and out[2].any()


def test_orthogonal_core_initialisation_gives_orthogonal_table():
    # Algorithm 2 and Claim 1: cores with semi-orthogonal unfoldings make W^T W a multiple of I.
    # This pins the forward over ALL ids of a table without any reference implementation.
    import workloads as wl
    for n, d, r in [((6, 5, 7), (2, 2, 3), (3, 2)), ((4, 8, 12), (2, 2, 2), (4, 4))]:
        s = Shape(n, d, r)
        g = wl.make_orthogonal_cores(n, d, r, seed=12)
        W = ora.forward_f64(s, *g, np.arange(s.N))
        gram = W.T @ W
        alpha = np.trace(gram) / s.D
        assert alpha > 0.5
        np.testing.assert_allclose(gram, alpha * np.eye(s.D), atol=1e-5 * alpha)
    with pytest.raises(ValueError):
        wl.make_orthogonal_cores((10, 10, 4), (2, 2, 5), (4, 4), seed=1)   # 5*4 > 4*1 vectors


# ----------------------------------------------------------------------------- sizes

def test_parameter_counts_and_memory_reduction_table():
    for row in _golden_rows("param_counts.txt"):
        name, nodes, dim = row[0], int(row[1]), int(row[2])
        m1, n1, m2, n2, m3, n3 = [int(x) for x in row[3:9]]
        params = [int(x) for x in row[9:12]]
        reductions = [int(x) for x in row[12:15]]
        assert n1 * n2 * n3 == dim and m1 * m2 * m3 >= nodes
        for R, p_ref, red_ref in zip((16, 32, 64), params, reductions):
            p = ora.param_count(Shape((m1, m2, m3), (n1, n2, n3), (R, R)))
            assert p == p_ref, (name, R)
            # the products row of the printed table is consistent with width 128, not its listed
            # 100 (2,449,029*128/198,400 = 1580); the other two rows use their listed width
            width = 128 if name == "ogbn-products" else dim
            assert abs(nodes * width / p - red_ref) < 1.0, (name, R)
    # unequal inner ranks: sum_k R_{k-1} m_k n_k R_k written out
    assert ora.param_count(Shape((3, 4, 5), (2, 3, 2), (3, 5))) == 1 * 3 * 2 * 3 + 3 * 4 * 3 * 5 + 5 * 5 * 2 * 1
    # "81,362x" for papers100M at rank 8 (Section 5)
    p8 = ora.param_count(Shape((480, 500, 500), (8, 4, 4), (8, 8)))
    assert abs(111059956 * 128 / p8 - 81362) < 1.0


# ----------------------------------------------------------------------------- backward

def _loss(shape, g, ids, grad):
    return float((ora.forward_f64(shape, *g, ids) * grad.astype(np.float64)).sum())


@pytest.mark.parametrize("n,d,r", [((3, 4, 4), (2, 3, 2), (3, 5)), ((10, 10, 10), (2, 2, 2), (4, 4))])
def test_gradients_against_central_differences(n, d, r):
    s = Shape(n, d, r)
    rng = np.random.default_rng(7)
    g = list(_rand_cores(s, rng, 0.5))
    # duplicates, shared prefixes, shared i3, and ids that are never drawn
    ids = np.concatenate([rng.integers(0, s.N, 40), [7, 7, 7, 8, 9, 7 + s.n[2]], [-3, s.N]])
    grad = rng.standard_normal((ids.size, s.D)).astype(np.float32)
    dg = ora.grads(s, *g, ids, grad)
    h = np.float32(0.25)                       # exactly representable; L is affine in each entry
    for k in range(3):
        flat = g[k].reshape(-1)
        num = np.zeros(flat.size)
        for e in range(flat.size):
            keep = flat[e]
            flat[e] = keep + h
            xp = float(flat[e])                # the fp32 value actually stored
            up = _loss(s, g, ids, grad)
            flat[e] = keep - h
            xm = float(flat[e])
            dn = _loss(s, g, ids, grad)
            flat[e] = keep
            num[e] = (up - dn) / (xp - xm)
        scale = np.abs(num).max()
        np.testing.assert_allclose(dg[k].reshape(-1), num, rtol=0, atol=1e-9 * scale)


@pytest.mark.parametrize("cfg", [1, 2])
def test_euler_identity_on_benchmark_shapes(cfg):
    # L is linear in each core separately, hence <dGk, Gk> = L for k = 1, 2, 3
    import workloads as wl
    w = wl.CONFIGS[cfg]
    s = Shape(w.n, w.d, w.r)
    B = min(w.batch, 4000)
    g = wl.make_cores(w, cfg)
    ids = wl.make_ids(w, cfg, B)
    grad = wl.make_grads(w, cfg, B)
    L = _loss(s, g, ids, grad)
    dg = ora.grads(s, *g, ids, grad)
    for k in range(3):
        assert abs(float((dg[k] * g[k].astype(np.float64)).sum()) - L) <= 1e-10 * max(1.0, abs(L))


def test_gradient_of_duplicates_adds():
    s = Shape((3, 4, 4), (2, 2, 2), (2, 3))
    rng = np.random.default_rng(8)
    g = _rand_cores(s, rng)
    ids = np.array([11, 11, 11], dtype=np.int64)
    grad = rng.standard_normal((3, s.D)).astype(np.float32)
    a = ora.grads(s, *g, ids, grad)
    b = ora.grads(s, *g, ids[:1], grad.astype(np.float64).sum(0, keepdims=True).astype(np.float32))
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-6, atol=1e-7)   # the summed grad is rounded to fp32


# ----------------------------------------------------------------------------- update

def test_update_properties():
    s = Shape((5, 4, 6), (2, 2, 3), (3, 4))
    rng = np.random.default_rng(9)
    g = _rand_cores(s, rng)
    ids = np.array([0, 1, 1, 30, 31, 7, 7, 7], dtype=np.int64)        # touches i1 in {0,1} only
    grad = rng.standard_normal((ids.size, s.D)).astype(np.float32)
    lr = np.float32(0.01)

    same = ora.backward_update(s, *g, ids, grad, 0.0)
    for a, b in zip(same, g):
        np.testing.assert_array_equal(a, b)                           # lr = 0: bit-identical

    new = ora.backward_update(s, *g, ids, grad, float(lr))
    dg = ora.grads(s, *g, ids, grad)
    coords = [ora.decompose(s, int(i)) for i in ids]
    for k in range(3):
        touched = sorted({c[k] for c in coords})
        untouched = [x for x in range(s.n[k]) if x not in touched]
        np.testing.assert_array_equal(new[k][untouched], g[k][untouched])
        assert all(np.any(new[k][t] != g[k][t]) for t in touched)
        want = (g[k].astype(np.float64) - float(lr) * dg[k]).astype(np.float32)
        np.testing.assert_array_equal(new[k], want)                   # G_new = G_old - lr*dG

    twice = ora.backward_update(s, *g, ids, grad, float(np.float32(2) * lr))
    for k in range(3):
        d1 = new[k].astype(np.float64) - g[k]
        d2 = twice[k].astype(np.float64) - g[k]
        np.testing.assert_allclose(d2, 2 * d1, rtol=0, atol=4e-7 * np.abs(g[k]).max())


def test_f32_build_agrees_with_f64_build():
    # the timed build is the same loops with float accumulators
    import workloads as wl
    w = wl.CONFIGS[1]
    s = Shape(w.n, w.d, w.r)
    g = wl.make_cores(w, 1)
    ids = wl.make_ids(w, 1)
    grad = wl.make_grads(w, 1)
    np.testing.assert_allclose(ora.forward(s, *g, ids, tag="f32"), ora.forward(s, *g, ids),
                               rtol=1e-5, atol=1e-7)
    a = ora.backward_update(s, *g, ids, grad, w.lr, tag="f32")
    b = ora.backward_update(s, *g, ids, grad, w.lr)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-5, atol=1e-7)


def test_adagrad_first_step_moves_every_touched_entry_by_lr():
    """Textbook special case that pins the Adagrad rule of the oracle without re-typing it: from a
    zero state and with eps -> 0 the first step is  -lr * dG / |dG| = -lr * sign(dG)  wherever the
    gradient is nonzero, and nothing moves elsewhere; the state becomes dG^2."""
    s = Shape((5, 4, 6), (2, 3, 2), (3, 2))
    rng = np.random.default_rng(5)
    cores = [rng.standard_normal(cs).astype(np.float32) for cs in s.core_shapes()]
    ids = np.array([0, 1, 7, 30, 31, 31], dtype=np.int64)    # leaves slices of every core untouched
    grad = rng.standard_normal((ids.size, s.D)).astype(np.float32)
    dg = ora.grads(s, *cores, ids, grad)                     # pinned by the finite-difference tests
    zero = [np.zeros_like(c) for c in cores]
    lr = 0.125
    new, state = ora.adagrad_update(s, *cores, zero, ids, grad, lr, 1e-30)
    for G, Gn, S, d in zip(cores, new, state, dg):
        moved = d != 0
        assert moved.any() and (~moved).any()
        np.testing.assert_array_equal(Gn[~moved], G[~moved])
        np.testing.assert_allclose(Gn[moved], (G.astype(np.float64) - lr * np.sign(d))[moved], rtol=2e-7)
        np.testing.assert_allclose(S, (d * d).astype(np.float32), rtol=1e-6)
    # a second step from that state with the same gradient would move by lr/sqrt(2): the state adds up
    new2, _ = ora.adagrad_update(s, *cores, state, ids, grad, lr, 1e-30)
    for G, Gn, d in zip(cores, new2, dg):
        moved = np.abs(d) > 1e-3
        np.testing.assert_allclose((G.astype(np.float64) - Gn)[moved],
                                   (lr / np.sqrt(2.0) * np.sign(d))[moved], rtol=1e-5)


def test_adam_first_step_constant_gradient_and_untouched_slices():
    """Pins of the oracle's Adam rule that do not re-type it.  (a) From zero moments the first step
    is -lr * dG / (|dG| + eps): the bias corrections cancel the (1 - beta) factors, so with
    eps -> 0 every entry with a nonzero gradient moves by exactly lr against the sign of its
    gradient, whatever beta1 and beta2 are.  (b) With beta1 = beta2 = 0 there is no memory and every
    step has that form.  (c) Slices no id touches keep core and moments bit for bit, even when
    their moments are nonzero.  (d) Feeding the same gradient again: the corrected moments of a
    constant gradient are that gradient and its square at every step (closed form of the two
    geometric sums), so the second step moves by lr * sign(dG) again."""
    s = Shape((5, 4, 6), (2, 3, 2), (3, 2))
    rng = np.random.default_rng(11)
    cores = [rng.standard_normal(cs).astype(np.float32) for cs in s.core_shapes()]
    ids = np.array([0, 1, 7, 30, 31, 31], dtype=np.int64)
    grad = rng.standard_normal((ids.size, s.D)).astype(np.float32)
    dg = ora.grads(s, *cores, ids, grad)
    masks = ora.touched_slices(s, ids)
    # by hand (n2*n3 = 24): ids 0,1,7 -> (0,0,0),(0,0,1),(0,1,1); 30,31 -> (1,1,0),(1,1,1)
    for mk in masks:
        assert list(np.nonzero(mk)[0]) == [0, 1]
    lr = 0.125
    zero = [np.zeros_like(c) for c in cores]
    for b1, b2 in ((0.9, 0.999), (0.5, 0.25), (0.0, 0.0)):
        new, m, v = ora.adam_update(s, *cores, zero, zero, 1, ids, grad, lr, b1, b2, 1e-30)
        for G, Gn, d, mk in zip(cores, new, dg, masks):
            moved = d != 0
            assert moved.any() and (~moved).any()
            np.testing.assert_array_equal(Gn[~moved], G[~moved])
            np.testing.assert_allclose(Gn[moved], (G.astype(np.float64) - lr * np.sign(d))[moved],
                                       rtol=2e-7)
        if b1 == 0.0:   # (b) any step number, any moments coming in: same step
            junk = [np.abs(rng.standard_normal(c.shape)).astype(np.float32) for c in cores]
            again, _, _ = ora.adam_update(s, *cores, junk, junk, 7, ids, grad, lr, 0.0, 0.0, 1e-30)
            for Gn, Ga, mk in zip(new, again, masks):
                np.testing.assert_array_equal(Ga[mk], Gn[mk])
    # (c) untouched slices
    m0 = [rng.standard_normal(c.shape).astype(np.float32) for c in cores]
    v0 = [np.abs(rng.standard_normal(c.shape)).astype(np.float32) for c in cores]
    new, m1, v1 = ora.adam_update(s, *cores, m0, v0, 3, ids, grad, lr, 0.9, 0.999, 1e-8)
    for G, Gn, a, an, b, bn, mk in zip(cores, new, m0, m1, v0, v1, masks):
        assert (~mk).any()
        np.testing.assert_array_equal(Gn[~mk], G[~mk])
        np.testing.assert_array_equal(an[~mk], a[~mk])
        np.testing.assert_array_equal(bn[~mk], b[~mk])
        assert not np.array_equal(an[mk], a[mk])
    # (d) constant gradient: the loss is linear in each core, so dG3 does not depend on G3; keep
    # G1, G2 fixed and step G3 twice with the moments carried along
    b1, b2 = 0.9, 0.999
    st1, m, v = ora.adam_update(s, *cores, zero, zero, 1, ids, grad, lr, b1, b2, 1e-30)
    mixed = (cores[0], cores[1], st1[2])
    st2, _, _ = ora.adam_update(s, *mixed, m, v, 2, ids, grad, lr, b1, b2, 1e-30)
    d3 = dg[2]
    moved = np.abs(d3) > 1e-3
    np.testing.assert_allclose((st1[2].astype(np.float64) - st2[2])[moved], (lr * np.sign(d3))[moved],
                               rtol=1e-5)



def test_adam_two_steps_with_a_changing_gradient():
    """Pins the decay rates to their moments.  Every pin above feeds a constant gradient, where the
    bias corrections cancel the decay weights and a swap of beta1 and beta2 between the two moments
    would go unseen.  Here the gradient changes between the steps by a known factor: the loss is
    linear in each core, so dG3 does not depend on G3, and with G1, G2 held fixed a batch whose row
    gradients are four times larger (exact in fp32) gives exactly 4*dG3.  For one entry with first
    gradient d, worked by hand from the textbook recursion (zero moments, eps -> 0):
        step 1:  m = (1-b1) d,             v = (1-b2) d^2
        step 2:  m = b1 (1-b1) d + (1-b1) 4d = (1-b1)(b1+4) d
                 v = b2 (1-b2) d^2 + (1-b2) 16 d^2 = (1-b2)(b2+16) d^2
                 m / (1-b1^2) = (b1+4)/(1+b1) d,   v / (1-b2^2) = (b2+16)/(1+b2) d^2
                 second move = lr * sign(d) * [(b1+4)/(1+b1)] / sqrt[(b2+16)/(1+b2)]
    With b1 = 1/2, b2 = 1/4:  (4.5/1.5) / sqrt(16.25/1.25) = 3/sqrt(13) = 0.832050...; the swapped
    assignment would give (4.25/1.25) / sqrt(16.5/1.5) = 1.025141..."""
    s = Shape((5, 4, 6), (2, 3, 2), (3, 2))
    rng = np.random.default_rng(23)
    cores = [rng.standard_normal(cs).astype(np.float32) for cs in s.core_shapes()]
    ids = np.array([0, 1, 7, 30, 31, 31], dtype=np.int64)
    grad = rng.standard_normal((ids.size, s.D)).astype(np.float32)
    d3 = ora.grads(s, *cores, ids, grad)[2]
    np.testing.assert_allclose(ora.grads(s, *cores, ids, 4 * grad)[2], 4 * d3, rtol=1e-14)
    lr, b1, b2 = 0.125, 0.5, 0.25
    zero = [np.zeros_like(c) for c in cores]
    st1, m, v = ora.adam_update(s, *cores, zero, zero, 1, ids, grad, lr, b1, b2, 1e-30)
    np.testing.assert_allclose(m[2], 0.5 * d3, rtol=1e-6)            # (1-b1) d
    np.testing.assert_allclose(v[2], 0.75 * d3 * d3, rtol=1e-6)      # (1-b2) d^2
    mixed = (cores[0], cores[1], st1[2])
    st2, m2, v2 = ora.adam_update(s, *mixed, m, v, 2, ids, 4 * grad, lr, b1, b2, 1e-30)
    np.testing.assert_allclose(m2[2], 0.5 * 4.5 * d3, rtol=1e-6)     # (1-b1)(b1+4) d
    np.testing.assert_allclose(v2[2], 0.75 * 16.25 * d3 * d3, rtol=1e-6)
    factor = 3.0 / np.sqrt(13.0)
    moved = np.abs(d3) > 1e-3
    assert moved.sum() >= 8
    np.testing.assert_allclose((st1[2].astype(np.float64) - st2[2])[moved],
                               (lr * factor * np.sign(d3))[moved], rtol=1e-5)


def test_eps_sits_outside_the_square_root():
    """Pins the place of eps in both adaptive rules with an eps as large as the gradients (all other
    pins run at eps = 1e-30, where sqrt(S) + eps and sqrt(S + eps) cannot be told apart).  From a
    zero state the first step has S = dG^2 (Adagrad) and bias-corrected moments dG and dG^2 (Adam),
    so both rules move an entry by  lr * d / (|d| + eps);  the other placement would give
    lr * d / sqrt(d^2 + eps), which at eps = 1/2 differs in the first digit."""
    s = Shape((5, 4, 6), (2, 3, 2), (3, 2))
    rng = np.random.default_rng(29)
    cores = [rng.standard_normal(cs).astype(np.float32) for cs in s.core_shapes()]
    ids = np.array([0, 1, 7, 30, 31, 31], dtype=np.int64)
    grad = rng.standard_normal((ids.size, s.D)).astype(np.float32)
    dg = ora.grads(s, *cores, ids, grad)
    zero = [np.zeros_like(c) for c in cores]
    lr, eps = 0.125, 0.5
    ada, _ = ora.adagrad_update(s, *cores, zero, ids, grad, lr, eps)
    adam, _, _ = ora.adam_update(s, *cores, zero, zero, 1, ids, grad, lr, 0.9, 0.999, eps)
    for G, Ga, Gm, d in zip(cores, ada, adam, dg):
        want = lr * d / (np.abs(d) + eps)
        other = lr * d / np.sqrt(d * d + eps)
        moved = np.abs(d) > 1e-2
        assert moved.sum() >= 8 and np.abs(want - other)[moved].min() > 1e-4
        for got in (Ga, Gm):
            np.testing.assert_allclose((G.astype(np.float64) - got)[moved], want[moved], rtol=2e-5,
                                       atol=2e-7)


def test_ttsvd_initialisation_reproduces_its_matrix():
    """Algorithm 1 of the paper (TT-SVD of a matrix into the TT-matrix format).  With ranks as large
    as the unfoldings' ranks the decomposition is exact, so the oracle's forward over every id must
    give back the matrix that was decomposed - for the default input, a random matrix with
    orthonormal columns, that is W^T W = I, the property the paper wants from this initialisation.
    With smaller ranks the result is an approximation whose Frobenius error TT-SVD bounds by the
    discarded singular values (the root of their summed squares over both steps)."""
    n, d = (6, 5, 7), (2, 2, 3)
    N = 6 * 5 * 7
    # ranks of the unfoldings: at most n1*d1 = 12 rows in the first, at most n3*d3 = 21 columns in
    # the second
    cores, info = wl.make_ttsvd_cores(n, d, (12, 21), seed=8, return_info=True)
    s = Shape(n, d, (12, 21))
    for g, cs in zip(cores, s.core_shapes()):
        assert g.shape == cs and g.dtype == np.float32
    assert all(t.size == 0 or np.abs(t).max() < 1e-12 for t in info["dropped"])
    W = ora.forward_f64(s, *cores, np.arange(N, dtype=np.int64))
    np.testing.assert_allclose(W, info["matrix"], atol=5e-6)
    np.testing.assert_allclose(W.T @ W, np.eye(s.D), atol=2e-5)
    # an arbitrary matrix, truncated ranks: the error bound of the decomposition
    rng = np.random.default_rng(80)
    A = rng.standard_normal((N, 12))
    cores, info = wl.make_ttsvd_cores(n, d, (5, 6), seed=0, matrix=A, return_info=True)
    s = Shape(n, d, (5, 6))
    W = ora.forward_f64(s, *cores, np.arange(N, dtype=np.int64))
    err = np.linalg.norm(W - A)
    bound = np.sqrt(sum(float((t * t).sum()) for t in info["dropped"]))
    assert 0.05 * bound < err <= bound * (1 + 1e-5) + 1e-4
    # the first core's unfolding has orthonormal columns (left singular vectors)
    U1 = cores[0].reshape(6 * 2, 5).astype(np.float64)
    np.testing.assert_allclose(U1.T @ U1, np.eye(5), atol=1e-5)
