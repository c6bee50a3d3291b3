"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Tolerances (fp32 path, fp64 oracle), written out here:
  rows   max over rows b of ||gpu_b - ora_b||_inf / ||ora_b||_inf          <= 1e-5
  cores  per core ||gpu - ora||_inf / ||ora||_inf                          <= 1e-4
  step   per core, with dG = (G_old - G_new)/lr recovered from both sides,
         ||dG_gpu - dG_ora||_inf / ||dG_ora||_inf                          <= 1e-4
The third line is stricter than the second (a step is lr = 0.01 times a gradient, so a wrong
gradient on a cold slice would hide inside the second).  Integer results (U, Q, out-of-range
count) are compared exactly.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import tt_oracle as ora
from oracle.tt_oracle import Shape

pytestmark = pytest.mark.gpu

ROW_TOL = 1e-5
CORE_TOL = 1e-4
STEP_TOL = 1e-4


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def row_error(gpu, ref):
    """max_b ||gpu_b - ref_b||_inf / ||ref_b||_inf (rows whose reference is all zero must match exactly)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.abs(gpu - ref).max(axis=1)
    den = np.abs(ref).max(axis=1)
    zero = den == 0
    assert not num[zero].any(), "a row that must be zero is not"
    return float((num[~zero] / den[~zero]).max()) if (~zero).any() else 0.0


def core_error(gpu, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(gpu, dtype=np.float64) - ref).max() / np.abs(ref).max())


def run_gpu(n, d, r, cores, ids, grad, lr, max_batch=None, flags=0):
    """One forward + backward_update through the C ABI; returns rows, new cores, stats."""
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    B = int(ids.size)
    emb = TTEmbedding(n, d, r, max_batch or max(B, 1), cores, flags=flags)
    t_ids = torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int64)).cuda()
    out = emb.forward(t_ids)
    stats = emb.stats(check=False)
    t_grad = torch.from_numpy(np.ascontiguousarray(grad, dtype=np.float32)).cuda()
    emb.backward_update(t_grad, lr)
    torch.cuda.synchronize()
    emb.stats(check=False)  # raises on an internal-error flag
    res = out.cpu().numpy(), [c.cpu().numpy() for c in emb.cores], stats
    emb.close()
    return res


def check_against_oracle(n, d, r, cores, ids, grad, lr, **kw):
    s = Shape(tuple(n), tuple(d), tuple(r))
    out, new, stats = run_gpu(n, d, r, cores, ids, grad, lr, **kw)
    ref_out = ora.forward(s, *cores, ids)
    assert row_error(out, ref_out) <= ROW_TOL
    ref_new = ora.backward_update(s, *cores, ids, grad, lr)
    ok = ids[(ids >= 0) & (ids < s.N)]
    assert stats["U"] == np.unique(ok).size
    assert stats["Q"] == np.unique(ok // n[2]).size
    assert stats["out_of_range"] == ids.size - ok.size
    for k in range(3):
        if ok.size == 0:
            np.testing.assert_array_equal(new[k], cores[k])
            continue
        assert core_error(new[k], ref_new[k]) <= CORE_TOL, f"core {k + 1}"
        step_gpu = (cores[k].astype(np.float64) - new[k]) / lr
        step_ref = (cores[k].astype(np.float64) - ref_new[k]) / lr
        # the recovered step carries the rounding of G itself: allow 2 ulp of |G| / lr on top
        slack = 2 * np.finfo(np.float32).eps * np.abs(cores[k]).max() / lr
        err = np.abs(step_gpu - step_ref).max()
        assert err <= STEP_TOL * np.abs(step_ref).max() + slack, f"step of core {k + 1}"
        # slices no id touches are not written at all
        touched = np.zeros(n[k], dtype=bool)
        coord = [ok // (n[1] * n[2]), (ok // n[2]) % n[1], ok % n[2]][k]
        touched[coord] = True
        np.testing.assert_array_equal(new[k][~touched], cores[k][~touched])
    return out, new, stats


def _workload(cfg, seed=None, batch=None):
    w = wl.CONFIGS[cfg]
    seed = cfg if seed is None else seed
    return w, wl.make_cores(w, seed), wl.make_ids(w, seed, batch), wl.make_grads(w, seed, batch)


# ----------------------------------------------------------------------------- small, in full

def test_config1_tiny_in_full():
    w, cores, ids, grad = _workload(1)
    check_against_oracle(w.n, w.d, w.r, cores, ids, grad, w.lr)


@pytest.mark.parametrize("n,d,r,B", [
    ((3, 4, 4), (2, 3, 2), (3, 5), 200),       # odd factors, r1 != r2, every id many times
    ((7, 5, 9), (1, 2, 5), (2, 7), 1000),
    ((5, 300, 6), (3, 1, 2), (6, 1), 5000),    # wide middle factor, rank-1 tail
    ((40, 33, 70), (2, 2, 3), (8, 8), 4097),   # one item past a 4096 sort block
    ((6, 9, 11), (8, 8, 2), (4, 64), 1500),    # staged row kernel with three wavefronts per block
    ((5, 7, 6), (8, 8, 1), (2, 260), 700),     # too large for the staged row and G3-gradient kernels
    ((9, 8, 7), (3, 7, 5), (5, 3), 2500),      # several 64-wide tiles with ragged edges (D = 105)
    ((4, 6, 5), (20, 1, 9), (70, 2), 900),     # stacked prefixes exceed one tile (16 * d1 = 320 rows)
])
def test_generic_shapes(n, d, r, B):
    rng = np.random.default_rng(B)
    s = Shape(n, d, r)
    cores = tuple((rng.standard_normal(cs) * 0.5).astype(np.float32) for cs in s.core_shapes())
    ids = rng.integers(0, s.N, size=B, dtype=np.int64)
    grad = rng.standard_normal((B, s.D)).astype(np.float32)
    check_against_oracle(n, d, r, cores, ids, grad, 0.01)


@pytest.mark.parametrize("flags", [0, 2])          # 2 = TT_EMB_FLAG_GENERIC_KERNELS
@pytest.mark.parametrize("R,d3", [(8, 4), (8, 8), (16, 4), (16, 8), (32, 8), (64, 8), (32, 4), (64, 4),
                                  (128, 4), (128, 8)])
@pytest.mark.parametrize("n,B", [((9, 21, 13), 6000), ((40, 50, 60), 5000), ((3, 2, 700), 3000)])
def test_matrix_core_shape_family(n, B, R, d3, flags):
    # d1 = d2 = 4 with equal ranks: the shapes that have matrix-core kernels; dense sharing
    # (small table), sparse sharing (large table) and long runs of ids under one prefix
    rng = np.random.default_rng(R * d3 + B)
    d, r = (4, 4, d3), (R, R)
    s = Shape(n, d, r)
    cores = tuple((rng.standard_normal(cs) / np.sqrt(R)).astype(np.float32) for cs in s.core_shapes())
    ids = rng.integers(0, s.N, size=B, dtype=np.int64)
    ids[: B // 10] = ids[0]
    grad = rng.standard_normal((B, s.D)).astype(np.float32)
    check_against_oracle(n, d, r, cores, ids, grad, 0.01, flags=flags)


@pytest.mark.parametrize("n,R,B", [((48, 50, 60), 32, 5000), ((70, 60, 9), 16, 6000)])
def test_prefix_ordered_chunk_schedule(n, R, B):
    # enough prefixes that the cached products can exceed one L2 (4 MiB): the G3-gradient chunks
    # are then walked in prefix order, one eighth of the order per XCD
    rng = np.random.default_rng(R + B)
    d, r = (4, 4, 8), (R, R)
    s = Shape(n, d, r)
    assert min(B, n[0] * n[1]) * 16 * R * 4 > 4 << 20
    cores = tuple((rng.standard_normal(cs) / np.sqrt(R)).astype(np.float32) for cs in s.core_shapes())
    ids = rng.integers(0, s.N, size=B, dtype=np.int64)
    ids[: B // 8] = ids[1]
    grad = rng.standard_normal((B, s.D)).astype(np.float32)
    check_against_oracle(n, d, r, cores, ids, grad, 0.01)


@pytest.mark.parametrize("B", [1, 2, 31, 32, 33, 63, 64, 65, 1023, 1025, 4095, 4096, 8193])
def test_ragged_batch_sizes(B):
    w, cores, _, _ = _workload(2)
    ids = wl.make_ids(w, 100 + B, B)
    grad = wl.make_grads(w, 100 + B, B)
    check_against_oracle(w.n, w.d, w.r, cores, ids, grad, w.lr, max_batch=10_000)


def test_duplicates_out_of_range_and_one_hot_id():
    w, cores, _, _ = _workload(2)
    rng = np.random.default_rng(5)
    hot = np.full(3000, 12345, dtype=np.int64)                    # one id, thousands of times
    near = 12345 + rng.integers(-40, 40, size=500)                # same and neighbouring prefixes
    bad = np.array([-1, w.N, w.N + 5, -2**40, 2**40], dtype=np.int64)
    ids = np.concatenate([hot, near, bad, rng.integers(0, w.N, 2000)]).astype(np.int64)
    rng.shuffle(ids)
    grad = rng.standard_normal((ids.size, w.D)).astype(np.float32)
    out, _, stats = check_against_oracle(w.n, w.d, w.r, cores, ids, grad, w.lr)
    assert stats["out_of_range"] == 5
    assert not out[(ids < 0) | (ids >= w.N)].any()


@pytest.mark.parametrize("flags", [0, 2])
def test_long_runs_cut_at_block_boundaries(flags):
    """Runs of one id longer than the 1024-slot unit of the gradient sums are carried as several
    pieces; the counts still name distinct ids, and pieces of one slot, runs that end exactly on a
    boundary and a run that covers whole units all add up to the oracle's gradient."""
    w, cores, _, _ = _workload(2)
    # sorted order: id 7 x 1023 | id 9 x 1 (slot 1023) | id 11 x 2049 (slots 1024..3072: two whole
    # units and one slot) | id 500 x 1023 (ends exactly at slot 4096) | id 501 x 1025 | ids above
    ids = np.concatenate([np.full(1023, 7), np.full(1, 9), np.full(2049, 11), np.full(1023, 500),
                          np.full(1025, 501), 600 + np.arange(300)]).astype(np.int64)
    rng = np.random.default_rng(21)
    rng.shuffle(ids)
    grad = rng.standard_normal((ids.size, w.D)).astype(np.float32)
    _, _, stats = check_against_oracle(w.n, w.d, w.r, cores, ids, grad, w.lr, flags=flags)
    assert stats["U"] == 305


def test_all_ids_out_of_range_and_empty_batch():
    w, cores, _, _ = _workload(1)
    ids = np.array([-5, w.N, w.N + 1], dtype=np.int64)
    grad = np.ones((3, w.D), dtype=np.float32)
    out, new, stats = run_gpu(w.n, w.d, w.r, cores, ids, grad, w.lr)
    assert not out.any() and stats == {"U": 0, "Q": 0, "out_of_range": 3}
    for a, b in zip(new, cores):
        np.testing.assert_array_equal(a, b)
    out, new, stats = run_gpu(w.n, w.d, w.r, cores, ids[:0], grad[:0], w.lr)
    assert out.shape == (0, w.D) and stats == {"U": 0, "Q": 0, "out_of_range": 0}
    for a, b in zip(new, cores):
        np.testing.assert_array_equal(a, b)


def test_config2_in_full():
    w, cores, ids, grad = _workload(2)
    _, _, stats = check_against_oracle(w.n, w.d, w.r, cores, ids, grad, w.lr)
    assert stats["Q"] == 56 * 56


# ----------------------------------------------------------------------------- the paper's own shapes

@pytest.mark.parametrize("name,n,d,R,B", [
    ("ogbn-arxiv", (55, 55, 56), (8, 4, 4), 16, 20_000),
    ("ogbn-products", (125, 140, 140), (4, 5, 5), 8, 20_000),       # D = 100, rows of 400 bytes
    ("ogbn-papers100M", (480, 500, 500), (8, 4, 4), 8, 30_000),
    ("ogbn-papers100M rank 16", (480, 500, 500), (8, 4, 4), 16, 30_000),   # slab split, d1 = 2*4
    ("ogbn-arxiv rank 32", (55, 55, 56), (8, 4, 4), 32, 20_000),
    ("d1 = 12, d3 = 8, rank 64", (20, 30, 25), (12, 4, 8), 64, 6_000),     # three slabs
    ("unequal ranks", (40, 60, 50), (4, 4, 8), (16, 32), 10_000),
])
def test_paper_table_shapes(name, n, d, R, B):
    # Table "ogb-dim-tt": the factorisations and dimension orderings the paper itself uses; they
    # run on the any-shape kernels
    rng = np.random.default_rng(len(name))
    r = R if isinstance(R, tuple) else (R, R)
    s = Shape(n, d, r)
    cores = tuple((rng.standard_normal(cs) / np.sqrt(r[0])).astype(np.float32) for cs in s.core_shapes())
    ids = rng.integers(0, s.N, size=B, dtype=np.int64)
    ids[: B // 20] = ids[0]
    ids[B // 20: B // 10] = ids[0] + rng.integers(0, 30, size=B // 10 - B // 20)   # shared prefixes
    ids = np.minimum(ids, s.N - 1)
    grad = rng.standard_normal((B, s.D)).astype(np.float32)
    check_against_oracle(n, d, r, cores, ids, grad, 0.01)


def test_orthogonal_initialisation_on_the_gpu():
    # Claim 1 of the paper, checked on the GPU forward over every id of a small table: no oracle
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    for n, d, r in [((4, 8, 128), (4, 4, 8), (16, 16)), ((6, 5, 7), (2, 2, 3), (3, 2))]:
        s = Shape(n, d, r)
        cores = wl.make_orthogonal_cores(n, d, r, seed=3)
        emb = TTEmbedding(n, d, r, s.N, cores)
        W = emb.forward(torch.arange(s.N, dtype=torch.int64, device="cuda")).double().cpu().numpy()
        emb.close()
        gram = W.T @ W
        alpha = np.trace(gram) / s.D
        np.testing.assert_allclose(gram, alpha * np.eye(s.D), atol=2e-5 * alpha)


# ----------------------------------------------------------------------------- full benchmark sizes

def _check_full(cfg, seed=None, ids=None):
    # the benchmark's launch configuration: max_batch = batch, default flags
    w, cores, gen_ids, grad = _workload(cfg, seed)
    ids = gen_ids if ids is None else ids
    out, new, stats = check_against_oracle(w.n, w.d, w.r, cores, ids, grad, w.lr)
    print(f"config {cfg}: B={ids.size} U={stats['U']} Q={stats['Q']}")
    return w, ids, stats


def test_config3_full_size_zipf_batch():
    w, ids, stats = _check_full(3)
    # the skew this workload is about: one id holds more than a tenth of the batch
    assert np.bincount(np.unique(ids, return_inverse=True)[1]).max() > 20_000


def test_config3_full_size_second_seed():
    _check_full(3, seed=103)


def test_config4_full_size_permuted_and_rank_order():
    w, ids, stats = _check_full(4)
    # secondary reading of the workload: Zipf rank = id (hot ids contiguous, fewer prefixes)
    rng = np.random.default_rng(4)
    ranks = wl.bounded_zipf_ranks(rng, w.N, w.zipf_s, w.batch)
    _, _, stats2 = _check_full(4, ids=ranks)
    assert stats2["Q"] < stats["Q"]


def test_config5_full_size_clustered_rank64():
    w, ids, stats = _check_full(5)
    assert stats["Q"] < 4000 and stats["U"] > 250_000     # few prefixes, mostly distinct ids


# ----------------------------------------------------------------------------- properties

def test_bit_reproducible_and_lr_zero():
    w, cores, ids, grad = _workload(3, batch=60_000)
    a = run_gpu(w.n, w.d, w.r, cores, ids, grad, w.lr)
    b = run_gpu(w.n, w.d, w.r, cores, ids, grad, w.lr)
    np.testing.assert_array_equal(a[0], b[0])
    for x, y in zip(a[1], b[1]):
        np.testing.assert_array_equal(x, y)
    c = run_gpu(w.n, w.d, w.r, cores, ids, grad, 0.0)
    for x, y in zip(c[1], cores):
        np.testing.assert_array_equal(x, y)


@pytest.mark.parametrize("flags", [0, 4])
def test_prepare_pipeline_matches_oracle_over_three_steps(flags):
    # flags = 4: the ids are complete in memory at every prepare (they are: synchronised uploads)
    # the next batch's index work is enqueued between forward and backward of the current one;
    # three different batches, cores carried from step to step on both sides
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    w, cores, _, _ = _workload(2)
    s = Shape(w.n, w.d, w.r)
    sizes = [7000, 2500, 9000]
    batches = [(wl.make_ids(w, 40 + k, B), wl.make_grads(w, 40 + k, B)) for k, B in enumerate(sizes)]
    batches[1][0][:400] = batches[1][0][0]                       # a hot id in the middle batch
    emb = TTEmbedding(w.n, w.d, w.r, 10_000, cores, flags=flags)
    t_ids = [torch.from_numpy(b[0]).cuda() for b in batches]
    t_grad = [torch.from_numpy(b[1]).cuda() for b in batches]
    outs = []
    for k in range(3):
        outs.append(emb.forward(t_ids[k]))
        if k + 1 < 3:
            emb.prepare(t_ids[k + 1])
        else:
            emb.prepare(t_ids[0])          # prepared but never used: must be harmless
        emb.backward_update(t_grad[k], w.lr)
    torch.cuda.synchronize()
    emb.stats()
    ref = [c.copy() for c in cores]
    for k in range(3):
        ids, grad = batches[k]
        assert row_error(outs[k].cpu().numpy(), ora.forward(s, *ref, ids)) <= ROW_TOL, f"step {k}"
        ref = list(ora.backward_update(s, *ref, ids, grad, w.lr))
    for k in range(3):
        assert core_error(emb.cores[k].cpu().numpy(), ref[k]) <= CORE_TOL
    # two batches ahead: prepare(next) is called before the forward of the current batch
    emb2 = TTEmbedding(w.n, w.d, w.r, 10_000, cores, flags=flags)
    outs2 = []
    emb2.prepare(t_ids[0])
    for k in range(3):
        if k + 1 < 3:
            emb2.prepare(t_ids[k + 1])
        outs2.append(emb2.forward(t_ids[k]))
        emb2.backward_update(t_grad[k], w.lr)
    torch.cuda.synchronize()
    emb2.stats()
    for k in range(3):
        assert torch.equal(outs2[k], outs[k]), f"step {k}"
        assert torch.equal(emb2.cores[k], emb.cores[k])
    emb2.close()
    # the batch after next prepared before every forward (three index sets: one in flight, two
    # ahead), then a fourth prepare that has to overwrite the oldest waiting batch
    emb3 = TTEmbedding(w.n, w.d, w.r, 10_000, cores, flags=flags)
    outs3 = []
    emb3.prepare(t_ids[0])
    emb3.prepare(t_ids[1])
    for k in range(3):
        if k + 2 < 3:
            emb3.prepare(t_ids[k + 2])
        outs3.append(emb3.forward(t_ids[k]))
        emb3.backward_update(t_grad[k], w.lr)
    torch.cuda.synchronize()
    for k in range(3):
        assert torch.equal(outs3[k], outs[k]), f"step {k}"
        assert torch.equal(emb3.cores[k], emb.cores[k])
    snap = [c.clone() for c in emb3.cores]
    for k in (0, 1, 2, 0):                 # one more than there are sets
        emb3.prepare(t_ids[k])
    out_x = emb3.forward(t_ids[1]).clone()  # still waiting: served from its prepared set
    emb3.backward_update(t_grad[1], w.lr)
    after_x = [c.clone() for c in emb3.cores]
    for c, b in zip(emb3.cores, snap):
        c.copy_(b)
    out_y = emb3.forward(t_ids[1]).clone()  # nothing matches any more: index work done in place
    emb3.backward_update(t_grad[1], w.lr)
    torch.cuda.synchronize()
    emb3.stats()
    assert torch.equal(out_x, out_y)
    for x, y in zip(after_x, emb3.cores):
        assert torch.equal(x, y)
    emb3.close()
    # a prepared batch that does not match the next forward is dropped, results unchanged
    base = [c.clone() for c in emb.cores]
    emb.prepare(t_ids[1])
    out_a = emb.forward(t_ids[2]).clone()
    emb.backward_update(t_grad[2], w.lr)
    after_a = [c.clone() for c in emb.cores]
    for c, b in zip(emb.cores, base):
        c.copy_(b)
    out_b = emb.forward(t_ids[2]).clone()
    emb.backward_update(t_grad[2], w.lr)
    torch.cuda.synchronize()
    assert torch.equal(out_a, out_b)
    for x, y in zip(after_a, emb.cores):
        assert torch.equal(x, y)
    emb.close()


@pytest.mark.parametrize("flags", [0, 4])
def test_prepare_with_reused_ids_buffers(flags):
    """Ten steps through two ids buffers whose contents change every step (the index sets rotate
    underneath, every set meets every buffer several times), each step against the oracle."""
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    n, d, r, B, steps = (9, 21, 13), (4, 4, 8), (16, 16), 3000, 10
    s = Shape(n, d, r)
    rng = np.random.default_rng(4242 + flags)
    cur = [(rng.standard_normal(cs) / 4).astype(np.float32) for cs in s.core_shapes()]
    batches = [rng.integers(0, s.N, B).astype(np.int64) for _ in range(steps)]
    for b in batches:
        b[:200] = b[0]
    grad = rng.standard_normal((B, s.D)).astype(np.float32)
    g = torch.from_numpy(grad).cuda()
    emb = TTEmbedding(n, d, r, B, cur, flags=flags)
    bufs = [torch.empty(B, dtype=torch.int64, device="cuda") for _ in range(2)]
    bufs[0].copy_(torch.from_numpy(batches[0]))
    torch.cuda.synchronize()
    emb.prepare(bufs[0])
    for k in range(steps):
        if k + 1 < steps:
            torch.cuda.synchronize()                      # the buffer's earlier reader is done
            bufs[(k + 1) % 2].copy_(torch.from_numpy(batches[k + 1]))
            torch.cuda.synchronize()                      # ids complete before prepare (flag 4)
            emb.prepare(bufs[(k + 1) % 2])
        out = emb.forward(bufs[k % 2]).cpu().numpy()
        assert row_error(out, ora.forward(s, *cur, batches[k])) <= ROW_TOL, k
        st = emb.stats(check=False)
        assert st["U"] == np.unique(batches[k]).size, k
        emb.backward_update(g, 0.01)
        cur = [c.astype(np.float32) for c in ora.backward_update(s, *cur, batches[k], grad, 0.01)]
        for j in range(3):
            assert core_error(emb.cores[j].cpu().numpy(), cur[j]) <= CORE_TOL, (k, j)
    emb.close()


def test_wait_backward_flow_control():
    """tt_emb_wait_backward(age) returns once that backward_update has finished on the device: after
    age 0 the stream is idle; an age the handle cannot know about, a handle that never prepared,
    and a fresh handle return at once; results are what they are without it."""
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    w, cores, ids, grad = _workload(2, batch=20_000)
    s = Shape(w.n, w.d, w.r)
    t_ids, t_grad = torch.from_numpy(ids).cuda(), torch.from_numpy(grad).cuda()
    emb = TTEmbedding(w.n, w.d, w.r, ids.size, cores, flags=4)
    emb.wait_backward(0)                                   # nothing has happened yet
    ref = [c.copy() for c in cores]
    emb.prepare(t_ids)
    emb.prepare(t_ids)
    for k in range(6):
        emb.wait_backward(1)
        if k < 4:
            emb.prepare(t_ids)
        emb.forward(t_ids)
        emb.backward_update(t_grad, w.lr * 0.01)
        ref = [c.astype(np.float32) for c in ora.backward_update(s, *ref, ids, grad, w.lr * 0.01)]
    emb.wait_backward(0)
    assert torch.cuda.current_stream().query()             # the update kernel was the last launch
    emb.wait_backward(2)
    emb.wait_backward(7)
    for k in range(3):
        assert core_error(emb.cores[k].cpu().numpy(), ref[k]) <= CORE_TOL
    emb.close()
    plain = TTEmbedding(w.n, w.d, w.r, ids.size, cores)    # no prepare, no flag: nothing tracked
    plain.forward(t_ids)
    plain.backward_update(t_grad, w.lr)
    plain.wait_backward(0)
    plain.close()


def test_lookup_only_calls_and_dense_materialisation():
    """forward_eval gives the rows of forward and arms no backward; materialize writes the dense
    table the cores define (all of config 1's 1000 rows, and a window of a rank-32 table that is
    longer than max_batch, so it is produced in several pieces)."""
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    from paper_2206_10581_amd.binding import TTEmbError, TT_EMB_ESTATE
    w, cores, ids, grad = _workload(1)
    s = Shape(w.n, w.d, w.r)
    emb = TTEmbedding(w.n, w.d, w.r, 256, cores)
    t_ids = torch.from_numpy(ids).cuda()
    out = emb.forward_eval(t_ids)
    assert row_error(out.cpu().numpy(), ora.forward(s, *cores, ids)) <= ROW_TOL
    with pytest.raises(TTEmbError) as e:
        emb.backward_update(torch.from_numpy(grad).cuda(), w.lr)
    assert e.value.code == TT_EMB_ESTATE
    table = emb.materialize().cpu().numpy()                       # 1000 rows, four pieces of 256
    ref = ora.forward(s, *cores, np.arange(s.N, dtype=np.int64))
    assert table.shape == ref.shape and row_error(table, ref) <= ROW_TOL
    for c_gpu, c in zip(emb.cores, cores):                        # lookups never write the cores
        np.testing.assert_array_equal(c_gpu.cpu().numpy(), c)
    emb.close()

    w, cores, _, _ = _workload(3)
    s = Shape(w.n, w.d, w.r)
    emb = TTEmbedding(w.n, w.d, w.r, 3000, cores)
    first, count = 136 * 136 * 5 - 4000, 10_001                   # crosses an i1 boundary
    part = emb.materialize(first, count).cpu().numpy()
    ref = ora.forward(s, *cores, np.arange(first, first + count, dtype=np.int64))
    assert row_error(part, ref) <= ROW_TOL
    emb.close()


def test_slab_split_shape_through_every_entry_point():
    """d = (8,4,4), rank 16 runs as a table with twice the first-core slices and d1 = 4 (each row
    two half rows); counts, out-of-range handling, the prepared pipeline, the lookup-only calls,
    the re-indexing table and Adagrad must all look as for any other shape."""
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    n, d, r = (6, 7, 9), (8, 4, 4), (16, 16)
    s = Shape(n, d, r)
    rng = np.random.default_rng(844)
    cores = tuple((rng.standard_normal(cs) / 4).astype(np.float32) for cs in s.core_shapes())
    B = 3000
    ids = rng.integers(0, s.N, B).astype(np.int64)
    ids[:500] = ids[0]
    ids[600:606] = [-1, s.N, s.N + 3, 1 << 40, s.N - 1, 0]
    grad = rng.standard_normal((B, s.D)).astype(np.float32)
    out, new, stats = check_against_oracle(n, d, r, cores, ids, grad, 0.01)
    assert stats["out_of_range"] == 4
    with_generic = run_gpu(n, d, r, cores, ids, grad, 0.01, flags=2)     # the any-shape kernels
    assert row_error(out, with_generic[0]) <= ROW_TOL and with_generic[2] == stats

    emb = TTEmbedding(n, d, r, 1000, cores)
    table = emb.materialize().cpu().numpy()                              # 378 rows
    assert row_error(table, ora.forward(s, *cores, np.arange(s.N, dtype=np.int64))) <= ROW_TOL
    part = emb.materialize(100, 200).cpu().numpy()
    np.testing.assert_array_equal(part, table[100:300])
    # three steps with the index work prepared ahead, then the same rows from a lookup-only call
    cur = [c.copy() for c in cores]
    batches = [rng.integers(0, s.N, 1000).astype(np.int64) for _ in range(3)]
    t_b = [torch.from_numpy(b).cuda() for b in batches]
    g = torch.from_numpy(grad[:1000]).cuda()
    emb.prepare(t_b[0])
    for k in range(3):
        if k + 1 < 3:
            emb.prepare(t_b[k + 1])
        o = emb.forward(t_b[k]).cpu().numpy()
        assert row_error(o, ora.forward(s, *cur, batches[k])) <= ROW_TOL
        emb.backward_update(g, 0.01)
        cur = [c.astype(np.float32) for c in ora.backward_update(s, *cur, batches[k], grad[:1000], 0.01)]
    for k in range(3):
        assert core_error(emb.cores[k].cpu().numpy(), cur[k]) <= CORE_TOL
    # re-indexing table in front of the split
    perm = rng.permutation(s.N).astype(np.int32)
    emb.set_reindex(torch.from_numpy(perm).cuda())
    o = emb.forward_eval(t_b[0]).cpu().numpy()
    now = [c.cpu().numpy() for c in emb.cores]
    assert row_error(o, ora.forward(s, *now, perm[batches[0]].astype(np.int64))) <= ROW_TOL
    emb.set_reindex(None)
    # Adagrad from a zero state
    emb.set_adagrad(1e-6)
    emb.forward(t_b[1])
    emb.backward_update(g, 0.05)
    torch.cuda.synchronize()
    ref_new, ref_state = ora.adagrad_update(s, *now, [np.zeros_like(c) for c in now], batches[1],
                                            grad[:1000], 0.05, 1e-6)
    for k in range(3):
        assert core_error(emb.cores[k].cpu().numpy(), ref_new[k]) <= CORE_TOL
        assert core_error(emb.adagrad_state[k].cpu().numpy(), ref_state[k]) <= CORE_TOL
    emb.close()


def test_node_reindexing_table():
    """With a re-indexing table the row of id i is W[new_id_of[i]] in forward and in the gradients;
    ids outside the table and entries outside [0, N) count as out of range."""
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    w, cores, _, _ = _workload(2)
    s = Shape(w.n, w.d, w.r)
    rng = np.random.default_rng(77)
    n_nodes = 150_000                                             # fewer nodes than table rows
    table = rng.permutation(s.N)[:n_nodes].astype(np.int32)
    table[:3] = [-1, s.N, s.N + 5]                                # entries that point outside
    B = 20_000
    ids = rng.integers(0, n_nodes, B).astype(np.int64)
    ids[:40] = ids[40]                                            # a repeated node
    ids[100:110] = [n_nodes, n_nodes + 7, -1, 0, 1, 2, -5, 1 << 40, n_nodes - 1, 3]
    grad = rng.standard_normal((B, s.D)).astype(np.float32)
    # what the table means, written out with NumPy: look the id up, out-of-table ids stay invalid
    inside = (ids >= 0) & (ids < n_nodes)
    rows = np.where(inside, table[np.clip(ids, 0, n_nodes - 1)].astype(np.int64), -1)
    emb = TTEmbedding(w.n, w.d, w.r, B, cores)
    emb.set_reindex(torch.from_numpy(table).cuda())
    out = emb.forward(torch.from_numpy(ids).cuda())
    stats = emb.stats(check=False)
    emb.backward_update(torch.from_numpy(grad).cuda(), w.lr)
    torch.cuda.synchronize()
    ok = rows[(rows >= 0) & (rows < s.N)]
    assert stats["U"] == np.unique(ok).size and stats["out_of_range"] == B - ok.size
    assert row_error(out.cpu().numpy(), ora.forward(s, *cores, rows)) <= ROW_TOL
    ref_new = ora.backward_update(s, *cores, rows, grad, w.lr)
    for k in range(3):
        assert core_error(emb.cores[k].cpu().numpy(), ref_new[k]) <= CORE_TOL
        step_gpu = (cores[k].astype(np.float64) - emb.cores[k].cpu().numpy()) / w.lr
        step_ref = (cores[k].astype(np.float64) - ref_new[k]) / w.lr
        slack = 2 * np.finfo(np.float32).eps * np.abs(cores[k]).max() / w.lr
        assert np.abs(step_gpu - step_ref).max() <= STEP_TOL * np.abs(step_ref).max() + slack
    # without the table the same ids mean table rows again
    emb.set_reindex(None)
    out2 = emb.forward_eval(torch.from_numpy(ids).cuda()).cpu().numpy()
    new_cores = [c.cpu().numpy() for c in emb.cores]
    assert row_error(out2, ora.forward(s, *new_cores, ids)) <= ROW_TOL
    emb.close()


def test_adagrad_update_two_steps():
    """Row-sparse Adagrad as the update rule: two steps with the state carried along, against the
    oracle's textbook rule; then back to SGD."""
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    for cfg, B in ((1, 256), (2, 12_000)):
        w, cores, _, _ = _workload(cfg)
        s = Shape(w.n, w.d, w.r)
        lr, eps = 0.05, 1e-8
        emb = TTEmbedding(w.n, w.d, w.r, B, cores)
        emb.set_adagrad(eps)
        ref = [c.copy() for c in cores]
        state = [np.zeros_like(c) for c in cores]
        for step in range(2):
            ids, grad = wl.make_ids(w, 60 + step, B), wl.make_grads(w, 60 + step, B)
            ids[:30] = ids[0]
            out = emb.forward(torch.from_numpy(ids).cuda())
            emb.backward_update(torch.from_numpy(grad).cuda(), lr)
            torch.cuda.synchronize()
            assert row_error(out.cpu().numpy(), ora.forward(s, *ref, ids)) <= ROW_TOL
            old = ref
            ref, state = ora.adagrad_update(s, *ref, state, ids, grad, lr, eps)
            for k in range(3):
                got = emb.cores[k].cpu().numpy()
                assert core_error(got, ref[k]) <= CORE_TOL, (cfg, step, k)
                # the step itself (at most lr per entry) to 1e-4 of lr, plus the rounding of G
                slack = 2 * np.finfo(np.float32).eps * np.abs(old[k]).max()
                assert np.abs((old[k].astype(np.float64) - got) - (old[k].astype(np.float64) - ref[k])).max() \
                    <= STEP_TOL * lr + slack, (cfg, step, k)
                st = emb.adagrad_state[k].cpu().numpy()
                assert core_error(st, state[k]) <= CORE_TOL
                # entries whose gradient was zero keep core and state bit for bit
                same = state[k] == 0
                np.testing.assert_array_equal(got[same], cores[k][same])
                np.testing.assert_array_equal(st[same], 0.0)
        emb.set_adagrad(enable=False)
        ids, grad = wl.make_ids(w, 70, B), wl.make_grads(w, 70, B)
        emb.forward(torch.from_numpy(ids).cuda())
        emb.backward_update(torch.from_numpy(grad).cuda(), w.lr)
        torch.cuda.synchronize()
        ref2 = ora.backward_update(s, *ref, ids, grad, w.lr)
        for k in range(3):
            assert core_error(emb.cores[k].cpu().numpy(), ref2[k]) <= CORE_TOL
        emb.close()


@pytest.mark.parametrize("n,d,r,B", [
    ((10, 10, 10), (2, 2, 2), (4, 4), 256),          # any-shape kernels
    ((56, 56, 56), (4, 4, 4), (16, 16), 12_000),     # matrix-core kernels
    ((9, 11, 13), (8, 4, 8), (32, 32), 4_000),       # ... through the slab split
])
def test_adam_update_three_steps(n, d, r, B):
    """Row-sparse Adam as the update rule: three steps with the moments carried along (batches that
    leave slices untouched, so that lazily kept moments matter), against the oracle's textbook
    rule; then the moments are handed to a second handle with steps_done and both take a step."""
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    from paper_2206_10581_amd.binding import tt_emb_set_adam
    s = Shape(n, d, r)
    rng = np.random.default_rng(B)
    cores = [(rng.standard_normal(cs) / np.sqrt(r[0])).astype(np.float32) for cs in s.core_shapes()]
    lr, b1, b2, eps = 0.01, 0.9, 0.99, 1e-6
    emb = TTEmbedding(n, d, r, B, cores)
    emb.set_adam(b1, b2, eps)
    ref = [c.copy() for c in cores]
    m = [np.zeros_like(c) for c in cores]
    v = [np.zeros_like(c) for c in cores]
    for step in range(1, 4):
        ids = rng.integers(0, s.N // 2 if step == 2 else s.N, B).astype(np.int64)   # step 2: half the i1
        ids[:40] = ids[0]
        grad = rng.standard_normal((B, s.D)).astype(np.float32)
        out = emb.forward(torch.from_numpy(ids).cuda())
        emb.backward_update(torch.from_numpy(grad).cuda(), lr)
        torch.cuda.synchronize()
        assert row_error(out.cpu().numpy(), ora.forward(s, *ref, ids)) <= ROW_TOL
        old = ref
        ref, m, v = ora.adam_update(s, *ref, m, v, step, ids, grad, lr, b1, b2, eps)
        for k in range(3):
            got = emb.cores[k].cpu().numpy()
            assert core_error(got, ref[k]) <= CORE_TOL, (step, k)
            # the step itself (about lr per entry) to 1e-4 of lr, plus the rounding of G
            slack = 2 * np.finfo(np.float32).eps * np.abs(old[k]).max()
            moved_gpu = old[k].astype(np.float64) - got
            moved_ref = old[k].astype(np.float64) - ref[k]
            assert np.abs(moved_gpu - moved_ref).max() <= STEP_TOL * max(lr, np.abs(moved_ref).max()) + slack
            assert core_error(emb.adam_state[0][k].cpu().numpy(), m[k]) <= CORE_TOL
            assert core_error(emb.adam_state[1][k].cpu().numpy(), v[k]) <= CORE_TOL
    # a second handle over copies of cores and moments, told that three steps were made
    cores2 = [c.cpu().numpy().copy() for c in emb.cores]
    emb2 = TTEmbedding(n, d, r, B, cores2)
    m2 = [t.clone() for t in emb.adam_state[0]]
    v2 = [t.clone() for t in emb.adam_state[1]]
    rc = tt_emb_set_adam(emb2.handle, [t.data_ptr() for t in m2], [t.data_ptr() for t in v2],
                         b1, b2, eps, 3)
    assert rc == 0
    ids = torch.from_numpy(rng.integers(0, s.N, B).astype(np.int64)).cuda()
    grad = torch.from_numpy(rng.standard_normal((B, s.D)).astype(np.float32)).cuda()
    for e in (emb, emb2):
        e.forward(ids)
        e.backward_update(grad, lr)
    torch.cuda.synchronize()
    for k in range(3):
        np.testing.assert_array_equal(emb.cores[k].cpu().numpy(), emb2.cores[k].cpu().numpy())
    emb2.close()
    emb.set_adam(enable=False)                               # back to SGD
    ids_np = rng.integers(0, s.N, B).astype(np.int64)
    grad_np = rng.standard_normal((B, s.D)).astype(np.float32)
    now = [c.cpu().numpy() for c in emb.cores]
    emb.forward(torch.from_numpy(ids_np).cuda())
    emb.backward_update(torch.from_numpy(grad_np).cuda(), lr)
    torch.cuda.synchronize()
    ref2 = ora.backward_update(s, *now, ids_np, grad_np, lr)
    for k in range(3):
        assert core_error(emb.cores[k].cpu().numpy(), ref2[k]) <= CORE_TOL
    emb.close()


def test_side_stream_and_graph_replays():
    """The calls only enqueue on the stream they are given: a step on a non-default stream, and a step
    captured into a HIP graph and replayed three times (eager work and synchronisation between the
    replays), give bit for bit what the eager default-stream step gives."""
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    w, cores, ids, grad = _workload(2, batch=20_000)
    ids[:500] = ids[0]
    t_ids, t_grad = torch.from_numpy(ids).cuda(), torch.from_numpy(grad).cuda()
    emb = TTEmbedding(w.n, w.d, w.r, ids.size, cores)
    snap = [c.clone() for c in emb.cores]
    out_ref = emb.forward(t_ids).clone()
    emb.backward_update(t_grad, w.lr)
    torch.cuda.synchronize()
    cores_ref = [c.clone() for c in emb.cores]

    def restore():
        for c, b in zip(emb.cores, snap):
            c.copy_(b)

    side = torch.cuda.Stream()
    restore()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        out_s = emb.forward(t_ids)
        emb.backward_update(t_grad, w.lr)
    side.synchronize()
    assert torch.equal(out_s, out_ref)
    for x, y in zip(emb.cores, cores_ref):
        assert torch.equal(x, y)

    restore()
    out_g = torch.empty_like(out_ref)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        emb.forward(t_ids, out_g)
        emb.backward_update(t_grad, w.lr)
    for replay in range(3):
        restore()
        out_g.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_ref), f"replay {replay}"
        for x, y in zip(emb.cores, cores_ref):
            assert torch.equal(x, y), f"replay {replay}"
        scratch = (out_g * 2).sum().item()          # eager work between the replays
        assert np.isfinite(scratch)
    emb.close()


def test_abi_error_codes():
    torch = _torch()
    import paper_2206_10581_amd as lib
    from paper_2206_10581_amd.binding import (TT_EMB_EINVAL, TT_EMB_ENOSPC, TT_EMB_ESTATE,
                                              TT_EMB_ERANGE, TT_EMB_FLAG_CHECK_RANGE, make_config)
    w, cores, ids, grad = _workload(1)
    assert lib.tt_emb_workspace_bytes(make_config((0, 10, 10), w.d, w.r, 10))[0] == TT_EMB_EINVAL
    assert lib.tt_emb_workspace_bytes(make_config((2000, 2000, 2000), w.d, w.r, 10))[0] == TT_EMB_EINVAL
    assert lib.tt_emb_workspace_bytes(make_config(w.n, w.d, (0, 4), 10))[0] == TT_EMB_EINVAL
    assert lib.tt_emb_workspace_bytes(make_config(w.n, w.d, w.r, 0))[0] == TT_EMB_EINVAL
    emb = lib.TTEmbedding(w.n, w.d, w.r, 100, cores, flags=TT_EMB_FLAG_CHECK_RANGE)
    t_grad = torch.from_numpy(grad[:100]).cuda()
    assert lib.tt_emb_backward_update(emb.handle, t_grad.data_ptr(), 0.01, 0) == TT_EMB_ESTATE
    t_ids = torch.from_numpy(ids).cuda()
    out = torch.empty((ids.size, w.D), device="cuda")
    assert lib.tt_emb_forward(emb.handle, t_ids.data_ptr(), ids.size, out.data_ptr(), 0) == TT_EMB_ENOSPC
    assert lib.tt_emb_forward(emb.handle, t_ids.data_ptr(), -1, out.data_ptr(), 0) == TT_EMB_EINVAL
    assert lib.tt_emb_forward(emb.handle, 0, 10, out.data_ptr(), 0) == TT_EMB_EINVAL
    bad = t_ids[:100].clone()
    bad[7] = w.N
    emb.forward(bad)
    rc, U, Q, oob = lib.tt_emb_get_stats(emb.handle)
    assert rc == TT_EMB_ERANGE and oob == 1
    emb.backward_update(t_grad, 0.01)
    assert lib.tt_emb_backward_update(emb.handle, t_grad.data_ptr(), 0.01, 0) == TT_EMB_ESTATE
    torch.cuda.synchronize()
    emb.close()
    rc, _ = lib.tt_emb_create(make_config(w.n, w.d, w.r, 100), 0, 0, 0, 0, 0)
    assert rc == TT_EMB_EINVAL


# ----------------------------------------------------------------------------- more properties

def _step_close(old, new_a, new_b, lr):
    """The updates two runs applied to one core agree to STEP_TOL of the larger update."""
    da = (old.astype(np.float64) - new_a) / lr
    db = (old.astype(np.float64) - new_b) / lr
    slack = 4 * np.finfo(np.float32).eps * np.abs(old).max() / lr
    assert np.abs(da - db).max() <= STEP_TOL * np.abs(db).max() + slack


def test_batch_permutation_invariance():
    """Shuffling the batch (ids and gradient rows together) permutes the output rows and leaves the
    update unchanged up to the order of the sums."""
    w, cores, ids, grad = _workload(3, batch=50_000)
    perm = np.random.default_rng(9).permutation(ids.size)
    out_a, new_a, st_a = run_gpu(w.n, w.d, w.r, cores, ids, grad, w.lr)
    out_b, new_b, st_b = run_gpu(w.n, w.d, w.r, cores, ids[perm], grad[perm], w.lr)
    assert st_a == st_b
    assert row_error(out_b, out_a[perm]) <= ROW_TOL
    for k in range(3):
        _step_close(cores[k], new_a[k], new_b[k], w.lr)


def test_every_id_twice_with_halved_gradients():
    """Every position of the batch doubled with half its gradient: the rows repeat, and the summed
    gradient, hence the update, is the same (halving is exact in fp32)."""
    w, cores, ids, grad = _workload(3, batch=40_000)
    ids2 = np.concatenate([ids, ids])
    grad2 = np.concatenate([grad * np.float32(0.5), grad * np.float32(0.5)])
    out_a, new_a, st_a = run_gpu(w.n, w.d, w.r, cores, ids, grad, w.lr)
    out_b, new_b, st_b = run_gpu(w.n, w.d, w.r, cores, ids2, grad2, w.lr)
    assert (st_a["U"], st_a["Q"]) == (st_b["U"], st_b["Q"])
    assert row_error(out_b[: ids.size], out_a) <= ROW_TOL
    assert row_error(out_b[ids.size:], out_a) <= ROW_TOL
    for k in range(3):
        _step_close(cores[k], new_a[k], new_b[k], w.lr)


# ----------------------------------------------------------------------------- sizes as quoted

def test_products_shape_rank32_full_size():
    """The paper's ogbn-products factorisation (Table "ogb-dim-tt": (125,140,140) x (4,5,5)) at the
    rank and batch its step time is quoted at: rank 32, the 200,000-row Zipf batch."""
    w, cores, ids, grad = _workload(7)
    check_against_oracle(w.n, w.d, w.r, cores, ids, grad, w.lr)


def test_rank128_through_the_slab_split_at_sweep_size():
    """Rank 128 on the paper's ogbn-arxiv factorisation ((55,55,56) x (8,4,4): two slabs of d1 = 4),
    50,000 uniform ids as in the rank sweep."""
    n, d, r, B = (55, 55, 56), (8, 4, 4), (128, 128), 50_000
    s = Shape(n, d, r)
    rng = np.random.default_rng(128)
    cores = tuple((rng.standard_normal(cs) / np.sqrt(128)).astype(np.float32) for cs in s.core_shapes())
    ids = rng.integers(0, s.N, size=B, dtype=np.int64)
    ids[:2000] = ids[0]
    grad = rng.standard_normal((B, s.D)).astype(np.float32)
    check_against_oracle(n, d, r, cores, ids, grad, 0.01)


def test_prepare_then_capture_is_refused():
    """A handle that has used tt_emb_prepare is not captured into a graph: its calls return
    TT_EMB_ESTATE while the stream is being captured, the capture itself stays valid, and the handle
    works as before afterwards."""
    torch = _torch()
    import paper_2206_10581_amd as lib
    from paper_2206_10581_amd.binding import TT_EMB_ESTATE
    w, cores, ids, grad = _workload(2, batch=5000)
    s = Shape(w.n, w.d, w.r)
    t_ids, t_grad = torch.from_numpy(ids).cuda(), torch.from_numpy(grad).cuda()
    emb = lib.TTEmbedding(w.n, w.d, w.r, ids.size, cores)
    out = torch.empty((ids.size, w.D), device="cuda")
    emb.prepare(t_ids)
    emb.forward(t_ids, out)
    emb.backward_update(t_grad, w.lr)
    torch.cuda.synchronize()
    now = [c.cpu().numpy() for c in emb.cores]
    dummy = torch.zeros(8, device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st = int(torch.cuda.current_stream().cuda_stream)
        rcs = (lib.tt_emb_prepare(emb.handle, t_ids.data_ptr(), ids.size, st),
               lib.tt_emb_forward(emb.handle, t_ids.data_ptr(), ids.size, out.data_ptr(), st),
               lib.tt_emb_forward_eval(emb.handle, t_ids.data_ptr(), ids.size, out.data_ptr(), st))
        dummy.add_(1.0)
    assert rcs == (TT_EMB_ESTATE,) * 3
    graph.replay()
    torch.cuda.synchronize()
    assert float(dummy[0]) == 1.0
    o = emb.forward(t_ids, out)                      # eager again: unchanged behaviour
    emb.backward_update(t_grad, w.lr)
    torch.cuda.synchronize()
    assert row_error(o.cpu().numpy(), ora.forward(s, *now, ids)) <= ROW_TOL
    ref = ora.backward_update(s, *now, ids, grad, w.lr)
    for k in range(3):
        assert core_error(emb.cores[k].cpu().numpy(), ref[k]) <= CORE_TOL
    emb.close()


def test_rejected_backward_keeps_the_forward_pending():
    torch = _torch()
    import paper_2206_10581_amd as lib
    from paper_2206_10581_amd.binding import TT_EMB_EINVAL
    w, cores, ids, grad = _workload(2, batch=3000)
    s = Shape(w.n, w.d, w.r)
    emb = lib.TTEmbedding(w.n, w.d, w.r, ids.size, cores)
    emb.forward(torch.from_numpy(ids).cuda())
    t_grad = torch.from_numpy(grad).cuda()
    assert lib.tt_emb_backward_update(emb.handle, 0, w.lr, 0) == TT_EMB_EINVAL
    assert lib.tt_emb_backward_update(emb.handle, t_grad.data_ptr() + 4, w.lr, 0) == TT_EMB_EINVAL
    emb.backward_update(t_grad, w.lr)                # the forward is still pending
    torch.cuda.synchronize()
    ref = ora.backward_update(s, *cores, ids, grad, w.lr)
    for k in range(3):
        assert core_error(emb.cores[k].cpu().numpy(), ref[k]) <= CORE_TOL
    emb.close()


# ----------------------------------------------------------------------------- the loops bench.py times

@pytest.mark.parametrize("loop", ["lookahead", "plain"])
def test_benchmark_loops_at_config3_full_size(loop):
    """bench.py's own loop functions at the benchmark's size and launch configuration: the
    200,000-row Zipf batches of config 3, three different batches in rotating buffers, six steps
    without any synchronisation between them.  "lookahead" is the headline loop: a handle with
    TT_EMB_FLAG_IDS_READY, tt_emb_prepare two batches ahead on the library's own streams,
    tt_emb_wait_backward(1) before every step.  Every step is checked element by element against
    the oracle started from the cores the GPU itself had before that step (device-side snapshots
    taken on the stream, no host wait), with the usual tolerances."""
    torch = _torch()
    import bench
    from paper_2206_10581_amd import TTEmbedding
    w = wl.CONFIGS[3]
    s = Shape(w.n, w.d, w.r)
    seeds, steps, lr = (3, 103, 203), 6, 2e-4
    cores = wl.make_cores(w, 3)
    ids_np = [wl.make_ids(w, sd) for sd in seeds]
    grad_np = [wl.make_grads(w, sd) for sd in seeds]
    ids = [torch.from_numpy(a).cuda() for a in ids_np]
    grad = [torch.from_numpy(a).cuda() for a in grad_np]
    out = [torch.empty((w.batch, w.D), device="cuda") for _ in seeds]
    torch.cuda.synchronize()
    emb = TTEmbedding(w.n, w.d, w.r, w.batch, cores, flags=4 if loop == "lookahead" else 0)
    core_snaps = [[c.clone() for c in emb.cores]]
    out_snaps = []

    def after(k):
        out_snaps.append(out[k % 3].clone())
        core_snaps.append([c.clone() for c in emb.cores])

    if loop == "lookahead":
        bench.prime_lookahead(emb, ids)
        bench.run_lookahead(emb, ids, grad, out, lr, steps, after_step=after)
    else:
        bench.run_plain(emb, ids, grad, out, lr, steps, after_step=after)
    torch.cuda.synchronize()
    emb.stats()                                              # raises on an internal-error flag
    for k in range(steps):
        before = [c.cpu().numpy() for c in core_snaps[k]]
        after_k = [c.cpu().numpy() for c in core_snaps[k + 1]]
        i, g = ids_np[k % 3], grad_np[k % 3]
        assert row_error(out_snaps[k].cpu().numpy(), ora.forward(s, *before, i)) <= ROW_TOL, k
        ref = ora.backward_update(s, *before, i, g, lr)
        for c in range(3):
            assert core_error(after_k[c], ref[c]) <= CORE_TOL, (k, c)
            step_gpu = (before[c].astype(np.float64) - after_k[c]) / lr
            step_ref = (before[c].astype(np.float64) - ref[c]) / lr
            slack = 2 * np.finfo(np.float32).eps * np.abs(before[c]).max() / lr
            assert np.abs(step_gpu - step_ref).max() <= STEP_TOL * np.abs(step_ref).max() + slack, (k, c)
    emb.close()


def test_ttsvd_initialisation_on_the_gpu():
    """Algorithm 1 of the paper (TT-SVD initialisation) at full ranks reproduces the matrix it
    decomposes; the HIP forward over every id gives that matrix back (no oracle involved), on an
    any-shape table and on a matrix-core shape."""
    torch = _torch()
    from paper_2206_10581_amd import TTEmbedding
    for n, d, r in [((6, 5, 7), (2, 2, 3), (12, 21)), ((4, 5, 4), (4, 4, 4), (16, 16))]:
        s = Shape(n, d, r)
        cores, info = wl.make_ttsvd_cores(n, d, r, seed=17, return_info=True)
        emb = TTEmbedding(n, d, r, s.N, cores)
        W = emb.forward(torch.arange(s.N, dtype=torch.int64, device="cuda")).double().cpu().numpy()
        emb.close()
        np.testing.assert_allclose(W, info["matrix"], atol=2e-5)
        np.testing.assert_allclose(W.T @ W, np.eye(s.D), atol=1e-4)


@pytest.mark.parametrize("flags", [0, 2])
def test_table_at_the_size_limits(flags):
    """The largest table the library accepts: 2048 values of i2 and of i3 (the bucket limit of the
    grouping passes, eleven-bit digits with the top bit in use) and N just below 2^31 (31-bit sort
    keys: three radix passes of eleven bits).  Ids from all over the range, the two ends of it,
    repeats, and ids just past the table."""
    n, d, r = (511, 2048, 2048), (4, 4, 4), (8, 8)
    s = Shape(n, d, r)
    assert 2 ** 31 - 2 ** 23 < s.N < 2 ** 31
    rng = np.random.default_rng(77 + flags)
    cores = tuple((rng.standard_normal(cs) * 0.35).astype(np.float32) for cs in s.core_shapes())
    ids = np.concatenate([
        rng.integers(0, s.N, size=4000, dtype=np.int64),
        rng.integers(s.N - 3000, s.N, size=700, dtype=np.int64),
        rng.integers(0, 3000, size=700, dtype=np.int64),
        np.array([0, s.N - 1, s.N - 1, s.N, s.N + 1, 2 ** 31, 2 ** 40, -1, -2 ** 35], dtype=np.int64),
    ])
    ids = np.concatenate([ids, ids[:600]])        # every one of these twice
    rng.shuffle(ids)
    grad = rng.standard_normal((ids.size, s.D)).astype(np.float32)
    check_against_oracle(n, d, r, cores, ids, grad, 0.01, flags=flags)


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes_and_batches(seed):
    """Seeded random tables and batches: factors, ranks, batch size, share of repeated ids, of ids
    sharing a prefix and of out-of-range ids all drawn at random; even seeds draw from the shapes
    that have matrix-core kernels (d1 a multiple of 4, d2 = 4, equal ranks), odd seeds from anything."""
    rng = np.random.default_rng(7000 + seed)
    if seed % 2 == 0:
        R = int(rng.choice([8, 16, 32, 64]))
        d = (int(rng.choice([4, 8])), 4, int(rng.choice([4, 8])))
        r = (R, R)
    else:
        d = tuple(int(x) for x in rng.integers(1, 7, size=3))
        r = tuple(int(x) for x in rng.integers(1, 20, size=2))
    n = tuple(int(x) for x in rng.integers(2, 40, size=3))
    s = Shape(n, d, r)
    B = int(rng.integers(1, 9000))
    cores = tuple((rng.standard_normal(cs) / np.sqrt(max(r))).astype(np.float32) for cs in s.core_shapes())
    ids = rng.integers(0, s.N, size=B, dtype=np.int64)
    k = int(B * rng.random() * 0.5)
    ids[:k] = ids[rng.integers(0, B)]                               # one id many times
    k2 = int(B * rng.random() * 0.3)
    ids[k:k + k2] = np.minimum(ids[0] // n[2] * n[2] + rng.integers(0, n[2], size=k2), s.N - 1)  # one prefix
    bad = rng.random(B) < 0.01
    ids[bad] = rng.choice([-1, s.N, s.N + 7, -(1 << 40), 1 << 40], size=int(bad.sum()))
    rng.shuffle(ids)
    grad = rng.standard_normal((B, s.D)).astype(np.float32)
    check_against_oracle(n, d, r, cores, ids, grad, 0.01, max_batch=B + int(rng.integers(0, 100)))
