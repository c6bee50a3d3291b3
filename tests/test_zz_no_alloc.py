"""The allocation-free lookup against the lookup it is a variant of (tt_emb_forward_eval), through
the C ABI: same kernels over a different workspace, so the rows must agree bit for bit (and, to
the usual tolerance, with the oracle).  Two calls in a row on the same device array, the second
with a smaller batch; then the size limit and the argument checks."""
import numpy as np
import pytest

import workloads as wl
from oracle import tt_oracle as ora
from oracle.tt_oracle import Shape

pytestmark = pytest.mark.gpu

ROW_TOL = 1e-5


def _row_error(gpu, ref):
    num = np.abs(np.asarray(gpu, np.float64) - ref).max(axis=1)
    den = np.abs(ref).max(axis=1)
    assert not num[den == 0].any()
    return float((num[den > 0] / den[den > 0]).max())


@pytest.mark.parametrize("cfg_no,sizes", [(3, (20_000, 7_001)), (2, (50_000, 333)), (1, (256, 100))])
def test_lookup_static_matches_forward_eval(cfg_no, sizes):
    import torch
    assert torch.cuda.is_available()
    import paper_2206_10581_amd as lib
    from paper_2206_10581_amd.binding import (TT_EMB_EINVAL, TT_EMB_ENOSPC, make_config)
    w = wl.CONFIGS[cfg_no]
    s = Shape(w.n, w.d, w.r)
    cores_np = wl.make_cores(w, cfg_no)
    emb = lib.TTEmbedding(w.n, w.d, w.r, max(sizes), cores_np)      # the existing entry point
    cfg = make_config(w.n, w.d, w.r, max(sizes), 0, 0)
    g = [c.data_ptr() for c in emb.cores]
    st = int(torch.cuda.current_stream().cuda_stream)
    assert lib.tt_emb_lookup_static(cfg, *g, 0, 0, 0, st) == 0          # B = 0: set-up only
    for k, B in enumerate(sizes):
        ids_np = wl.make_ids(w, 900 + k, B)
        ids_np[: B // 10] = ids_np[0]                                    # a repeated id
        if B > 50:
            ids_np[5] = -1                                               # out of range: a zero row
            ids_np[6] = w.N
        ids = torch.from_numpy(ids_np).cuda()
        want = emb.forward_eval(ids)
        got = torch.full((B, w.D), float("nan"), device="cuda")
        rc = lib.tt_emb_lookup_static(cfg, *g, ids.data_ptr(), B, got.data_ptr(), st)
        assert rc == 0, lib.tt_emb_strerror(rc)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"call {k}, B={B}"
        assert _row_error(got.cpu().numpy(), ora.forward(s, *cores_np, ids_np)) <= ROW_TOL
    # the cores are never written by a lookup
    for t, c in zip(emb.cores, cores_np):
        np.testing.assert_array_equal(t.cpu().numpy(), c)
    # argument checks (host side, nothing is enqueued)
    ids = torch.zeros(8, dtype=torch.int64, device="cuda")
    o = torch.empty((8, w.D), device="cuda")
    assert lib.tt_emb_lookup_static(cfg, 0, g[1], g[2], ids.data_ptr(), 8, o.data_ptr(), st) == TT_EMB_EINVAL
    assert lib.tt_emb_lookup_static(cfg, *g, 0, 8, o.data_ptr(), st) == TT_EMB_EINVAL
    assert lib.tt_emb_lookup_static(cfg, *g, ids.data_ptr(), max(sizes) + 1, o.data_ptr(), st) == TT_EMB_ENOSPC
    other = make_config(w.n, w.d, w.r, max(sizes), 1, 0)                 # not the current device
    assert lib.tt_emb_lookup_static(other, *g, ids.data_ptr(), 8, o.data_ptr(), st) == TT_EMB_EINVAL
    emb.close()


def test_lookup_static_rejects_batches_beyond_the_array():
    import torch
    import paper_2206_10581_amd as lib
    from paper_2206_10581_amd.binding import TT_EMB_ENOSPC, make_config
    w = wl.CONFIGS[4]              # 230,400 possible prefixes of 1 KiB: 500,000 ids cannot fit 64 MiB
    cores = [torch.zeros(cs, device="cuda") for cs in w.core_shapes()]
    g = [c.data_ptr() for c in cores]
    B = w.batch
    cfg = make_config(w.n, w.d, w.r, B, 0, 0)
    ids = torch.zeros(B, dtype=torch.int64, device="cuda")
    out = torch.empty((B, w.D), device="cuda")
    assert lib.tt_emb_lookup_static(cfg, *g, ids.data_ptr(), B, out.data_ptr(), 0) == TT_EMB_ENOSPC
    # the same table takes a batch that does fit
    B = 40_000
    ids_np = wl.make_ids(w, 4, B)
    t_ids = torch.from_numpy(ids_np).cuda()
    assert lib.tt_emb_lookup_static(cfg, *g, t_ids.data_ptr(), B, out.data_ptr(), 0) == 0
    torch.cuda.synchronize()
    assert not out[:B].any()       # zero cores: zero rows
