"""CPU-side checks of the C-ABI library: it loads, exports every function the header declares,
and its host-only logic (argument checks, workspace sizing, error strings) behaves as documented.
No kernel is launched here."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2206_10581_amd import build as b
    if not os.path.exists(b.lib_path()):
        b.build()
    import paper_2206_10581_amd as p
    p.load_library()
    return p


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "tt_emb.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(tt_emb_[a-z_]+)\s*\(", header)))
    assert len(names) >= 10
    cdll = lib.load_library()
    for name in names:
        assert hasattr(cdll, name), name


def test_workspace_sizing_and_argument_checks(lib):
    from paper_2206_10581_amd.binding import TT_EMB_EINVAL, TT_EMB_ENOSPC, make_config
    import workloads as wl
    sizes = []
    for k in (1, 2, 3, 4, 5):
        w = wl.CONFIGS[k]
        rc, nbytes = lib.tt_emb_workspace_bytes(make_config(w.n, w.d, w.r, w.batch))
        assert rc == 0 and nbytes > 0 and nbytes % 256 == 0
        sizes.append(nbytes)
    assert sizes[0] < sizes[1] < sizes[2] < sizes[4] < 8 << 30
    w = wl.CONFIGS[1]
    # a bigger batch bound never shrinks the workspace
    assert lib.tt_emb_workspace_bytes(make_config(w.n, w.d, w.r, 1000))[1] >= sizes[0]
    for bad in (make_config((10, 10, -1), w.d, w.r, 8), make_config(w.n, (2, 0, 2), w.r, 8),
                make_config(w.n, w.d, (4, 0), 8), make_config(w.n, w.d, w.r, 0),
                make_config(w.n, w.d, w.r, 1 << 30), make_config((1 << 11, 1 << 11, 1 << 11), w.d, w.r, 8),
                make_config((10, 4096, 10), w.d, w.r, 8), make_config(w.n, (32, 32, 32), w.r, 8)):
        assert lib.tt_emb_workspace_bytes(bad)[0] == TT_EMB_EINVAL
    cfg = make_config(w.n, w.d, w.r, 8)
    assert lib.tt_emb_create(cfg, 0, 0, 0, 0, 0)[0] == TT_EMB_EINVAL           # null pointers
    assert lib.tt_emb_create(cfg, 256, 256, 256, 256 + 1, 1 << 30)[0] == TT_EMB_EINVAL  # misaligned
    assert lib.tt_emb_create(cfg, 256, 256, 256, 256, 16)[0] == TT_EMB_ENOSPC  # workspace too small


def test_handle_state_machine_without_launches(lib):
    from paper_2206_10581_amd.binding import TT_EMB_EINVAL, TT_EMB_ENOSPC, TT_EMB_ESTATE, make_config
    import workloads as wl
    w = wl.CONFIGS[1]
    cfg = make_config(w.n, w.d, w.r, 8)
    nbytes = lib.tt_emb_workspace_bytes(cfg)[1]
    # fake, never dereferenced device addresses: only host-side paths are exercised
    rc, h = lib.tt_emb_create(cfg, 256, 512, 768, 1024, nbytes)
    assert rc == 0
    assert lib.tt_emb_backward_update(h, 256, 0.01, 0) == TT_EMB_ESTATE
    assert lib.tt_emb_forward(h, 256, 9, 256, 0) == TT_EMB_ENOSPC
    assert lib.tt_emb_forward(h, 256, -1, 256, 0) == TT_EMB_EINVAL
    assert lib.tt_emb_forward(h, 0, 0, 0, 0) == 0                 # B = 0 is a valid no-op
    assert lib.tt_emb_get_stats(h) == (0, 0, 0, 0)
    assert lib.tt_emb_backward_update(h, 0, 0.01, 0) == 0         # consumes the empty forward
    assert lib.tt_emb_backward_update(h, 0, 0.01, 0) == TT_EMB_ESTATE
    # lookup-only calls and the re-indexing table: argument checks and the pending-forward rule
    assert lib.tt_emb_forward_eval(h, 256, 9, 256, 0) == TT_EMB_ENOSPC
    assert lib.tt_emb_forward_eval(h, 0, 0, 0, 0) == 0
    assert lib.tt_emb_backward_update(h, 0, 0.01, 0) == TT_EMB_ESTATE   # eval leaves nothing pending
    assert lib.tt_emb_materialize(h, 0, 0, 0, 0) == 0
    assert lib.tt_emb_materialize(h, -1, 1, 256, 0) == TT_EMB_EINVAL
    assert lib.tt_emb_materialize(h, 999, 2, 256, 0) == TT_EMB_EINVAL   # past the 1000-row table
    assert lib.tt_emb_set_reindex(h, 0, 5) == TT_EMB_EINVAL
    assert lib.tt_emb_set_reindex(h, 258, 5) == TT_EMB_EINVAL           # misaligned int32 table
    assert lib.tt_emb_set_reindex(h, 256, 5) == 0
    assert lib.tt_emb_set_reindex(h, 0, 0) == 0
    assert lib.tt_emb_forward(h, 0, 0, 0, 0) == 0
    assert lib.tt_emb_forward_eval(h, 0, 0, 0, 0) == TT_EMB_ESTATE      # a forward is pending
    assert lib.tt_emb_materialize(h, 0, 0, 0, 0) == TT_EMB_ESTATE
    assert lib.tt_emb_set_reindex(h, 256, 5) == TT_EMB_ESTATE
    assert lib.tt_emb_backward_update(h, 0, 0.01, 0) == 0
    assert lib.tt_emb_set_adagrad(h, 256, 0, 256, 1e-8) == TT_EMB_EINVAL   # all three or none
    assert lib.tt_emb_set_adagrad(h, 256, 512, 768, 0.0) == TT_EMB_EINVAL  # eps must be positive
    assert lib.tt_emb_set_adagrad(h, 256, 512, 772, 1e-8) == TT_EMB_EINVAL # misaligned
    assert lib.tt_emb_set_adagrad(h, 256, 512, 768, 1e-8) == 0
    assert lib.tt_emb_set_adagrad(h, 0, 0, 0, 0.0) == 0                    # back to SGD
    adam = lambda ptrs, b1, b2, eps, t=0: lib.tt_emb_set_adam(h, ptrs[:3], ptrs[3:], b1, b2, eps, t)
    six = (256, 512, 768, 1024, 1280, 1536)
    assert adam((256, 512, 768, 0, 0, 0), 0.9, 0.999, 1e-8) == TT_EMB_EINVAL   # all six or none
    assert adam(six, 1.0, 0.999, 1e-8) == TT_EMB_EINVAL                        # beta below one
    assert adam(six, 0.9, -0.1, 1e-8) == TT_EMB_EINVAL
    assert adam(six, 0.9, 0.999, 0.0) == TT_EMB_EINVAL                         # eps must be positive
    assert adam(six, 0.9, 0.999, 1e-8, -1) == TT_EMB_EINVAL                    # steps done so far
    assert adam(six[:5] + (1540,), 0.9, 0.999, 1e-8) == TT_EMB_EINVAL          # misaligned
    assert adam(six, 0.9, 0.999, 1e-8, 12) == 0
    assert adam((0,) * 6, 0.0, 0.0, 0.0) == 0                                  # back to SGD
    assert lib.tt_emb_profile_slots() >= 10
    assert lib.tt_emb_profile_read(h, 0)[0] == 0 and lib.tt_emb_profile_read(h, 999)[0] == TT_EMB_EINVAL
    assert lib.tt_emb_destroy(h) == 0
    for code in range(0, -8, -1):
        assert isinstance(lib.tt_emb_strerror(code), str) and lib.tt_emb_strerror(code)
