"""ctypes binding of libtt_emb.so: same names as the C ABI, argument marshalling only.

There is no fallback: if the shared library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t, \
    c_uint32, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtt_emb.so")

TT_EMB_OK, TT_EMB_EINVAL, TT_EMB_ENOSPC, TT_EMB_ESTATE, TT_EMB_EHIP, TT_EMB_ERANGE, \
    TT_EMB_EINTERNAL = 0, -1, -2, -3, -4, -5, -6
TT_EMB_FLAG_CHECK_RANGE = 1
TT_EMB_FLAG_GENERIC_KERNELS = 2
TT_EMB_FLAG_IDS_READY = 4


class TTEmbConfig(ctypes.Structure):
    _fields_ = [("n", c_int64 * 3), ("d", c_int32 * 3), ("r", c_int32 * 2), ("max_batch", c_int64),
                ("device", c_int32), ("flags", c_uint32)]


class TTEmbError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {tt_emb_strerror(code)} (code {code})")


_lib = None


def load_library():
    """Loads libtt_emb.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2206_10581_amd.build` "
                          "(there is no CPU fallback)")
    # PyTorch carries its own copy of the HIP runtime; importing it first makes this library bind
    # to that same copy (one runtime per process), whatever order the caller imports things in.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    cfgp = POINTER(TTEmbConfig)
    lib.tt_emb_workspace_bytes.argtypes = [cfgp, POINTER(c_size_t)]
    lib.tt_emb_create.argtypes = [POINTER(c_void_p), cfgp, c_void_p, c_void_p, c_void_p, c_void_p,
                                  c_size_t]
    lib.tt_emb_forward.argtypes = [c_void_p, c_void_p, c_int64, c_void_p, c_void_p]
    lib.tt_emb_backward_update.argtypes = [c_void_p, c_void_p, c_float, c_void_p]
    lib.tt_emb_forward_eval.argtypes = [c_void_p, c_void_p, c_int64, c_void_p, c_void_p]
    lib.tt_emb_materialize.argtypes = [c_void_p, c_int64, c_int64, c_void_p, c_void_p]
    lib.tt_emb_lookup_static.argtypes = [cfgp, c_void_p, c_void_p, c_void_p, c_void_p, c_int64,
                                         c_void_p, c_void_p]
    lib.tt_emb_set_reindex.argtypes = [c_void_p, c_void_p, c_int64]
    lib.tt_emb_set_adagrad.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_float]
    lib.tt_emb_wait_backward.argtypes = [c_void_p, c_int]
    lib.tt_emb_set_adam.argtypes = [c_void_p] + [c_void_p] * 6 + [c_float, c_float, c_float, c_int64]
    lib.tt_emb_prepare.argtypes = [c_void_p, c_void_p, c_int64, c_void_p]
    lib.tt_emb_get_stats.argtypes = [c_void_p, POINTER(c_int64), POINTER(c_int64), POINTER(c_int64)]
    lib.tt_emb_profile_enable.argtypes = [c_void_p, c_int]
    lib.tt_emb_profile_slots.argtypes = []
    lib.tt_emb_profile_read.argtypes = [c_void_p, c_int, POINTER(c_char_p), POINTER(c_int64),
                                        POINTER(c_double)]
    lib.tt_emb_profile_peaks.argtypes = [c_void_p, c_size_t, c_void_p, POINTER(c_double),
                                         POINTER(c_double), POINTER(c_double), POINTER(c_double)]
    lib.tt_emb_destroy.argtypes = [c_void_p]
    lib.tt_emb_strerror.argtypes = [c_int]
    lib.tt_emb_strerror.restype = c_char_p
    for name in ("tt_emb_workspace_bytes", "tt_emb_create", "tt_emb_forward", "tt_emb_prepare",
                 "tt_emb_backward_update", "tt_emb_forward_eval", "tt_emb_materialize", "tt_emb_lookup_static",
                 "tt_emb_set_reindex", "tt_emb_set_adagrad", "tt_emb_set_adam", "tt_emb_wait_backward", "tt_emb_get_stats", "tt_emb_profile_enable",
                 "tt_emb_profile_slots", "tt_emb_profile_read", "tt_emb_profile_peaks", "tt_emb_destroy"):
        getattr(lib, name).restype = c_int
    _lib = lib
    return lib


def make_config(n, d, r, max_batch: int, device: int = 0, flags: int = 0) -> TTEmbConfig:
    c = TTEmbConfig()
    for k in range(3):
        c.n[k] = int(n[k])
        c.d[k] = int(d[k])
    c.r[0], c.r[1] = int(r[0]), int(r[1])
    c.max_batch, c.device, c.flags = int(max_batch), int(device), int(flags)
    return c


# ---- the C entry points, one to one (integers are raw pointers: tensor.data_ptr(), stream handles)

def tt_emb_strerror(code: int) -> str:
    return load_library().tt_emb_strerror(int(code)).decode()


def tt_emb_workspace_bytes(cfg: TTEmbConfig):
    out = c_size_t(0)
    rc = load_library().tt_emb_workspace_bytes(byref(cfg), byref(out))
    return rc, int(out.value)


def tt_emb_create(cfg: TTEmbConfig, g1_ptr: int, g2_ptr: int, g3_ptr: int, ws_ptr: int, ws_bytes: int):
    h = c_void_p(None)
    rc = load_library().tt_emb_create(byref(h), byref(cfg), c_void_p(g1_ptr), c_void_p(g2_ptr),
                                      c_void_p(g3_ptr), c_void_p(ws_ptr), c_size_t(ws_bytes))
    return rc, h


def tt_emb_forward(h, ids_ptr: int, B: int, out_ptr: int, stream: int) -> int:
    return load_library().tt_emb_forward(h, c_void_p(ids_ptr), c_int64(B), c_void_p(out_ptr),
                                         c_void_p(stream))


def tt_emb_forward_eval(h, ids_ptr: int, B: int, out_ptr: int, stream: int) -> int:
    return load_library().tt_emb_forward_eval(h, c_void_p(ids_ptr), c_int64(B), c_void_p(out_ptr),
                                              c_void_p(stream))


def tt_emb_materialize(h, first_row: int, count: int, out_ptr: int, stream: int) -> int:
    return load_library().tt_emb_materialize(h, c_int64(first_row), c_int64(count),
                                             c_void_p(out_ptr), c_void_p(stream))


def tt_emb_lookup_static(cfg: TTEmbConfig, g1_ptr: int, g2_ptr: int, g3_ptr: int, ids_ptr: int, B: int,
                         out_ptr: int, stream: int) -> int:
    return load_library().tt_emb_lookup_static(byref(cfg), c_void_p(g1_ptr), c_void_p(g2_ptr),
                                               c_void_p(g3_ptr), c_void_p(ids_ptr), c_int64(B),
                                               c_void_p(out_ptr), c_void_p(stream))


def tt_emb_set_reindex(h, table_ptr: int, n_ids: int) -> int:
    return load_library().tt_emb_set_reindex(h, c_void_p(table_ptr), c_int64(n_ids))


def tt_emb_wait_backward(h, age: int) -> int:
    return load_library().tt_emb_wait_backward(h, c_int(age))


def tt_emb_set_adam(h, m_ptrs, v_ptrs, beta1: float, beta2: float, eps: float, steps_done: int = 0) -> int:
    ptrs = [c_void_p(p) for p in (*m_ptrs, *v_ptrs)]
    return load_library().tt_emb_set_adam(h, *ptrs, c_float(beta1), c_float(beta2), c_float(eps),
                                          c_int64(steps_done))


def tt_emb_set_adagrad(h, s1_ptr: int, s2_ptr: int, s3_ptr: int, eps: float) -> int:
    return load_library().tt_emb_set_adagrad(h, c_void_p(s1_ptr), c_void_p(s2_ptr), c_void_p(s3_ptr),
                                             c_float(eps))


def tt_emb_prepare(h, ids_ptr: int, B: int, stream: int) -> int:
    return load_library().tt_emb_prepare(h, c_void_p(ids_ptr), c_int64(B), c_void_p(stream))


def tt_emb_backward_update(h, grad_ptr: int, lr: float, stream: int) -> int:
    return load_library().tt_emb_backward_update(h, c_void_p(grad_ptr), c_float(lr), c_void_p(stream))


def tt_emb_get_stats(h):
    U, Q, oob = c_int64(0), c_int64(0), c_int64(0)
    rc = load_library().tt_emb_get_stats(h, byref(U), byref(Q), byref(oob))
    return rc, int(U.value), int(Q.value), int(oob.value)


def tt_emb_profile_enable(h, enable: bool) -> int:
    return load_library().tt_emb_profile_enable(h, c_int(1 if enable else 0))


def tt_emb_profile_slots() -> int:
    return load_library().tt_emb_profile_slots()


def tt_emb_profile_read(h, slot: int):
    name, n, ms = c_char_p(None), c_int64(0), c_double(0.0)
    rc = load_library().tt_emb_profile_read(h, c_int(slot), byref(name), byref(n), byref(ms))
    return rc, (name.value or b"").decode(), int(n.value), float(ms.value)


def tt_emb_profile_peaks(buf_ptr: int, nbytes: int, stream: int):
    copy, mfma, gather, far = c_double(0.0), c_double(0.0), c_double(0.0), c_double(0.0)
    rc = load_library().tt_emb_profile_peaks(c_void_p(buf_ptr), c_size_t(nbytes), c_void_p(stream),
                                             byref(copy), byref(mfma), byref(gather), byref(far))
    return rc, float(copy.value), float(mfma.value), float(gather.value), float(far.value)


def tt_emb_destroy(h) -> int:
    return load_library().tt_emb_destroy(h)


# ---- convenience wrapper over torch tensors (memory and streams only)

class TTEmbedding:
    """Owns the device tensors the library borrows: three cores and the workspace."""

    def __init__(self, n, d, r, max_batch: int, cores, device="cuda:0", flags: int = 0):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.n, self.d, self.r = tuple(n), tuple(d), tuple(r)
        self.D = self.d[0] * self.d[1] * self.d[2]
        shapes = ((n[0], d[0], r[0]), (n[1], r[0], d[1], r[1]), (n[2], r[1], d[2]))
        self.cores = []
        for c, s in zip(cores, shapes):
            if (isinstance(c, torch.Tensor) and c.device == self.device and c.dtype == torch.float32
                    and c.is_contiguous()):
                t = c                      # caller-owned device tensor: borrowed, updated in place
            else:
                t = torch.as_tensor(c).to(device=self.device, dtype=torch.float32).contiguous().clone()
            if tuple(t.shape) != tuple(s):
                raise ValueError(f"core shape {tuple(t.shape)} != {s}")
            self.cores.append(t)
        index = self.device.index if self.device.index is not None else 0
        self.cfg = make_config(n, d, r, max_batch, index, flags)
        rc, nbytes = tt_emb_workspace_bytes(self.cfg)
        if rc:
            raise TTEmbError(rc, "tt_emb_workspace_bytes")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) & ~255
        self.workspace_bytes = nbytes
        rc, self.handle = tt_emb_create(self.cfg, *(t.data_ptr() for t in self.cores), self._ws_ptr,
                                        nbytes)
        if rc:
            raise TTEmbError(rc, "tt_emb_create")

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream(self.device).cuda_stream)

    def forward(self, ids, out=None):
        torch = self.torch
        assert ids.dtype == torch.int64 and ids.is_contiguous() and ids.device == self.device
        B = ids.numel()
        if out is None:
            out = torch.empty((B, self.D), dtype=torch.float32, device=self.device)
        assert out.is_contiguous() and out.shape == (B, self.D) and out.dtype == torch.float32
        rc = tt_emb_forward(self.handle, ids.data_ptr() if B else 0, B, out.data_ptr() if B else 0,
                            self._stream())
        if rc:
            raise TTEmbError(rc, "tt_emb_forward")
        return out

    def forward_eval(self, ids, out=None):
        """Lookup without keeping anything for a backward pass."""
        torch = self.torch
        assert ids.dtype == torch.int64 and ids.is_contiguous() and ids.device == self.device
        B = ids.numel()
        if out is None:
            out = torch.empty((B, self.D), dtype=torch.float32, device=self.device)
        assert out.is_contiguous() and out.shape == (B, self.D) and out.dtype == torch.float32
        rc = tt_emb_forward_eval(self.handle, ids.data_ptr() if B else 0, B,
                                 out.data_ptr() if B else 0, self._stream())
        if rc:
            raise TTEmbError(rc, "tt_emb_forward_eval")
        return out

    def materialize(self, first_row: int = 0, count: int | None = None, out=None):
        """Rows first_row .. first_row+count-1 of the dense table the cores define."""
        torch = self.torch
        N = self.n[0] * self.n[1] * self.n[2]
        count = N - first_row if count is None else count
        if out is None:
            out = torch.empty((count, self.D), dtype=torch.float32, device=self.device)
        assert out.is_contiguous() and out.shape == (count, self.D) and out.dtype == torch.float32
        rc = tt_emb_materialize(self.handle, first_row, count, out.data_ptr() if count else 0,
                                self._stream())
        if rc:
            raise TTEmbError(rc, "tt_emb_materialize")
        return out

    def set_reindex(self, new_id_of):
        """Installs (or, with None, removes) an old-id -> table-row table: device int32 tensor."""
        torch = self.torch
        if new_id_of is None:
            self._reindex = None
            rc = tt_emb_set_reindex(self.handle, 0, 0)
        else:
            assert new_id_of.dtype == torch.int32 and new_id_of.is_contiguous()
            assert new_id_of.device == self.device
            self._reindex = new_id_of          # keeps the borrowed table alive
            rc = tt_emb_set_reindex(self.handle, new_id_of.data_ptr(), new_id_of.numel())
        if rc:
            raise TTEmbError(rc, "tt_emb_set_reindex")

    def set_adagrad(self, eps: float = 1e-10, enable: bool = True):
        """Switches backward_update to row-sparse Adagrad (state tensors are created here, zeroed)
        or back to SGD."""
        torch = self.torch
        if not enable:
            self.adagrad_state = None
            rc = tt_emb_set_adagrad(self.handle, 0, 0, 0, 0.0)
        else:
            self.adagrad_state = [torch.zeros_like(c) for c in self.cores]
            rc = tt_emb_set_adagrad(self.handle, *(t.data_ptr() for t in self.adagrad_state), eps)
        if rc:
            raise TTEmbError(rc, "tt_emb_set_adagrad")

    def set_adam(self, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                 enable: bool = True):
        """Switches backward_update to row-sparse Adam (moment tensors are created here, zeroed) or
        back to SGD."""
        torch = self.torch
        self.adagrad_state = None
        if not enable:
            self.adam_state = None
            rc = tt_emb_set_adam(self.handle, (0, 0, 0), (0, 0, 0), 0.0, 0.0, 0.0)
        else:
            self.adam_state = ([torch.zeros_like(c) for c in self.cores],
                               [torch.zeros_like(c) for c in self.cores])
            rc = tt_emb_set_adam(self.handle, [t.data_ptr() for t in self.adam_state[0]],
                                 [t.data_ptr() for t in self.adam_state[1]], beta1, beta2, eps)
        if rc:
            raise TTEmbError(rc, "tt_emb_set_adam")

    def wait_backward(self, age: int = 1):
        """Host-side flow control: returns once the backward_update made `age` calls before the
        latest one has finished on the device."""
        rc = tt_emb_wait_backward(self.handle, age)
        if rc:
            raise TTEmbError(rc, "tt_emb_wait_backward")

    def prepare(self, ids):
        """Index work of the next batch, overlapped with whatever follows on the current stream."""
        torch = self.torch
        assert ids.dtype == torch.int64 and ids.is_contiguous() and ids.device == self.device
        rc = tt_emb_prepare(self.handle, ids.data_ptr() if ids.numel() else 0, ids.numel(),
                            self._stream())
        if rc:
            raise TTEmbError(rc, "tt_emb_prepare")

    def backward_update(self, grad_out, lr: float):
        torch = self.torch
        assert grad_out.dtype == torch.float32 and grad_out.is_contiguous()
        assert grad_out.device == self.device
        rc = tt_emb_backward_update(self.handle, grad_out.data_ptr() if grad_out.numel() else 0,
                                    float(lr), self._stream())
        if rc:
            raise TTEmbError(rc, "tt_emb_backward_update")

    def stats(self, check: bool = True):
        rc, U, Q, oob = tt_emb_get_stats(self.handle)
        if rc and (check or rc not in (TT_EMB_ERANGE,)):
            raise TTEmbError(rc, "tt_emb_get_stats")
        return {"U": U, "Q": Q, "out_of_range": oob}

    def profile(self, enable: bool):
        rc = tt_emb_profile_enable(self.handle, enable)
        if rc:
            raise TTEmbError(rc, "tt_emb_profile_enable")

    def profile_read(self):
        res = {}
        for k in range(tt_emb_profile_slots()):
            rc, name, n, ms = tt_emb_profile_read(self.handle, k)
            if rc:
                raise TTEmbError(rc, "tt_emb_profile_read")
            res[name] = {"launches": n, "ms": ms}
        return res

    def close(self):
        if getattr(self, "handle", None) is not None:
            tt_emb_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
