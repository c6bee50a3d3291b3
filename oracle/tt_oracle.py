"""Python face of the CPU oracle (oracle/tt_emb_oracle.c).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the CPU-baseline leg of the benchmark
may import this module; nothing on the product path does.  It never imports the GPU package.

Two shared objects are built from the one C source with gcc:
  * ``libtt_oracle_f64.so``  every accumulator is a double; this is the parity reference;
  * ``libtt_oracle_f32.so``  the same loops with float accumulators; only ever timed.
Both use OpenMP over batch positions.

Arrays are numpy, cores are fp32 in slice-contiguous layout:
  g1[n1, d1, r1], g2[n2, r1, d2, r2], g3[n3, r2, d3].
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tt_emb_oracle.c")


class _CShape(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64 * 3), ("d", ctypes.c_int32 * 3), ("r", ctypes.c_int32 * 2)]


@dataclass(frozen=True)
class Shape:
    """Factorisation of the table: N = n1*n2*n3 rows of D = d1*d2*d3 floats, ranks (1, r1, r2, 1)."""

    n: tuple
    d: tuple
    r: tuple

    @property
    def N(self) -> int:
        return int(self.n[0]) * int(self.n[1]) * int(self.n[2])

    @property
    def D(self) -> int:
        return int(self.d[0]) * int(self.d[1]) * int(self.d[2])

    def core_shapes(self):
        (n1, n2, n3), (d1, d2, d3), (r1, r2) = self.n, self.d, self.r
        return (n1, d1, r1), (n2, r1, d2, r2), (n3, r2, d3)

    def _c(self) -> _CShape:
        c = _CShape()
        for k in range(3):
            c.n[k] = int(self.n[k])
            c.d[k] = int(self.d[k])
        c.r[0], c.r[1] = int(self.r[0]), int(self.r[1])
        return c


def build(force: bool = False) -> None:
    """Compile both shared objects with gcc (a few seconds)."""
    for tag, acc in (("f64", "double"), ("f32", "float")):
        out = os.path.join(_HERE, f"libtt_oracle_{tag}.so")
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O3", "-march=native", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               f"-DTT_ACC={acc}", _SRC, "-o", out]
        subprocess.run(cmd, check=True)


_LIBS: dict = {}


def _lib(tag: str):
    if tag in _LIBS:
        return _LIBS[tag]
    build()
    lib = ctypes.CDLL(os.path.join(_HERE, f"libtt_oracle_{tag}.so"))
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    sp = ctypes.POINTER(_CShape)
    lib.tto_param_count.restype = i64
    lib.tto_param_count.argtypes = [sp]
    lib.tto_decompose.restype = ctypes.c_int
    lib.tto_decompose.argtypes = [sp, i64] + [ctypes.POINTER(i64)] * 3
    lib.tto_forward.restype = None
    lib.tto_forward.argtypes = [sp, vp, vp, vp, vp, i64, vp]
    lib.tto_forward_acc.restype = None
    lib.tto_forward_acc.argtypes = [sp, vp, vp, vp, vp, i64, vp]
    lib.tto_grads.restype = None
    lib.tto_grads.argtypes = [sp, vp, vp, vp, vp, i64, vp, vp, vp, vp]
    lib.tto_backward_update.restype = None
    lib.tto_backward_update.argtypes = [sp, vp, vp, vp, vp, i64, vp, ctypes.c_float]
    lib.tto_threads.restype = ctypes.c_int
    lib.tto_acc_bytes.restype = ctypes.c_int
    _LIBS[tag] = lib
    return lib


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _check_cores(shape: Shape, g1, g2, g3):
    for g, cs in zip((g1, g2, g3), shape.core_shapes()):
        assert g.dtype == np.float32 and g.flags.c_contiguous, "cores are C-contiguous fp32"
        assert tuple(g.shape) == tuple(cs), (g.shape, cs)


def _ids(ids) -> np.ndarray:
    return np.ascontiguousarray(ids, dtype=np.int64)


def threads(tag: str = "f64") -> int:
    return int(_lib(tag).tto_threads())


def param_count(shape: Shape) -> int:
    c = shape._c()
    return int(_lib("f64").tto_param_count(ctypes.byref(c)))


def decompose(shape: Shape, node_id: int):
    """(i1, i2, i3) of a node id, or None when the id is outside the table."""
    c = shape._c()
    a, b, d = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    ok = _lib("f64").tto_decompose(ctypes.byref(c), int(node_id), ctypes.byref(a), ctypes.byref(b),
                                   ctypes.byref(d))
    return (a.value, b.value, d.value) if ok else None


def forward(shape: Shape, g1, g2, g3, ids, tag: str = "f64") -> np.ndarray:
    """Embedding rows out[B, D] in fp32 (accumulated in the build's accumulator type)."""
    _check_cores(shape, g1, g2, g3)
    ids = _ids(ids)
    out = np.empty((ids.size, shape.D), dtype=np.float32)
    c = shape._c()
    _lib(tag).tto_forward(ctypes.byref(c), _p(g1), _p(g2), _p(g3), _p(ids), ids.size, _p(out))
    return out


def forward_f64(shape: Shape, g1, g2, g3, ids) -> np.ndarray:
    """Embedding rows out[B, D] kept in fp64 (no rounding)."""
    _check_cores(shape, g1, g2, g3)
    ids = _ids(ids)
    out = np.empty((ids.size, shape.D), dtype=np.float64)
    c = shape._c()
    _lib("f64").tto_forward_acc(ctypes.byref(c), _p(g1), _p(g2), _p(g3), _p(ids), ids.size, _p(out))
    return out


def grads(shape: Shape, g1, g2, g3, ids, grad, tag: str = "f64"):
    """Core gradients (dG1, dG2, dG3) of L = sum_b <grad_b, row_b>, in the accumulator type."""
    _check_cores(shape, g1, g2, g3)
    ids = _ids(ids)
    grad = np.ascontiguousarray(grad, dtype=np.float32)
    assert grad.shape == (ids.size, shape.D)
    dt = np.float64 if tag == "f64" else np.float32
    dg = [np.empty(cs, dtype=dt) for cs in shape.core_shapes()]
    c = shape._c()
    _lib(tag).tto_grads(ctypes.byref(c), _p(g1), _p(g2), _p(g3), _p(ids), ids.size, _p(grad),
                        _p(dg[0]), _p(dg[1]), _p(dg[2]))
    return tuple(dg)


def backward_update(shape: Shape, g1, g2, g3, ids, grad, lr: float, tag: str = "f64"):
    """One SGD step; returns NEW core arrays (the inputs are left untouched)."""
    _check_cores(shape, g1, g2, g3)
    ids = _ids(ids)
    grad = np.ascontiguousarray(grad, dtype=np.float32)
    assert grad.shape == (ids.size, shape.D)
    n1, n2, n3 = g1.copy(), g2.copy(), g3.copy()
    c = shape._c()
    _lib(tag).tto_backward_update(ctypes.byref(c), _p(n1), _p(n2), _p(n3), _p(ids), ids.size,
                                  _p(grad), ctypes.c_float(lr))
    return n1, n2, n3


def adagrad_update(shape: Shape, g1, g2, g3, state, ids, grad, lr: float, eps: float):
    """One Adagrad step on the batch-summed core gradients (the paper names no optimiser; this is
    the textbook rule, elementwise per core):  S <- S + dG^2,  G <- G - lr * dG / (sqrt(S) + eps).
    fp64 throughout, rounded to fp32 once.  Entries no id touches have dG = 0 and stay as they are.
    Returns (new cores, new state); the inputs are left untouched."""
    dg = grads(shape, g1, g2, g3, ids, grad)
    new_cores, new_state = [], []
    for G, S, d in zip((g1, g2, g3), state, dg):
        s64 = S.astype(np.float64) + d * d
        g64 = G.astype(np.float64) - lr * d / (np.sqrt(s64) + eps)
        new_state.append(s64.astype(np.float32))
        new_cores.append(g64.astype(np.float32))
    return tuple(new_cores), tuple(new_state)


def touched_slices(shape: Shape, ids):
    """Boolean masks over the slices of the three cores: which G1[i1], G2[i2], G3[i3] some in-range
    id of the batch selects (index split of Section 3)."""
    ids = _ids(ids)
    ok = ids[(ids >= 0) & (ids < shape.N)]
    n1, n2, n3 = shape.n
    masks = [np.zeros(n, dtype=bool) for n in (n1, n2, n3)]
    masks[0][ok // (n2 * n3)] = True
    masks[1][(ok // n3) % n2] = True
    masks[2][ok % n3] = True
    return masks


def adam_update(shape: Shape, g1, g2, g3, m, v, step: int, ids, grad, lr: float,
                beta1: float, beta2: float, eps: float):
    """One Adam step in the row-sparse ("lazy") form on the batch-summed core gradients; the paper
    names no optimiser, this is the textbook rule (Kingma & Ba, Algorithm 1) applied to the slices
    the batch touches and to nothing else:
        m <- beta1 m + (1 - beta1) dG,   v <- beta2 v + (1 - beta2) dG^2,
        G <- G - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps),   t = step = 1, 2, ...
    Slices no id touches keep core, m and v as they are (their moments do not decay).  fp64
    throughout, rounded to fp32 once.  Returns (new cores, new m, new v)."""
    assert step >= 1
    dg = grads(shape, g1, g2, g3, ids, grad)
    masks = touched_slices(shape, ids)
    c1, c2 = 1.0 - beta1 ** step, 1.0 - beta2 ** step
    out_g, out_m, out_v = [], [], []
    for G, M, V, d, mask in zip((g1, g2, g3), m, v, dg, masks):
        G64, M64, V64 = G.astype(np.float64), M.astype(np.float64), V.astype(np.float64)
        t = mask.reshape((-1,) + (1,) * (G.ndim - 1))        # broadcast over the slice
        m_new = beta1 * M64 + (1.0 - beta1) * d
        v_new = beta2 * V64 + (1.0 - beta2) * d * d
        g_new = G64 - lr * (m_new / c1) / (np.sqrt(v_new / c2) + eps)
        out_m.append(np.where(t, m_new, M64).astype(np.float32))
        out_v.append(np.where(t, v_new, V64).astype(np.float32))
        out_g.append(np.where(t, g_new, G64).astype(np.float32))
    return tuple(out_g), tuple(out_m), tuple(out_v)

