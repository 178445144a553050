"""ctypes binding of the C oracle (oracle/pasgd_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg; never by the HIP path.  It imports nothing from
the product package.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .build import LIB, LIB_F32ACC, build

MAX_LAYERS = 8
KIND_QUAD, KIND_MLP = 0, 1


class OrcModel(C.Structure):
    _fields_ = [
        ("kind", C.c_int),
        ("n_layers", C.c_int),
        ("dims", C.c_int * (MAX_LAYERS + 1)),
        ("B", C.c_int),
        ("N", C.c_int64),
        ("E", C.c_int),
        ("lr", C.c_float),
        ("beta", C.c_float),
        ("wd", C.c_float),
        ("bf16", C.c_int),
        ("sampler", C.c_int),
    ]


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB):
        build()
    L = C.CDLL(LIB)
    fp, ip, lp = C.POINTER(C.c_float), C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    mp = C.POINTER(OrcModel)
    L.orc_mix64.restype = C.c_uint64
    L.orc_mix64.argtypes = [C.c_uint64]
    L.orc_index.restype = C.c_int64
    L.orc_index.argtypes = [C.c_uint64, C.c_int, C.c_int64, C.c_int, C.c_int64]
    L.orc_index_partition.restype = C.c_int64
    L.orc_index_partition.argtypes = [C.c_uint64, C.c_int, C.c_int64, C.c_int, C.c_int64, C.c_int, C.c_int]
    L.orc_bf16_round.restype = C.c_float
    L.orc_bf16_round.argtypes = [C.c_float]
    L.orc_param_count.restype = C.c_int64
    L.orc_param_count.argtypes = [mp]
    L.orc_mlp_loss_grad.restype = C.c_float
    L.orc_mlp_loss_grad.argtypes = [mp, fp, fp, ip, lp, fp]
    L.orc_mlp_preactivations.restype = None
    L.orc_mlp_preactivations.argtypes = [mp, fp, fp, lp, fp]
    L.orc_sgd_update.restype = None
    L.orc_sgd_update.argtypes = [C.c_int64, fp, fp, fp, C.c_float, C.c_float, C.c_float]
    L.orc_next_tau.restype = C.c_int
    L.orc_next_tau.argtypes = [C.c_double, C.c_double, C.c_int]
    L.orc_create.restype = C.c_void_p
    L.orc_create.argtypes = [C.c_int, mp, C.c_uint64, fp, fp, ip, fp, fp]
    L.orc_destroy.restype = None
    L.orc_destroy.argtypes = [C.c_void_p]
    L.orc_set_threads.restype = C.c_int
    L.orc_set_threads.argtypes = [C.c_int]
    L.orc_set_lr.restype = None
    L.orc_set_lr.argtypes = [C.c_void_p, C.c_float]
    L.orc_k.restype = C.c_int64
    L.orc_k.argtypes = [C.c_void_p]
    L.orc_X.restype = fp
    L.orc_X.argtypes = [C.c_void_p]
    L.orc_V.restype = fp
    L.orc_V.argtypes = [C.c_void_p]
    L.orc_last_losses.restype = fp
    L.orc_last_losses.argtypes = [C.c_void_p]
    L.orc_local_steps.restype = None
    L.orc_local_steps.argtypes = [C.c_void_p, C.c_int]
    L.orc_local_steps_subset.restype = None
    L.orc_local_steps_subset.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_int), C.c_int]
    L.orc_update_from_grad.restype = None
    L.orc_update_from_grad.argtypes = [C.c_void_p, fp]
    L.orc_average.restype = None
    L.orc_average.argtypes = [C.c_void_p]
    L.orc_loss.restype = C.c_double
    L.orc_loss.argtypes = [C.c_void_p]
    L.orc_run.restype = C.c_int
    L.orc_run.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_int64, lp, C.POINTER(C.c_int),
                          C.c_int, C.POINTER(C.c_int), lp]
    L.orc_block_begin.restype = None
    L.orc_block_begin.argtypes = [C.c_void_p, C.c_float]
    L.orc_block_end.restype = None
    L.orc_block_end.argtypes = [C.c_void_p]
    L.orc_block_u.restype = fp
    L.orc_block_u.argtypes = [C.c_void_p]
    L.orc_next_tau_ex.restype = C.c_int
    L.orc_next_tau_ex.argtypes = [C.c_double, C.c_double, C.c_int, C.c_int, C.c_double, C.c_int, C.c_double,
                                  C.c_double, C.c_int]
    L.orc_run_ex.restype = C.c_int
    L.orc_run_ex.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int64, C.c_int, C.c_double, C.c_int, C.c_int, lp, fp,
                             C.c_int, lp, C.POINTER(C.c_int), fp, C.c_int, C.POINTER(C.c_int), lp]
    L.orc_acc_bytes.restype = C.c_int
    L.orc_acc_bytes.argtypes = []
    assert L.orc_acc_bytes() == 8, "the oracle accumulates in double"
    _lib = L
    return L


_probe = None


def f32acc_probe() -> C.CDLL:
    """The same source compiled with fp32 accumulators in the matrix products (same order of
    additions).  A sensitivity probe: tests use it to SHOW how far gradients move and which ReLU
    gates change side when only the summation precision changes.  Only the two stateless pieces
    are exposed, and nothing is ever compared with the HIP path through it."""
    global _probe
    if _probe is not None:
        return _probe
    if not os.path.exists(LIB_F32ACC):
        build()
    L = C.CDLL(LIB_F32ACC)
    fp, ip, lp = C.POINTER(C.c_float), C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    mp = C.POINTER(OrcModel)
    L.orc_acc_bytes.restype = C.c_int
    L.orc_acc_bytes.argtypes = []
    assert L.orc_acc_bytes() == 4
    L.orc_mlp_loss_grad.restype = C.c_float
    L.orc_mlp_loss_grad.argtypes = [mp, fp, fp, ip, lp, fp]
    L.orc_mlp_preactivations.restype = None
    L.orc_mlp_preactivations.argtypes = [mp, fp, fp, lp, fp]
    _probe = L
    return L


def _f(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def make_model(kind: int, dims: Sequence[int], B: int = 1, N: int = 1, E: int = 1, lr: float = 0.1,
               beta: float = 0.0, wd: float = 0.0, bf16: bool = False, sampler: int = 0) -> OrcModel:
    md = OrcModel()
    md.sampler = int(sampler)
    md.kind = kind
    md.n_layers = len(dims) - 1 if kind == KIND_MLP else 0
    for j, d in enumerate(dims):
        md.dims[j] = int(d)
    md.B, md.N, md.E = int(B), int(N), int(E)
    md.lr, md.beta, md.wd = float(lr), float(beta), float(wd)
    md.bf16 = int(bool(bf16))
    return md


def mix64(z: int) -> int:
    return int(lib().orc_mix64(C.c_uint64(z & (2**64 - 1))))


def index(seed: int, i: int, k: int, b: int, N: int) -> int:
    return int(lib().orc_index(C.c_uint64(seed & (2**64 - 1)), i, k, b, N))


def index_partition(seed: int, i: int, k: int, b: int, N: int, m: int, B: int) -> int:
    return int(lib().orc_index_partition(C.c_uint64(seed & (2**64 - 1)), i, k, b, N, m, B))


def bf16_round(a) -> np.ndarray:
    a = np.asarray(a, dtype=np.float32)
    out = np.empty_like(a)
    L = lib()
    flat_in, flat_out = a.reshape(-1), out.reshape(-1)
    for j in range(flat_in.size):
        flat_out[j] = L.orc_bf16_round(C.c_float(float(flat_in[j])))
    return out


def next_tau(F0: float, Fl: float, tau0: int) -> int:
    return int(lib().orc_next_tau(float(F0), float(Fl), int(tau0)))


def next_tau_ex(F0: float, Fl: float, tau0: int, tau_prev: int, gamma: float = 0.5, slack: int = 0,
                lr0: float = 1.0, lrl: float = 1.0, lr_changed: bool = False) -> int:
    return int(lib().orc_next_tau_ex(float(F0), float(Fl), int(tau0), int(tau_prev), float(gamma), int(slack),
                                     float(lr0), float(lrl), int(bool(lr_changed))))


def mlp_loss_grad(md: OrcModel, x: np.ndarray, data: np.ndarray, labels: np.ndarray,
                  idx: Sequence[int], want_grad: bool = True, f32acc: bool = False) -> Tuple[float, Optional[np.ndarray]]:
    """f32acc=True asks the fp32-accumulation probe instead of the oracle (sensitivity only)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    data = np.ascontiguousarray(data, dtype=np.float32)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    ix = np.ascontiguousarray(idx, dtype=np.int64)
    assert ix.size == md.B
    g = np.zeros_like(x) if want_grad else None
    L = f32acc_probe() if f32acc else lib()
    loss = L.orc_mlp_loss_grad(C.byref(md), _f(x), _f(data), labels.ctypes.data_as(C.POINTER(C.c_int32)),
                                   ix.ctypes.data_as(C.POINTER(C.c_int64)), _f(g) if want_grad else None)
    return float(loss), g


def mlp_preactivations(md: OrcModel, x: np.ndarray, data: np.ndarray, idx: Sequence[int],
                       f32acc: bool = False) -> List[np.ndarray]:
    """Pre-ReLU values of the hidden layers, one [B, d_l] array per hidden layer.
    f32acc=True asks the fp32-accumulation probe instead of the oracle (sensitivity only)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    data = np.ascontiguousarray(data, dtype=np.float32)
    ix = np.ascontiguousarray(idx, dtype=np.int64)
    hidden = [md.dims[l] for l in range(1, md.n_layers)]
    z = np.zeros((md.B, max(1, sum(hidden))), np.float32)
    if hidden:
        L = f32acc_probe() if f32acc else lib()
        L.orc_mlp_preactivations(C.byref(md), _f(x), _f(data), ix.ctypes.data_as(C.POINTER(C.c_int64)), _f(z))
    out, o = [], 0
    for d in hidden:
        out.append(z[:, o:o + d].copy())
        o += d
    return out


def sgd_update(x: np.ndarray, v: np.ndarray, g: np.ndarray, lr: float, beta: float, wd: float) -> None:
    assert x.dtype == v.dtype == g.dtype == np.float32
    lib().orc_sgd_update(x.size, _f(x), _f(v), _f(g), lr, beta, wd)


def set_threads(n: int) -> int:
    return int(lib().orc_set_threads(int(n)))


class Run:
    """One m-worker PASGD run held by the oracle."""

    def __init__(self, m: int, md: OrcModel, seed: int, x1: np.ndarray,
                 data: Optional[np.ndarray] = None, labels: Optional[np.ndarray] = None,
                 qa: Optional[np.ndarray] = None, qc: Optional[np.ndarray] = None):
        self.m, self.md = int(m), md
        self._keep: List[np.ndarray] = []

        def keep(a, dt):
            if a is None:
                return None
            a = np.ascontiguousarray(a, dtype=dt)
            self._keep.append(a)
            return a

        x1 = keep(x1, np.float32)
        data, labels = keep(data, np.float32), keep(labels, np.int32)
        qa, qc = keep(qa, np.float32), keep(qc, np.float32)
        self.P = int(x1.size)
        if md.kind == KIND_MLP:
            assert self.P == lib().orc_param_count(C.byref(md))
            assert data.shape == (md.N, md.dims[0]) and labels.shape == (md.N,)
        else:
            assert md.dims[0] == self.P and qa.shape == (m, self.P) and qc.shape == (m, self.P)
        self._h = lib().orc_create(
            m, C.byref(md), C.c_uint64(seed & (2**64 - 1)), _f(x1),
            _f(data) if data is not None else None,
            labels.ctypes.data_as(C.POINTER(C.c_int32)) if labels is not None else None,
            _f(qa) if qa is not None else None, _f(qc) if qc is not None else None)

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_destroy(self._h)
            self._h = None

    @property
    def X(self) -> np.ndarray:  # live view [m,P]
        return np.ctypeslib.as_array(lib().orc_X(self._h), shape=(self.m, self.P))

    @property
    def V(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().orc_V(self._h), shape=(self.m, self.P))

    @property
    def k(self) -> int:
        return int(lib().orc_k(self._h))

    @property
    def last_losses(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().orc_last_losses(self._h), shape=(self.m,)).copy()

    def set_lr(self, lr: float) -> None:
        lib().orc_set_lr(self._h, lr)

    def local_steps(self, tau: int, ids: Optional[Sequence[int]] = None) -> None:
        if ids is None:
            lib().orc_local_steps(self._h, int(tau))
        else:
            arr = (C.c_int * len(ids))(*[int(i) for i in ids])
            lib().orc_local_steps_subset(self._h, int(tau), arr, len(ids))

    def update_from_grad(self, G: np.ndarray) -> None:
        G = np.ascontiguousarray(G, dtype=np.float32)
        assert G.shape == (self.m, self.P)
        lib().orc_update_from_grad(self._h, _f(G))

    def average(self) -> None:
        lib().orc_average(self._h)

    def loss(self) -> float:
        return float(lib().orc_loss(self._h))

    def block_begin(self, beta_glob: float) -> None:
        lib().orc_block_begin(self._h, float(beta_glob))

    def block_end(self) -> None:
        lib().orc_block_end(self._h)

    @property
    def block_u(self) -> np.ndarray:
        return np.ctypeslib.as_array(lib().orc_block_u(self._h), shape=(self.P,)).copy()

    def run(self, K: int, tau0: int, adaptive: bool = False, interval: int = 0, cap: int = 4096):
        sk = (C.c_int64 * cap)()
        st = (C.c_int * cap)()
        ns, rounds = C.c_int(0), C.c_int64(0)
        rc = lib().orc_run(self._h, int(K), int(tau0), int(bool(adaptive)), int(interval), sk, st, cap,
                           C.byref(ns), C.byref(rounds))
        if rc != 0:
            raise RuntimeError(f"orc_run failed: {rc}")
        n = min(ns.value, cap)
        return [(int(sk[j]), int(st[j])) for j in range(n)], int(rounds.value)

    def run_ex(self, K: int, tau0: int, interval: int, refine: bool = True, gamma: float = 0.5, slack: int = 0,
               lr_schedule: Sequence[Tuple[int, float]] = (), postpone_lr: bool = True, cap: int = 4096):
        """Driver with the AdaComm refinements; returns ([(k, tau, lr)], rounds)."""
        n = len(lr_schedule)
        at = (C.c_int64 * max(n, 1))(*[int(a) for a, _ in lr_schedule])
        val = (C.c_float * max(n, 1))(*[float(v) for _, v in lr_schedule])
        sk = (C.c_int64 * cap)()
        st = (C.c_int * cap)()
        sl = (C.c_float * cap)()
        ns, rounds = C.c_int(0), C.c_int64(0)
        rc = lib().orc_run_ex(self._h, int(K), int(tau0), int(interval), int(bool(refine)), float(gamma), int(slack),
                              n, at, val, int(bool(postpone_lr)), sk, st, sl, cap, C.byref(ns), C.byref(rounds))
        if rc != 0:
            raise RuntimeError(f"orc_run_ex failed: {rc}")
        m = min(ns.value, cap)
        return [(int(sk[j]), int(st[j]), float(sl[j])) for j in range(m)], int(rounds.value)
