"""Thin Python binding of liblocalcomm (include/localcomm.h).

Argument marshalling only: torch allocates device memory and owns the stream;
every step of the method runs in the library's HIP kernels.  There is no CPU
fallback: if the shared library is missing, loading fails with an error.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblocalcomm.so")

MAX_LAYERS = 8
KIND_QUAD, KIND_MLP = 0, 1
GEMM_FP32, GEMM_BF16 = 0, 1
SAMPLE_REPLACEMENT, SAMPLE_PARTITION = 0, 1
TIME_BWD, TIME_FWD, TIME_AVG, TIME_UPD, TIME_UPDAVG, TIME_NONE = 0, 1, 2, 3, 4, -1
# kernels of class TIME_BWD, for lc_timing_select()
BWD_ANY, BWD_ROW_OWNER, BWD_FIRST_LAYER, BWD_TILE_OWNER, BWD_HEAD, BWD_RESIDENT = 0, 1, 2, 3, 4, 5


class LcModel(C.Structure):
    _fields_ = [
        ("kind", C.c_int32),
        ("n_layers", C.c_int32),
        ("dims", C.c_int32 * (MAX_LAYERS + 1)),
        ("B", C.c_int32),
        ("N", C.c_int64),
        ("E", C.c_int32),
        ("lr", C.c_float),
        ("beta", C.c_float),
        ("wd", C.c_float),
        ("gemm", C.c_int32),
        ("sampler", C.c_int32),
    ]


class LcError(RuntimeError):
    def __init__(self, status: int, where: str, hip: int = 0):
        self.status = status
        msg = f"{where}: {_strerror(status)} ({status})"
        if hip:
            msg += f" [hipError {hip}]"
        super().__init__(msg)


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Load liblocalcomm.so (built by paper_1810_08313_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = C.CDLL(LIB_PATH)
    vp, mp = C.c_void_p, C.POINTER(LcModel)
    L.lc_strerror.restype = C.c_char_p
    L.lc_strerror.argtypes = [C.c_int]
    L.lc_last_hip_error.restype = C.c_int
    L.lc_last_hip_error.argtypes = [vp]
    L.lc_param_count.restype = C.c_int64
    L.lc_param_count.argtypes = [mp]
    L.lc_row_stride.restype = C.c_int64
    L.lc_row_stride.argtypes = [C.c_int64]
    L.lc_init.restype = C.c_int
    L.lc_init.argtypes = [C.c_int, C.c_int64, mp, C.c_uint64, C.POINTER(vp)]
    L.lc_destroy.restype = None
    L.lc_destroy.argtypes = [vp]
    L.lc_workspace_bytes.restype = C.c_size_t
    L.lc_workspace_bytes.argtypes = [vp]
    L.lc_attach.restype = C.c_int
    L.lc_attach.argtypes = [vp, vp, vp, vp, C.c_size_t, vp, vp, vp]
    L.lc_attach_quad.restype = C.c_int
    L.lc_attach_quad.argtypes = [vp, vp, vp]
    L.lc_local_steps.restype = C.c_int
    L.lc_local_steps.argtypes = [vp, C.c_int]
    L.lc_local_periods.restype = C.c_int
    L.lc_local_periods.argtypes = [vp, C.c_int, C.c_int]
    L.lc_average.restype = C.c_int
    L.lc_average.argtypes = [vp]
    L.lc_set_lazy_broadcast.restype = C.c_int
    L.lc_set_lazy_broadcast.argtypes = [vp, C.c_int]
    L.lc_set_implicit_momentum.restype = C.c_int
    L.lc_set_implicit_momentum.argtypes = [vp, C.c_int]
    L.lc_set_resident.restype = C.c_int
    L.lc_set_resident.argtypes = [vp, C.c_int]
    L.lc_set_fused_averaging.restype = C.c_int
    L.lc_set_fused_averaging.argtypes = [vp, C.c_int]
    L.lc_implicit_momentum_layers.restype = C.c_int
    L.lc_implicit_momentum_layers.argtypes = [vp]
    L.lc_resident_active.restype = C.c_int
    L.lc_resident_active.argtypes = [vp]
    L.lc_set_barrier_polls.restype = C.c_int
    L.lc_set_barrier_polls.argtypes = [vp, C.c_int]
    L.lc_materialize.restype = C.c_int
    L.lc_materialize.argtypes = [vp]
    L.lc_loss.restype = C.c_int
    L.lc_loss.argtypes = [vp, C.POINTER(C.c_double)]
    L.adacomm_next_tau.restype = C.c_int
    L.adacomm_next_tau.argtypes = [C.c_double, C.c_double, C.c_int]
    L.lc_run.restype = C.c_int
    L.lc_run.argtypes = [vp, C.c_int64, C.c_int, C.c_int, C.c_int64, C.POINTER(C.c_int64),
                         C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int64)]
    L.adacomm_next_tau_ex.restype = C.c_int
    L.adacomm_next_tau_ex.argtypes = [C.c_double, C.c_double, C.c_int, C.c_int, C.c_double, C.c_int, C.c_double,
                                      C.c_double, C.c_int]
    L.lc_run_ex.restype = C.c_int
    L.lc_run_ex.argtypes = [vp, C.c_int64, C.c_int, C.c_int64, C.c_int, C.c_double, C.c_int, C.c_int,
                            C.POINTER(C.c_int64), C.POINTER(C.c_float), C.c_int, C.POINTER(C.c_int64),
                            C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_int, C.POINTER(C.c_int32),
                            C.POINTER(C.c_int64)]
    L.lc_block_momentum_begin.restype = C.c_int
    L.lc_block_momentum_begin.argtypes = [vp, C.c_float]
    L.lc_block_momentum_end.restype = C.c_int
    L.lc_block_momentum_end.argtypes = [vp]
    L.lc_get_block_momentum.restype = C.c_int
    L.lc_get_block_momentum.argtypes = [vp, vp, vp]
    L.lc_set_grad.restype = C.c_int
    L.lc_set_grad.argtypes = [vp, vp]
    L.lc_update_from_grad.restype = C.c_int
    L.lc_update_from_grad.argtypes = [vp]
    L.lc_update_from_grad_and_average.restype = C.c_int
    L.lc_update_from_grad_and_average.argtypes = [vp]
    L.lc_get_state.restype = C.c_int
    L.lc_get_state.argtypes = [vp, vp, vp, C.POINTER(C.c_int64)]
    L.lc_set_state.restype = C.c_int
    L.lc_set_state.argtypes = [vp, vp, vp, C.c_int64]
    L.lc_set_lr.restype = C.c_int
    L.lc_set_lr.argtypes = [vp, C.c_float]
    L.lc_get_local_losses.restype = C.c_int
    L.lc_get_local_losses.argtypes = [vp, vp]
    L.lc_get_last_indices.restype = C.c_int
    L.lc_get_last_indices.argtypes = [vp, vp]
    L.lc_timing_begin.restype = C.c_int
    L.lc_timing_begin.argtypes = [vp, C.c_int]
    L.lc_average_block_momentum_static.restype = C.c_int
    L.lc_average_block_momentum_static.argtypes = [vp, vp, C.c_int, C.c_int64, C.c_int64, C.c_float, C.c_float,
                                                   C.c_int, vp]
    L.lc_timing_select.restype = C.c_int
    L.lc_timing_select.argtypes = [vp, C.c_int, C.c_int]
    L.lc_timing_read.restype = C.c_int
    L.lc_timing_read.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    _lib = L
    return L


def _strerror(status: int) -> str:
    return lib().lc_strerror(int(status)).decode()


def make_model(kind: int, dims: Sequence[int], B: int = 1, N: int = 1, E: int = 1, lr: float = 0.1,
               beta: float = 0.0, wd: float = 0.0, bf16: bool = False, sampler: int = 0) -> LcModel:
    md = LcModel()
    md.sampler = int(sampler)
    md.kind = kind
    md.n_layers = len(dims) - 1 if kind == KIND_MLP else 0
    for j, d in enumerate(dims):
        md.dims[j] = int(d)
    md.B, md.N, md.E = int(B), int(N), int(E)
    md.lr, md.beta, md.wd = float(lr), float(beta), float(wd)
    md.gemm = GEMM_BF16 if bf16 else GEMM_FP32
    return md


def lc_param_count(md: LcModel) -> int:
    return int(lib().lc_param_count(C.byref(md)))


def lc_row_stride(P: int) -> int:
    return int(lib().lc_row_stride(int(P)))


def adacomm_next_tau(F0: float, Fl: float, tau0: int) -> int:
    """AdaComm basic update rule; raises LcError on invalid input."""
    t = int(lib().adacomm_next_tau(float(F0), float(Fl), int(tau0)))
    if t < 0:
        raise LcError(t, "adacomm_next_tau")
    return t


STATIC_MAX_PARAMS = 4456448


def average_block_momentum_static(X, V, P: int, lr: float, beta_glob: float, begin: bool, stream=None) -> None:
    """lc_average_block_momentum_static on torch device tensors X (and V or None) of shape
    [m, row_stride]; raises LcError on a negative status."""
    import torch
    assert X.dtype == torch.float32 and X.is_contiguous() and X.dim() == 2
    st = (stream or torch.cuda.current_stream(X.device)).cuda_stream
    rc = lib().lc_average_block_momentum_static(X.data_ptr(), V.data_ptr() if V is not None else None, int(X.shape[0]),
                                                int(P), int(X.shape[1]), float(lr), float(beta_glob), int(bool(begin)), st)
    if rc != 0:
        raise LcError(rc, "lc_average_block_momentum_static")


def adacomm_next_tau_ex(F0: float, Fl: float, tau0: int, tau_prev: int, gamma: float = 0.5, slack: int = 0,
                        lr0: float = 1.0, lrl: float = 1.0, lr_changed: bool = False) -> int:
    """AdaComm with the saturation and learning-rate refinements; raises LcError on invalid input."""
    t = int(lib().adacomm_next_tau_ex(float(F0), float(Fl), int(tau0), int(tau_prev), float(gamma), int(slack),
                                      float(lr0), float(lrl), int(bool(lr_changed))))
    if t < 0:
        raise LcError(t, "adacomm_next_tau_ex")
    return t


class LocalSGD:
    """One m-replica run on the current CUDA/HIP device.

    Holds the torch tensors whose memory the library works on:
      X, V : fp32 [m, row_stride] (use .X[:, :P] for the logical view)
    """

    def __init__(self, m: int, md: LcModel, seed: int, x1: Optional[np.ndarray] = None,
                 data: Optional[np.ndarray] = None, labels: Optional[np.ndarray] = None,
                 qa: Optional[np.ndarray] = None, qc: Optional[np.ndarray] = None, device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("LocalSGD needs a GPU: there is no CPU path")
        self._torch = torch
        self._L = lib()
        self.m, self.md = int(m), md
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        P = lc_param_count(md)
        if P < 0:
            raise LcError(P, "lc_param_count")
        self.P, self.Ps = P, lc_row_stride(P)
        h = C.c_void_p()
        self._check(self._L.lc_init(self.m, P, C.byref(md), C.c_uint64(seed & (2**64 - 1)), C.byref(h)), "lc_init")
        self._h = h
        self.X = torch.zeros((self.m, self.Ps), dtype=torch.float32, device=self.device)
        self.V = torch.zeros((self.m, self.Ps), dtype=torch.float32, device=self.device)
        self.G = None
        ws = int(self._L.lc_workspace_bytes(self._h))
        self.scratch = torch.empty(ws, dtype=torch.uint8, device=self.device)
        self.data = self.labels = self.qa = self.qc = None
        if md.kind == KIND_MLP:
            d = torch.from_numpy(np.ascontiguousarray(data, dtype=np.float32))
            assert d.shape == (md.N, md.dims[0])
            self.data = d.to(self.device, dtype=torch.bfloat16 if md.gemm == GEMM_BF16 else torch.float32).contiguous()
            self.labels = torch.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)).to(self.device)
        self.stream = torch.cuda.current_stream(self.device)
        self._check(self._L.lc_attach(self._h, self.X.data_ptr(), self.V.data_ptr(), self.scratch.data_ptr(), ws,
                                      self.data.data_ptr() if self.data is not None else None,
                                      self.labels.data_ptr() if self.labels is not None else None,
                                      self.stream.cuda_stream), "lc_attach")
        if md.kind == KIND_QUAD:
            self.qa = self._padded(qa)
            self.qc = self._padded(qc)
            self._check(self._L.lc_attach_quad(self._h, self.qa.data_ptr(), self.qc.data_ptr()), "lc_attach_quad")
        if x1 is not None:
            x1 = np.ascontiguousarray(x1, dtype=np.float32).reshape(-1)
            assert x1.size == P
            self.set_state(np.broadcast_to(x1, (self.m, P)).copy(), np.zeros((self.m, P), np.float32), 0)

    # ---- helpers
    def _check(self, status: int, where: str) -> None:
        if status != 0:
            hip = int(self._L.lc_last_hip_error(self._h)) if getattr(self, "_h", None) else 0
            raise LcError(status, where, hip)

    def _padded(self, a: np.ndarray):
        torch = self._torch
        a = np.ascontiguousarray(a, dtype=np.float32)
        assert a.shape == (self.m, self.P)
        t = torch.zeros((self.m, self.Ps), dtype=torch.float32, device=self.device)
        t[:, :self.P] = torch.from_numpy(a).to(self.device)
        return t

    def close(self) -> None:
        if getattr(self, "_h", None):
            self._torch.cuda.synchronize(self.device)
            self._L.lc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the C ABI, one method per entry point
    def local_steps(self, tau: int) -> None:
        self._check(self._L.lc_local_steps(self._h, int(tau)), "lc_local_steps")

    def local_periods(self, tau: int, n_periods: int) -> None:
        self._check(self._L.lc_local_periods(self._h, int(tau), int(n_periods)), "lc_local_periods")

    def average(self) -> None:
        self._check(self._L.lc_average(self._h), "lc_average")

    def set_lazy_broadcast(self, on: bool) -> None:
        self._check(self._L.lc_set_lazy_broadcast(self._h, int(bool(on))), "lc_set_lazy_broadcast")

    def grid_search_tau0(self, taus, K: int):
        """lc_grid_search_tau0: (index of the best candidate, losses, seconds)."""
        arr = np.ascontiguousarray(taus, dtype=np.int32)
        loss = np.zeros(len(arr), np.float64)
        sec = np.zeros(len(arr), np.float64)
        best = C.c_int32(-1)
        self._check(self._L.lc_grid_search_tau0(self._h, arr.ctypes.data_as(C.c_void_p), len(arr), C.c_int64(int(K)),
                                                loss.ctypes.data_as(C.c_void_p), sec.ctypes.data_as(C.c_void_p),
                                                C.byref(best)), "lc_grid_search_tau0")
        return int(best.value), loss, sec

    def set_xcd_local_exchange(self, on: bool) -> None:
        self._check(self._L.lc_set_xcd_local_exchange(self._h, int(bool(on))), "lc_set_xcd_local_exchange")

    def set_deferred_update(self, on: bool) -> None:
        self._check(self._L.lc_set_deferred_update(self._h, int(bool(on))), "lc_set_deferred_update")

    def set_implicit_momentum(self, mode: int) -> None:
        """0 off, 1 where it pays (default), 2 wherever the kernels allow (see lc_set_implicit_momentum)."""
        self._check(self._L.lc_set_implicit_momentum(self._h, int(mode)), "lc_set_implicit_momentum")

    def set_first_layer_fusion(self, on: bool) -> None:
        self._check(self._L.lc_set_first_layer_fusion(self._h, int(bool(on))), "lc_set_first_layer_fusion")

    def set_resident(self, on) -> None:
        """False/0: launch-per-layer kernels; True/1: resident step kernel where it applies; 2: and
        in-kernel averaging steps at every shape it handles (see lc_local_periods)."""
        self._check(self._L.lc_set_resident(self._h, int(on)), "lc_set_resident")

    def set_fused_averaging(self, mode: int) -> None:
        """0 off, 1 the first layer, 2 large hidden layers too (default) (see lc_set_fused_averaging)."""
        self._check(self._L.lc_set_fused_averaging(self._h, int(mode)), "lc_set_fused_averaging")

    def implicit_momentum_layers(self) -> int:
        """Layers whose steps inside a period keep two consecutive models instead of model and momentum."""
        rc = self._L.lc_implicit_momentum_layers(self._h)
        self._check(min(rc, 0), "lc_implicit_momentum_layers")
        return rc

    def resident_active(self) -> bool:
        rc = self._L.lc_resident_active(self._h)
        self._check(min(rc, 0), "lc_resident_active")
        return rc == 1

    def set_barrier_polls(self, polls: int) -> None:
        self._check(self._L.lc_set_barrier_polls(self._h, int(polls)), "lc_set_barrier_polls")

    def materialize(self) -> None:
        self._check(self._L.lc_materialize(self._h), "lc_materialize")

    def loss(self) -> float:
        out = C.c_double(0.0)
        self._check(self._L.lc_loss(self._h, C.byref(out)), "lc_loss")
        return float(out.value)

    def run(self, K: int, tau0: int, adaptive: bool = False, interval: int = 0, cap: int = 4096
            ) -> Tuple[List[Tuple[int, int]], int]:
        sk = (C.c_int64 * cap)()
        st = (C.c_int32 * cap)()
        ns, rounds = C.c_int32(0), C.c_int64(0)
        self._check(self._L.lc_run(self._h, int(K), int(tau0), int(bool(adaptive)), int(interval), sk, st, cap,
                                   C.byref(ns), C.byref(rounds)), "lc_run")
        n = min(ns.value, cap)
        return [(int(sk[j]), int(st[j])) for j in range(n)], int(rounds.value)

    def run_ex(self, K: int, tau0: int, interval: int, refine: bool = True, gamma: float = 0.5, slack: int = 0,
               lr_schedule: Sequence[Tuple[int, float]] = (), postpone_lr: bool = True, cap: int = 4096):
        n = len(lr_schedule)
        at = (C.c_int64 * max(n, 1))(*[int(a) for a, _ in lr_schedule])
        val = (C.c_float * max(n, 1))(*[float(v) for _, v in lr_schedule])
        sk = (C.c_int64 * cap)()
        st = (C.c_int32 * cap)()
        sl = (C.c_float * cap)()
        ns, rounds = C.c_int32(0), C.c_int64(0)
        self._check(self._L.lc_run_ex(self._h, int(K), int(tau0), int(interval), int(bool(refine)), float(gamma),
                                      int(slack), n, at, val, int(bool(postpone_lr)), sk, st, sl, cap, C.byref(ns),
                                      C.byref(rounds)), "lc_run_ex")
        m = min(ns.value, cap)
        return [(int(sk[j]), int(st[j]), float(sl[j])) for j in range(m)], int(rounds.value)

    def block_momentum_begin(self, beta_glob: float) -> None:
        self._check(self._L.lc_block_momentum_begin(self._h, float(beta_glob)), "lc_block_momentum_begin")

    def block_momentum_end(self) -> None:
        self._check(self._L.lc_block_momentum_end(self._h), "lc_block_momentum_end")

    def get_block_momentum(self) -> Tuple[np.ndarray, np.ndarray]:
        u, xs = np.empty(self.P, np.float32), np.empty(self.P, np.float32)
        self._check(self._L.lc_get_block_momentum(self._h, u.ctypes.data, xs.ctypes.data), "lc_get_block_momentum")
        return u, xs

    def set_grad(self, G) -> None:
        """G: numpy [m, P] (copied, padded) or a torch device tensor [m, Ps]."""
        torch = self._torch
        if isinstance(G, np.ndarray):
            G = self._padded(G)
        assert G.shape == (self.m, self.Ps) and G.dtype == torch.float32 and G.is_contiguous()
        self.G = G
        self._check(self._L.lc_set_grad(self._h, G.data_ptr()), "lc_set_grad")

    def update_from_grad(self) -> None:
        self._check(self._L.lc_update_from_grad(self._h), "lc_update_from_grad")

    def update_from_grad_and_average(self) -> None:
        self._check(self._L.lc_update_from_grad_and_average(self._h), "lc_update_from_grad_and_average")

    def get_state(self) -> Tuple[np.ndarray, np.ndarray, int]:
        X = np.empty((self.m, self.P), np.float32)
        V = np.empty((self.m, self.P), np.float32)
        k = C.c_int64(0)
        self._check(self._L.lc_get_state(self._h, X.ctypes.data, V.ctypes.data, C.byref(k)), "lc_get_state")
        return X, V, int(k.value)

    @property
    def k(self) -> int:
        k = C.c_int64(0)
        self._check(self._L.lc_get_state(self._h, None, None, C.byref(k)), "lc_get_state")
        return int(k.value)

    def set_state(self, X: Optional[np.ndarray], V: Optional[np.ndarray], k: int) -> None:
        if X is not None:
            X = np.ascontiguousarray(X, dtype=np.float32)
            assert X.shape == (self.m, self.P)
        if V is not None:
            V = np.ascontiguousarray(V, dtype=np.float32)
            assert V.shape == (self.m, self.P)
        self._check(self._L.lc_set_state(self._h, X.ctypes.data if X is not None else None,
                                         V.ctypes.data if V is not None else None, int(k)), "lc_set_state")

    def set_lr(self, lr: float) -> None:
        self._check(self._L.lc_set_lr(self._h, float(lr)), "lc_set_lr")

    def local_losses(self) -> np.ndarray:
        out = np.empty(self.m, np.float32)
        self._check(self._L.lc_get_local_losses(self._h, out.ctypes.data), "lc_get_local_losses")
        return out

    def last_indices(self) -> np.ndarray:
        out = np.empty((self.m, self.md.B), np.int32)
        self._check(self._L.lc_get_last_indices(self._h, out.ctypes.data), "lc_get_last_indices")
        return out

    def timing_begin(self, which: int) -> None:
        self._check(self._L.lc_timing_begin(self._h, int(which)), "lc_timing_begin")

    def timing_select(self, layer: int, kernel: int) -> None:
        self._check(self._L.lc_timing_select(self._h, int(layer), int(kernel)), "lc_timing_select")

    def timing_read(self) -> Tuple[int, float]:
        n, ms = C.c_int64(0), C.c_double(0.0)
        self._check(self._L.lc_timing_read(self._h, C.byref(n), C.byref(ms)), "lc_timing_read")
        return int(n.value), float(ms.value)
