"""Which ReLU gates can the summation order decide?  Host-side helper of the GPU parity tests.

ReLU'(z) is a step at zero.  The oracle adds every product in double, the GPU adds in fp32 on the
matrix cores, so the two pre-activations of one unit and sample differ by summation error.  Where
the oracle's |z| is smaller than that difference the gate may open on one side and stay shut on the
other; both outcomes are valid results of the method, and the unit's own column of dW_l (one of B
terms) then differs by far more than any tolerance.  Such units are left out of their own layer's
comparison -- and only those, so the bound has to be tight.  It is an interval propagation over the
oracle's own forward pass, layer by layer:

    dz_l[b, j]  bound on |z_gpu - z_oracle| for sample b, unit j of hidden layer l
      = eps_sum * max(1, rms(z_l))                        fp32 against double summation
      + min(sum_k t_k, IN_SIGMAS * sqrt(sum_k t_k^2)),  t_k = da_{l-1}[b, k] |W_l[k, j]|   uncertainty of the layer's inputs
      + the same with t_k = |a_{l-1}[b, k]| dw_l[k, j]                                     uncertainty of the weight operand
    da_l[b, k]  bound on the difference of the activations handed to the next layer
      fp32 operands:  dz_l[b, k]                           (continuous)
      bf16 operands:  one bf16 ulp where relu(z) lies within dz of a bf16 rounding boundary,
                      else 0                               (the rounding absorbs smaller changes)
    dw_l[k, j]   0 while both sides hold bit-identical master weights (right after the state was
                 set from the oracle, x = x0).  After unforced steps the masters differ, because the
                 gradients of the steps in between do (by summation order with fp32 operands; with
                 bf16 operands also by activations and deltas that rounded the other way):
                     |x_gpu - x| <= REL_GRAD * (|x - x0| + rms of |x - x0| over the layer) + 2 ulp
                 i.e. a share of the distance travelled since the state was forced.  fp32 operands
                 take that as it is; bf16 operands take one bf16 ulp for the weights whose master
                 lies that close to a point where its bf16 rounding changes.
                 A unit that had an undecided gate in an earlier unforced step (`suspect`) is another
                 matter: if its gate did fall the other way, its whole column of W_l differs by one
                 sample's term of that step's update, which is of the size of the column's movement
                 itself.  For such columns dw = |x - x0| + rms, with any operands, and what their
                 activations then may differ by reaches the layer above like any other input
                 uncertainty.

A gate is undecided where |z_l[b, j]| <= dz_l[b, j]; a unit is masked when any sample's gate is.
Inputs (layer 0) are exact on both sides.  All of it uses oracle values only.

Both uncertainty terms are capped by a root-sum-square instead of the sum of magnitudes: with bf16 operands from the third
layer on, most activations of an affected sample could round either way, few of them do, and the
signs are mixed; the plain sum would flag a quarter of a 2048-unit layer per step where the fp32-
accumulation build of the oracle's source moves z by a tenth of that bound (tests/
test_gate_bounds.py measures both).  A bound that is too small cannot hide a defect: a gate that
flips without being masked makes the comparison fail, not pass.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

EPS_SUM = 4e-6       # fp32 MFMA accumulation against the double sum, relative to the layer's rms (K <= 3072 terms)
IN_SIGMAS = 4.0      # root-sum-square of the input uncertainties, times this
REL_GRAD_BF16 = 1e-4        # relative discrepancy of an accumulated gradient entry, bf16 operands (measured: up to 5e-5)
REL_GRAD_F32 = 1e-5         # ... fp32 operands (measured: 2e-6)


def _ulp32(v: np.ndarray) -> np.ndarray:
    """Spacing of fp32 numbers at |v| (as float64)."""
    v = np.abs(np.asarray(v, np.float32))
    e = np.frexp(np.maximum(v, np.float32(1.2e-38)))[1]     # v = f * 2^e, 0.5 <= f < 1
    return np.ldexp(1.0, e - 24)


def _to_boundary_ulps(v: np.ndarray) -> np.ndarray:
    """Distance of fp32 v from the nearest point where its bf16 rounding changes (the midpoint
    between two neighbouring bf16 values), in fp32 ulps."""
    low = (np.asarray(v, np.float32).view(np.uint32) & np.uint32(0xFFFF)).astype(np.int64)
    return np.abs(low - 0x8000).astype(np.float64)


def _bf16(v: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(v, np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + (((u >> 16) & 1) + 0x7FFF)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(np.shape(v))


def undecided_gates(orc, omd, x: np.ndarray, data: np.ndarray, idx: Sequence[int],
                    x0: np.ndarray = None, eps_sum: float = EPS_SUM,
                    suspect: Dict[int, np.ndarray] = None) -> Dict[int, np.ndarray]:
    """{hidden layer l: bool [B, d_l]} of the gates that summation order may decide, for one
    worker with master parameters x on the samples idx.  x0: the parameters at which both sides
    were last bit-identical (None: they are now).  suspect: {layer: bool [d_l]} units that had an
    undecided gate in a step since then."""
    L = omd.n_layers
    dims = [omd.dims[l] for l in range(L + 1)]
    bf16 = bool(omd.bf16)
    zs = orc.mlp_preactivations(omd, x, data, idx)
    a = np.abs(np.asarray(data, np.float32)[np.asarray(idx)].astype(np.float64))
    da = np.zeros_like(a)
    out, off = {}, 0
    for l in range(1, L):
        din, dout = dims[l - 1], dims[l]
        W = np.asarray(x[off:off + din * dout], np.float32).reshape(din, dout)
        off += din * dout + dout
        Wabs = np.abs((_bf16(W) if bf16 else W).astype(np.float64))
        z = zs[l - 1].astype(np.float64)
        rms = max(1.0, float(np.sqrt(np.mean(z * z))))
        dz = np.full_like(z, eps_sum * rms)
        if da.any():
            dz += np.minimum(da @ Wabs, IN_SIGMAS * np.sqrt((da * da) @ (Wabs * Wabs)))
        if x0 is not None:
            moved = np.abs(W.astype(np.float64) - np.asarray(x0[off - din * dout - dout:off - dout], np.float32)
                           .reshape(din, dout).astype(np.float64))
            rel = REL_GRAD_BF16 if bf16 else REL_GRAD_F32
            drift = rel * (moved + np.sqrt(np.mean(moved * moved))) + 2.0 * _ulp32(W)
            if bf16:
                dw = np.where(_to_boundary_ulps(W) * _ulp32(W) <= drift, 65536.0 * _ulp32(W), 0.0)
            else:
                dw = drift
            if suspect and l in suspect and suspect[l].any():
                dw[:, suspect[l]] = (moved + np.sqrt(np.mean(moved * moved)))[:, suspect[l]]
            dz += np.minimum(a @ dw, IN_SIGMAS * np.sqrt((a * a) @ (dw * dw)))
        out[l] = np.abs(z) <= dz
        act = np.maximum(zs[l - 1], np.float32(0.0))
        if bf16:
            near = (_to_boundary_ulps(act) * _ulp32(act) <= dz) & (z > -dz)
            da = np.where(near, np.maximum(65536.0 * _ulp32(np.maximum(act, dz.astype(np.float32))), dz), 0.0)
            a = _bf16(act).astype(np.float64)
        else:
            da = np.where(z > -dz, dz, 0.0)
            a = act.astype(np.float64)
    return out


class UnitMasks:
    """Per worker and hidden layer, the units with an undecided gate in any step so far; and per
    worker the parameters at which both sides were last bit-identical (`origin`)."""

    def __init__(self):
        self.units: Dict[int, Dict[int, np.ndarray]] = {}
        self.origin: Dict[int, np.ndarray] = {}

    def add(self, worker: int, gates: Dict[int, np.ndarray]) -> None:
        mine = self.units.setdefault(worker, {})
        for l, g in gates.items():
            u = g.any(axis=0)
            mine[l] = (mine[l] | u) if l in mine else u

    def of(self, worker: int) -> Dict[int, np.ndarray]:
        return self.units.get(worker, {})

    def union(self, workers: Sequence[int]) -> Dict[int, np.ndarray]:
        """Units undecided in any of the workers (for quantities all of them feed, like the mean)."""
        out: Dict[int, np.ndarray] = {}
        for i in workers:
            for l, u in self.of(i).items():
                out[l] = (out[l] | u) if l in out else u.copy()
        return out

    def counts(self, worker: int) -> Dict[int, int]:
        return {l: int(u.sum()) for l, u in self.of(worker).items() if u.any()}


def batch_indices(orc, md, seed: int, worker: int, k: int, m: int) -> List[int]:
    """The mini-batch of one worker at local iteration k, from the oracle's index streams."""
    if md.sampler:
        return [orc.index_partition(seed, worker, k, b, md.N, m, md.B) for b in range(md.B)]
    return [orc.index(seed, worker, k, b, md.N) for b in range(md.B)]
