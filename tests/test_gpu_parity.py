"""GPU parity: the HIP path, called through the C ABI, against the oracle on the
same seeded inputs.  Integers (index stream, tau schedule, counters) and the
averaging step are compared bit for bit; parameters, buffers and losses within
1e-4 relative for fp32 operands and 2e-2 for bf16 operands (relative to the
largest magnitude of the compared block, per layer block) -- these two bars and
no multiples of them.

Runs of several steps are teacher-forced: after each comparison the GPU state is
set from the oracle's (lc_set_state), so every comparison starts from bit-identical
models and covers exactly the calls under test.

ReLU gates.  A hidden unit whose pre-activation lies within summation error of
zero may open on one side (double sums in the oracle) and stay shut on the other
(fp32 sums on the matrix cores); both are valid results.  tests/gate_bounds.py
bounds that error from oracle values alone; units with such a gate are left out
of the comparison of their own layer's block (their column of W_l, their entry
of b_l), the count is printed and bounded, and every other entry is held to the
bar."""
import ctypes as C
import sys

import os

import numpy as np
import pytest

import synth
from gate_bounds import UnitMasks, batch_indices, undecided_gates

pytestmark = pytest.mark.gpu

TOL32, TOL16 = 1e-4, 2e-2


@pytest.fixture(scope="module")
def pkg():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1810_08313_amd as p
    p.lib()
    return p


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _blocks(dims):
    """(name, slice) of every W_l and b_l inside a flat parameter vector."""
    out, off = [], 0
    for l in range(len(dims) - 1):
        nw = dims[l] * dims[l + 1]
        out.append((f"W{l + 1}", slice(off, off + nw)))
        out.append((f"b{l + 1}", slice(off + nw, off + nw + dims[l + 1])))
        off += nw + dims[l + 1]
    return out


def _assert_close(got, want, dims, tol, what, masked=None, max_masked=0.5, skip_layers=(), over="fail"):
    """Per block: max |got - want| / max |want| < tol.  masked = {layer: bool [d_l]}: units whose
    gate summation order may decide (see the module text) are left out of their own layer's block.
    If they are more than max_masked of the layer the test fails (over="fail": the comparison
    would say too little), or the block is skipped with a printed note (over="skip": runs of many
    unforced steps, where that is expected and the short runs carry the comparison).
    masked["bias_only"]: leave the units out of the bias blocks only (see _xmask).
    skip_layers: blocks not compared at all (the caller says why)."""
    masked = dict(masked or {})
    bias_only = masked.pop("bias_only", False)
    for name, sl in _blocks(dims):
        layer = int(name[1:])
        if layer in skip_layers:
            continue
        g, w = got[..., sl].astype(np.float64), want[..., sl].astype(np.float64)
        if layer in masked and masked[layer].any() and not (bias_only and name[0] == "W"):
            keep = ~masked[layer]
            if ((~keep).mean() > max_masked or not keep.any()) and over == "skip":
                _say(f"  {what} {name}: {int((~keep).sum())} of {keep.size} units undecided, block not compared")
                continue
            assert (~keep).mean() <= max_masked, f"{what} {name}: {int((~keep).sum())} of {keep.size} units masked"
            if name[0] == "W":
                g = g.reshape(g.shape[:-1] + (dims[layer - 1], dims[layer]))[..., keep]
                w = w.reshape(w.shape[:-1] + (dims[layer - 1], dims[layer]))[..., keep]
            else:
                g, w = g[..., keep], w[..., keep]
        scale = np.abs(w).max()
        if scale == 0.0:
            assert np.abs(g).max() == 0.0, (what, name)
            continue
        err = np.abs(g - w).max() / scale
        assert err < tol, f"{what} {name}: rel err {err:.3e} >= {tol}"


def _errors(got, want, dims, masked=None):
    """{block: max |got - want| / max |want|} outside the masked units, for printing."""
    out = {}
    for name, sl in _blocks(dims):
        layer = int(name[1:])
        g, w = got[..., sl].astype(np.float64), want[..., sl].astype(np.float64)
        if masked and layer in masked and masked[layer].any() and not masked[layer].all():
            keep = ~masked[layer]
            if name[0] == "W":
                g, w = g.reshape(dims[layer - 1], dims[layer])[:, keep], w.reshape(dims[layer - 1], dims[layer])[:, keep]
            else:
                g, w = g[keep], w[keep]
        out[name] = float(f"{np.abs(g - w).max() / max(np.abs(w).max(), 1e-30):.2e}")
    return out


def _drift(got, want, origin, dims, masked=None):
    """How far the master weights of the two sides have come apart after unforced steps, as a
    share of the distance travelled since they were identical: per weight block the maximum,
    outside the masked units, of |got - want| / (|want - origin| + rms(want - origin)) -- the
    quantity gate_bounds.REL_GRAD_* bound.  For printing."""
    out = {}
    for name, sl in _blocks(dims):
        layer = int(name[1:])
        if name[0] != "W":
            continue
        shape = (dims[layer - 1], dims[layer])
        moved = np.abs(want[sl].astype(np.float64) - origin[sl]).reshape(shape)
        q = np.abs(got[sl].astype(np.float64) - want[sl]).reshape(shape) / (moved + np.sqrt(np.mean(moved ** 2)) + 1e-30)
        if masked and layer in masked:
            q = q[:, ~masked[layer]]
        out[name] = float(f"{q.max():.2e}") if q.size else None
    return out


def _xmask(ref, masked):
    """Mask for a comparison of PARAMETERS.  With fp32 operands (bar 1e-4) a gate that fell the
    other way shows in its unit's weights, so the undecided units are left out as for the buffers.
    With bf16 operands (bar 2e-2) it does not -- one sample's term of one step times the learning
    rate is far below a fiftieth of the largest weight -- and every weight is compared; the biases
    start at zero, are nothing but accumulated gradient, and keep the mask."""
    return dict(masked or {}, bias_only=True) if ref.md.bf16 else masked


def _note_gates(orc, ref, seed, masks, ids, fresh):
    """Before a step of the oracle: which gates of that step may summation order decide?
    fresh: both sides hold bit-identical master weights at this point."""
    data = ref._keep[1]
    for i in ids:
        if fresh:
            masks.origin[i] = ref.X[i].copy()
        idx = batch_indices(orc, ref.md, seed, i, ref.k, ref.m)
        masks.add(i, undecided_gates(orc, ref.md, ref.X[i], data, idx, None if fresh else masks.origin[i],
                                     suspect=None if fresh else masks.of(i)))


def _ref_steps(orc, ref, seed, tau, masks=None, ids=None, fresh=True):
    """tau local steps of the oracle, one at a time (the same arithmetic as one call of tau),
    noting before each step the gates it leaves undecided.  ids: advance these workers only."""
    every = ids is None
    ids = list(range(ref.m)) if every else list(ids)
    for t in range(tau):
        if masks is not None and ref.md.n_layers > 1:
            _note_gates(orc, ref, seed, masks, ids, fresh and t == 0)
        ref.local_steps(1, ids=None if every else ids)


def _check_workers(run, ref, dims, tol, what, masks=None, ids=None, buffers=True, max_masked=0.5, over="fail",
                   below="assert"):
    """State of the GPU run against the oracle's, worker by worker, at the bar `tol`.
    below="skip": a layer's gradient passes through the gates of every layer above it, so a gate
    that fell the other way up there moves all of the blocks below a little (by unit it cannot be
    left out): the buffers -- and with the 1e-4 bar of fp32 operands the parameters -- of layers
    below a layer with an undecided unit are then not compared for that worker.  The tests on
    chosen shapes do not need this; the sweep over random shapes, some of them deep and narrow, does."""
    X, V, k = run.get_state()
    assert k == ref.k, (what, k, ref.k)
    for i in (range(ref.m) if ids is None else ids):
        mk = masks.of(i) if masks is not None else None
        skip = set()
        if below == "skip" and mk:
            skip = {l for l in range(1, len(dims) - 1) if any(mk[j].any() for j in mk if j > l)}
        if buffers:
            _assert_close(V[i], ref.V[i], dims, tol, f"{what}: V[{i}]", mk, max_masked, skip, over=over)
        _assert_close(X[i], ref.X[i], dims, tol, f"{what}: X[{i}]", _xmask(ref, mk), max_masked,
                      set() if ref.md.bf16 else skip, over=over)
    return X, V


def _check_losses(run, ref, tol, what, ids=None):
    ll, want = run.local_losses(), ref.last_losses
    ids = list(range(ref.m)) if ids is None else list(ids)
    assert np.abs(ll[ids] - want[ids]).max() < tol * max(np.abs(want[ids]).max(), 1e-3), what


def _force(run, ref):
    """Teacher forcing: the GPU run continues from the oracle's state."""
    run.set_state(ref.X, ref.V, ref.k)


def _forced_periods(orc, run, ref, seed, dims, tol, tau, n, what):
    """n communication periods (tau local steps + the averaging step, one lc_local_periods call
    each), every one started from the oracle's synchronised state with the broadcast of that model
    still pending -- the state after any averaging step under the deferred broadcast, in which all
    replicas read the one model and, at tau = 1, the deferred update and the tile-owner kernels run.
    The model after the averaging step is one vector (units undecided in any worker are left out);
    the momentum buffers are compared worker by worker."""
    m = ref.m
    for it in range(n):
        assert all(np.array_equal(ref.X[i], ref.X[0]) for i in range(1, m))
        _force(run, ref)
        run.average()   # identical rows: their mean is the model itself, bit for bit; leaves the broadcast pending
        masks = UnitMasks()
        _ref_steps(orc, ref, seed, tau, masks)
        ref.average()
        run.local_periods(tau, 1)
        _check_losses(run, ref, tol, f"{what}, period {it}: local losses")
        X, V, k = run.get_state()
        assert k == ref.k
        assert bool((X[1:] == X[0:1]).all())
        _assert_close(X[0], ref.X[0], dims, tol, f"{what}, period {it}: X", _xmask(ref, masks.union(range(m))))
        for i in range(m):
            _assert_close(V[i], ref.V[i], dims, tol, f"{what}, period {it}: V[{i}]", masks.of(i))
        _say(f"  {what}, period {it}: masked units (any worker) { {l: int(u.sum()) for l, u in masks.union(range(m)).items()} }")


@pytest.fixture(autouse=True)
def _oracle_threads(orc):
    """The oracle runs its workers on several host threads here (same results at any count)."""
    orc.set_threads(8)
    yield
    orc.set_threads(1)


def _problem(pkg, orc, dims, m, B, N=400, lr=0.1, beta=0.9, wd=0.0, bf16=False, seed=11, E=None, mean_sd=1.0,
             resident=True):
    data, labels = synth.gaussian_mixture(seed, N, dims[0], dims[-1], mean_sd=mean_sd)
    if bf16:
        data = synth.bf16_representable(data)
    x1 = synth.init_params(seed, dims)
    # non-zero biases so that the bias path matters from the first step
    for name, sl in _blocks(dims):
        if name.startswith("b"):
            x1[sl] = 0.05
    E = min(N, 300) if E is None else E
    omd = orc.make_model(orc.KIND_MLP, dims, B=B, N=N, E=E, lr=lr, beta=beta, wd=wd, bf16=bf16)
    gmd = pkg.make_model(pkg.KIND_MLP, dims, B=B, N=N, E=E, lr=lr, beta=beta, wd=wd, bf16=bf16)
    ref = orc.Run(m, omd, seed, x1, data, labels)
    run = pkg.LocalSGD(m, gmd, seed, x1, data, labels)
    run.set_resident(resident)   # False: launch-per-layer kernels also where the resident kernel applies
    ref.seed = seed
    return ref, run


SHAPES = [
    # dims, m, B        -- ragged everywhere, one tile
    ([50, 37, 5], 3, 5),
    # softmax regression of the small configuration
    ([64, 10], 4, 32),
    # three layers, several row/column tiles with ragged tails, B not a multiple of 16
    ([130, 70, 33, 7], 2, 48),
    # widths that are not multiples of 4 (unaligned weight rows)
    ([67, 129, 10], 2, 33),
    # the 2-layer configuration's layer shapes
    ([784, 256, 10], 8, 64),
    # full 128-row batch tile
    ([200, 128, 10], 3, 128),
    # more classes than one 64-column tile: separate softmax kernel, two-chunk last layer
    ([40, 50, 70], 2, 16),
    # enough replicas x column tiles that one block keeps the whole 128-row batch (activations
    # are then read feature-major, tiles hold interleaved batch rows), ragged batch
    ([100, 512, 24, 10], 32, 120),
    # the same in the last layer, with the loss and dZ_L formed in the forward epilogue
    ([200, 10], 256, 128),
]


# ------------------------------------------------------------------ integers

def test_index_stream_bit_exact(pkg, orc):
    _say("index stream")
    dims, m, B, N = [20, 6], 5, 37, 1000
    ref, run = _problem(pkg, orc, dims, m, B, N=N, lr=0.0)
    for k in (0, 1, 123456789):
        run.set_state(None, None, k)
        run.local_steps(1)
        got = run.last_indices()
        want = np.array([[orc.index(11, i, k, b, N) for b in range(B)] for i in range(m)], dtype=np.int32)
        assert np.array_equal(got, want), k
        assert run.k == k + 1
    run.close()


def test_partition_sampler_bit_exact_and_run(pkg, orc):
    """Per-worker partitions reshuffled every epoch: the index stream of every worker
    over more than two epochs, then a short run against the oracle."""
    _say("partition sampler")
    dims, m, B, N = [20, 12, 6], 5, 9, 203          # 40 or 41 samples per worker: 4 iterations per epoch
    data, labels = synth.gaussian_mixture(3, N, dims[0], dims[-1], mean_sd=1.0)
    x1 = synth.init_params(3, dims)
    kw = dict(B=B, N=N, E=100, lr=0.05, beta=0.9, sampler=1)
    ref = orc.Run(m, orc.make_model(orc.KIND_MLP, dims, **kw), 77, x1, data, labels)
    run = pkg.LocalSGD(m, pkg.make_model(pkg.KIND_MLP, dims, **kw), 77, x1, data, labels)
    masks = UnitMasks()
    for k in range(10):
        run.local_steps(1)
        want = np.array([[orc.index_partition(77, i, k, b, N, m, B) for b in range(B)] for i in range(m)], np.int32)
        assert np.array_equal(run.last_indices(), want), k
        _ref_steps(orc, ref, 77, 1, masks, fresh=k % 5 == 0)
        if k % 5 == 4:
            _check_workers(run, ref, dims, TOL32, f"after {k + 1} steps", masks)
            _force(run, ref)
            masks = UnitMasks()
    ref.average()
    run.average()
    X, V, kk = run.get_state()
    assert kk == ref.k == 10
    _assert_close(X, ref.X, dims, TOL32, "X")
    run.close()
    L = pkg.lib()
    h = C.c_void_p()
    bad = pkg.make_model(pkg.KIND_MLP, dims, B=64, N=N, E=100, sampler=1)     # 40 samples per worker < 64
    assert L.lc_init(m, pkg.lc_param_count(bad), C.byref(bad), 1, C.byref(h)) == -2


# ------------------------------------------------------------------ averaging

@pytest.mark.parametrize("m,P", [(1, 7), (3, 50), (5, 1000), (16, 70001), (64, 257), (7, 4096)])
def test_average_bit_exact(pkg, orc, m, P):
    _say(f"average m={m} P={P}")
    X, _ = synth.flat_stress(m * 1000 + P, m, P)
    X[:, ::7] *= 1000.0          # mixed magnitudes
    Vv = (X * 0.5).astype(np.float32)
    md_o = orc.make_model(orc.KIND_QUAD, [P])
    ref = orc.Run(m, md_o, 0, X[0], qa=np.ones((m, P), np.float32), qc=np.zeros((m, P), np.float32))
    ref.X[:] = X
    ref.average()
    run = pkg.LocalSGD(m, pkg.make_model(pkg.KIND_QUAD, [P]), 0, qa=np.ones((m, P), np.float32),
                       qc=np.zeros((m, P), np.float32))
    run.set_state(X, Vv, 0)
    run.average()
    got, gotV, _ = run.get_state()
    assert np.array_equal(got.view(np.uint32), ref.X.view(np.uint32))
    assert np.array_equal(gotV.view(np.uint32), Vv.view(np.uint32))       # buffers are not communicated
    for i in range(m):
        assert np.array_equal(got[i].view(np.uint32), got[0].view(np.uint32))
    run.average()                                                          # J J = J
    again, _, _ = run.get_state()
    assert np.array_equal(again.view(np.uint32), got.view(np.uint32))
    # the row padding stays zero
    assert float(run.X[:, P:].abs().max().item()) == 0.0 if run.Ps > P else True
    run.close()


@pytest.mark.parametrize("m,P", [(3, 50), (8, 10007)])
def test_update_from_grad_and_fused_average(pkg, orc, m, P):
    _say(f"update_from_grad m={m} P={P}")
    X, G = synth.flat_stress(5, m, P)
    kw = dict(lr=0.05, beta=0.9, wd=1e-3)
    ones, zeros = np.ones((m, P), np.float32), np.zeros((m, P), np.float32)
    ref = orc.Run(m, orc.make_model(orc.KIND_QUAD, [P], **kw), 0, X[0], qa=ones, qc=zeros)
    ref.X[:] = X
    run = pkg.LocalSGD(m, pkg.make_model(pkg.KIND_QUAD, [P], **kw), 0, qa=ones, qc=zeros)
    run.set_state(X, zeros, 0)
    run.set_grad(G)
    for _ in range(3):
        ref.update_from_grad(G)
        run.update_from_grad()
    gx, gv, k = run.get_state()
    assert k == 0
    assert np.abs(gx - ref.X).max() < 1e-6 * np.abs(ref.X).max()
    assert np.abs(gv - ref.V).max() < 1e-6 * np.abs(ref.V).max()
    # tau = 1 fusion: update then average in one pass
    ref.update_from_grad(G)
    ref.average()
    run.update_from_grad_and_average()
    gx, gv, _ = run.get_state()
    assert np.abs(gx - ref.X).max() < 1e-6 * np.abs(ref.X).max()
    assert np.abs(gv - ref.V).max() < 1e-6 * np.abs(ref.V).max()
    for i in range(m):
        assert np.array_equal(gx[i].view(np.uint32), gx[0].view(np.uint32))
    run.close()


# ------------------------------------------------------------- one local step

def _resident_shape(dims, m, B):
    """Shapes lc_set_resident documents as taking the resident step kernel."""
    up64 = lambda d: (d + 63) // 64 * 64
    if len(dims) == 2:
        return dims[1] <= 16 and B <= 64 and up64(dims[0]) <= 256
    return (len(dims) == 3 and dims[2] <= 16 and B <= 64 and up64(dims[0]) <= 1024 and up64(dims[1]) <= 256
            and m <= 64 and m * up64(dims[1]) // 16 <= 256)


@pytest.mark.parametrize("resident", [True, False])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("dims,m,B", SHAPES)
def test_one_local_step(pkg, orc, dims, m, B, bf16, resident):
    if not resident and not _resident_shape(dims, m, B):
        pytest.skip("only one engine handles this shape")
    _say(f"one step dims={dims} m={m} B={B} bf16={bf16} resident={resident}")
    ref, run = _problem(pkg, orc, dims, m, B, wd=1e-3, bf16=bf16, resident=resident)
    tol = TOL16 if bf16 else TOL32
    masks = UnitMasks()
    _ref_steps(orc, ref, 11, 1, masks)
    run.local_steps(1)
    # after the first step V is the gradient (+ wd x): the sensitive comparison
    _check_workers(run, ref, dims, tol, "one step", masks)
    _say(f"  masked units of worker 0: {masks.counts(0)}")
    _check_losses(run, ref, tol, "local losses")
    run.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_round_of_local_steps_then_average(pkg, orc, bf16):
    dims, m, B, tau = [130, 70, 33, 7], 4, 48, 5
    _say(f"round dims={dims} bf16={bf16}")
    ref, run = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, lr=0.03)
    tol = TOL16 if bf16 else TOL32
    for r in range(2):
        masks = UnitMasks()
        x_start = ref.X[0].copy()
        _ref_steps(orc, ref, 11, tau, masks)
        run.local_steps(tau)
        _say(f"  masked units of worker 0 {masks.counts(0)}; drift of the masters "
             f"{_drift(run.get_state()[0][0], ref.X[0], x_start, dims, masks.of(0))}")
        # (five unforced steps: the 33 units of the second hidden layer may all have had an undecided gate by then)
        _check_workers(run, ref, dims, tol, f"before average {r}", masks, over="skip")
        ref.average()
        run.average()
        X, V, k = run.get_state()
        _assert_close(X[0], ref.X[0], dims, tol, f"X round {r}", _xmask(ref, masks.union(range(m))), over="skip")
        for i in range(1, m):
            assert np.array_equal(X[i].view(np.uint32), X[0].view(np.uint32))
        assert k == ref.k == tau * (r + 1)
        _force(run, ref)
    run.close()


def test_plain_sgd_without_momentum_and_repeatability(pkg, orc):
    dims, m, B = [64, 10], 4, 32
    _say("plain SGD, repeatability")
    outs = []
    for rep in range(2):
        ref, run = _problem(pkg, orc, dims, m, B, beta=0.0, lr=0.05)
        run.local_steps(4)
        run.average()
        outs.append(run.get_state())
        if rep == 0:
            ref.local_steps(4)
            ref.average()
            _assert_close(outs[0][0], ref.X, dims, TOL32, "X")
        run.close()
    assert np.array_equal(outs[0][0].view(np.uint32), outs[1][0].view(np.uint32))   # bit-identical reruns
    assert np.array_equal(outs[0][1].view(np.uint32), outs[1][1].view(np.uint32))


RESIDENT_CASES = [
    # dims, m, B: softmax regression (one workgroup per replica, no exchange), ragged; then two layers:
    # unaligned rows and a ragged batch; two column slices and one; the 2-layer configuration
    ([70, 7], 5, 20),
    ([64, 10], 4, 32),
    ([67, 129, 10], 3, 33),
    ([96, 64, 16], 5, 64),
    ([784, 256, 10], 8, 64),
]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("dims,m,B", RESIDENT_CASES)
def test_resident_rounds_against_oracle_and_layer_kernels(pkg, orc, dims, m, B, bf16):
    """Runs of local steps inside one launch each (5 steps, then 11; the state goes back to
    memory and is reloaded in between) with averaging in between, deferred broadcast on: against
    the oracle, and against the launch-per-layer kernels (same arithmetic, other summation order)."""
    assert _resident_shape(dims, m, B)
    _say(f"resident rounds dims={dims} m={m} B={B} bf16={bf16}")
    tol = TOL16 if bf16 else TOL32
    ref, run = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, lr=0.05)
    _, lay = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, lr=0.05, resident=False)
    run.set_lazy_broadcast(True)
    lay.set_lazy_broadcast(True)
    done = 0
    for tau in (5, 11):
        masks = UnitMasks()
        _ref_steps(orc, ref, 11, tau, masks)
        run.local_steps(tau)
        lay.local_steps(tau)
        done += tau
        X, V = _check_workers(run, ref, dims, tol, f"after {done}", masks)
        _check_workers(lay, ref, dims, tol, f"layer kernels after {done}", masks)
        assert run.k == done
        _check_losses(run, ref, tol, f"local losses after {done}")
        ref.average()
        run.average()
        lay.average()
        assert abs(run.loss() - ref.loss()) < tol * max(ref.loss(), 1e-3)
        X, V, _ = run.get_state()
        for i in range(1, m):
            assert np.array_equal(X[i].view(np.uint32), X[0].view(np.uint32))
        # both engines continue from the oracle's state, with a broadcast pending as after any averaging step
        for r in (run, lay):
            _force(r, ref)
            r.average()
    run.close()
    lay.close()


def test_resident_repeatable_and_barrier_timeout_reported(pkg, orc):
    dims, m, B = [96, 64, 10], 4, 32
    _say("resident repeatability, forced barrier time-out")
    outs = []
    for rep in range(2):
        _, run = _problem(pkg, orc, dims, m, B)
        run.local_steps(6)
        outs.append(run.get_state())
        run.close()
    assert np.array_equal(outs[0][0].view(np.uint32), outs[1][0].view(np.uint32))   # bit-identical reruns
    assert np.array_equal(outs[0][1].view(np.uint32), outs[1][1].view(np.uint32))
    # a wait that may not poll at all gives up: the kernel still ends, and the error is reported once
    ref, run = _problem(pkg, orc, dims, m, B)
    x1 = ref.X.copy()
    run.set_barrier_polls(0)
    run.local_steps(3)
    with pytest.raises(pkg.LcError) as ei:
        run.get_state()
    assert ei.value.status == -9
    run.set_barrier_polls(400000)
    run.set_state(x1, np.zeros_like(x1), 0)
    masks = UnitMasks()
    _ref_steps(orc, ref, 11, 3, masks)
    run.local_steps(3)
    _check_workers(run, ref, dims, TOL32, "after recovery", masks)
    run.close()


FIRST_LAYER_CASES = [
    # dims, m, B: shapes the column-owner first-layer kernel takes (m * d1 / 64 >= 192, d0 a
    # multiple of 16): 2, 4 and 8 batch tiles; 6, 5 and 7 sixteen-row steps over 4 wavefronts; then
    # the 8-wavefront kernel of bf16 operands at 65..128 samples (d0 a multiple of 128): three rounds
    # (a pair and a single one) and one round
    ([96, 256, 24, 10], 48, 30),
    ([80, 192, 10], 64, 64),
    ([112, 512, 24, 10], 32, 120),
    ([384, 512, 24, 10], 32, 100),
    ([128, 256, 10], 48, 128),
]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("dims,m,B", FIRST_LAYER_CASES)
def test_first_layer_fusion_across_steps(pkg, orc, dims, m, B, bf16):
    """Runs of local steps in which the first layer's backward kernel also produces the next
    step's first hidden activations: against the oracle, and against the same steps with the
    separate forward launch (same arithmetic, other summation order); a second call and an
    averaging step with deferred broadcast in between."""
    assert not _resident_shape(dims, m, B)
    _say(f"first-layer fusion dims={dims} m={m} B={B} bf16={bf16}")
    tol = TOL16 if bf16 else TOL32
    ref, run = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, lr=0.05)
    _, sep = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, lr=0.05)
    sep.set_first_layer_fusion(False)
    run.set_lazy_broadcast(True)
    sep.set_lazy_broadcast(True)
    done = 0
    # (the last call is longer than the 32 steps one gather launch prepares: a step without a gathered
    # successor in mid-call)
    for tau in (3, 1, 4, 35) if (B == 30 and not bf16) else (3, 1, 4):
        masks = UnitMasks()
        _ref_steps(orc, ref, 11, tau, masks)
        run.local_steps(tau)
        sep.local_steps(tau)
        done += tau
        over = "skip" if tau > 1 else "fail"   # (unforced steps: a 24-unit layer fills up with undecided units)
        _check_workers(run, ref, dims, tol, f"after {done}", masks, over=over)
        _check_workers(sep, ref, dims, tol, f"separate forward after {done}", masks, over=over)
        _check_losses(run, ref, tol, f"local losses after {done}")
        ref.average()
        run.average()
        sep.average()
        assert abs(run.loss() - ref.loss()) < tol * max(ref.loss(), 1e-3)
        for r in (run, sep):
            _force(r, ref)
            r.average()   # (a broadcast pending, as after any averaging step)
    run.close()
    sep.close()


@pytest.mark.parametrize("dims,m,B", [([784, 256, 10], 8, 64), ([96, 64, 16], 16, 32), ([96, 64, 16], 5, 64)])
def test_resident_exchange_inside_one_xcd_is_bit_identical(pkg, orc, dims, m, B):
    """The resident kernel's per-step exchange through the XCD's L2 (first two shapes: one replica
    per XCD, two replicas per XCD) against the agent-scope exchange: same arithmetic, so the same
    bits; the third shape does not place a replica inside one XCD and uses the agent scope in
    both runs.  Also against the oracle."""
    _say(f"xcd-local exchange dims={dims} m={m} B={B}")
    ref, run = _problem(pkg, orc, dims, m, B, wd=5e-4, lr=0.05)
    _, far = _problem(pkg, orc, dims, m, B, wd=5e-4, lr=0.05)
    far.set_xcd_local_exchange(False)
    masks = UnitMasks()
    for tau in (7, 2):
        run.local_steps(tau)
        far.local_steps(tau)
        _ref_steps(orc, ref, 11, tau, masks, fresh=tau == 7)
        if tau == 7:
            _check_workers(run, ref, dims, TOL32, "against the oracle", masks)
        run.average()
        far.average()
        ref.average()
    X, V, k = run.get_state()
    Xf, Vf, _ = far.get_state()
    assert k == 9
    assert np.array_equal(X.view(np.uint32), Xf.view(np.uint32))
    assert np.array_equal(V.view(np.uint32), Vf.view(np.uint32))
    _assert_close(X[0], ref.X[0], dims, TOL32, "X after two periods", _xmask(ref, masks.union(range(m))))
    # a longer run through the schedule driver (400 steps, 80 averaging steps): still the same bits
    run.run(400, 5)
    far.run(400, 5)
    X, V, _ = run.get_state()
    Xf, Vf, _ = far.get_state()
    assert np.array_equal(X.view(np.uint32), Xf.view(np.uint32))
    assert np.array_equal(V.view(np.uint32), Vf.view(np.uint32))
    # the bounded wait of this form of the barrier gives up the same way
    run.set_barrier_polls(0)
    run.local_steps(2)
    with pytest.raises(pkg.LcError) as ei:
        run.get_state()
    assert ei.value.status == -9
    run.set_barrier_polls(400000)
    run.set_state(Xf, Vf, 409)
    run.local_steps(3)
    far.local_steps(3)
    X, V, _ = run.get_state()
    Xf, Vf, _ = far.get_state()
    assert np.array_equal(X.view(np.uint32), Xf.view(np.uint32))
    assert np.array_equal(V.view(np.uint32), Vf.view(np.uint32))
    run.close()
    far.close()


PERIOD_CASES = [
    # dims, m, B, tau, periods: one launch holds several periods (32 steps at most); 7 periods of 5
    # need two launches; one period per launch at tau=20; tau=1 (an averaging step after every step);
    # a shape outside the resident kernel's limits (call-by-call fallback)
    ([70, 7], 5, 20, 4, 5),
    ([67, 129, 10], 3, 33, 5, 7),
    ([96, 64, 16], 5, 64, 1, 9),
    ([784, 256, 10], 8, 64, 20, 2),
    ([130, 70, 33, 7], 3, 16, 3, 2),
    ([96, 64, 16], 5, 64, 40, 1),   # a period longer than one gather launch prepares: two resident launches
]


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("dims,m,B,tau,periods", PERIOD_CASES)
def test_periods_in_one_launch(pkg, orc, dims, m, B, tau, periods, bf16):
    """lc_local_periods(tau, n): whole communication periods inside one resident launch, the
    averaging steps taken in the kernel.  Bit-identical to local_steps(tau) + average() call by
    call (same kernels, same averaging arithmetic).  Against the oracle: the first call, from the
    common initial state, at the bar (the model is one vector after the averaging step, so units
    undecided in any worker are left out; the buffers worker by worker); the second call starts
    from an unforced state and is held to the call-by-call form only."""
    _say(f"periods in one launch dims={dims} m={m} B={B} tau={tau} n={periods} bf16={bf16}")
    tol = TOL16 if bf16 else TOL32
    ref, run = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, lr=0.05)
    _, sep = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, lr=0.05)
    run.set_resident(2)   # in-kernel averaging also at the size where ending the launch is faster
    for lazy in (False, True):   # the second batch starts from a deferred broadcast
        run.set_lazy_broadcast(lazy)
        sep.set_lazy_broadcast(lazy)
        if lazy:
            run.local_steps(2)
            run.average()
            sep.local_steps(2)
            sep.average()
        run.local_periods(tau, periods)
        masks = UnitMasks()
        for j in range(periods):
            sep.local_steps(tau)
            sep.average()
            if not lazy:
                _ref_steps(orc, ref, 11, tau, masks, fresh=j == 0)
                ref.average()
        X, V, k = run.get_state()
        Xs, Vs, ks = sep.get_state()
        assert k == ks and (lazy or k == ref.k)
        assert np.array_equal(X.view(np.uint32), Xs.view(np.uint32))
        assert np.array_equal(V.view(np.uint32), Vs.view(np.uint32))
        for i in range(1, m):
            assert np.array_equal(X[i].view(np.uint32), X[0].view(np.uint32))
        assert np.array_equal(run.local_losses().view(np.uint32), sep.local_losses().view(np.uint32))
        if not lazy:
            _assert_close(X[0], ref.X[0], dims, tol, "X against the oracle", _xmask(ref, masks.union(range(m))), over="skip")
            for i in range(m):
                _assert_close(V[i], ref.V[i], dims, tol, f"V[{i}] against the oracle", masks.of(i), over="skip")
            assert abs(run.loss() - ref.loss()) < tol * max(ref.loss(), 1e-3)
    run.close()
    sep.close()


def test_periods_in_one_launch_timeout_reported(pkg, orc):
    """The all-replica barrier of the in-kernel averaging step gives up like the per-step one."""
    dims, m, B = [64, 10], 4, 32   # one workgroup per replica: only the averaging barrier waits
    _say("periods in one launch, forced barrier time-out")
    ref, run = _problem(pkg, orc, dims, m, B)
    x1 = ref.X.copy()
    run.set_barrier_polls(0)
    run.local_periods(2, 3)
    with pytest.raises(pkg.LcError) as ei:
        run.get_state()
    assert ei.value.status == -9
    run.set_barrier_polls(400000)
    run.set_state(x1, np.zeros_like(x1), 0)
    for _ in range(3):
        ref.local_steps(2)
        ref.average()
    run.local_periods(2, 3)
    X, V, k = run.get_state()
    assert k == 6
    _assert_close(X, ref.X, dims, TOL32, "X after recovery")
    with pytest.raises(pkg.LcError):
        run.local_periods(0, 1)
    with pytest.raises(pkg.LcError):
        run.local_periods(1, 0)
    run.close()


# --------------------------------------------------------------- loss + driver

@pytest.mark.parametrize("bf16", [False, True])
def test_loss_of_averaged_model(pkg, orc, bf16):
    dims, m, B = [130, 70, 33, 7], 3, 16
    _say(f"loss bf16={bf16}")
    # E = 300 is not a multiple of the 128-sample evaluation chunk
    ref, run = _problem(pkg, orc, dims, m, B, bf16=bf16, E=300)
    assert abs(run.loss() - ref.loss()) < 1e-5 * ref.loss()
    ref.local_steps(2)
    run.local_steps(2)
    before = run.get_state()
    Fg, Fr = run.loss(), ref.loss()          # workers differ here: the loss is that of their mean
    assert abs(Fg - Fr) < (TOL16 if bf16 else TOL32) * Fr
    after = run.get_state()
    assert np.array_equal(before[0], after[0]) and np.array_equal(before[1], after[1])
    run.close()


def test_loss_many_chunks(pkg, orc):
    dims = [40, 10]
    _say("loss over several passes")
    ref, run = _problem(pkg, orc, dims, 2, 8, N=9000, E=8500)   # > 64 chunks: two passes
    assert abs(run.loss() - ref.loss()) < 1e-5 * ref.loss()
    run.close()


def test_cfg1_full_run(pkg, orc):
    """The small configuration end to end: softmax regression, m=4, B=32,
    tau=4, 200 iterations, plain SGD from zero (convex: errors do not amplify)."""
    _say("cfg1 full run")
    w = synth.make_workload("cfg1")
    omd = orc.make_model(orc.KIND_MLP, w.dims, B=w.B, N=w.N, E=w.E, lr=w.lr, beta=w.beta)
    gmd = pkg.make_model(pkg.KIND_MLP, w.dims, B=w.B, N=w.N, E=w.E, lr=w.lr, beta=w.beta)
    ref = orc.Run(w.m, omd, w.seed, w.x1, w.data, w.labels)
    run = pkg.LocalSGD(w.m, gmd, w.seed, w.x1, w.data, w.labels)
    F0 = run.loss()
    assert abs(F0 - np.log(10.0)) < 1e-6            # zero init: uniform prediction
    s_ref, r_ref = ref.run(w.K, w.tau0)
    s_gpu, r_gpu = run.run(w.K, w.tau0)
    assert s_gpu == s_ref == [(0, 4)] and r_gpu == r_ref == 50
    X, V, k = run.get_state()
    assert k == ref.k == 200
    _assert_close(X, ref.X, w.dims, TOL32, "X")
    Fg, Fr = run.loss(), ref.loss()
    assert abs(Fg - Fr) < TOL32 * Fr and Fg < 0.5 * F0
    run.close()


def test_adaptive_schedule_bit_exact(pkg, orc):
    """AdaComm on a small MLP: same tau decisions, rounds and counters as the
    oracle.  Every decision is checked to sit far enough from an integer that
    the 1e-4 loss tolerance cannot flip the ceil."""
    dims, m, B = [64, 32, 10], 4, 32
    _say("adaptive schedule")
    ref, run = _problem(pkg, orc, dims, m, B, N=2000, lr=0.05, beta=0.0, E=1024, mean_sd=2.0)
    K, tau0, I = 120, 8, 24
    s_ref, r_ref = ref.run(K, tau0, adaptive=True, interval=I)
    # the margins, from a second oracle run that follows the schedule step by step: at every decision
    # p = sqrt(F_l / F_0) tau_0 must be further from an integer than ten times what a relative loss
    # discrepancy of 1e-4 (5e-5 in p) can move it -- otherwise another seed is needed
    chk, unused = _problem(pkg, orc, dims, m, B, N=2000, lr=0.05, beta=0.0, E=1024, mean_sd=2.0)
    unused.close()
    F0 = chk.loss()
    masks = UnitMasks()   # (and the gates any step of the run leaves undecided, for the final comparison)
    for (k0, tau), (k1, tau_next) in zip(s_ref, s_ref[1:] + [(K, None)]):
        while chk.k < k1:
            _ref_steps(orc, chk, 11, min(tau, K - chk.k), masks, fresh=chk.k == 0)
            chk.average()
        assert chk.k == k1
        if tau_next is not None:
            Fl = chk.loss()
            pval = float(np.sqrt(Fl / F0)) * tau0
            assert orc.next_tau(F0, Fl, tau0) == tau_next
            assert abs(pval - round(pval)) > 10 * 5e-5 * pval, (k1, pval)
    assert np.array_equal(chk.X, ref.X)
    s_gpu, r_gpu = run.run(K, tau0, adaptive=True, interval=I)
    assert len(s_ref) >= 4 and s_ref[-1][1] < tau0      # the loss fell, so tau fell
    assert s_gpu == s_ref and r_gpu == r_ref
    assert run.k == ref.k == K
    X, V, _ = run.get_state()
    _assert_close(X[0], ref.X[0], dims, TOL32, "X after adaptive run", _xmask(ref, masks.union(range(m))), max_masked=0.5)
    run.close()


@pytest.mark.parametrize("dims,m,B", [([64, 10], 4, 32), ([64, 32, 10], 4, 32), ([130, 70, 33, 7], 3, 16)])
def test_grid_search_for_tau0(pkg, orc, dims, m, B):
    """The tau_0 helper: every candidate's loss is the loss of K iterations with that fixed
    period from the same start (against the oracle's own runs), the state is back where it
    was afterwards, bit for bit, and the index returned is the largest loss decrease per second
    of the two arrays it hands back."""
    _say(f"grid search dims={dims} m={m}")
    ref, run = _problem(pkg, orc, dims, m, B, N=2000, lr=0.05, beta=0.9, E=512, mean_sd=2.0)
    run.local_steps(3)
    run.average()
    ref.local_steps(3)
    ref.average()
    X0, V0, k0 = run.get_state()
    F0 = run.loss()
    taus, K = [1, 4, 16, 5], 32
    best, loss, sec = run.grid_search_tau0(taus, K)
    X1, V1, k1 = run.get_state()
    assert k1 == k0 == 3
    assert np.array_equal(X1.view(np.uint32), X0.view(np.uint32))
    assert np.array_equal(V1.view(np.uint32), V0.view(np.uint32))
    assert (sec > 0).all() and np.isfinite(loss).all()
    assert best == int(np.argmax((F0 - loss) / sec))
    for i, tau in enumerate(taus):   # the oracle from the same start: a fresh run brought to iteration 3
        r, g = _problem(pkg, orc, dims, m, B, N=2000, lr=0.05, beta=0.9, E=512, mean_sd=2.0)
        g.close()
        r.local_steps(3)
        r.average()
        r.run(K, tau)
        assert abs(loss[i] - r.loss()) < TOL32 * max(r.loss(), 1e-2), (tau, loss[i], r.loss())
    with pytest.raises(pkg.LcError):
        run.grid_search_tau0([4, 0], K)
    run.close()


# ------------------------------------------------------------------ quadratic

def test_quadratic_closed_form_and_schedule(pkg, orc):
    _say("quadratic")
    m, P, lr, tau, R = 4, 333, 0.2, 4, 5
    a, c, x0 = synth.quad_problem(2, m, P)
    run = pkg.LocalSGD(m, pkg.make_model(pkg.KIND_QUAD, [P], lr=lr), 0, x0, qa=a, qc=c)
    for _ in range(R):
        run.local_steps(tau)
        run.average()
    rho = 1.0 - lr * a.astype(np.float64)
    alpha = (rho ** tau).mean(axis=0)
    bt = ((1.0 - rho ** tau) * c).mean(axis=0)
    want = alpha ** R * x0 + bt * (1.0 - alpha ** R) / (1.0 - alpha)
    X, V, k = run.get_state()
    assert k == tau * R
    assert np.abs(X[0] - want).max() < 2e-5
    xbar = X[0].astype(np.float64)
    F = float(np.mean([0.5 * np.sum(a[i].astype(np.float64) * (xbar - c[i].astype(np.float64)) ** 2) for i in range(m)]))
    assert abs(run.loss() - F) < 1e-9 * F
    run.close()

    # momentum + adaptive schedule against the oracle
    kw = dict(lr=0.02, beta=0.5)
    a, c, x0 = synth.quad_problem(8, m, P, common_a=True)
    c = (c * 0.05).astype(np.float32)
    ref = orc.Run(m, orc.make_model(orc.KIND_QUAD, [P], **kw), 0, x0, qa=a, qc=c)
    run = pkg.LocalSGD(m, pkg.make_model(pkg.KIND_QUAD, [P], **kw), 0, x0, qa=a, qc=c)
    s_ref, r_ref = ref.run(150, 12, adaptive=True, interval=20)
    s_gpu, r_gpu = run.run(150, 12, adaptive=True, interval=20)
    assert s_gpu == s_ref and r_gpu == r_ref and len(s_ref) > 3
    X, V, k = run.get_state()
    assert k == ref.k
    assert np.abs(X - ref.X).max() < 1e-4 * np.abs(ref.X).max()
    assert np.abs(V - ref.V).max() < 1e-4 * max(np.abs(ref.V).max(), 1e-3)
    run.close()


def test_refined_schedule_bit_exact(pkg, orc):
    """AdaComm with saturation decay, learning-rate coupling and postponed rate
    change: same (iteration, tau, lr) decisions as the oracle, on the quadratic
    (exactly predictable losses) and on a small MLP."""
    _say("refined schedule")
    m, P = 4, 333
    a, c, x0 = synth.quad_problem(8, m, P, common_a=True)
    c = (c * 0.05).astype(np.float32)
    kw = dict(lr=0.02)
    ref = orc.Run(m, orc.make_model(orc.KIND_QUAD, [P], **kw), 0, x0, qa=a, qc=c)
    run = pkg.LocalSGD(m, pkg.make_model(pkg.KIND_QUAD, [P], **kw), 0, x0, qa=a, qc=c)
    args = dict(refine=True, gamma=0.5, slack=0, lr_schedule=[(70, 0.005)], postpone_lr=True)
    s_ref, r_ref = ref.run_ex(260, 12, 20, **args)
    s_gpu, r_gpu = run.run_ex(260, 12, 20, **args)
    assert s_gpu == s_ref and r_gpu == r_ref and len(s_ref) > 6
    assert any(lr == pytest.approx(0.005) for _, _, lr in s_ref)
    X, V, k = run.get_state()
    assert k == ref.k == 260
    assert np.abs(X - ref.X).max() < 1e-4 * np.abs(ref.X).max()
    run.close()

    dims = [64, 32, 10]
    ref, run = _problem(pkg, orc, dims, 4, 32, N=2000, lr=0.05, beta=0.0, E=1024, mean_sd=2.0)
    args = dict(refine=True, gamma=0.5, slack=1, lr_schedule=[(60, 0.0125)], postpone_lr=False)
    s_ref, r_ref = ref.run_ex(140, 8, 24, **args)
    s_gpu, r_gpu = run.run_ex(140, 8, 24, **args)
    assert s_gpu == s_ref and r_gpu == r_ref
    X, V, k = run.get_state()
    _assert_close(X, ref.X, dims, TOL32, "X after refined run")
    run.close()


@pytest.mark.parametrize("dims", [[130, 70, 33, 7], [96, 64, 10]])   # per-layer kernels; resident kernel
@pytest.mark.parametrize("bf16", [False, True])
def test_block_momentum_rounds(pkg, orc, bf16, dims):
    """Block momentum (global factor 0.3, local 0.9, local buffers restarted at every
    averaging step) over several periods against the oracle."""
    m, B, tau = 4, 48, 3
    _say(f"block momentum bf16={bf16} dims={dims}")
    ref, run = _problem(pkg, orc, dims, m, B, lr=0.05, beta=0.9, bf16=bf16)
    tol = TOL16 if bf16 else TOL32
    ref.block_begin(0.3)
    run.block_momentum_begin(0.3)
    # (the global buffer u lives in the library's scratch and cannot be set from outside, so these
    # three periods run unforced; model and u are one vector each: units undecided in any worker
    # and any step so far are left out)
    masks = UnitMasks()
    for r in range(3):
        _ref_steps(orc, ref, 11, tau, masks, fresh=r == 0)
        run.local_steps(tau)
        ref.average()
        run.average()
        X, V, k = run.get_state()
        u, xs = run.get_block_momentum()
        every = masks.union(range(m))
        _assert_close(X[0], ref.X[0], dims, tol, f"X round {r}", _xmask(ref, every), over="skip")
        _assert_close(u, ref.block_u, dims, tol, f"u round {r}", every, over="skip")
        assert np.array_equal(xs, X[0]) and np.abs(V).max() == 0.0 and np.abs(ref.V).max() == 0.0
        for i in range(1, m):
            assert np.array_equal(X[i].view(np.uint32), X[0].view(np.uint32))
    # back to plain averaging: buffers survive the averaging step again
    ref.block_end()
    run.block_momentum_end()
    _force(run, ref)
    masks = UnitMasks()
    _ref_steps(orc, ref, 11, 2, masks)
    run.local_steps(2)
    _check_workers(run, ref, dims, tol, "after leaving the mode", masks)
    ref.average()
    run.average()
    X, V, _ = run.get_state()
    _assert_close(X[0], ref.X[0], dims, tol, "X after leaving the mode", _xmask(ref, masks.union(range(m))))
    assert np.abs(V).max() > 0
    run.close()


def test_block_momentum_quadratic_closed_form_and_driver(pkg, orc):
    _say("block momentum quadratic")
    m, P, lr, bg, tau, R = 4, 333, 0.1, 0.3, 5, 6
    a, c, x0 = synth.quad_problem(12, m, P, common_a=True)
    run = pkg.LocalSGD(m, pkg.make_model(pkg.KIND_QUAD, [P], lr=lr), 0, x0, qa=a, qc=c)
    run.block_momentum_begin(bg)
    sched, rounds = run.run(tau * R, tau)
    assert rounds == R
    a64, cbar = a[0].astype(np.float64), c.astype(np.float64).mean(axis=0)
    lr64 = np.float64(np.float32(lr))
    rho_t = (1.0 - lr64 * a64) ** tau
    e, u = x0.astype(np.float64) - cbar, np.zeros(P)
    for _ in range(R):
        u = bg * u + (1.0 - rho_t) * e / lr64
        e = e - lr64 * u
    X, V, k = run.get_state()
    gu, _ = run.get_block_momentum()
    assert k == tau * R
    assert np.abs(X[0] - (cbar + e)).max() < 2e-5
    assert np.abs(gu - u).max() < 2e-4 * max(1.0, np.abs(u).max())
    run.close()


@pytest.mark.parametrize("bf16", [False, True])
def test_lazy_broadcast_is_bit_identical_to_eager(pkg, orc, bf16):
    """Deferred broadcast: the averaging step only reduces, the next local step reads
    the one averaged model.  Same bits as the eager form at every observable point."""
    dims, m, B = [130, 70, 33, 7], 4, 48
    _say(f"lazy broadcast bf16={bf16}")
    _, eager = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16)
    ref, lazy = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16)
    lazy.set_lazy_broadcast(True)
    for tau in (1, 1, 3, 2):
        for r in (eager, lazy):
            r.local_steps(tau)
            r.average()
        assert lazy.loss() == eager.loss()                     # evaluated while the broadcast is pending
        for r in (eager, lazy):
            r.average()                                        # averaging twice changes nothing
    Xe, Ve, ke = eager.get_state()
    Xl, Vl, kl = lazy.get_state()                              # materialises
    assert ke == kl == 7
    assert np.array_equal(Xe.view(np.uint32), Xl.view(np.uint32))
    assert np.array_equal(Ve.view(np.uint32), Vl.view(np.uint32))
    # and both follow the oracle
    masks = UnitMasks()
    for j, tau in enumerate((1, 1, 3, 2)):
        _ref_steps(orc, ref, 11, tau, masks, fresh=j == 0)
        ref.average()
    _assert_close(Xl[0], ref.X[0], dims, TOL16 if bf16 else TOL32, "X", _xmask(ref, masks.union(range(m))), over="skip")
    # a pending broadcast is visible in device memory until materialised
    lazy.local_steps(2)
    lazy.average()
    assert not bool((lazy.X[1:] == lazy.X[0:1]).all().item())
    lazy.materialize()
    assert bool((lazy.X[1:] == lazy.X[0:1]).all().item())
    # drivers and block momentum work on top of it
    eager.local_steps(2)
    eager.average()
    for r in (eager, lazy):
        r.block_momentum_begin(0.3)
        r.run(7, 3)
    Xe, Ve, _ = eager.get_state()
    Xl, Vl, _ = lazy.get_state()
    assert np.array_equal(Xe.view(np.uint32), Xl.view(np.uint32))
    assert np.array_equal(Ve.view(np.uint32), Vl.view(np.uint32))
    eager.close()
    lazy.close()


DEFER_CASES = [
    # last layer with more than 128 inputs (its backward pass is the row-owner kernel), ragged everywhere
    ([130, 70, 200, 7], 4, 48, False),
    ([130, 70, 200, 7], 4, 48, True),
    # unaligned weight rows, resident kernel switched off
    ([67, 129, 10], 3, 33, False),
]


@pytest.mark.parametrize("dims,m,B,bf16", DEFER_CASES)
def test_deferred_update_at_tau_1_is_bit_identical(pkg, orc, dims, m, B, bf16):
    """tau = 1 under the deferred broadcast: the backward kernels write V only and the
    averaging step forms x_bar - lr v_i itself.  Same bits as with the rows written."""
    _say(f"deferred update dims={dims} bf16={bf16}")
    ref, plain = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, resident=False)
    _, defer = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, resident=False)
    for r in (plain, defer):
        r.set_lazy_broadcast(True)
    plain.set_deferred_update(False)
    for r in (plain, defer):
        r.run(6, 1)
    # the switch did something: from the second iteration on the rows of X stay unwritten
    assert not bool((plain.X == defer.X).all().item())
    assert plain.loss() == defer.loss()
    for r in (plain, defer):
        r.run(6, 3)              # longer periods in between write the rows again
        r.local_periods(1, 4)    # ... and the other driver
        r.set_lr(0.03)
        r.run(3, 1)
    Xp, Vp, kp = plain.get_state()
    Xd, Vd, kd = defer.get_state()
    assert kp == kd == 19
    assert np.array_equal(Xp.view(np.uint32), Xd.view(np.uint32))
    assert np.array_equal(Vp.view(np.uint32), Vd.view(np.uint32))
    # against the oracle: deferred iterations one at a time, each from the oracle's state
    ref.set_lr(0.03)
    _forced_periods(orc, defer, ref, 11, dims, TOL16 if bf16 else TOL32, 1, 3, "deferred update")
    # ... and three of them in a row, unforced in between: the model (the buffers of the last one
    # depend on gates of earlier steps in ways the masks of one step do not describe)
    _force(defer, ref)
    defer.average()
    masks = UnitMasks()
    for j in range(3):
        _ref_steps(orc, ref, 11, 1, masks, fresh=j == 0)
        ref.average()
    defer.run(3, 1)
    Xd, _, kd = defer.get_state()
    assert kd == ref.k
    _assert_close(Xd[0], ref.X[0], dims, TOL16 if bf16 else TOL32, "X after three deferred iterations",
                  _xmask(ref, masks.union(range(m))), max_masked=0.5)
    plain.close()
    defer.close()


@pytest.mark.parametrize("bf16,m,d0,d1,mode,implicit", [
    (True, 16, 2048, 1152, 1, 1),              # first layer; momentum implicit inside the period (the default at this size)
    (False, 12, 2000, 1152, 1, 0),             # fp32 operands, a last row block that is partly padding
    (False, 12, 2048, 1152, 1, 2),             # ... with the implicit form forced on
    (True, 8, 2048, (1152, 1856), 2, 1),       # a hidden layer above 8 MB as well (after the dA-only pass)
    (False, 16, 2048, (1152, 1856), 2, 0),
])
def test_fused_averaging_is_bit_identical(pkg, orc, bf16, m, d0, d1, mode, implicit):
    """The last step of a period and the averaging of the large layers in one kernel
    (lc_set_fused_averaging) against the same periods with the step and the averaging step apart:
    periods of 3, 2 and 4 through the schedule driver and lc_local_periods, a learning-rate change
    in between; model, buffers, losses bit for bit.  (Against the oracle these periods are held
    by the other tests of this file, which run with the fusion on wherever it applies.)"""
    dims, B = [d0, *(d1 if isinstance(d1, tuple) else (d1,)), 10], 24
    _say(f"fused averaging bf16={bf16} m={m} dims={dims} mode={mode} implicit={implicit}")
    runs = []
    for fused in (mode, 0):
        _, r = _problem(pkg, orc, dims, m, B, N=300, lr=0.05, wd=1e-4, bf16=bf16, mean_sd=0.03)
        assert not r.resident_active()
        r.set_lazy_broadcast(True)
        r.set_implicit_momentum(implicit)
        r.set_fused_averaging(fused)
        runs.append(r)
    for step, (tau, n) in enumerate([(3, 2), (2, 1), (4, 1)]):
        outs = []
        for r in runs:
            if step == 0:
                r.run(tau * n, tau)
            else:
                r.local_periods(tau, n)
            outs.append((r.loss(), r.local_losses(), *r.get_state()))
            if step == 1:
                r.set_lr(0.02)
        (la, lla, Xa, Va, ka), (lb, llb, Xb, Vb, kb) = outs
        assert ka == kb
        assert la == lb and np.array_equal(lla, llb), (tau, n)
        assert np.array_equal(Xa.view(np.uint32), Xb.view(np.uint32)), (tau, n)
        assert np.array_equal(Va.view(np.uint32), Vb.view(np.uint32)), (tau, n)
        assert bool((Xa[1:] == Xa[0:1]).all())
    for r in runs:
        r.close()


@pytest.mark.parametrize("bf16,m,d0,d1,tau,K", [
    (True, 16, 2048, 1100, 1, 3), (False, 16, 2048, 1100, 1, 3),   # two sets of 8 replicas
    (False, 12, 2048, 1100, 1, 3),                                 # one set of 12
    (True, 16, 2048, 1152, 2, 4),      # first layer by the column-owner kernel, first step of a period
    (True, 16, 2048, 1152, 1, 3), (False, 12, 2048, 1152, 1, 3),   # first layer by the tile-owner kernel that also averages it
    (False, 16, 2000, 1152, 1, 3), (True, 16, 2000, 1152, 1, 3),   # ... with a last row block that is partly padding
    (False, 16, 2048, (1152, 1856), 1, 3),   # a second layer above 8 MB: dZ_1 by the dA-only backward pass, then
    (True, 8, 2048, (1152, 1856), 1, 3),     # the tile-owner kernel for it as well; biases and the last layer averaged apart
])
def test_shared_model_block_order_against_oracle(pkg, orc, bf16, m, d0, d1, tau, K, B=24, bitwise=True):
    """A first layer above 8 MB in a state above 256 MB: the steps that read one model for all
    replicas hand the same weight tile to neighbouring blocks (another block numbering in the
    forward, backward and first-layer kernels).  K / tau periods against the oracle, model and
    momentum buffers at the bar: the first from the common initial state (rows written by the step),
    the others each from the oracle's state with the broadcast pending (deferred update and
    tile-owner kernels at tau = 1)."""
    dims = [d0, *(d1 if isinstance(d1, tuple) else (d1,)), 10]
    _say(f"shared-model block order bf16={bf16} m={m} d0={d0} d1={d1} tau={tau} B={B}")
    ref, run = _problem(pkg, orc, dims, m, B, N=300, lr=0.05, wd=1e-4, bf16=bf16, mean_sd=0.03)   # overlapping classes
    assert not run.resident_active()
    run.set_lazy_broadcast(True)
    tol = TOL16 if bf16 else TOL32
    masks = UnitMasks()
    _ref_steps(orc, ref, 11, tau, masks)
    ref.average()
    run.run(tau, tau)
    X, V, k = run.get_state()
    assert k == ref.k == tau
    assert bool((X[1:] == X[0:1]).all())
    _assert_close(X[0], ref.X[0], dims, tol, "first period: X", _xmask(ref, masks.union(range(m))))
    for i in range(m):
        _assert_close(V[i], ref.V[i], dims, tol, f"first period: V[{i}]", masks.of(i))
    _forced_periods(orc, run, ref, 11, dims, tol, tau, K // tau - 1, "shared model")
    np.testing.assert_allclose(run.loss(), ref.loss(), rtol=2e-3 if bf16 else 1e-4)
    # the tile-owner kernels against the same iterations without them, unforced: bit for bit
    if tau == 1:
        os.environ["LC_SYNC_FIRST_LAYER"] = "0"
        try:
            _, plain = _problem(pkg, orc, dims, m, B, N=300, lr=0.05, wd=1e-4, bf16=bf16, mean_sd=0.03)
        finally:
            del os.environ["LC_SYNC_FIRST_LAYER"]
        plain.set_lazy_broadcast(True)
        for r in (run, plain):
            _force(r, ref)
            r.run(K, tau)
        X, V, _ = run.get_state()
        Xp, Vp, _ = plain.get_state()
        if bitwise:
            assert np.array_equal(X.view(np.uint32), Xp.view(np.uint32))
            assert np.array_equal(V.view(np.uint32), Vp.view(np.uint32))
        else:   # (another summation order in the dA-only pass: see the caller)
            for i in range(m):
                _assert_close(V[i], Vp[i], dims, tol, f"with and without the tile-owner kernels: V[{i}]")
            _assert_close(X[0], Xp[0], dims, tol, "with and without the tile-owner kernels: X")
        plain.close()
        # ... and those unforced iterations against the oracle: the buffers at the bar outside the units
        # whose gate is open to summation order or, from the second iteration on, to weights that
        # have drifted across a bf16 rounding boundary
        masks = UnitMasks()
        for j in range(K // tau):
            _ref_steps(orc, ref, 11, tau, masks, fresh=j == 0)
            ref.average()
        _say(f"  unforced: masked units (any worker) { {l: int(u.sum()) for l, u in masks.union(range(m)).items()} }")
        _assert_close(X[0], ref.X[0], dims, tol, "unforced: X", _xmask(ref, masks.union(range(m))), over="skip")
        # (a buffer passes through the gates of every layer above its own: only the blocks with no
        # undecided unit above them can be held to the bar after unforced steps; the forced periods
        # above hold all of them)
        for i in range(m):
            mk = masks.of(i)
            below = {l for l in range(1, len(dims) - 1) if any(mk[j].any() for j in mk if j > l)}
            _assert_close(V[i], ref.V[i], dims, tol, f"unforced: V[{i}]", mk, over="skip", skip_layers=below)
    run.close()


def test_deferred_update_with_chunked_averaging(pkg, orc):
    """The same on a state above 512 MB, where the averaging step is the chunked reduce kernel:
    against the run that writes the rows, bit for bit (that run is held to the oracle elsewhere)."""
    dims, m, B = [8192, 8320, 10], 2, 32
    _say("deferred update, chunked averaging")
    data, labels = synth.gaussian_mixture(5, 200, dims[0], dims[-1], mean_sd=1.0)
    data = synth.bf16_representable(data)
    x1 = synth.init_params(5, dims)
    out = []
    for on in (False, True):
        md = pkg.make_model(pkg.KIND_MLP, dims, B=B, N=200, E=100, lr=0.05, beta=0.9, wd=1e-4, bf16=True)
        run = pkg.LocalSGD(m, md, 5, x1, data, labels)
        run.set_lazy_broadcast(True)
        run.set_deferred_update(on)
        run.run(4, 1)
        loss = run.loss()
        X, V, k = run.get_state()
        out.append((loss, X[:, ::97].copy(), V[:, ::97].copy(), X[0, -70000:].copy(), k))
        run.close()
        del X, V
    assert out[0][0] == out[1][0] and out[0][4] == out[1][4] == 4
    for a, b in zip(out[0][1:4], out[1][1:4]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.isfinite(out[0][0])


@pytest.mark.parametrize("bf16,m,d0,d1,tau,K,B", [
    (True, 32, 2048, (1152, 1856), 1, 2, 32),    # forward passes and the dA-only pass with two replicas per block
    (False, 32, 2048, (1152, 1856), 1, 2, 32),
    (False, 64, 256, 1024, 3, 6, 32),            # first step of a period: four replicas per block in the first layer
    (True, 32, 256, 1024, 2, 4, 64),             # 64 samples: two replicas per block
])
def test_grouped_batches_at_shared_steps(pkg, orc, bf16, m, d0, d1, tau, K, B):
    """Steps in which all replicas read one model hand the batches of several replicas to one block
    (forward passes; at tau = 1 also the dA-only backward pass) when every batch row is a sample
    (B = 16, 32, 64) and enough blocks remain: the periods of the shared-model test at such batch
    sizes, against the oracle.  (The dA-only pass with two replicas per block starts its walk over
    the columns elsewhere than the full backward pass does, so its deltas are no longer the same
    bits as those of the run without the tile-owner kernels: that comparison is at the bar here.)"""
    test_shared_model_block_order_against_oracle(pkg, orc, bf16, m, d0, d1, tau, K, B=B, bitwise=False)


# ---------------------------------------------------------- implicit momentum

IMPLICIT_CASES = [
    # dims, m, B: row-owner backward kernel on three layers, ragged; the column-owner first-layer kernel
    # with the next forward in it; unaligned rows; the 8-wavefront first-layer kernel (bf16 operands)
    ([130, 70, 33, 7], 4, 48),
    ([96, 256, 24, 10], 48, 30),
    ([67, 129, 10], 3, 33),
    ([256, 512, 24, 10], 32, 100),
]


@pytest.mark.parametrize("lazy", [False, True])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("dims,m,B", IMPLICIT_CASES)
def test_implicit_momentum_inside_periods(pkg, orc, dims, m, B, bf16, lazy):
    """Inside a call the large layers may keep two consecutive models instead of model and momentum
    (lc_set_implicit_momentum; forced on here at small shapes and for both operand types).  Calls of
    2, 5, 1 and 7 steps -- two to seven of them without the momentum in memory, through both row
    buffers in turn, from separate rows and from a pending broadcast -- against the oracle, each from
    the oracle's state: model, momentum (explicit again at the end of every call) and losses at the
    bar; then the averaging step."""
    _say(f"implicit momentum dims={dims} m={m} B={B} bf16={bf16} lazy={lazy}")
    tol = TOL16 if bf16 else TOL32
    ref, run = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, lr=0.05, resident=False)
    run.set_implicit_momentum(2)
    run.set_lazy_broadcast(lazy)
    for tau in (2, 5, 1, 7):
        masks = UnitMasks()
        _ref_steps(orc, ref, 11, tau, masks)
        run.local_steps(tau)
        _check_workers(run, ref, dims, tol, f"call of {tau}", masks, over="skip")
        _check_losses(run, ref, tol, f"local losses, call of {tau}")
        ref.average()
        run.average()
        X, _, _ = run.get_state()
        _assert_close(X[0], ref.X[0], dims, tol, f"mean after {tau}", _xmask(ref, masks.union(range(m))), over="skip")
        assert all(np.array_equal(X[i], X[0]) for i in range(1, m))
        _force(run, ref)
        if lazy:
            run.average()   # identical rows: exact; leaves the broadcast pending, the next call starts from the one model
    # the schedule driver: periods of 3, the last one shortened
    masks = UnitMasks()
    for j, tau in enumerate((3, 3, 2)):
        _ref_steps(orc, ref, 11, tau, masks, fresh=j == 0)
        ref.average()
    run.run(8, 3)
    X, V, k = run.get_state()
    assert k == ref.k
    _assert_close(X[0], ref.X[0], dims, tol, "after the driver", _xmask(ref, masks.union(range(m))), over="skip")
    run.close()
    if dims[0] == 96 and not bf16 and not lazy:
        # A call longer than the 32 steps one gather launch prepares: the implicit form carries over
        # from one launch's steps to the next's (twice in 70 steps).  No two runs agree to the bar
        # after 70 unforced steps; what is checked is that this run stays with the one that writes
        # model and momentum in every step as closely as 30 steps (no launch boundary) leave them
        # (measured: 3e-5 in the model, 8e-4 in the momentum after 70 steps, 2e-5 and 2e-4 after 30)
        # -- a step that read the wrong buffer would show as an error of order one.
        ends = []
        for mode in (2, 0):
            _, r = _problem(pkg, orc, dims, m, B, wd=5e-4, bf16=bf16, lr=0.05, resident=False)
            r.set_implicit_momentum(mode)
            r.local_steps(70)
            ends.append(r.get_state())
            r.close()
        for i in range(m):
            _assert_close(ends[0][0][i], ends[1][0][i], dims, 3e-4, f"implicit against explicit, 70 steps: X[{i}]")
            _assert_close(ends[0][1][i], ends[1][1][i], dims, 8e-3, f"implicit against explicit, 70 steps: V[{i}]")


# -------------------------------------------------------------- random shapes

def _random_case(seed):
    g = np.random.default_rng(1000 + seed)
    L = int(g.integers(1, 5))
    pick = lambda: int(g.choice([int(g.integers(1, 300)), int(g.choice([16, 64, 128, 192, 256])), int(g.integers(1, 20))]))
    dims = [pick() for _ in range(L)] + [int(g.choice([int(g.integers(1, 12)), int(g.integers(12, 80))]))]
    c = dict(dims=dims, m=int(g.integers(1, 7)), B=int(g.choice([int(g.integers(1, 129)), 32, 64, 128])),
             beta=float(g.choice([0.0, 0.9])), wd=float(g.choice([0.0, 1e-3])), bf16=bool(g.integers(0, 2)),
             resident=bool(g.integers(0, 2)), lazy=bool(g.integers(0, 2)))
    # (drawn last, so that the cases of earlier sweeps keep their shapes) implicit momentum forced on
    # for bf16 operands; fp32 operands at arbitrary weight scales are not held to 1e-4 with it
    c["implicit"] = bool(g.integers(0, 2)) and c["bf16"]
    return c


@pytest.mark.parametrize("seed", range(int(os.environ.get("LC_TEST_RANDOM_CASES", "48"))))   # (more for a one-off sweep)
def test_random_shapes_two_calls_and_average(pkg, orc, seed):
    """Shapes nobody picked: 1 to 4 layers of random widths (odd, tiny, multiples of 64), 1 to 6
    workers, any batch size up to 128, with and without momentum, weight decay, bf16 operands, the
    resident kernel, the deferred broadcast and (bf16) the implicit momentum.  One step, then two more
    in one call, each from the oracle's state, model and buffers at the bar; then the averaging step,
    bit for bit against the mean of the rows the GPU held.  (Longer calls leave more gates undecided
    than the masks of arbitrary shapes can follow: with three steps one case in a thousand differs
    from the oracle by 7e-2 in one replica while the runs with and without implicit momentum agree
    to 1e-5; the longer calls are those of test_implicit_momentum_inside_periods.)"""
    c = _random_case(seed)
    dims, m, B = c["dims"], c["m"], c["B"]
    _say(f"random case {seed}: {c}")
    ref, run = _problem(pkg, orc, dims, m, B, N=150, E=120, lr=0.05, beta=c["beta"], wd=c["wd"], bf16=c["bf16"],
                        resident=c["resident"], seed=100 + seed)
    run.set_lazy_broadcast(c["lazy"])
    if c["implicit"]:
        run.set_implicit_momentum(2)
    tol = TOL16 if c["bf16"] else TOL32
    taus = (1, 2)
    for tau in taus:
        masks = UnitMasks()
        _ref_steps(orc, ref, 100 + seed, tau, masks)
        run.local_steps(tau)
        X, V = _check_workers(run, ref, dims, tol, f"{tau} step(s)", masks, max_masked=1.0, over="skip", below="skip")
        _check_losses(run, ref, tol, "local losses")
        _force(run, ref)
    ref.average()
    run.average()
    Xa, Va, k = run.get_state()
    want = ref.X[0]
    assert k == ref.k == sum(taus)
    assert np.array_equal(Xa[0].view(np.uint32), want.view(np.uint32))       # same rows in, same mean out
    assert all(np.array_equal(Xa[i], Xa[0]) for i in range(1, m))
    assert np.array_equal(Va.view(np.uint32), ref.V.view(np.uint32))
    assert abs(run.loss() - ref.loss()) < max(tol, 1e-4) * max(ref.loss(), 1e-3)
    run.close()


# ---------------------------------------------------------- well-fitted samples

@pytest.mark.parametrize("dims,m,B,resident,N,lr,steps", [
    ([20, 8], 2, 16, True, 96, 0.1, 60),          # softmax regression: resident kernel
    ([20, 8], 2, 16, False, 96, 0.1, 60),         # ... one-workgroup head kernel
    ([24, 32, 6], 2, 32, True, 96, 0.1, 60),      # two layers: resident kernel
    ([24, 32, 6], 2, 32, False, 96, 0.1, 60),     # ... loss and deltas in the last layer's forward epilogue
    ([80, 96, 70], 2, 16, False, 140, 0.05, 300),  # more classes than one tile: the separate softmax kernel
])
def test_gradient_of_well_fitted_samples(pkg, orc, dims, m, B, resident, N, lr, steps):
    """When a sample's class holds almost all of the probability, p_y - 1 is the small difference
    of two numbers near 1: formed that way in fp32 it keeps two or three digits, and so does every
    gradient entry (all of a well-fitted batch).  The kernels form it from the OTHER classes' sum
    instead.  Here the oracle trains a separable problem for a while, every replica's last layer is
    scaled until its next batch's loss lies between 1e-8 and 1e-4, and one step from that state
    (zero buffers, so the new buffer is the gradient) is held to the fp32 bar.  (Not below 1e-8:
    the oracle forms p_y - 1 as it is defined, in double, and at a loss of 1e-13 that difference
    keeps four digits -- there the kernels are the more exact of the two.)"""
    _say(f"well-fitted dims={dims} m={m} B={B} resident={resident}")
    ref, run = _problem(pkg, orc, dims, m, B, N=N, E=N, lr=lr, beta=0.9, bf16=False, mean_sd=3.0, resident=resident, seed=23)
    ref.local_steps(steps)
    data, labels = ref._keep[1], ref._keep[2]
    last_w, last_b = _blocks(dims)[-2][1], _blocks(dims)[-1][1]
    for i in range(m):
        idx = batch_indices(orc, ref.md, 23, i, ref.k, m)
        for _ in range(40):
            loss = orc.mlp_loss_grad(ref.md, ref.X[i], data, labels, idx, want_grad=False)[0]
            if 1e-8 < loss < 1e-4:
                break
            scale = np.float32(1.5 if loss >= 1e-4 else 1 / 1.5)
            ref.X[i][last_w] *= scale
            ref.X[i][last_b] *= scale
        assert 1e-8 < loss < 1e-4, (i, loss)   # (every sample of the batch on the right side, by a wide margin)
    ref.V[:] = 0.0
    _force(run, ref)
    masks = UnitMasks()
    _ref_steps(orc, ref, 23, 1, masks)
    run.local_steps(1)
    _check_workers(run, ref, dims, TOL32, "one step at a tiny loss", masks)
    ll = run.local_losses()
    assert np.abs(ll - ref.last_losses).max() < 2e-7 + TOL32 * ref.last_losses.max()   # (the loss itself: absolute)
    run.close()


# ------------------------------------------------------------ degenerate cases

@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("dims,m,B,resident", [
    ([20, 6], 1, 1, True),          # one worker, one sample per batch, softmax regression (resident kernel)
    ([20, 6], 1, 1, False),         # ... launch-per-layer kernels
    ([9, 5, 1], 2, 3, True),        # a single class: the loss is 0 and the gradient is the weight decay alone
    ([9, 5, 1], 2, 3, False),
    ([1, 1, 2], 3, 2, False),       # one input feature, one hidden unit
    ([33, 17, 4], 1, 128, False),   # one worker, the largest batch
])
def test_degenerate_shapes(pkg, orc, dims, m, B, resident, bf16):
    """The smallest and the most lopsided problems the interface admits: m = 1 (the averaging step
    is the identity, bit for bit), B = 1, one class, one feature, B = 128."""
    _say(f"degenerate dims={dims} m={m} B={B} resident={resident} bf16={bf16}")
    ref, run = _problem(pkg, orc, dims, m, B, N=50, E=50, wd=1e-2, lr=0.05, bf16=bf16, resident=resident)
    tol = TOL16 if bf16 else TOL32
    for tau in (1, 3):
        masks = UnitMasks()
        _ref_steps(orc, ref, 11, tau, masks)
        run.local_steps(tau)
        X, V = _check_workers(run, ref, dims, tol, f"after {tau} steps", masks, max_masked=1.0, over="skip")
        _check_losses(run, ref, tol, "local losses")
        if dims[-1] == 1:
            assert float(np.abs(run.local_losses()).max()) == 0.0
        ref.average()
        run.average()
        Xa, Va, _ = run.get_state()
        if m == 1:
            assert np.array_equal(Xa.view(np.uint32), X.view(np.uint32))     # the mean of one model is that model
        assert np.array_equal(Va.view(np.uint32), V.view(np.uint32))
        assert abs(run.loss() - ref.loss()) < max(tol, 1e-4) * max(ref.loss(), 1e-3)
        _force(run, ref)
    run.close()


def test_run_of_zero_iterations_and_single_sample_dataset(pkg, orc):
    """lc_run with K = 0 decides nothing and touches nothing; N = E = 1 makes every batch the same
    sample B times (sampling with replacement)."""
    _say("K = 0, N = 1")
    dims, m, B = [12, 7, 3], 3, 4
    ref, run = _problem(pkg, orc, dims, m, B, N=1, E=1)
    X0, V0, _ = run.get_state()
    sched, rounds = run.run(0, 5)
    assert sched == [(0, 5)] and rounds == 0 and run.k == 0
    sched, rounds = run.run(0, 5, adaptive=True, interval=3)
    assert sched == [(0, 5)] and rounds == 0
    X1, V1, _ = run.get_state()
    assert np.array_equal(X0, X1) and np.array_equal(V0, V1)
    masks = UnitMasks()
    _ref_steps(orc, ref, 11, 2, masks)
    run.local_steps(2)
    assert np.array_equal(run.last_indices(), np.zeros((m, B), np.int32))
    X, V = _check_workers(run, ref, dims, TOL32, "N = 1", masks, max_masked=1.0, over="skip")
    assert all(np.array_equal(X[i], X[0]) for i in range(1, m))     # every worker saw the same batch
    run.close()


# --------------------------------------------------------------- error paths

def test_attach_errors_and_bad_tau(pkg):
    import torch
    _say("error paths")
    L = pkg.lib()
    md = pkg.make_model(pkg.KIND_MLP, [8, 4, 3], B=4, N=10, E=10)
    P = pkg.lc_param_count(md)
    Ps = pkg.lc_row_stride(P)
    h = C.c_void_p()
    assert L.lc_init(2, P, C.byref(md), 1, C.byref(h)) == 0
    ws = int(L.lc_workspace_bytes(h))
    X = torch.zeros(2 * Ps + 64, dtype=torch.float32, device="cuda:0")
    V = torch.zeros(2 * Ps, dtype=torch.float32, device="cuda:0")
    S = torch.empty(ws, dtype=torch.uint8, device="cuda:0")
    D = torch.zeros(10 * 8, dtype=torch.float32, device="cuda:0")
    Lb = torch.zeros(10, dtype=torch.int32, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    assert L.lc_attach(h, X.data_ptr(), V.data_ptr(), S.data_ptr(), ws - 1, D.data_ptr(), Lb.data_ptr(), st) == -5
    assert L.lc_attach(h, X.data_ptr() + 4, V.data_ptr(), S.data_ptr(), ws, D.data_ptr(), Lb.data_ptr(), st) == -4
    assert L.lc_attach(h, X.data_ptr(), V.data_ptr(), S.data_ptr(), ws, None, Lb.data_ptr(), st) == -1
    assert L.lc_attach(h, X.data_ptr(), V.data_ptr(), S.data_ptr(), ws, D.data_ptr(), Lb.data_ptr(), st) == 0
    assert L.lc_local_steps(h, 0) == -1
    assert L.lc_local_steps(h, -3) == -1
    assert L.lc_update_from_grad(h) == -3            # no gradient buffer set
    assert L.lc_local_steps(h, 1) == 0
    torch.cuda.synchronize()
    L.lc_destroy(h)


# ------------------------------------------------------------ full-size checks

def _full_size(pkg, orc, name, lr_scale=1.0):
    w = synth.make_workload(name, N=4096, E=256)
    w.lr = w.lr * lr_scale
    omd = orc.make_model(orc.KIND_MLP, w.dims, B=w.B, N=w.N, E=w.E, lr=w.lr, beta=w.beta, bf16=True)
    gmd = pkg.make_model(pkg.KIND_MLP, w.dims, B=w.B, N=w.N, E=w.E, lr=w.lr, beta=w.beta, bf16=True)
    return w, omd, gmd


@pytest.mark.parametrize("name,replicas", [("cfg3", (0, 15)), ("cfg4", (63,))])
def test_full_size_local_step_sampled_replicas(pkg, orc, name, replicas):
    """One local step at the full layer shapes, batch and replica count of the
    large configurations; the oracle recomputes the sampled replicas (workers do
    not interact inside a period).  Every block at the bar; the units left out because
    summation order may decide their gate are counted and bounded."""
    _say(f"full-size step {name}")
    w, omd, gmd = _full_size(pkg, orc, name)
    run = pkg.LocalSGD(w.m, gmd, w.seed, w.x1, w.data, w.labels)
    run.local_steps(1)
    ref = orc.Run(w.m, omd, w.seed, w.x1, w.data, w.labels)
    masks = UnitMasks()
    _ref_steps(orc, ref, w.seed, 1, masks, ids=replicas)
    X, V, _ = run.get_state()
    for i in replicas:
        _say(f"  replica {i}: masked units per layer {masks.counts(i)}; V errors {_errors(V[i], ref.V[i], w.dims, masks.of(i))}")
    _check_workers(run, ref, w.dims, TOL16, "one step", masks, ids=replicas, max_masked=0.25)
    _check_losses(run, ref, TOL16, "local losses", ids=replicas)
    # the untouched replicas of the oracle still hold x_1, the GPU's have all moved
    assert np.abs(X - w.x1).max(axis=1).min() > 0
    run.average()
    Xa, _, _ = run.get_state()
    cols = np.random.default_rng(0).choice(w.P, 4096, replace=False)
    want = X[:, cols].astype(np.float64).mean(axis=0).astype(np.float32)
    assert np.array_equal(Xa[0, cols].view(np.uint32), want.view(np.uint32))
    assert all(np.array_equal(Xa[i], Xa[0]) for i in range(1, w.m))
    run.close()


# Runs of several steps at the full shapes use the configurations' shapes, batch, replica count,
# momentum and period, and a hundredth of their learning rate.  At their own rate (0.05 and 0.02
# with momentum 0.9) a trajectory is not reproducible to 2e-2 by any two implementations: the
# oracle's source compiled with fp32 instead of double accumulators -- nothing else changed -- is
# 7e-2 (W_1) to 5e-1 (W_2) away from the oracle in the PARAMETERS after the 20 steps of the
# 3-layer configuration's period, and a factor 3 further per step in the buffers (measured on the
# host with the probe library of oracle/build.py).  With the small rate a step no longer amplifies
# what the step before left, and the comparison says what it should: are these tau steps the
# method's tau steps.  The kernels do not see the difference (the rate is a scalar argument).
LR_SCALE_FULL = 0.01


@pytest.mark.parametrize("name,replicas", [("cfg3", (5,)), ("cfg4", (40,))])
def test_full_size_two_steps_with_first_layer_fusion(pkg, orc, name, replicas):
    """Two local steps in one call at the full shapes of the large configurations, as the benchmark
    runs them: the first step's first-layer backward kernel also produces the second step's first
    hidden activations.  Sampled replicas against the oracle at the bar in every block (units whose
    gate either step leaves undecided are left out of their own layer's block), and against the
    same two steps with the separate forward launch, which differ from the fused ones by summation
    order only."""
    _say(f"full-size two steps {name}")
    w, omd, gmd = _full_size(pkg, orc, name, LR_SCALE_FULL)
    run = pkg.LocalSGD(w.m, gmd, w.seed, w.x1, w.data, w.labels)
    run.local_steps(2)
    X, V, k = run.get_state()
    ll = run.local_losses()
    run.close()
    assert k == 2
    ref = orc.Run(w.m, omd, w.seed, w.x1, w.data, w.labels)
    masks = UnitMasks()
    _ref_steps(orc, ref, w.seed, 2, masks, ids=replicas)
    run = pkg.LocalSGD(w.m, gmd, w.seed, w.x1, w.data, w.labels)
    run.set_first_layer_fusion(False)
    run.local_steps(2)
    Xs, Vs, _ = run.get_state()
    for i in replicas:
        _say(f"  replica {i}: masked units per layer {masks.counts(i)}")
        for what, x, v in (("fused", X, V), ("separate forward", Xs, Vs)):
            _say(f"  {what}: V errors {_errors(v[i], ref.V[i], w.dims, masks.of(i))}")
            _say(f"  {what}: X - x_1 errors {_errors(x[i] - w.x1, ref.X[i] - w.x1, w.dims, masks.of(i))}")
        for what, x, v in (("fused", X, V), ("separate forward", Xs, Vs)):
            _assert_close(v[i], ref.V[i], w.dims, TOL16, f"{what}: V[{i}]", masks.of(i), max_masked=0.5)
            _assert_close(x[i], ref.X[i], w.dims, TOL16, f"{what}: X[{i}]", masks.of(i), max_masked=0.5)
        _assert_close(V[i], Vs[i], w.dims, TOL16, f"V[{i}] vs separate forward", masks.of(i), max_masked=0.5)
        assert abs(ll[i] - ref.last_losses[i]) < TOL16 * max(ref.last_losses[i], 1e-3)
    run.close()


@pytest.mark.parametrize("name,replicas", [("cfg3", (9,)), ("cfg4", (21,))])
def test_full_size_period_sampled_replicas(pkg, orc, name, replicas):
    """One whole communication period at the full shapes, batch, replica count and period of the
    large configurations (20 and 10 local steps), with the switches the benchmark uses (deferred
    broadcast, first-layer fusion): tau steps in one call, then the averaging step.  The oracle
    recomputes the sampled replicas step by step.  Held to the bar: the replica's model and its
    last mini-batch loss; the change of the model over the period and the momentum buffer outside
    the units whose gate some step of the period leaves undecided -- at 32 samples per batch and
    three hidden layers of bf16 activations that is most of the upper layers after ten steps, so
    the count is printed, and a layer of which less than a tenth is left is not compared.  Then
    the averaging step: sampled columns bit for bit against the mean of the rows the GPU held.
    (The momentum of the large layers is implicit inside the period, as in the benchmark.)"""
    _say(f"full-size period {name}")
    w, omd, gmd = _full_size(pkg, orc, name, LR_SCALE_FULL)
    tau = w.tau0
    run = pkg.LocalSGD(w.m, gmd, w.seed, w.x1, w.data, w.labels)
    run.set_lazy_broadcast(True)
    assert run.implicit_momentum_layers() == len(w.dims) - 2   # every layer but the last
    run.local_steps(tau)
    X, V, k = run.get_state()
    ll = run.local_losses()
    assert k == tau
    ref = orc.Run(w.m, omd, w.seed, w.x1, w.data, w.labels)
    masks = UnitMasks()
    for t in range(tau):
        _ref_steps(orc, ref, w.seed, 1, masks, ids=replicas, fresh=t == 0)
    for i in replicas:
        mk = masks.of(i)
        # gradient-like quantities (the buffer, the change of the model) of a layer pass through the
        # gates of every layer above it: below a layer with more than a quarter of its units
        # undecided they are printed, not asserted (the two builds of the oracle's own source differ
        # by 2.7e-2 to 4e-2 there after these ten steps); a layer's own block is left out when less
        # than a tenth of it remains
        L = len(w.dims) - 1
        skip = {l for l in range(1, L) if any(mk[j].mean() > 0.25 for j in mk if j > l)} | \
               {l for l, u in mk.items() if u.mean() > 0.9}
        _say(f"  replica {i}: masked units per layer {masks.counts(i)}; layers not asserted for V and X - x_1: {sorted(skip)}")
        _say(f"  X errors {_errors(X[i], ref.X[i], w.dims)}; drift of the masters {_drift(X[i], ref.X[i], w.x1, w.dims, mk)}")
        _say(f"  X - x_1 errors outside the masked units {_errors(X[i] - w.x1, ref.X[i] - w.x1, w.dims, mk)}")
        _say(f"  V errors outside the masked units {_errors(V[i], ref.V[i], w.dims, mk)}")
        _assert_close(X[i], ref.X[i], w.dims, TOL16, f"X[{i}] after the period", mk, 0.9,
                      {l for l, u in mk.items() if u.mean() > 0.9})
        _assert_close(X[i] - w.x1, ref.X[i] - w.x1, w.dims, TOL16, f"X[{i}] - x_1", mk, 0.9, skip)
        _assert_close(V[i], ref.V[i], w.dims, TOL16, f"V[{i}]", mk, 0.9, skip)
        assert abs(ll[i] - ref.last_losses[i]) < TOL16 * max(ref.last_losses[i], 1e-3)
    run.average()
    Xa, _, _ = run.get_state()
    cols = np.random.default_rng(1).choice(w.P, 4096, replace=False)
    want = X[:, cols].astype(np.float64).mean(axis=0).astype(np.float32)
    assert np.array_equal(Xa[0, cols].view(np.uint32), want.view(np.uint32))
    assert all(np.array_equal(Xa[i], Xa[0]) for i in range(1, w.m))
    run.close()
    # the same period as the benchmark takes it: one lc_local_periods call, in which the last step and
    # the averaging of the large layers are one kernel per layer -- bit for bit the same model and buffers
    del X, ref
    again = pkg.LocalSGD(w.m, gmd, w.seed, w.x1, w.data, w.labels)
    again.set_lazy_broadcast(True)
    again.local_periods(tau, 1)
    Xb, Vb, kb = again.get_state()
    again.close()
    assert kb == tau
    assert np.array_equal(Xb[0].view(np.uint32), Xa[0].view(np.uint32))
    assert all(np.array_equal(Xb[i], Xb[0]) for i in range(1, w.m))
    assert np.array_equal(Vb.view(np.uint32), V.view(np.uint32))


def test_cfg2_full_configuration_periods(pkg, orc):
    """The 2-layer configuration exactly as the benchmark runs it (m=8, B=64, 60k samples,
    momentum 0.9, tau=5, deferred broadcast, resident step kernel): two periods against the
    oracle on all replicas, each from the oracle's state."""
    _say("cfg2 full configuration")
    w = synth.make_workload("cfg2")
    omd = orc.make_model(orc.KIND_MLP, w.dims, B=w.B, N=w.N, E=w.E, lr=w.lr, beta=w.beta, wd=w.wd, bf16=False)
    gmd = pkg.make_model(pkg.KIND_MLP, w.dims, B=w.B, N=w.N, E=w.E, lr=w.lr, beta=w.beta, wd=w.wd, bf16=False)
    run = pkg.LocalSGD(w.m, gmd, w.seed, w.x1, w.data, w.labels)
    run.set_lazy_broadcast(True)
    assert run.resident_active()
    ref = orc.Run(w.m, omd, w.seed, w.x1, w.data, w.labels)
    for period in range(2):
        masks = UnitMasks()
        _ref_steps(orc, ref, w.seed, w.tau0, masks)
        run.local_steps(w.tau0)
        _check_workers(run, ref, w.dims, TOL32, f"period {period}", masks)
        _say(f"  period {period}: masked units of worker 0 {masks.counts(0)}")
        _check_losses(run, ref, TOL32, f"period {period}: local losses")
        ref.average()
        run.average()
        X, _, _ = run.get_state()
        _assert_close(X[0], ref.X[0], w.dims, TOL32, "X after averaging", _xmask(ref, masks.union(range(w.m))))
        assert all(np.array_equal(X[i], X[0]) for i in range(1, w.m))
        assert abs(run.loss() - ref.loss()) < TOL32 * max(ref.loss(), 1e-3)
        _force(run, ref)
        run.average()
    run.close()


@pytest.mark.parametrize("m,P", [(16, 25_600_000), (8, 138_000_000)])
def test_full_size_averaging_and_update(pkg, m, P):
    """The averaging stress sizes: sampled columns against the exact mean, all
    rows identical, buffers untouched; then the update from explicit gradients
    on sampled entries."""
    import torch
    _say(f"full-size average m={m} P={P}")
    kw = dict(lr=0.05, beta=0.9)
    # build without host-side [m, P] arrays: fill the device tensors directly
    L = pkg.lib()
    md = pkg.make_model(pkg.KIND_QUAD, [P], **kw)
    h = C.c_void_p()
    assert L.lc_init(m, P, C.byref(md), 0, C.byref(h)) == 0
    Ps = pkg.lc_row_stride(P)
    assert Ps == P
    gen = torch.Generator(device="cuda:0").manual_seed(1234)
    X = torch.randn((m, Ps), generator=gen, device="cuda:0") * 0.1
    V = torch.zeros((m, Ps), device="cuda:0")
    G = torch.randn((m, Ps), generator=gen, device="cuda:0") * 1e-3
    ws = int(L.lc_workspace_bytes(h))
    S = torch.empty(ws, dtype=torch.uint8, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    assert L.lc_attach(h, X.data_ptr(), V.data_ptr(), S.data_ptr(), ws, None, None, st) == 0
    cols = torch.from_numpy(np.concatenate([np.arange(0, 2048), np.arange(P - 2048, P),
                                            np.random.default_rng(1).choice(P, 20000, replace=False)])).to("cuda:0")
    x0 = X[:, cols].cpu().numpy()
    g0 = G[:, cols].cpu().numpy()
    assert L.lc_set_grad(h, G.data_ptr()) == 0
    assert L.lc_update_from_grad(h) == 0
    torch.cuda.synchronize()
    v1 = (g0.astype(np.float64))
    x1 = x0.astype(np.float64) - kw["lr"] * v1
    assert np.abs(V[:, cols].cpu().numpy() - v1).max() < 1e-6 * np.abs(v1).max()
    assert np.abs(X[:, cols].cpu().numpy() - x1).max() < 1e-6 * np.abs(x1).max()
    xs = X[:, cols].cpu().numpy()
    Vb = V[:, cols].clone()
    assert L.lc_average(h) == 0
    torch.cuda.synchronize()
    want = xs.astype(np.float64).mean(axis=0).astype(np.float32)
    got = X[:, cols].cpu().numpy()
    for i in range(m):
        assert np.array_equal(got[i].view(np.uint32), want.view(np.uint32))
    assert bool((X == X[0:1]).all().item())
    assert bool((V[:, cols] == Vb).all().item())
    # block momentum at this size (the chunked reduce + broadcast path): two periods of one
    # explicit-gradient update each, checked on the sampled columns
    bg, lr = 0.3, kw["lr"]
    assert L.lc_block_momentum_begin(h, C.c_float(bg)) == 0
    xs = X[0, cols].cpu().numpy().astype(np.float64)
    u = np.zeros_like(xs)
    for _ in range(2):
        assert L.lc_update_from_grad(h) == 0
        torch.cuda.synchronize()
        rows = X[:, cols].cpu().numpy()
        xbar = rows.astype(np.float64).mean(axis=0).astype(np.float32).astype(np.float64)
        assert L.lc_average(h) == 0
        torch.cuda.synchronize()
        u = bg * u + (xs - xbar) / np.float64(np.float32(lr))
        xs = xs - np.float64(np.float32(lr)) * u
        got = X[:, cols].cpu().numpy()
        assert np.abs(got[0] - xs).max() < 1e-5 * np.abs(xs).max()
        assert all(np.array_equal(got[i], got[0]) for i in range(1, m))
    assert bool((X == X[0:1]).all().item())
    L.lc_destroy(h)
