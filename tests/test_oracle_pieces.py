"""Pins for the oracle's building blocks: index stream, bf16 rounding, the MLP
loss/gradient, the SGD update and the AdaComm controller.  Every check here
compares the oracle with something other than itself: published numbers,
library routines (torch autograd / optim, scipy), exact integer arithmetic,
or finite differences."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import synth

HERE = os.path.dirname(os.path.abspath(__file__))
M64 = 2**64 - 1
GAMMA = 0x9E3779B97F4A7C15


# ----------------------------------------------------------------- index stream

def test_mix64_matches_published_splitmix_sequence(orc):
    want = [int(l) for l in open(os.path.join(HERE, "golden", "splitmix64_seed1234567.txt"))
            if l.strip() and not l.startswith("#")]
    s, got = 1234567, []
    for _ in want:
        s = (s + GAMMA) & M64
        got.append(orc.mix64(s))
    assert got == want


def test_index_range_and_sensitivity(orc):
    N = 977
    base = orc.index(5, 1, 2, 3, N)
    assert 0 <= base < N
    # every argument moves the stream
    streams = {
        "seed": [orc.index(s, 1, 2, 3, 10**9) for s in range(64)],
        "i": [orc.index(5, i, 2, 3, 10**9) for i in range(64)],
        "k": [orc.index(5, 1, k, 3, 10**9) for k in range(64)],
        "b": [orc.index(5, 1, 2, b, 10**9) for b in range(64)],
    }
    for name, vals in streams.items():
        assert len(set(vals)) == 64, name
    # N = 1 has a single possible draw
    assert orc.index(5, 1, 2, 3, 1) == 0


def test_index_uniform_over_dataset(orc):
    # sampling with replacement from the whole set: each of N bins equally likely
    N, draws = 50, 40000
    counts = np.zeros(N)
    j = 0
    for k in range(100):
        for i in range(8):
            for b in range(50):
                counts[orc.index(42, i, k, b, N)] += 1
                j += 1
    assert j == draws
    chi2 = float(((counts - draws / N) ** 2 / (draws / N)).sum())
    # 49 degrees of freedom: mean 49, sd ~9.9; 110 is beyond 6 sigma
    assert chi2 < 110.0


def test_index_workers_are_independent_streams(orc):
    # the batches of two workers at the same iteration share no more indices than chance
    N, B = 10**6, 256
    a = {orc.index(9, 0, 7, b, N) for b in range(B)}
    c = {orc.index(9, 1, 7, b, N) for b in range(B)}
    assert len(a & c) <= 2


def _mix_py(z):
    """SplitMix64 output function (Steele, Lea & Flood 2014), written out in Python integers."""
    z &= M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def test_index_chaining_matches_the_stated_formula(orc):
    """The documented stream: idx = mix(mix(mix(seed + G (k+1)) + G (i+1)) + G (b+1)) mod N --
    iteration first, then worker, then position in the batch, all in arithmetic modulo 2^64.
    A transposed argument, a missing +1 or another order of the three draws fails here."""
    g = np.random.default_rng(17)
    cases = [(0, 0, 0, 0, 7), (2**64 - 1, 3, 2**40, 127, 50000), (11, 63, 123456789, 31, 2**31 - 1)]
    for _ in range(300):
        cases.append((int(g.integers(0, 2**63)) * 2 + int(g.integers(0, 2)), int(g.integers(0, 65535)),
                      int(g.integers(0, 2**45)), int(g.integers(0, 128)), int(g.integers(1, 2**31 - 1))))
    for seed, i, k, b, N in cases:
        h = _mix_py(seed + GAMMA * (k + 1))
        h = _mix_py(h + GAMMA * (i + 1))
        h = _mix_py(h + GAMMA * (b + 1))
        assert orc.index(seed, i, k, b, N) == h % N, (seed, i, k, b, N)
    # the three arguments are not interchangeable
    assert len({orc.index(5, 1, 2, 3, 10**9), orc.index(5, 2, 1, 3, 10**9), orc.index(5, 3, 2, 1, 10**9),
                orc.index(5, 1, 3, 2, 10**9)}) == 4


# ------------------------------------------------------------------ bf16 round

def test_bf16_round_matches_torch_conversion(orc):
    g = np.random.default_rng(0)
    vals = np.concatenate([
        g.standard_normal(2000).astype(np.float32),
        (g.standard_normal(500) * 1e-30).astype(np.float32),
        (g.standard_normal(500) * 1e30).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 1.0078125, 3.3895314e38, np.inf, -np.inf,
                  1e-40, -1e-40], dtype=np.float32),
    ])
    got = orc.bf16_round(vals)
    want = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # ties go to the even mantissa: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6
    assert orc.bf16_round(np.float32(1.00390625)) == np.float32(1.0)
    assert orc.bf16_round(np.float32(1.01171875)) == np.float32(1.015625)
    # the shared input generator's rounding agrees too
    assert np.array_equal(synth.bf16_representable(vals[:3000]).view(np.uint32),
                          got[:3000].view(np.uint32))


# ------------------------------------------------------------ MLP loss and grad

def _unpack(x, dims):
    out, off = [], 0
    for l in range(len(dims) - 1):
        nw = dims[l] * dims[l + 1]
        out.append((x[off:off + nw].reshape(dims[l], dims[l + 1]), x[off + nw:off + nw + dims[l + 1]]))
        off += nw + dims[l + 1]
    assert off == x.size
    return out


def _np_loss(x, dims, xb, yb):
    """Textbook definition in float64: ReLU MLP, mean softmax cross-entropy."""
    from scipy.special import logsumexp
    a = xb.astype(np.float64)
    layers = _unpack(x.astype(np.float64), dims)
    for l, (W, b) in enumerate(layers):
        a = a @ W + b
        if l < len(layers) - 1:
            a = np.maximum(a, 0.0)
    lse = logsumexp(a, axis=1)
    return float(np.mean(lse - a[np.arange(len(yb)), yb]))


@pytest.mark.parametrize("dims", [[6, 3], [5, 4, 3], [4, 6, 5, 3]])
def test_loss_and_grad_against_definition_and_finite_differences(orc, dims):
    g = np.random.default_rng(len(dims))
    N, B = 20, 4
    data = g.standard_normal((N, dims[0])).astype(np.float32)
    labels = g.integers(0, dims[-1], N).astype(np.int32)
    x = (g.standard_normal(synth.param_count(dims)) * 0.5).astype(np.float32)
    idx = [3, 17, 3, 8]  # a repeated sample counts twice (sampling with replacement)
    md = orc.make_model(orc.KIND_MLP, dims, B=B, N=N)
    loss, grad = orc.mlp_loss_grad(md, x, data, labels, idx)
    xb, yb = data[idx], labels[idx]
    assert abs(loss - _np_loss(x, dims, xb, yb)) < 2e-6 * max(1.0, abs(loss))
    h = 1e-5
    for j in g.choice(x.size, size=min(x.size, 40), replace=False):
        xp, xm = x.astype(np.float64), x.astype(np.float64)
        xp[j] += h
        xm[j] -= h
        fd = (_np_loss(xp, dims, xb, yb) - _np_loss(xm, dims, xb, yb)) / (2 * h)
        assert abs(fd - grad[j]) < 5e-6 + 1e-4 * abs(fd), (j, fd, grad[j])


def _np_preactivations(x, dims, xb, bf16):
    """Z_l of the hidden layers in float64 numpy; with bf16 the operands (inputs, weights, hidden
    activations) are rounded through torch's conversion, biases and sums are not."""
    q = (lambda t: torch.from_numpy(np.asarray(t, np.float32)).to(torch.bfloat16).to(torch.float64).numpy()) \
        if bf16 else (lambda t: np.asarray(t, np.float64))
    a = q(xb)
    out = []
    layers = _unpack(x, dims)
    for W, b in layers[:-1]:
        z = a @ q(W) + b.astype(np.float64)
        out.append(z)
        a = q(np.maximum(z, 0.0).astype(np.float32))   # activations are stored as fp32, then rounded
    return out


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("dims,B", [([7, 5, 3], 4), ([9, 6, 11, 4], 5), ([12, 8, 5, 7, 3], 3), ([6, 4], 2)])
def test_preactivations_against_numpy_forward_values_and_layout(orc, dims, B, bf16):
    """The observer that tells the GPU tests which ReLU gates are too close to zero to call: its
    values against a float64 numpy forward pass, and its layout -- one [B, d_l] block per hidden
    layer, sample-major, layers side by side in one row of d_1 + ... + d_{L-1} values.  The
    layer widths all differ, so a transposed or shifted block cannot pass."""
    g = np.random.default_rng(sum(dims) + B)
    N = 30
    data = g.standard_normal((N, dims[0])).astype(np.float32)
    if bf16:
        data = synth.bf16_representable(data)
    x = (g.standard_normal(synth.param_count(dims)) * 0.4).astype(np.float32)
    idx = g.integers(0, N, B)
    md = orc.make_model(orc.KIND_MLP, dims, B=B, N=N, bf16=bf16)
    got = orc.mlp_preactivations(md, x, data, idx)
    want = _np_preactivations(x, dims, data[idx], bf16)
    assert len(got) == len(dims) - 2 == len(want)
    for l, (zg, zw) in enumerate(zip(got, want), start=1):
        assert zg.shape == (B, dims[l]) and zg.dtype == np.float32
        # layer 1 sums exact products in double on both sides: agreement to the fp32 store.  Above
        # it a hidden activation that sits on a bf16 rounding boundary may round the other way in
        # the fp32-stored oracle than in float64 numpy (2^-8 of one term): allow for that.
        tol = 2e-7 if (not bf16 or l == 1) else 2e-3
        assert np.abs(zg - zw).max() <= tol * max(1.0, np.abs(zw).max()), (l, np.abs(zg - zw).max())
    # the gates the oracle's backward pass uses are the signs of these values: a unit whose
    # pre-activation is positive passes its delta on, any other does not
    if len(dims) == 3 and not bf16:
        labels = g.integers(0, dims[-1], N).astype(np.int32)
        _, grad = orc.mlp_loss_grad(md, x, data, labels, idx)
        W1g = grad[:dims[0] * dims[1]].reshape(dims[0], dims[1])
        dead = np.nonzero((got[0] <= 0).all(axis=0))[0]
        for j in dead:
            assert np.abs(W1g[:, j]).max() == 0.0


def test_f32acc_probe_is_the_same_computation_in_another_precision(orc):
    """The fp32-accumulation build of the oracle's source (a sensitivity probe, never a reference):
    same results to fp32 summation error, not the same bits, and where its pre-activations change
    sign against the oracle's they are tiny on both sides.  This is the evidence behind the gate
    masks of the GPU tests: which units can fall either way is decided by |z| against the
    summation error, nothing else."""
    dims, B, N = [300, 200, 60, 10], 16, 200
    g = np.random.default_rng(3)
    data = g.standard_normal((N, dims[0])).astype(np.float32)
    labels = g.integers(0, dims[-1], N).astype(np.int32)
    x = synth.init_params(9, dims)
    idx = g.integers(0, N, B)
    md = orc.make_model(orc.KIND_MLP, dims, B=B, N=N)
    z64 = orc.mlp_preactivations(md, x, data, idx)
    z32 = orc.mlp_preactivations(md, x, data, idx, f32acc=True)
    l64, g64 = orc.mlp_loss_grad(md, x, data, labels, idx)
    l32, g32 = orc.mlp_loss_grad(md, x, data, labels, idx, f32acc=True)
    assert not np.array_equal(g64, g32)
    assert abs(l64 - l32) < 1e-5 * abs(l64)
    for a, b in zip(z64, z32):
        rms = float(np.sqrt(np.mean(a.astype(np.float64) ** 2)))
        assert np.abs(a - b).max() < 2e-5 * rms
        flipped = (a > 0) != (b > 0)
        assert np.abs(a[flipped]).max(initial=0.0) < 2e-5 * rms
    # with no gate between the two sides the gradients agree to summation error
    if not any(((a > 0) != (b > 0)).any() for a, b in zip(z64, z32)):
        assert np.abs(g64 - g32).max() < 1e-4 * np.abs(g64).max()


def _torch_params(x, dims, dtype=torch.float64):
    ps = []
    for W, b in _unpack(x, dims):
        ps.append(torch.tensor(W, dtype=dtype, requires_grad=True))
        ps.append(torch.tensor(b, dtype=dtype, requires_grad=True))
    return ps


def _flat(ps, attr=None):
    return np.concatenate([(p if attr is None else getattr(p, attr)).detach().numpy().reshape(-1) for p in ps])


def _q(t):
    return t.to(torch.float32).to(torch.bfloat16).to(t.dtype)


class _RoundSTE(torch.autograd.Function):
    """bf16 rounding with an identity backward."""

    @staticmethod
    def forward(ctx, t):
        return _q(t)

    @staticmethod
    def backward(ctx, gout):
        return gout


def _torch_loss(ps, xb, yb, bf16):
    a = torch.tensor(xb, dtype=torch.float64)
    L = len(ps) // 2
    for l in range(L):
        W, b = ps[2 * l], ps[2 * l + 1]
        if bf16:
            z = _RoundSTE.apply(a) @ _RoundSTE.apply(W) + b
            z.register_hook(_q)  # the delta of every layer is rounded when it is produced
        else:
            z = a @ W + b
        a = z
        if l < L - 1:
            a = torch.relu(z)
            if bf16:
                a = _RoundSTE.apply(a)
    return torch.nn.functional.cross_entropy(a, torch.tensor(yb, dtype=torch.long))


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("beta,wd", [(0.0, 0.0), (0.9, 0.0), (0.9, 5e-4)])
def test_steps_against_torch_autograd_and_optim_sgd(orc, bf16, beta, wd):
    """Several (momentum-)SGD steps of one worker against PyTorch CPU autograd in
    fp64 driving torch.optim.SGD -- the library's buffer form v = beta v + g,
    x = x - lr v, weight decay added to the gradient."""
    dims = [12, 9, 7, 4]
    g = np.random.default_rng(7)
    N, B, lr = 64, 8, 0.05
    data = g.standard_normal((N, dims[0])).astype(np.float32)
    if bf16:
        data = synth.bf16_representable(data)
    labels = g.integers(0, dims[-1], N).astype(np.int32)
    x = synth.init_params(3, dims)
    x[-4:] = 0.1  # non-zero biases so that their path is exercised
    md = orc.make_model(orc.KIND_MLP, dims, B=B, N=N, lr=lr, beta=beta, wd=wd, bf16=bf16)
    ps = _torch_params(x, dims)
    opt = torch.optim.SGD(ps, lr=lr, momentum=beta, weight_decay=wd)
    xo, vo = x.copy(), np.zeros_like(x)
    for step in range(5):
        idx = g.integers(0, N, B)
        loss, grad = orc.mlp_loss_grad(md, xo, data, labels, idx)
        opt.zero_grad()
        tl = _torch_loss(ps, data[idx], labels[idx], bf16)
        tl.backward()
        tg = _flat(ps, "grad")
        scale = np.abs(tg).max()
        assert abs(loss - tl.item()) < 5e-6 * max(1.0, abs(loss))
        assert np.abs(grad - tg).max() < 2e-6 * scale + (1e-3 * scale if bf16 else 0.0), step
        orc.sgd_update(xo, vo, grad, lr, beta, wd)
        opt.step()
        tx = _flat(ps)
        tol = 2e-3 if bf16 else 1e-5
        assert np.abs(xo - tx).max() < tol * np.abs(tx).max(), step


def test_bf16_mode_differs_from_fp32_mode_but_stays_close(orc):
    dims = [32, 16, 5]
    g = np.random.default_rng(11)
    N, B = 40, 8
    data = synth.bf16_representable(g.standard_normal((N, dims[0])).astype(np.float32))
    labels = g.integers(0, dims[-1], N).astype(np.int32)
    x = synth.init_params(5, dims)
    idx = g.integers(0, N, B)
    l32, g32 = orc.mlp_loss_grad(orc.make_model(orc.KIND_MLP, dims, B=B, N=N), x, data, labels, idx)
    l16, g16 = orc.mlp_loss_grad(orc.make_model(orc.KIND_MLP, dims, B=B, N=N, bf16=True), x, data, labels, idx)
    assert not np.array_equal(g32, g16)
    assert abs(l32 - l16) < 2e-2 * abs(l32)
    assert np.abs(g32 - g16).max() < 2e-2 * np.abs(g32).max()


# ------------------------------------------------------------------ controller

def test_controller_closed_forms(orc):
    # F_l = F_0 keeps tau_0; a quarter of the loss halves an even tau_0
    for tau0 in (1, 2, 4, 10, 20, 100):
        assert orc.next_tau(2.5, 2.5, tau0) == tau0
        if tau0 % 2 == 0:
            assert orc.next_tau(2.0, 0.5, tau0) == tau0 // 2
    assert orc.next_tau(1.0, 0.0, 20) == 1          # never below the fully synchronous limit
    assert orc.next_tau(1.0, 1e-12, 20) == 1
    assert orc.next_tau(1.0, 4.0, 10) == 20         # no upper clamp in the basic rule
    # monotone in the current loss
    last = 0
    for f in np.linspace(0.0, 3.0, 301):
        t = orc.next_tau(1.7, float(f), 13)
        assert t >= max(last, 1)
        last = t
    for bad in [(0.0, 1.0, 5), (-1.0, 1.0, 5), (1.0, -0.1, 5), (float("nan"), 1.0, 5),
                (1.0, float("inf"), 5), (1.0, 1.0, 0)]:
        assert orc.next_tau(*bad) < 0


def test_controller_against_exact_rational_arithmetic(orc):
    """ceil(sqrt(Fl/F0) tau0) is the least integer n with n^2 F0 >= tau0^2 Fl.
    Checked wherever the exact value is at least 1e-9 away from an integer
    (closer than that the double evaluation may legitimately land on the other
    side; exactly representable perfect squares are checked separately above)."""
    checked = 0
    for F0 in range(1, 40):
        for Fl in range(0, 60):
            for tau0 in (1, 3, 7, 10, 20, 64):
                n = max(1, math.isqrt(tau0 * tau0 * Fl // F0))
                while n * n * F0 < tau0 * tau0 * Fl:
                    n += 1
                while n > 1 and (n - 1) * (n - 1) * F0 >= tau0 * tau0 * Fl:
                    n -= 1
                exact = math.sqrt(Fraction(tau0 * tau0 * Fl, F0))
                if abs(exact - round(exact)) < 1e-9:
                    continue
                assert orc.next_tau(float(F0), float(Fl), tau0) == n, (F0, Fl, tau0)
                checked += 1
    assert checked > 10000
