"""The entry point that allocates nothing (lc_average_block_momentum_static), through the C ABI,
against the entry points it is a variant of: lc_block_momentum_begin() + lc_average() of a run
with a handle and a workspace.  Same kernel, same arithmetic: the models must agree bit for bit
(the bar for this path; that path is held to the oracle in test_gpu_parity.py).  Two runs in a
row on the one static array, the second smaller, so that what the first left behind is there to
be cleared."""
import sys

import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pkg():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1810_08313_amd as p
    p.lib()
    return p


def _one_run(pkg, m, P, lr, bg, periods, seed):
    """A block-momentum run of `periods` periods (one explicit-gradient update per period makes the
    workers differ) with the handle path, and the same run with the static entry point fed the
    handle path's models right before each averaging step."""
    import torch
    print(f"static block-momentum averaging m={m} P={P}", flush=True)
    sys.stdout.flush()
    X0, G = synth.flat_stress(seed, m, P)
    X0[:] = X0[0]                                   # synchronised start
    ones, zeros = np.ones((m, P), np.float32), np.zeros((m, P), np.float32)
    run = pkg.LocalSGD(m, pkg.make_model(pkg.KIND_QUAD, [P], lr=lr, beta=0.9), 0, qa=ones, qc=zeros)
    run.set_state(X0, zeros, 0)
    run.set_grad(G)
    run.block_momentum_begin(bg)
    Xs = run.X.clone()                              # [m, row_stride], padding zero
    Vs = torch.full_like(Xs, 3.0)                   # must come back cleared
    Vs[:, P:] = 0.0
    pkg.average_block_momentum_static(Xs, Vs, P, lr, bg, begin=True)
    torch.cuda.synchronize()
    assert bool((Xs == run.X).all().item()) and float(Vs.abs().max().item()) == 0.0
    for r in range(periods):
        run.update_from_grad()
        torch.cuda.synchronize()
        Xs.copy_(run.X)                             # the workers' models before the averaging step
        Vs.fill_(1.0)
        Vs[:, P:] = 0.0
        run.average()
        pkg.average_block_momentum_static(Xs, Vs, P, lr, bg, begin=False)
        torch.cuda.synchronize()
        want, _, _ = run.get_state()
        got = Xs[:, :P].cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), r
        assert all(np.array_equal(got[i], got[0]) for i in range(1, m))
        assert float(Vs.abs().max().item()) == 0.0
        assert float(Xs[:, P:].abs().max().item()) == 0.0 if Xs.shape[1] > P else True
    u, xs = run.get_block_momentum()
    assert np.abs(u).max() > 0 and np.array_equal(xs, got[0])
    run.close()


def test_static_entry_point_matches_the_handle_path_twice_in_a_row(pkg):
    import torch
    _one_run(pkg, 5, 70001, 0.05, 0.3, 3, seed=21)
    _one_run(pkg, 3, 1000, 0.1, 0.5, 2, seed=22)    # smaller: u and x_sync of the first run are still in the array
    # sizes beyond the static array, and other bad arguments, are refused before anything is launched
    L = pkg.lib()
    X = torch.zeros((2, 64), device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    big = pkg.STATIC_MAX_PARAMS + 1
    assert L.lc_average_block_momentum_static(X.data_ptr(), None, 2, big, big + 3, 0.1, 0.3, 0, st) == -11
    assert L.lc_average_block_momentum_static(X.data_ptr(), None, 2, 64, 62, 0.1, 0.3, 0, st) == -1     # stride < P
    assert L.lc_average_block_momentum_static(X.data_ptr(), None, 2, 60, 63, 0.1, 0.3, 0, st) == -1     # stride % 4
    assert L.lc_average_block_momentum_static(X.data_ptr() + 4, None, 2, 60, 64, 0.1, 0.3, 0, st) == -4
    assert L.lc_average_block_momentum_static(None, None, 2, 60, 64, 0.1, 0.3, 0, st) == -1
    assert L.lc_average_block_momentum_static(X.data_ptr(), None, 2, 60, 64, 0.0, 0.3, 0, st) == -1
    assert L.lc_average_block_momentum_static(X.data_ptr(), None, 2, 60, 64, 0.1, 1.0, 0, st) == -1
    with pytest.raises(pkg.LcError):
        pkg.average_block_momentum_static(X, None, big, 0.1, 0.3, False)
    torch.cuda.synchronize()
