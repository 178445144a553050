"""Pins for the oracle's partition sampler (Sec. 5.1: each worker owns a partition
of the data set which is reshuffled after every epoch)."""
import numpy as np
import pytest

from test_oracle_runs import _small_problem


@pytest.mark.parametrize("N,m,B", [(1000, 4, 32), (1003, 7, 10), (64, 2, 32), (50000, 16, 128)])
def test_every_epoch_is_a_shuffled_pass_over_the_own_partition(orc, N, m, B):
    S = (N // m) // B
    workers = range(m) if N <= 2000 else (0, m - 1)
    seen_all = []
    for i in workers:
        lo, hi = i * N // m, (i + 1) * N // m
        orders = []
        for e in range(3):
            idx = [orc.index_partition(7, i, e * S + k, b, N, m, B) for k in range(S) for b in range(B)]
            assert all(lo <= j < hi for j in idx)            # never leaves the worker's partition
            assert len(set(idx)) == len(idx) == S * B         # no sample twice within an epoch
            orders.append(idx)
        assert orders[0] != orders[1] != orders[2]            # reshuffled every epoch
        if S * B >= 64:
            # a real shuffle: positions are not correlated with the sample order (the correlation of
            # a random permutation of n items has standard deviation 1 / sqrt(n - 1))
            r = np.corrcoef(np.arange(S * B), np.array(orders[0]))[0, 1]
            assert abs(r) < 4.5 / np.sqrt(S * B - 1)
        seen_all.append(set(orders[0]))
    for a in range(len(seen_all)):
        for c in range(a + 1, len(seen_all)):
            assert not (seen_all[a] & seen_all[c])            # partitions are disjoint


def test_partition_permutation_is_a_bijection_of_the_whole_partition(orc):
    # n = 25 samples per worker, B = 5: S * B = n, so one epoch must visit every sample exactly once
    N, m, B = 100, 4, 5
    for i in range(m):
        idx = sorted(orc.index_partition(3, i, k, b, N, m, B) for k in range(5) for b in range(B))
        assert idx == list(range(i * 25, (i + 1) * 25))
    assert orc.index_partition(3, 0, 0, 0, 100, 4, 26) == -1   # partition smaller than a batch


def test_sampler_choice_changes_the_run_only_through_the_batches(orc):
    a = _small_problem(orc, m=3)[0]
    run, md, data, labels, x1 = _small_problem(orc, m=3)
    md2 = orc.make_model(orc.KIND_MLP, list(md.dims[:md.n_layers + 1]), B=md.B, N=md.N, E=md.E, lr=md.lr, sampler=1)
    b = orc.Run(3, md2, 1810_08313, x1, data, labels)
    a.local_steps(2)
    b.local_steps(2)
    assert not np.array_equal(a.X, b.X)
    # replaying worker 1's partition batches through the gradient routine reproduces its model
    x, v = x1.copy(), np.zeros_like(x1)
    for k in range(2):
        idx = [orc.index_partition(1810_08313, 1, k, bb, md.N, 3, md.B) for bb in range(md.B)]
        _, g = orc.mlp_loss_grad(md, x, data, labels, idx)
        orc.sgd_update(x, v, g, md.lr, 0.0, 0.0)
    assert np.array_equal(b.X[1], x)
