"""The gate-uncertainty bound of the GPU parity tests (tests/gate_bounds.py), checked on the CPU
against the one other summation precision at hand: the fp32-accumulation build of the oracle's
source.  Every ReLU gate that changes side between double and fp32 accumulation must be among the
gates the bound calls undecided, and the bound must stay small enough to leave a test."""
import numpy as np
import pytest

import synth
from gate_bounds import UnitMasks, batch_indices, undecided_gates

# sequential fp32 summation (the probe) errs more than the blocked sums of the matrix cores
EPS_PROBE = 1.5e-5


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("dims,B", [([300, 200, 10], 32), ([400, 300, 200, 10], 48), ([256, 512, 384, 256, 10], 32),
                                    ([1024, 2048, 2048, 2048, 10], 32)])
def test_flips_between_summation_precisions_are_all_flagged(orc, dims, B, bf16):
    N = 400
    flagged_total = flips_total = gates_total = 0
    deep = len(dims) == 5 and dims[1] >= 2048     # the widths, batch and image-like inputs of the largest configuration
    for seed in range(6 if deep else 3):
        data, labels = (synth.image_like if deep else synth.gaussian_mixture)(seed + 1, N, dims[0], dims[-1], 0.5)
        if bf16:
            data = synth.bf16_representable(data)
        x = synth.init_params(seed + 1, dims)
        md = orc.make_model(orc.KIND_MLP, dims, B=B, N=N, bf16=bf16)
        idx = batch_indices(orc, md, seed, 0, 0, 1)
        und = undecided_gates(orc, md, x, data, idx, eps_sum=EPS_PROBE)
        z64 = orc.mlp_preactivations(md, x, data, idx)
        z32 = orc.mlp_preactivations(md, x, data, idx, f32acc=True)
        assert sorted(und) == list(range(1, len(dims) - 1))
        for l, (a, b) in enumerate(zip(z64, z32), start=1):
            flips = (a > 0) != (b > 0)
            assert not (flips & ~und[l]).any(), (seed, l, int((flips & ~und[l]).sum()))
            flips_total += int(flips.sum())
            flagged_total += int(und[l].sum())
            gates_total += flips.size
    # the bound is not vacuous: well under a per cent of the gates (fp32: a handful) ...
    assert flagged_total < (0.01 if bf16 else 0.001) * gates_total, (flagged_total, gates_total)
    # ... and neither is this test: the deep bf16 case does have gates that change side
    if bf16 and len(dims) == 5 and dims[1] >= 1024:
        assert flips_total > 0
    print(f"bf16={bf16} dims={dims}: {flips_total} flips, {flagged_total} flagged of {gates_total} gates")


def test_weight_drift_widens_the_bound_and_masks_accumulate(orc):
    dims, B, N = [300, 200, 100, 10], 32, 400
    data, _ = synth.gaussian_mixture(4, N, dims[0], dims[-1], mean_sd=0.5)
    data = synth.bf16_representable(data)
    x = synth.init_params(4, dims)
    md = orc.make_model(orc.KIND_MLP, dims, B=B, N=N, bf16=True)
    idx = batch_indices(orc, md, 4, 0, 0, 1)
    fresh = undecided_gates(orc, md, x, data, idx)
    moved = (x + np.float32(0.5) * synth.init_params(5, dims)).astype(np.float32)   # far from where the sides agreed
    drift = undecided_gates(orc, md, moved, data, idx, x0=x)
    again = undecided_gates(orc, md, moved, data, idx)
    for l in again:
        assert not (again[l] & ~drift[l]).any()          # a wider bound flags a superset
    fresh = again
    for l in fresh:
        assert not (fresh[l] & ~drift[l]).any()          # a wider bound flags a superset
    assert sum(int(g.sum()) for g in drift.values()) > sum(int(g.sum()) for g in fresh.values())
    masks = UnitMasks()
    masks.add(0, fresh)
    masks.add(0, drift)
    masks.add(1, fresh)
    assert masks.counts(0) == {l: int(g.any(axis=0).sum()) for l, g in drift.items() if g.any()}
    u = masks.union([0, 1])
    for l in u:
        assert np.array_equal(u[l], drift[l].any(axis=0))
    assert masks.of(7) == {}
