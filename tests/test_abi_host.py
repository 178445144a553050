"""CPU-side checks of the C ABI: the library loads, exports every symbol the
header declares, validates its arguments, and its pure host function (the
AdaComm controller) agrees bit for bit with the oracle.  No kernel is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pkg():
    import paper_1810_08313_amd as p
    p.lib()
    return p


def _declared_functions():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if fn.endswith(".h"):
            src = open(os.path.join(ROOT, "include", fn)).read()
            src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
            names += re.findall(r"\b((?:lc|adacomm)_[a-z_0-9]+)\s*\(", src)
    return sorted(set(names))


def test_library_exports_every_declared_symbol(pkg):
    names = _declared_functions()
    assert {"lc_init", "lc_local_steps", "lc_average", "lc_loss", "adacomm_next_tau", "lc_attach",
            "lc_run", "lc_update_from_grad"} <= set(names)
    L = pkg.lib()
    for n in names:
        assert hasattr(L, n), n


def test_param_count_and_row_stride(pkg):
    import synth
    for dims in ([64, 10], [784, 256, 10], [3072, 1024, 1024, 10], [3072, 2048, 2048, 2048, 10]):
        md = pkg.make_model(pkg.KIND_MLP, dims, B=32, N=100, E=10)
        assert pkg.lc_param_count(md) == synth.param_count(dims)
    assert pkg.lc_param_count(pkg.make_model(pkg.KIND_MLP, [3072, 2048, 2048, 2048, 10], B=32, N=9, E=9)) == 14706698
    assert pkg.lc_row_stride(650) == 704 and pkg.lc_row_stride(64) == 64 and pkg.lc_row_stride(1) == 64
    assert pkg.lc_row_stride(25_600_000) == 25_600_000
    assert pkg.lc_row_stride(0) < 0


def test_init_rejects_bad_arguments(pkg):
    L = pkg.lib()
    h = C.c_void_p()
    good = pkg.make_model(pkg.KIND_MLP, [8, 4, 3], B=4, N=10, E=10)
    P = pkg.lc_param_count(good)
    assert L.lc_init(0, P, C.byref(good), 1, C.byref(h)) == -1           # m < 1
    assert L.lc_init(2, P + 1, C.byref(good), 1, C.byref(h)) == -2       # P != P(model)
    assert L.lc_init(2, P, None, 1, C.byref(h)) == -1
    for kw in (dict(B=0), dict(B=129), dict(E=11), dict(N=0)):
        args = dict(B=4, N=10, E=10)
        args.update(kw)
        bad = pkg.make_model(pkg.KIND_MLP, [8, 4, 3], **args)
        assert L.lc_init(2, P, C.byref(bad), 1, C.byref(h)) < 0, kw
    bad = pkg.make_model(pkg.KIND_MLP, [8, 0, 3], B=4, N=10, E=10)
    assert L.lc_init(2, P, C.byref(bad), 1, C.byref(h)) < 0
    assert L.lc_init(2, P, C.byref(good), 1, C.byref(h)) == 0 and h.value
    # not attached yet: every device entry point refuses
    assert L.lc_local_steps(h, 1) == -3
    assert L.lc_local_periods(h, 1, 1) == -3 and L.lc_local_periods(None, 1, 1) == -1
    assert L.lc_grid_search_tau0(h, None, 1, 1, None, None, None) == -3
    assert L.lc_average(h) == -3
    out = C.c_double()
    assert L.lc_loss(h, C.byref(out)) == -3
    assert L.lc_update_from_grad(h) == -3
    assert L.lc_workspace_bytes(h) > 0
    # switches of the resident step kernel: argument checks need no device
    assert L.lc_set_xcd_local_exchange(h, 0) == 0 and L.lc_set_xcd_local_exchange(None, 1) == -1
    assert L.lc_set_first_layer_fusion(h, 0) == 0 and L.lc_set_first_layer_fusion(None, 1) == -1
    assert L.lc_set_deferred_update(h, 0) == 0 and L.lc_set_deferred_update(None, 1) == -1
    assert L.lc_set_resident(h, 0) == 0 and L.lc_set_resident(h, 1) == 0 and L.lc_set_resident(None, 1) == -1
    assert L.lc_set_barrier_polls(h, -1) == -1 and L.lc_set_barrier_polls(h, 0) == 0
    assert L.lc_resident_active(h) == -3 and L.lc_resident_active(None) == -1
    assert pkg.lib().lc_strerror(-9).decode().startswith("replica barrier timed out")
    L.lc_destroy(h)
    assert pkg.lib().lc_strerror(-5).decode() == "scratch buffer too small"


def test_controller_bit_exact_against_oracle(pkg, orc):
    g = np.random.default_rng(3)
    L = pkg.lib()
    n = 0
    for tau0 in (1, 2, 5, 10, 20, 37, 100, 1000):
        for F0 in np.concatenate([g.uniform(1e-3, 5.0, 40), [1.0, 2.302585092994046, 0.1]]):
            for Fl in np.concatenate([g.uniform(0.0, 6.0, 40), [0.0, F0, F0 / 4, F0 * 4, 1e-300]]):
                a = L.adacomm_next_tau(float(F0), float(Fl), tau0)
                assert a == orc.next_tau(float(F0), float(Fl), tau0)
                assert a >= 1
                n += 1
    assert n > 10000
    for bad in [(0.0, 1.0, 5), (-1.0, 1.0, 5), (1.0, -0.1, 5), (float("nan"), 1.0, 5), (1.0, float("inf"), 5),
                (1.0, 1.0, 0), (1e-300, 1e300, 1000)]:
        assert L.adacomm_next_tau(*bad) < 0
        assert orc.next_tau(*bad) < 0
    with pytest.raises(pkg.LcError):
        pkg.adacomm_next_tau(0.0, 1.0, 5)


def test_refined_controller_bit_exact_against_oracle(pkg, orc):
    g = np.random.default_rng(5)
    L = pkg.lib()
    n = 0
    for _ in range(20000):
        F0, Fl = float(g.uniform(1e-3, 5.0)), float(g.uniform(0.0, 6.0))
        tau0, tau_prev = int(g.integers(1, 100)), int(g.integers(1, 120))
        gamma = float(g.choice([0.5, 0.25, 0.75, 0.9]))
        slack = int(g.integers(0, 3))
        lr0, lrl = float(g.choice([0.4, 0.2, 0.1])), float(g.choice([0.4, 0.04, 0.004, 0.1]))
        ch = int(g.integers(0, 2))
        a = L.adacomm_next_tau_ex(F0, Fl, tau0, tau_prev, gamma, slack, lr0, lrl, ch)
        assert a == orc.next_tau_ex(F0, Fl, tau0, tau_prev, gamma, slack, lr0, lrl, bool(ch)) and a >= 1
        n += 1
    for bad in [(0.0, 1.0, 5, 5, 0.5, 0, 1.0, 1.0, 0), (1.0, 1.0, 5, 0, 0.5, 0, 1.0, 1.0, 0),
                (1.0, 1.0, 5, 5, 0.0, 0, 1.0, 1.0, 0), (1.0, 1.0, 5, 5, 0.5, -1, 1.0, 1.0, 0),
                (1.0, 1.0, 5, 5, 0.5, 0, 0.0, 1.0, 0), (1.0, 1.0, 5, 5, 0.5, 0, 1.0, float("nan"), 0)]:
        assert L.adacomm_next_tau_ex(*bad) < 0 and orc.next_tau_ex(*bad[:8], bool(bad[8])) < 0
    assert pkg.adacomm_next_tau_ex(2.0, 2.0, 20, 20) == 10


def test_no_cpu_fallback_without_gpu(pkg):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    md = pkg.make_model(pkg.KIND_MLP, [8, 4, 3], B=4, N=10, E=10)
    with pytest.raises(RuntimeError):
        pkg.LocalSGD(2, md, 1, np.zeros(pkg.lc_param_count(md), np.float32),
                     np.zeros((10, 8), np.float32), np.zeros(10, np.int32))


def test_product_path_does_not_touch_the_oracle():
    pk = os.path.join(ROOT, "paper_1810_08313_amd")
    for dp, _, fns in os.walk(pk):
        for fn in fns:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dp, fn)).read()
                assert "oracle" not in src.lower().replace("no cpu path", ""), os.path.join(dp, fn)


def test_public_header_is_plain_c(tmp_path):
    """include/localcomm.h is the boundary: it must compile as C99 and as C++ on its own."""
    import shutil
    import subprocess
    inc = os.path.join(ROOT, "include")
    for cc, std, ext in (("gcc", "-std=c99", "c"), ("g++", "-std=c++17", "cpp")):
        if not shutil.which(cc):
            pytest.skip(f"{cc} not available")
        src = tmp_path / f"use_header.{ext}"
        src.write_text('#include "localcomm.h"\nint main(void) { return LC_OK; }\n')
        subprocess.run([cc, std, "-pedantic", "-Wall", "-Werror", "-I", inc, "-c", str(src), "-o", str(tmp_path / f"o_{ext}.o")],
                       check=True, capture_output=True)
