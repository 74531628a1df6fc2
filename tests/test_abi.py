"""The C ABI: the built library loads and exports every function the header
declares; host-only entry points (planner, packing, error text) behave."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import planner as OP
from paper_2408_10284_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2408_10284_amd import build
        build.build(verbose=False)
    return B.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "adapmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:adapmoe|cache|moe)_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert len(names) >= 25
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.exported_names()) == names     # the binding covers the same set


def test_strerror(lib):
    assert lib.adapmoe_strerror(0) == b"ok"
    assert b"resident" in lib.adapmoe_strerror(B.ENORES)


def test_bad_config_rejected_without_gpu(lib):
    cfg = B.Config(500, 1024, 8, 1, B.BF16, 1, 0, 0)   # H not a multiple of 512
    n = ctypes.c_size_t()
    assert lib.adapmoe_expert_bytes(ctypes.byref(cfg), ctypes.byref(n)) == B.EINVAL
    ctx = ctypes.c_void_p()
    assert lib.adapmoe_create(ctypes.byref(cfg), ctypes.byref(ctx)) == B.EINVAL
    cfg = B.Config(4096, 14336, 8, 32, B.BF16, 1, 0, 0)
    assert B.adapmoe_expert_bytes(cfg) == 352321536


def test_pack_layout(lib):
    cfg = B.Config(512, 1024, 2, 1, B.BF16, 1, 0, 0)
    rng = np.random.default_rng(0)
    w1 = rng.integers(0, 65536, (1024, 512), dtype=np.uint16)
    w3 = rng.integers(0, 65536, (1024, 512), dtype=np.uint16)
    w2 = rng.integers(0, 65536, (512, 1024), dtype=np.uint16)
    out = np.zeros(B.adapmoe_expert_bytes(cfg), dtype=np.uint8)
    B.adapmoe_pack_expert(cfg, w1, w3, w2, out)
    img = out.view(np.uint16)
    gu = img[: 2 * 1024 * 512].reshape(1024, 2, 512)
    np.testing.assert_array_equal(gu[:, 0], w1)
    np.testing.assert_array_equal(gu[:, 1], w3)
    np.testing.assert_array_equal(img[2 * 1024 * 512:].reshape(512, 1024), w2)


def test_planner_matches_checker(lib):
    rng = np.random.default_rng(5)
    for trial in range(60):
        L, N = int(rng.integers(1, 9)), int(rng.integers(2, 9))
        Ctot = int(rng.integers(0, L * N + 3))
        a = np.round(rng.uniform(0, 1, L) * 1024) / 1024
        beta = np.round(rng.uniform(0, 1, L) * 1024) / 1024
        t, cost = B.cache_plan(L, N, Ctot, a, beta)
        t_ref, cost_ref = OP.plan(L, N, Ctot, a, beta)
        assert abs(cost - cost_ref) < 1e-12
        assert t == t_ref
        for i in range(L):
            for s in range(N + 1):
                assert abs(B.cache_cost(N, s, a[i], beta[i]) - OP.cost(N, s, a[i], beta[i])) < 1e-15
    # Mixtral-sized instance: early layers harder to predict and less often single-expert get more slots
    L, N = 32, 8
    a = np.linspace(0.1, 0.4, L)
    beta = np.linspace(0.7, 0.95, L)
    t, cost = B.cache_plan(L, N, 64, a, beta)
    assert sum(t) == 64 and t == OP.plan(L, N, 64, a, beta)[0]
    assert t[0] >= t[-1]


def test_planner_argument_errors(lib):
    t = (ctypes.c_int32 * 2)()
    a = (ctypes.c_double * 2)(0.1, 0.2)
    assert lib.cache_plan(2, 1, 4, a, a, t, None) == B.EINVAL
    assert lib.cache_plan(2, 8, -1, a, a, t, None) == B.EINVAL
    assert lib.cache_plan(2, 8, 4, None, a, t, None) == B.EINVAL
