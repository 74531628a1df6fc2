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


def _decode_int4_row(row_bytes, n):
    """Independent reader of the documented int4 row format -> (codes[n], scale[n/64], zero[n/64])."""
    G = n // 64
    codes = np.zeros(n, dtype=np.uint8)
    raw = np.frombuffer(row_bytes, dtype=np.uint8)
    for g in range(G):
        blk, l = divmod(g, 64)
        nb = min(64, G - blk * 64)
        for half in range(2):
            off = blk * 2048 + half * nb * 16 + l * 16
            dwords = raw[off:off + 16].view(np.uint32)
            for d in range(4):
                w = int(dwords[d])
                for s in range(4):
                    codes[g * 64 + half * 32 + d * 8 + 2 * s] = (w >> (4 * s)) & 15
                    codes[g * 64 + half * 32 + d * 8 + 2 * s + 1] = (w >> (4 * s + 16)) & 15
    sz = raw[n // 2: n // 2 + 4 * G].view(np.uint16).reshape(G, 2)
    return codes, sz[:, 0].copy(), sz[:, 1].copy()


def test_pack_int4_layout(lib):
    H, F = 512, 4352     # W2 rows: 68 groups = one block of 64 + one of 4
    cfg = B.Config(H, F, 2, 1, B.INT4G64, 1, 0, 0)
    nbytes = B.adapmoe_expert_bytes(cfg)
    assert nbytes == 3 * H * F * 9 // 16
    rng = np.random.default_rng(1)
    mats = []
    for (r, c) in ((F, H), (F, H), (H, F)):
        mats.append((rng.integers(0, 16, (r, c), dtype=np.uint8),
                     rng.integers(0, 65536, (r, c // 64), dtype=np.uint16),
                     rng.integers(0, 65536, (r, c // 64), dtype=np.uint16)))
    out = np.zeros(nbytes, dtype=np.uint8)
    B.adapmoe_pack_expert_int4(cfg, *[a for m in mats for a in m], out)
    rbH, rbF = H // 2 + H // 16, F // 2 + F // 16
    for f in (0, 1, 77, F - 1):
        for which, m in ((0, mats[0]), (1, mats[1])):
            row = out[(2 * f + which) * rbH:(2 * f + which + 1) * rbH].tobytes()
            q, s, z = _decode_int4_row(row, H)
            np.testing.assert_array_equal(q, m[0][f])
            np.testing.assert_array_equal(s, m[1][f])
            np.testing.assert_array_equal(z, m[2][f])
    base = 2 * F * rbH
    for h in (0, 5, H - 1):
        q, s, z = _decode_int4_row(out[base + h * rbF: base + (h + 1) * rbF].tobytes(), F)
        np.testing.assert_array_equal(q, mats[2][0][h])
        np.testing.assert_array_equal(s, mats[2][1][h])
        np.testing.assert_array_equal(z, mats[2][2][h])
    # Mixtral-shaped int4 expert: 9/16 byte per weight
    assert B.adapmoe_expert_bytes(B.Config(4096, 14336, 8, 32, B.INT4G64, 1, 0, 0)) == 99090432


def test_int4_image_generators_match_library_packer(lib):
    """The torch-side quantiser/packer used for large stacks produces byte-identical images to
    quantize_int4_g64 + adapmoe_pack_expert_int4, and decode_int4_image inverts both."""
    import torch
    from paper_2408_10284_amd import synth
    H, F = 512, 4352
    cfg = B.Config(H, F, 2, 1, B.INT4G64, 1, 0, 0)
    rng = np.random.default_rng(3)
    ws = [synth.bf16_round((rng.standard_normal(s) * 0.02).astype(np.float32)) for s in ((F, H), (F, H), (H, F))]
    qs = [synth.quantize_int4_g64(w) for w in ws]
    ref = np.zeros(B.adapmoe_expert_bytes(cfg), dtype=np.uint8)
    B.adapmoe_pack_expert_int4(cfg, *[a for (q, s, z) in qs for a in (q, s.view(np.uint16), z.view(np.uint16))], ref)
    img = synth.int4_image_from_weights_torch(*[torch.from_numpy(w) for w in ws]).numpy()
    np.testing.assert_array_equal(img, ref)
    for got, (q, s, z) in zip(synth.decode_int4_image(ref, H, F), qs):
        np.testing.assert_array_equal(got[0], q)
        np.testing.assert_array_equal(got[1].view(np.uint16), s.view(np.uint16))
        np.testing.assert_array_equal(got[2].view(np.uint16), z.view(np.uint16))


def _decode_int2_row(row_bytes, n):
    """Independent reader of the documented 2-bit row format."""
    G = n // 64
    codes = np.zeros(n, dtype=np.uint8)
    raw = np.frombuffer(row_bytes, dtype=np.uint8)
    for g in range(G):
        blk, l = divmod(g, 64)
        off = blk * 1024 + l * 16          # a block of nb groups is nb x 16 bytes, groups in order
        dwords = raw[off:off + 16].view(np.uint32)
        for d in range(4):
            w = int(dwords[d])
            for s in range(8):
                codes[g * 64 + d * 16 + 2 * s] = (w >> (2 * s)) & 3
                codes[g * 64 + d * 16 + 2 * s + 1] = (w >> (2 * s + 16)) & 3
    sz = raw[n // 4: n // 4 + 4 * G].view(np.uint16).reshape(G, 2)
    return codes, sz[:, 0].copy(), sz[:, 1].copy()


def test_pack_int2_layout_and_generators(lib):
    import torch
    from paper_2408_10284_amd import synth
    H, F = 512, 4352
    cfg = B.Config(H, F, 2, 1, B.INT2G64, 1, 0, 0)
    nbytes = B.adapmoe_expert_bytes(cfg)
    assert nbytes == 3 * H * F * 5 // 16
    assert B.adapmoe_expert_bytes(B.Config(4096, 14336, 8, 32, B.INT2G64, 1, 0, 0)) == 55050240
    rng = np.random.default_rng(5)
    ws = [synth.bf16_round((rng.standard_normal(s) * 0.02).astype(np.float32)) for s in ((F, H), (F, H), (H, F))]
    qs = [synth.quantize_int2_g64(w) for w in ws]
    out = np.zeros(nbytes, dtype=np.uint8)
    B.adapmoe_pack_expert_int2(cfg, *[a for (q, s, z) in qs for a in (q, s.view(np.uint16), z.view(np.uint16))], out)
    rbH, rbF = H // 4 + H // 16, F // 4 + F // 16
    for f in (0, 3, F - 1):
        for which in (0, 1):
            q, s, z = _decode_int2_row(out[(2 * f + which) * rbH:(2 * f + which + 1) * rbH].tobytes(), H)
            np.testing.assert_array_equal(q, qs[which][0][f])
            np.testing.assert_array_equal(s, qs[which][1][f].view(np.uint16))
            np.testing.assert_array_equal(z, qs[which][2][f].view(np.uint16))
    base = 2 * F * rbH
    for h in (0, 9, H - 1):
        q, s, z = _decode_int2_row(out[base + h * rbF: base + (h + 1) * rbF].tobytes(), F)
        np.testing.assert_array_equal(q, qs[2][0][h])
        np.testing.assert_array_equal(s, qs[2][1][h].view(np.uint16))
    # the torch-side generator used for large stacks is byte-identical, and the image reader inverts it
    img = synth.int2_image_from_weights_torch(*[torch.from_numpy(w) for w in ws]).numpy()
    np.testing.assert_array_equal(img, out)
    for got, (q, s, z) in zip(synth.decode_int2_image(out, H, F), qs):
        np.testing.assert_array_equal(got[0], q)
        np.testing.assert_array_equal(got[1].view(np.uint16), s.view(np.uint16))
        np.testing.assert_array_equal(got[2].view(np.uint16), z.view(np.uint16))
    # a config of one type is refused by the other packer
    assert lib.adapmoe_pack_expert_int4(ctypes.byref(cfg), *([None] * 10)) == B.EINVAL


def test_product_and_checker_do_not_touch_each_other():
    """The library package never imports the checker (there is no CPU fallback), the checker never
    imports the library, and bench.py reaches the checker only from its CPU-baseline function."""
    import ast
    def imports(path):
        tree = ast.parse(open(path).read())
        out = []
        for node in ast.walk(tree):
            if isinstance(node, ast.Import):
                out += [(a.name, node.lineno) for a in node.names]
            elif isinstance(node, ast.ImportFrom) and node.module:
                out.append((node.module, node.lineno))
        return out
    pkg = os.path.join(ROOT, "paper_2408_10284_amd")
    for f in os.listdir(pkg):
        if f.endswith(".py"):
            assert not [m for m, _ in imports(os.path.join(pkg, f)) if m.split(".")[0] == "oracle"], f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            assert not [m for m, _ in imports(os.path.join(ROOT, "oracle", f)) if "paper_2408_10284_amd" in m], f
    # csrc never mentions the checker either
    for f in os.listdir(os.path.join(pkg, "csrc")):
        assert "oracle" not in open(os.path.join(pkg, "csrc", f)).read(), f
    src = open(os.path.join(ROOT, "bench.py")).read()
    tree = ast.parse(src)
    for node in tree.body:
        if isinstance(node, ast.FunctionDef):
            uses = [n for n in ast.walk(node) if isinstance(n, ast.ImportFrom) and n.module and n.module.startswith("oracle")]
            assert not uses or node.name.startswith("cpu_baseline_"), node.name   # only the CPU-baseline legs touch the checker
    assert not [n for n in tree.body if isinstance(n, (ast.Import, ast.ImportFrom)) and "oracle" in ast.dump(n)]


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_build_rejects_kernels_with_scratch_memory():
    """The build parses the compiler's per-kernel resource remarks; scratch use must be seen (it costs every
    dispatch a private-segment set-up) and the built library's kernels must all be at zero."""
    from paper_2408_10284_amd import build as BLD
    sample = (
        "a.hip:5:1: remark: Function Name: k_good [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hip:5:1: remark:     VGPRs: 12 [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hip:5:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hip:9:1: remark: Function Name: k_bad [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hip:9:1: remark:     ScratchSize [bytes/lane]: 32 [-Rpass-analysis=kernel-resource-usage]\n"
        "a.hip:9:1: remark:     Occupancy [waves/SIMD]: 4 [-Rpass-analysis=kernel-resource-usage]\n")
    res = BLD.kernel_resources(sample)
    assert res == {"k_good": {"VGPRs": 12, "ScratchSize": 0}, "k_bad": {"ScratchSize": 32, "Occupancy": 4}}
    if not os.path.exists(BLD.RESOURCES):
        BLD.build(verbose=False)
    rows = [l.split(" | ") for l in open(BLD.RESOURCES).read().splitlines()[1:]]
    assert len(rows) >= 30                      # every kernel instantiation of the library
    assert any("ffn_gateup_kernel" in r[0] for r in rows) and any("grouped_down_mfma_kernel" in r[0] for r in rows)
    assert all(int(r[4]) == 0 for r in rows), [r[0] for r in rows if int(r[4]) != 0]


def test_binding_refuses_buffers_that_are_too_small_or_misplaced():
    """The wrappers check size, contiguity and placement of every array they marshal (the C side
    sees raw addresses only); a short buffer must never reach a kernel."""
    cfg = B.Config(512, 512, 4, 2, B.BF16, 1, 0, 0)
    w = np.zeros((512, 512), dtype=np.uint16)
    out = np.zeros(3 * 512 * 512 * 2, dtype=np.uint8)
    B.adapmoe_pack_expert(cfg, w, w, w, out)                              # exact sizes pass
    with pytest.raises(ValueError, match="bytes given"):
        B.adapmoe_pack_expert(cfg, w, w, w, out[:-1])
    with pytest.raises(ValueError, match="bytes given"):
        B.adapmoe_pack_expert(cfg, w[:-1], w, w, out)
    with pytest.raises(ValueError, match="contiguous"):
        B.adapmoe_pack_expert(cfg, np.zeros((512, 1024), dtype=np.uint16)[:, ::2], w, w, out)
    # a context address the module does not know
    with pytest.raises(ValueError, match="unknown context"):
        B.moe_layer_step(ctypes.c_void_p(1234), 0, None, 1, None)
    # the checks themselves, on stand-ins for the step arguments
    with pytest.raises(ValueError, match="device tensor"):
        B._need_step(cfg, 1, x=np.zeros(512, np.uint16), y=None)          # a host array where HBM is expected
    B._need_step(cfg, 7, x=np.zeros(1, np.uint16))                        # B out of range: left to the library to report
    with pytest.raises(ValueError, match="x: 1022 bytes given, 1024 needed"):
        B._need("x", np.zeros(511, np.uint16), 1024)
    import torch
    with pytest.raises(ValueError, match="device tensor"):
        B._need("x", torch.zeros(512, dtype=torch.bfloat16), 1024, "dev")


def test_stream_probe_rejects_bad_patterns_without_gpu(lib):
    """The load-only probe checks its pattern before anything touches the GPU: rows that are no
    power-of-two number of KiB, chunks other than 512 bytes or a whole row, units that do not fill
    whole 16 KiB buffers, a row count that is no multiple of the unit, empty launches."""
    us = ctypes.c_double()
    buf = ctypes.c_void_p(4096)          # never dereferenced: every call below fails its argument check

    def rc(nrows, row_bytes, unit, chunk, wgs=64, reps=1, b=buf):
        return lib.adapmoe_stream_probe(b, nrows, row_bytes, unit, chunk, wgs, reps, ctypes.byref(us), None)

    assert rc(64, 8192, 2, 8192, b=None) == B.EINVAL
    assert rc(64, 12288, 2, 12288) == B.EINVAL        # 16384 is no multiple of the row
    assert rc(64, 8192, 32, 1024) == B.EINVAL         # neither 512 nor the whole row
    assert rc(64, 8192, 16, 512) == B.EINVAL          # 16 x 512 bytes do not fill a buffer
    assert rc(66, 8192, 4, 8192) == B.EINVAL          # 66 rows are no whole number of units
    assert rc(64, 8192, 2, 8192, wgs=0) == B.EINVAL
    assert rc(64, 8192, 2, 8192, reps=0) == B.EINVAL
    assert rc(0, 8192, 2, 8192) == B.EINVAL
