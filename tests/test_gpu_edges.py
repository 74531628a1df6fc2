"""GPU tests of the edges of the C ABI: argument errors, the largest supported sizes, degenerate inputs."""
import numpy as np
import pytest
import torch

from oracle import expert as OE
from oracle import gate as OG
from paper_2408_10284_amd import binding as B
from paper_2408_10284_amd import synth
from gpu_helpers import GpuLayerSet, rel_err_per_token, to_dev_act
from test_gpu_parity import TOL, check_gate, run_ffn, run_gate

pytestmark = pytest.mark.gpu


def _code(fn, *args):
    with pytest.raises(B.AdapMoEError) as ei:
        fn(*args)
    return ei.value.code


def test_argument_errors_are_reported():
    shape = synth.MoEShape(H=512, F=512, N=4, L=2, dtype="bf16")
    ls = GpuLayerSet(shape, seed=1, max_B=2, resident=False)
    try:
        x = torch.zeros((2, 512), dtype=torch.bfloat16, device="cuda")
        y = torch.zeros((2, 512), dtype=torch.float32, device="cuda")
        ids = torch.zeros((2, 2), dtype=torch.int32, device="cuda")
        w = torch.zeros((2, 2), dtype=torch.float32, device="cuda")
        k = torch.ones(2, dtype=torch.int32, device="cuda")
        # empty and oversized batches, layers out of range, null pointers
        assert _code(B.moe_gate, ls.ctx, 0, x, 0, ids, w, k) == B.EINVAL
        assert _code(B.moe_gate, ls.ctx, 0, x, 3, ids, w, k) == B.EINVAL
        assert _code(B.moe_gate, ls.ctx, 2, x, 1, ids, w, k) == B.EINVAL
        assert _code(B.moe_gate, ls.ctx, 0, None, 1, ids, w, k) == B.EINVAL
        assert _code(B.moe_expert_ffn, ls.ctx, 0, x, 0, ids, w, k, y) == B.EINVAL
        assert _code(B.moe_expert_ffn, ls.ctx, -1, x, 1, ids, w, k, y) == B.EINVAL
        assert _code(B.moe_layer_step, ls.ctx, 0, x, 3, y) == B.EINVAL
        assert _code(B.moe_layer_step, ls.ctx, 0, x, 1, None) == B.EINVAL
        # a layer step on offloaded experts before the cache exists
        assert _code(B.moe_layer_step, ls.ctx, 0, x, 1, y) == B.ESTATE
        assert _code(B.cache_alloc, ls.ctx, [5, 0]) == B.EINVAL        # more slots than experts
        assert _code(B.cache_alloc, ls.ctx, [-1, 0]) == B.EINVAL
        B.cache_alloc(ls.ctx, [1, 1])
        assert _code(B.cache_alloc, ls.ctx, [1, 1]) == B.ESTATE        # only once
        assert _code(B.moe_prefetch, ls.ctx, 0, [4]) == B.EINVAL        # expert id out of range
        assert _code(B.moe_prefetch, ls.ctx, 2, [0]) == B.EINVAL
        assert _code(B.adapmoe_set_tiles, ls.ctx, 65) == B.EINVAL
        assert _code(B.adapmoe_set_tiles, ls.ctx, -1) == B.EINVAL
        assert _code(B.adapmoe_set_lookahead, ls.ctx, 0) == B.EINVAL
        assert _code(B.adapmoe_set_lookahead, ls.ctx, 4) == B.EINVAL
        pinned = torch.empty(16, dtype=torch.uint8).pin_memory()
        assert _code(B.adapmoe_register_expert, ls.ctx, 0, 0, pinned, 16) == B.EINVAL   # wrong image size
        # the context still works after all of that
        B.moe_layer_step(ls.ctx, 0, x[:1], 1, y[:1])
        B.adapmoe_check(ls.ctx)
        assert torch.all(torch.isfinite(y))
    finally:
        ls.close()


def test_unregistered_expert_is_an_error_not_a_fault():
    shape = synth.MoEShape(H=512, F=512, N=4, L=1, dtype="bf16")
    ctx, cfg = B.adapmoe_create(shape.H, shape.F, shape.N, shape.L, B.BF16)
    try:
        B.adapmoe_set_router(ctx, 0, to_dev_act("bf16", synth.router_weights(shape, 0)))
        B.adapmoe_set_tau(ctx, [0.2])
        B.cache_alloc(ctx, [2])
        x = to_dev_act("bf16", synth.iid_tokens(1, 512, seed=1, dtype="bf16"))
        y = torch.zeros((1, 512), dtype=torch.float32, device="cuda")
        assert _code(B.moe_layer_step, ctx, 0, x, 1, y) == B.ENOTREG
    finally:
        torch.cuda.synchronize()
        B.adapmoe_destroy(ctx)


@pytest.mark.parametrize("dtype,H,F,N,max_B", [
    ("bf16", 512, 20480, 2, 1),      # largest F of the fp32/bf16 GEMV path: a_j of two experts fills the 160 KB of LDS
    ("int4g64", 8192, 512, 2, 1),    # largest H of the quantised path: two full blocks of x per lane
    ("int2g64", 8192, 2048, 2, 1),   # the same with 2-bit codes (F = 16384 is covered by the shape tests)
    ("bf16", 512, 512, 64, 64),      # most experts, largest batch: 64 tokens over 64 experts through the batched path
    ("f32", 256, 256, 2, 64),        # smallest shapes, largest batch, looped GEMV path
])
def test_largest_supported_sizes(dtype, H, F, N, max_B):
    shape = synth.MoEShape(H=H, F=F, N=N, L=1, dtype=dtype)
    ls = GpuLayerSet(shape, seed=5, max_B=max_B, taus=[0.3])
    try:
        n = max(max_B, 3)
        X = synth.ar1_tokens(n, H, 0.5, seed=6, dtype=dtype)
        g = run_gate(ls, 0, X)
        ref = OG.gate_batch(X, ls.routers_f32[0], np.float32(0.3))
        check_gate(g["ids"], g["k"], g["w"], ref, 0.3, 1e-5)
        y = run_ffn(ls, 0, g)
        Yref = OE.moe_block_rows(X, ls.experts_f32[0], g["ids"], g["w"].astype(np.float64), g["k"])
        err = rel_err_per_token(y, Yref)
        assert err.max() <= TOL[dtype], err.max()
    finally:
        ls.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16", "int4g64"])
def test_degenerate_inputs(dtype):
    """Zero input: all logits equal, so the tie rule picks experts 0 and 1 with weights 1/2 each, the test value
    is exactly 1/2 (two experts below a threshold of 1/2, one at it), and the block output is exactly zero.
    Identical tokens give identical outputs."""
    shape = synth.MoEShape(H=512, F=1024, N=8, L=1, dtype=dtype)
    ls = GpuLayerSet(shape, seed=8, max_B=4, taus=[0.3])
    try:
        Z = np.zeros((3, shape.H), dtype=np.float32)
        g = run_gate(ls, 0, Z)
        assert np.all(g["ids"] == [0, 1]) and np.all(g["k"] == 2)
        np.testing.assert_array_equal(g["w"], 0.5)
        assert OG.adaptive_gate(Z[0].astype(np.float64), ls.routers_f32[0], 0.3)["ids"] == (0, 1)
        y = run_ffn(ls, 0, g)
        assert np.all(y == 0.0)
        B.adapmoe_set_tau(ls.ctx, [0.5])
        g = run_gate(ls, 0, Z)
        assert np.all(g["k"] == 1) and np.all(g["w"] == [1.0, 0.0])
        B.adapmoe_set_tau(ls.ctx, [0.3])
        X = np.repeat(synth.iid_tokens(1, shape.H, seed=2, dtype=dtype), 4, axis=0)
        g = run_gate(ls, 0, X)
        y = run_ffn(ls, 0, g)
        assert np.all(g["ids"] == g["ids"][0]) and np.all(y == y[0])
        assert np.all(np.isfinite(y)) and np.abs(y).max() > 0
    finally:
        ls.close()


@pytest.mark.parametrize("Bt", [1, 6])
def test_resident_stack_step_can_be_captured_in_a_graph(Bt):
    """With every expert resident, moe_stack_token makes no host round trip, allocates nothing and clears
    its own counters in kernels, so a HIP graph can hold it.  The graph is replayed several times, on new
    inputs, with eager work in between, and every replay is compared with the eager result.  Bt = 6 takes
    the batched kernels (bucketing, streaming grouped GEMM, atomic adds onto a y cleared by a kernel)."""
    shape = synth.MoEShape(H=1024, F=2048, N=8, L=3, dtype="bf16")
    ls = GpuLayerSet(shape, seed=21, max_B=Bt, taus=[0.2, 0.3, 0.25])
    try:
        n = 5
        H0 = torch.from_numpy(synth.ar1_streams(n, Bt, shape.H, 0.8, seed=3, dtype="f32") * 2.0).cuda()
        x = torch.empty((Bt, shape.H), dtype=torch.bfloat16, device="cuda")
        y = torch.empty((Bt, shape.H), dtype=torch.float32, device="cuda")
        h = torch.empty((Bt, shape.H), dtype=torch.float32, device="cuda")

        def eager(t):
            h.copy_(H0[t])
            B.moe_stack_token(ls.ctx, t, h, x, y, Bt, 0.5, torch.cuda.current_stream())
            torch.cuda.synchronize()
            return h.clone(), y.clone()

        ref = [eager(t) for t in range(n)]
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            h.copy_(H0[0])
            B.moe_stack_token(ls.ctx, 0, h, x, y, Bt, 0.5, side)       # warm-up on the capture stream
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                B.moe_stack_token(ls.ctx, 0, h, x, y, Bt, 0.5, torch.cuda.current_stream())
        torch.cuda.current_stream().wait_stream(side)
        for rep in range(2):
            for t in range(n):
                h.copy_(H0[t])
                g.replay()
                torch.cuda.synchronize()
                assert torch.equal(h, ref[t][0]) and torch.equal(y, ref[t][1]), (rep, t)
                he, ye = eager((t + 1) % n)                              # eager work between replays
                assert torch.equal(he, ref[(t + 1) % n][0]) and torch.equal(ye, ref[(t + 1) % n][1])
        B.adapmoe_check(ls.ctx)
    finally:
        ls.close()


def test_two_contexts_are_independent():
    a = GpuLayerSet(synth.MoEShape(H=512, F=1024, N=4, L=1, dtype="bf16"), seed=31, max_B=2, taus=[0.3])
    b = GpuLayerSet(synth.MoEShape(H=1024, F=512, N=8, L=1, dtype="f32"), seed=32, max_B=2, taus=[0.25])
    try:
        Xa = synth.ar1_tokens(6, 512, 0.5, seed=1, dtype="bf16")
        Xb = synth.ar1_tokens(6, 1024, 0.5, seed=2, dtype="f32")
        ga, gb = run_gate(a, 0, Xa), run_gate(b, 0, Xb)
        ya_alone, yb_alone = run_ffn(a, 0, ga), run_ffn(b, 0, gb)
        # interleaved, two tokens at a time
        ya = torch.empty((6, 512), dtype=torch.float32, device="cuda")
        yb = torch.empty((6, 1024), dtype=torch.float32, device="cuda")
        for s in range(0, 6, 2):
            B.moe_layer_step(a.ctx, 0, ga["x_dev"][s:s + 2], 2, ya[s:s + 2])
            B.moe_layer_step(b.ctx, 0, gb["x_dev"][s:s + 2], 2, yb[s:s + 2])
        B.adapmoe_check(a.ctx)
        B.adapmoe_check(b.ctx)
        np.testing.assert_array_equal(ya.cpu().numpy(), ya_alone)
        np.testing.assert_array_equal(yb.cpu().numpy(), yb_alone)
    finally:
        a.close()
        b.close()


@pytest.mark.parametrize("dtype,blocks,pct", [("bf16", 40, 50), ("bf16", 7, 100), ("bf16", 1000, 15), ("bf16", 512, 0),
                                              ("int4g64", 10, 50), ("int4g64", 3, 100), ("int4g64", 37, 30), ("int2g64", 16, 40)])
def test_dynamic_tail_with_odd_grids(dtype, blocks, pct):
    """The gate/up kernel's dynamic tail must cover every row exactly once for any grid size and pool share
    (grids that are no multiple of 8 workgroups, fewer workgroups than queues, everything in the pool).
    The quantised kernels assign every row in advance whatever the option says: their cases check odd grid
    sizes (rows that do not divide over the wavefronts, wavefronts with one row pair or none)."""
    shape = synth.MoEShape(H=4096, F=1536, N=4, L=1, dtype=dtype)     # compile-time row length, 2 F no multiple of most grids
    ls = GpuLayerSet(shape, seed=51, max_B=3, taus=[0.3])
    try:
        B.adapmoe_set_option(ls.ctx, B.OPT_GATEUP_BLOCKS, blocks)
        B.adapmoe_set_option(ls.ctx, B.OPT_DYN_PCT, pct)
        assert B.adapmoe_get_option(ls.ctx, B.OPT_GATEUP_BLOCKS) == blocks and B.adapmoe_get_option(ls.ctx, B.OPT_DYN_PCT) == pct
        X = synth.ar1_tokens(9, shape.H, 0.5, seed=52, dtype="bf16")
        g = run_gate(ls, 0, X)
        for rep in range(3):      # repeated launches: the counters are cleared in between by the down kernel
            y = run_ffn(ls, 0, g)
            Yref = OE.moe_block_rows(X, ls.experts_f32[0], g["ids"], g["w"].astype(np.float64), g["k"])
            err = rel_err_per_token(y, Yref)
            assert err.max() <= TOL[dtype], (rep, err.max())
    finally:
        ls.close()


def test_stream_probe_runs_and_reports_a_plausible_rate():
    """The load-only probe of the kernels' access patterns: both patterns run over a small matrix (ragged
    share of units per wavefront, more wavefronts than units) and report a duration that corresponds to
    less than the chip's HBM peak."""
    rows, row_bytes = 64 * 1024, 8192                # 512 MiB
    buf = torch.ones(rows * row_bytes, dtype=torch.uint8, device="cuda")
    for unit, chunk, wgs in ((2, 8192, 512), (32, 512, 256), (2, 8192, 3), (32, 512, 1000)):
        us = B.adapmoe_stream_probe(buf, rows, row_bytes, unit, chunk, wgs, 3)
        gbs = rows * row_bytes / (us * 1e-6) / 1e9
        assert 50.0 < gbs < 8000.0, (unit, chunk, wgs, us, gbs)
    # fewer units than wavefronts, and a single unit
    assert B.adapmoe_stream_probe(buf, 64, row_bytes, 32, 512, 256, 2) > 0.0
    assert B.adapmoe_stream_probe(buf, 2, row_bytes, 2, 8192, 1, 2) > 0.0
    with pytest.raises(ValueError):
        B.adapmoe_stream_probe(buf, rows + 2, row_bytes, 2, 8192, 64, 1)     # larger than the buffer
