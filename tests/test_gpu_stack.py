"""GPU parity of the multi-layer token step on HBM-resident experts (moe_stack_token with every expert
bound): the path that fuses the residual update, the normalisation and the gate into one launch, makes no
host round trip, and takes the batched (matrix-core) kernels when a step carries several tokens."""
import numpy as np
import pytest
import torch

from oracle import expert as OE
from oracle import gate as OG
from oracle import stack as OS
from paper_2408_10284_amd import binding as B
from paper_2408_10284_amd import synth

from gpu_helpers import GpuLayerSet, check_outputs, to_dev_act
from test_gpu_parity import BAND, TIE_GAP, TOL

pytestmark = pytest.mark.gpu


def _stack_tokens(ctx, L, max_B, H0, Bt, gamma, dtype, log=True):
    """Runs H0[step] ([Bt,H] each) through moe_stack_token.  Returns (final h [steps,Bt,H] float64,
    ids [steps,L,Bt,2], k [steps,L,Bt]) with the decisions read from the decision log."""
    n_steps, H = H0.shape[0], H0.shape[2]
    act = torch.float32 if dtype == "f32" else torch.bfloat16
    x = torch.empty((Bt, H), dtype=act, device="cuda")
    y = torch.empty((Bt, H), dtype=torch.float32, device="cuda")
    logbuf = torch.full((n_steps * L, 6 * max_B), -7, dtype=torch.int32, device="cuda")
    if log:
        B.adapmoe_set_decision_log(ctx, logbuf, n_steps * L)
    out = np.zeros((n_steps, Bt, H), np.float64)
    for t in range(n_steps):
        h = torch.from_numpy(np.ascontiguousarray(H0[t], dtype=np.float32)).cuda()
        B.moe_stack_token(ctx, t, h, x, y, Bt, gamma)
        B.adapmoe_check(ctx)
        out[t] = h.cpu().numpy()
    if log:
        B.adapmoe_set_decision_log(ctx, None, 0)
    rec = logbuf.cpu().numpy().reshape(n_steps, L, 6 * max_B)
    ids = rec[:, :, :2 * Bt].reshape(n_steps, L, Bt, 2)
    k = rec[:, :, 2 * Bt:3 * Bt]
    return out, ids, k


@pytest.mark.parametrize("Bt", [1, 3])
def test_resident_stack_fp32_free_running_against_checker(Bt):
    """fp32, four layers, every expert bound: the library's token step and the checker's stack run on their
    own from the same tokens.  Every decision of every layer and the residual stream after the last layer must
    agree (the checker's smallest logit gaps and threshold margins are required to be far above fp32 rounding,
    so the agreement is not luck).  Bt = 3 takes the same kernels with three tokens per launch."""
    shape = synth.MoEShape(H=512, F=1024, N=8, L=4, dtype="f32")
    taus = [0.2, 0.3, 0.25, 0.35]
    n_steps, gamma = 12, 0.5
    ls = GpuLayerSet(shape, seed=4, max_B=4, taus=taus)
    try:
        B.adapmoe_set_option(ls.ctx, B.OPT_BATCH_MIN, 64)
        H0 = (synth.ar1_streams(n_steps, Bt, shape.H, 0.8, seed=9, dtype="f32") * 2.0).astype(np.float32)
        got_h, got_ids, got_k = _stack_tokens(ls.ctx, shape.L, 4, H0, Bt, gamma, "f32")
        for b in range(Bt):
            ref = OS.run_stack(H0[:, b].astype(np.float64), ls.routers_f32, [np.float32(t) for t in taus],
                               lambda l, e, x: OE.expert_ffn(x, *ls.experts_f32[l][e]), gamma,
                               store=lambda a: a.astype(np.float32))
            margin = np.abs(ref["v"] - np.asarray(taus)[None, :])
            assert ref["gap23"].min() > 1e-4 and margin.min() > 1e-5, (ref["gap23"].min(), margin.min())
            np.testing.assert_array_equal(got_k[:, :, b], ref["k"])
            np.testing.assert_array_equal(got_ids[:, :, b, 0], ref["ids"][:, :, 0])
            two = ref["k"] == 2
            np.testing.assert_array_equal(got_ids[:, :, b, 1][two], ref["ids"][:, :, 1][two])
            hL = ref["h"][:, shape.L]
            err = np.max(np.abs(got_h[:, b] - hL), axis=1) / np.max(np.abs(hL), axis=1)
            assert err.max() <= 1e-5, err.max()
    finally:
        ls.close()


class _LazyExperts:
    """experts[e] -> (W1, W3, W2) of one layer, unpacked from the device image on first use."""

    def __init__(self, images, H, F):
        self.images, self.H, self.F, self.cache = images, H, F, {}

    def __len__(self):
        return len(self.images)

    def __getitem__(self, e):
        if e not in self.cache:
            bits = self.images[e].view(torch.int16).cpu().numpy().view(np.uint16)
            self.cache[e] = synth.unpack_image_bf16(bits, self.H, self.F)
        return self.cache[e]


@pytest.mark.parametrize("H,F,N,L,Bt,n_steps", [
    (1024, 1536, 8, 3, 1, 6),      # small shapes, one token per step: normalise-and-gate launch, GEMV kernels
    (1024, 1536, 8, 3, 16, 3),     # 16 tokens per step: normalise-and-gate for 16 rows, grouped GEMM on the matrix cores
    (1024, 1536, 8, 3, 2, 4),      # 2 tokens per step: below the batched threshold, GEMV kernels with two rows
    (16384, 512, 4, 2, 1, 3),      # rows longer than 8192: the normalisation re-reads h instead of keeping it in registers
    (16384, 512, 4, 2, 5, 2),      # the same through the batched kernels
    (4096, 14336, 8, 2, 1, 4),     # Mixtral-8x7B shape, two layers, launch configuration of the resident-stack benchmark
    (4096, 14336, 8, 2, 16, 1),    # Mixtral-8x7B shape, 16 streams: launch configuration of the batched benchmark
])
def test_resident_stack_bf16_teacher_forced_against_checker(H, F, N, L, Bt, n_steps):
    """bf16 stack with every expert bound, free-running on the GPU through moe_stack_token.  The residual
    stream in front of layer l is taken from a context that holds the first l layers only (same images, same
    kernels, hence the same bits), so every layer can be checked on the GPU's own input: the decisions in the
    decision log against the checker's gate on x_l = bf16(h_l / rms(h_l)) (exact outside the exclusion bands),
    and the block output y_l = (h_{l+1} - h_l) / gamma against the checker's experts (2e-2)."""
    shape = synth.MoEShape(H=H, F=F, N=N, L=L, dtype="bf16")
    taus = [0.2, 0.3, 0.25][:L]
    gamma = 0.3
    seed = 21
    routers = [synth.router_bf16_torch(shape, l, seed) for l in range(L)]
    routers_f32 = [r.float().cpu().numpy() for r in routers]
    images = [[synth.expert_image_bf16_torch(shape, l, e, seed) for e in range(N)] for l in range(L)]
    torch.cuda.synchronize()
    ctxs = []
    try:
        for depth in range(1, L + 1):      # context `depth` holds layers 0 .. depth-1
            ctx, cfg = B.adapmoe_create(H, F, N, depth, B.BF16, max_B=Bt)
            ctxs.append(ctx)
            for l in range(depth):
                B.adapmoe_set_router(ctx, l, routers[l])
                for e in range(N):
                    B.adapmoe_bind_expert_dev(ctx, l, e, images[l][e])
            B.adapmoe_set_tau(ctx, taus[:depth])
        H0 = (synth.ar1_streams(n_steps, Bt, H, 0.8, seed=23, dtype="f32") * 1.5).astype(np.float32)
        h_after = [H0.astype(np.float64)]                     # h_after[l] = residual stream in front of layer l
        ids = k = None
        for depth in range(1, L + 1):
            hh, ids, k = _stack_tokens(ctxs[depth - 1], depth, Bt, H0, Bt, gamma, "bf16")
            h_after.append(hh)
        worst = worst_elem = 0.0
        compared = tied = 0
        for l in range(L):
            lazy = _LazyExperts(images[l], H, F)
            for t in range(n_steps):
                hl = h_after[l][t]
                X = np.stack([synth.bf16_round(OS.rmsnorm(hl[b]).astype(np.float32)) for b in range(Bt)]).astype(np.float64)
                ref = OG.gate_batch(X, routers_f32[l], np.float32(taus[l]))
                clear = (ref["gap23"] > TIE_GAP) & (ref["gap12"] > TIE_GAP)
                tied += int((~clear).sum())
                np.testing.assert_array_equal(ids[t, l][clear], ref["ids"][clear])
                clear_k = clear & (np.abs(ref["v"] - taus[l]) > BAND)
                np.testing.assert_array_equal(k[t, l][clear_k], ref["k"][clear_k])
                compared += int(clear_k.sum())
                # outputs on the GPU's own decision, so that a token inside an exclusion band still checks the arithmetic
                kk = k[t, l]
                w = np.where((kk == 1)[:, None], np.array([[1.0, 0.0]]), np.stack([1.0 - ref["v"], ref["v"]], axis=1))
                Yref = OE.moe_block_rows(X, lazy, ids[t, l], w, kk)
                Ygpu = (h_after[l + 1][t] - hl) / gamma
                # y is recovered from two fp32 residual streams: allow their rounding on top of the bar
                slack = 4 * 2.0 ** -24 * np.max(np.abs(hl)) / gamma / np.max(np.abs(Yref))
                a, b_ = check_outputs(Ygpu, Yref, TOL["bf16"] + slack, f"layer {l} step {t}")
                worst, worst_elem = max(worst, a), max(worst_elem, b_)
        print(f"H={H} F={F} L={L} B={Bt}: {compared} decisions compared, {tied} near-ties skipped, "
              f"max rel err {worst:.3e} (max-norm), {worst_elem:.3e} (element-wise, floor 1e-3 rms)")
        assert tied <= 1 and compared >= n_steps * Bt * L - 2
    finally:
        torch.cuda.synchronize()
        for ctx in ctxs:
            B.adapmoe_destroy(ctx)


def test_residual_rmsnorm_long_rows():
    """Rows longer than 8192 elements take the normalisation's second pass from memory."""
    for dtype, bd in (("f32", B.F32), ("bf16", B.BF16)):
        Hh = 16384 if dtype == "bf16" else 12288
        ctx, cfg = B.adapmoe_create(Hh, 512, 2, 1, bd, max_B=3)
        try:
            rng = np.random.default_rng(5)
            h = (rng.standard_normal((3, Hh)) * 2).astype(np.float32)
            y = rng.standard_normal((3, Hh)).astype(np.float32)
            hd, yd = torch.from_numpy(h).cuda(), torch.from_numpy(y).cuda()
            xd = torch.empty((3, Hh), dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device="cuda")
            B.moe_residual_rmsnorm(ctx, hd, yd, 0.25, xd, 3)
            torch.cuda.synchronize()
            h2 = h.astype(np.float64) + 0.25 * y.astype(np.float64)
            np.testing.assert_allclose(hd.cpu().numpy(), h2, rtol=1e-6, atol=1e-6)
            xref = np.stack([OS.rmsnorm(r) for r in h2])
            np.testing.assert_allclose(xd.float().cpu().numpy(), xref, rtol=1e-5 if dtype == "f32" else 2.0 ** -8, atol=1e-6)
        finally:
            B.adapmoe_destroy(ctx)
