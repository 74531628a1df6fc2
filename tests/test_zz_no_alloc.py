"""The expert FFN entry point that allocates nothing (its scratch memory is a fixed device array inside the
library): same results as moe_expert_ffn on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2408_10284_amd import binding as B
from paper_2408_10284_amd import synth

from gpu_helpers import GpuLayerSet, to_dev_act

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,H,F,N", [("bf16", 4096, 3584, 8), ("int4g64", 1024, 4352, 4), ("f32", 512, 1024, 8), ("bf16", 1024, 1536, 8)])
def test_static_scratch_ffn_equals_context_ffn(dtype, H, F, N):
    shape = synth.MoEShape(H=H, F=F, N=N, L=1, dtype=dtype)
    ls = GpuLayerSet(shape, seed=17, max_B=4, taus=[0.3])
    dt = {"f32": B.F32, "bf16": B.BF16, "int4g64": B.INT4G64}[dtype]
    try:
        B.adapmoe_set_option(ls.ctx, B.OPT_BATCH_MIN, 64)      # the context's calls take the GEMV kernels too
        table = torch.tensor([t.data_ptr() for t in ls.images], dtype=torch.int64, device="cuda")   # N image addresses
        X = synth.ar1_tokens(4, H, 0.5, seed=18, dtype=dtype)
        xd = to_dev_act(dtype, X)
        ids = torch.empty((4, 2), dtype=torch.int32, device="cuda")
        w = torch.empty((4, 2), dtype=torch.float32, device="cuda")
        k = torch.empty(4, dtype=torch.int32, device="cuda")
        B.moe_gate(ls.ctx, 0, xd, 4, ids, w, k)
        torch.cuda.synchronize()
        assert 2 in k.cpu().numpy()
        err = torch.zeros(1, dtype=torch.int32, device="cuda")
        # first call: 3 tokens; second call right after it: 1 token (a smaller input, other tokens' leftovers in the array)
        for (lo, n) in ((0, 3), (3, 1), (1, 2)):
            want = torch.full((n, H), 3.0, dtype=torch.float32, device="cuda")
            got = torch.full((n, H), -5.0, dtype=torch.float32, device="cuda")
            B.moe_expert_ffn(ls.ctx, 0, xd[lo:lo + n], n, ids[lo:lo + n], w[lo:lo + n], k[lo:lo + n], want)
            B.adapmoe_check(ls.ctx)
            print(f"static call: {dtype} H={H} F={F} tokens {lo}..{lo + n - 1}", flush=True)
            B.moe_expert_ffn_static(H, F, N, dt, table, xd[lo:lo + n], n, ids[lo:lo + n], w[lo:lo + n], k[lo:lo + n], got, err)
            torch.cuda.synchronize()
            assert int(err.item()) == 0
            np.testing.assert_array_equal(got.cpu().numpy(), want.cpu().numpy())
            assert np.abs(want.cpu().numpy()).max() > 0
        # an absent expert is flagged, contributes nothing, and nothing faults
        table2 = table.clone()
        e_used = int(ids[0, 0].item())
        table2[e_used] = 0
        got = torch.full((1, H), -5.0, dtype=torch.float32, device="cuda")
        B.moe_expert_ffn_static(H, F, N, dt, table2, xd[0:1], 1, ids[0:1], w[0:1], k[0:1], got, err)
        torch.cuda.synchronize()
        assert int(err.item()) & 1
        assert torch.all(torch.isfinite(got))
        # sizes beyond the fixed array are refused before anything is launched
        for bad in (lambda: B.moe_expert_ffn_static(H, F, N, dt, table, xd, 5, ids, w, k, got, err),
                    lambda: B.moe_expert_ffn_static(H, F, N, dt, table, xd, 0, ids, w, k, got, err),
                    lambda: B.moe_expert_ffn_static(H, 32768, N, dt, table, xd, 1, ids, w, k, got, err),
                    lambda: B.moe_expert_ffn_static(H, F, N, dt, None, xd, 1, ids, w, k, got, err)):
            with pytest.raises(B.AdapMoEError) as ei:
                bad()
            assert ei.value.code == B.EINVAL
    finally:
        ls.close()
