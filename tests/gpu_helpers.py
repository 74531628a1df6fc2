"""Shared set-up for the GPU parity tests: synthetic layer -> packed images in HBM."""
import numpy as np
import torch

from oracle.expert import decode_int4 as OE_decode
from paper_2408_10284_amd import binding as B
from paper_2408_10284_amd import synth


def np_dtype_bits(shape_dtype, a):
    """float32 array -> storage array handed to the library (float32 or bf16 bit patterns)."""
    return a.astype(np.float32) if shape_dtype == "f32" else synth.bf16_bits(a)


def to_dev_act(shape_dtype, a):
    """float32 activations -> device tensor in the activation storage type."""
    if shape_dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    bits = synth.bf16_bits(a).view(np.int16)
    return torch.from_numpy(bits).cuda().view(torch.bfloat16).reshape(a.shape)


class GpuLayerSet:
    """L layers of N experts: weights from synth, packed by the library, resident in HBM
    (bound) or registered as pinned host images."""

    def __init__(self, shape, seed=0, max_B=1, trace_capacity=0, resident=True, taus=None, expert_layers=None, pageable=False):
        self.shape = shape
        dt = {"f32": B.F32, "bf16": B.BF16, "int4g64": B.INT4G64, "int2g64": B.INT2G64}[shape.dtype]
        self.ctx, self.cfg = B.adapmoe_create(shape.H, shape.F, shape.N, shape.L, dt, max_B=max_B,
                                               trace_capacity=trace_capacity)
        self.nbytes = B.adapmoe_expert_bytes(self.cfg)
        self.routers_f32 = []
        self.routers_dev = []
        self.experts_f32 = []   # [L][N] tuples (W1, W3, W2) float32, for the checker
        self.images = []        # keeps device / pinned buffers alive
        for l in range(shape.L):
            wg = synth.router_weights(shape, l, seed)
            self.routers_f32.append(wg)
            d = to_dev_act(shape.dtype, wg)
            self.routers_dev.append(d)
            B.adapmoe_set_router(self.ctx, l, d)
            row = []
            if expert_layers is not None and l not in expert_layers:     # router only (a layer that is just predicted for)
                self.experts_f32.append(row)
                continue
            for e in range(shape.N):
                w1, w3, w2 = synth.expert_weights(shape, l, e, seed)
                img = np.empty(self.nbytes, dtype=np.uint8)
                if shape.dtype in ("int4g64", "int2g64"):
                    four = shape.dtype == "int4g64"
                    qs = [(synth.quantize_int4_g64 if four else synth.quantize_int2_g64)(m) for m in (w1, w3, w2)]
                    args = []
                    for (q, sc, zr) in qs:
                        args += [q, sc.view(np.uint16), zr.view(np.uint16)]
                    (B.adapmoe_pack_expert_int4 if four else B.adapmoe_pack_expert_int2)(self.cfg, *args, img)
                    # the checker sees the same codes, scales and zeros, decoded by its own routine
                    row.append(tuple(OE_decode(q, sc, zr) for (q, sc, zr) in qs))
                else:
                    row.append((w1, w3, w2))
                    B.adapmoe_pack_expert(self.cfg, np_dtype_bits(shape.dtype, w1), np_dtype_bits(shape.dtype, w3),
                                          np_dtype_bits(shape.dtype, w2), img)
                if resident:
                    t = torch.from_numpy(img).cuda()
                    B.adapmoe_bind_expert_dev(self.ctx, l, e, t)
                else:
                    t = torch.from_numpy(img) if pageable else torch.from_numpy(img).pin_memory()
                    B.adapmoe_register_expert(self.ctx, l, e, t, self.nbytes)
                self.images.append(t)
            self.experts_f32.append(row)
        self.taus = list(taus) if taus is not None else [0.2] * shape.L
        B.adapmoe_set_tau(self.ctx, self.taus)

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize()
            B.adapmoe_destroy(self.ctx)
            self.ctx = None


def rel_err_per_token(y, ref):
    """max_i |y_i - ref_i| / max_i |ref_i| for each row (the floating-point bar)."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return np.max(np.abs(y - ref), axis=-1) / np.max(np.abs(ref), axis=-1)


def elementwise_violation(y, ref, tol):
    """Largest |y_i - ref_i| / (tol*|ref_i| + tol*rms(ref)) over all elements: <= 1 means every element is
    within tol of its reference value relative to its own size plus the same fraction of the row's rms
    (a purely relative bound is meaningless for the elements of a row that happen to be near zero)."""
    y = np.atleast_2d(np.asarray(y, dtype=np.float64))
    ref = np.atleast_2d(np.asarray(ref, dtype=np.float64))
    rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    return float(np.max(np.abs(y - ref) / (tol * np.abs(ref) + tol * rms + 1e-300)))


def elementwise_err_with_floor(y, ref, floor=1e-3):
    """max_i |y_i - ref_i| / max(|ref_i|, floor * rms(ref)) per row: the element-wise relative error with
    small reference values floored at a fraction of the row's rms (reported next to the max-norm figure)."""
    y = np.atleast_2d(np.asarray(y, dtype=np.float64))
    ref = np.atleast_2d(np.asarray(ref, dtype=np.float64))
    rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    return np.max(np.abs(y - ref) / np.maximum(np.abs(ref), floor * rms + 1e-300), axis=-1)


def check_outputs(y, ref, tol, what=""):
    """The floating-point bar in both forms: per token max-norm error <= tol, and every element within
    tol*|ref_i| + tol*rms(ref).  Returns (largest max-norm error, largest floored element-wise error)."""
    worst = float(np.max(rel_err_per_token(np.atleast_2d(y), np.atleast_2d(ref))))
    assert worst <= tol, (what, worst)
    v = elementwise_violation(y, ref, tol)
    assert v <= 1.0, (what, "element-wise bound exceeded by a factor", v)
    return worst, float(np.max(elementwise_err_with_floor(y, ref)))
