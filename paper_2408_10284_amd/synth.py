"""Seeded synthetic inputs for the decode-time MoE block.

This module only *draws and stores numbers*: random weights, hidden-state
streams, storage-format rounding (bf16) and the group-quantised int4 storage
format of the weights.  It holds none of the method's arithmetic (no gating,
no expert evaluation, no cache policy, no dequantisation) and imports neither
the HIP binding nor the CPU checker, so both can be fed from it.

Shapes follow Mixtral-8x7B (the paper's evaluation model, Sec. 6.1): hidden
size H, FFN size F, N experts per layer, experts stored as W1[F,H] (gate
projection), W3[F,H] (up projection), W2[H,F] (down projection).  Values are
random stand-ins for the trained weights and benchmark prompts, which are not
available here.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

# ----------------------------------------------------------------------------
# storage formats
# ----------------------------------------------------------------------------


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bfloat16, returned as float32."""
    return bf16_to_f32(bf16_bits(a))


# ----------------------------------------------------------------------------
# configurations (the five workloads of the baseline description)
# ----------------------------------------------------------------------------


@dataclass(frozen=True)
class MoEShape:
    H: int
    F: int
    N: int
    L: int = 1
    dtype: str = "f32"  # "f32" | "bf16" | "int4g64" | "int2g64"


TINY = MoEShape(H=512, F=1024, N=8, L=1, dtype="f32")
MIXTRAL_LAYER = MoEShape(H=4096, F=14336, N=8, L=1, dtype="bf16")
MIXTRAL_STACK = MoEShape(H=4096, F=14336, N=8, L=32, dtype="bf16")
MIXTRAL_STACK_INT4 = MoEShape(H=4096, F=14336, N=8, L=32, dtype="int4g64")

WEIGHT_STD = 0.02


def _rng(*key: int) -> np.random.Generator:
    return np.random.default_rng([int(k) for k in key])


def router_weights(shape: MoEShape, layer: int, seed: int = 0) -> np.ndarray:
    """W_g of one layer, [N,H] float32, N(0, 0.02^2); bf16-rounded for bf16/int4 shapes."""
    w = _rng(seed, 1, layer).standard_normal((shape.N, shape.H), dtype=np.float32) * np.float32(WEIGHT_STD)
    return w if shape.dtype == "f32" else bf16_round(w)


def expert_weights(shape: MoEShape, layer: int, expert: int, seed: int = 0):
    """(W1[F,H], W3[F,H], W2[H,F]) of one expert, float32 storage, N(0, 0.02^2).

    Drawn from a generator keyed on (seed, layer, expert) so any expert can be
    regenerated without materialising the others.  For bf16 and int4 shapes
    the values are bf16-rounded (the int4 codes are then derived from them by
    `quantize_int4_g64`).
    """
    g = _rng(seed, 2, layer, expert)
    s = np.float32(WEIGHT_STD)
    w1 = g.standard_normal((shape.F, shape.H), dtype=np.float32) * s
    w3 = g.standard_normal((shape.F, shape.H), dtype=np.float32) * s
    w2 = g.standard_normal((shape.H, shape.F), dtype=np.float32) * s
    if shape.dtype != "f32":
        w1, w3, w2 = bf16_round(w1), bf16_round(w3), bf16_round(w2)
    return w1, w3, w2


def iid_tokens(n: int, H: int, seed: int = 1, dtype: str = "f32") -> np.ndarray:
    """n independent hidden states ~ N(0, I), [n,H] float32."""
    x = _rng(seed, 3).standard_normal((n, H), dtype=np.float32)
    return x if dtype == "f32" else bf16_round(x)


def ar1_tokens(n: int, H: int, rho: float = 0.8, seed: int = 1, dtype: str = "bf16") -> np.ndarray:
    """n hidden states following a per-element AR(1) process with N(0,1) marginals.

    x_0 ~ N(0,I); x_t = rho x_{t-1} + sqrt(1-rho^2) eps_t.  Successive tokens are
    correlated, which gives the routing locality an expert cache relies on.
    """
    g = _rng(seed, 4)
    x = np.empty((n, H), dtype=np.float32)
    x[0] = g.standard_normal(H, dtype=np.float32)
    c = np.float32(np.sqrt(1.0 - rho * rho))
    for t in range(1, n):
        x[t] = np.float32(rho) * x[t - 1] + c * g.standard_normal(H, dtype=np.float32)
    return x if dtype == "f32" else bf16_round(x)


def ar1_streams(n_steps: int, B: int, H: int, rho: float = 0.8, seed: int = 1, dtype: str = "bf16") -> np.ndarray:
    """B independent AR(1) streams, [n_steps,B,H] float32 (the batched workload)."""
    out = np.empty((n_steps, B, H), dtype=np.float32)
    for b in range(B):
        out[:, b, :] = ar1_tokens(n_steps, H, rho, seed=seed * 1000 + b, dtype=dtype)
    return out


def tau_profile(L: int, lo: float = 0.15, hi: float = 0.35) -> np.ndarray:
    """Per-layer gating thresholds tau_l = sqrt(T / S_l) for a synthetic
    sensitivity profile in which early layers are the most sensitive (Sec. 6.5):
    tau rises linearly from `lo` at layer 0 to `hi` at layer L-1.  float32."""
    if L == 1:
        return np.array([lo], dtype=np.float32)
    return np.linspace(lo, hi, L).astype(np.float32)


# ----------------------------------------------------------------------------
# int4 storage format (group 64 along the reduction axis, fp16 scale + zero)
# ----------------------------------------------------------------------------

INT4_GROUP = 64


def quantize_int4_g64(w: np.ndarray, levels: int = 15):
    """Round-to-nearest asymmetric 4-bit storage of a [rows, cols] matrix
    (levels = 15; `quantize_int2_g64` calls it with levels = 3 for 2-bit codes).

    Groups are 64 consecutive elements along the last axis (the axis a
    matrix-vector product reduces over).  Per group: zero = fp16(min),
    scale = fp16((max-min)/15), code = clamp(rint((w-zero)/scale), 0, 15) with
    the fp16-rounded scale/zero (scale == 0 -> code 0).  Returns
    (codes uint8 [rows, cols] with values 0..15, scale fp16 [rows, cols/64],
    zero fp16 [rows, cols/64]).  Packing into nibbles is the consumer's
    business (`pack_nibbles`).
    """
    rows, cols = w.shape
    assert cols % INT4_GROUP == 0
    g = np.ascontiguousarray(w, dtype=np.float32).reshape(rows, cols // INT4_GROUP, INT4_GROUP)
    lo = g.min(axis=2)
    hi = g.max(axis=2)
    zero = lo.astype(np.float16)
    scale = ((hi - lo) / np.float32(levels)).astype(np.float16)
    z32 = zero.astype(np.float32)[:, :, None]
    s32 = scale.astype(np.float32)[:, :, None]
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.rint((g - z32) / s32)
    q = np.where(s32 > 0, q, 0.0)
    q = np.clip(q, 0.0, float(levels)).astype(np.uint8)
    return q.reshape(rows, cols), scale, zero


def quantize_int2_g64(w: np.ndarray):
    """The same storage scheme with 2-bit codes 0..3: scale = fp16((max-min)/3)."""
    return quantize_int4_g64(w, levels=3)


def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """[rows, cols] codes 0..15 -> [rows, cols/2] bytes; element 2i in the low
    nibble, element 2i+1 in the high nibble."""
    c = codes.reshape(codes.shape[0], -1, 2)
    return (c[:, :, 0] | (c[:, :, 1] << 4)).astype(np.uint8)


# ----------------------------------------------------------------------------
# large stacks: expert images drawn on the GPU
# ----------------------------------------------------------------------------
# With i.i.d. weights the packed image of an expert is itself an i.i.d. array,
# so the multi-layer workloads (hundreds of experts, ~90 GB) draw each image
# directly, keyed on (seed, layer, expert), instead of drawing three matrices
# and packing them.  `unpack_image_bf16` recovers the canonical matrices of an
# image for the checker: rows of W1 and W3 interleaved ([F][2][H]), then W2
# ([H][F]).


def expert_image_bf16_torch(shape: MoEShape, layer: int, expert: int, seed: int = 0, device: str = "cuda"):
    """bfloat16 tensor [3*H*F] ~ N(0, 0.02^2): the image of expert (layer, expert)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(layer)) * 1009 + int(expert))
    n = 3 * shape.H * shape.F
    return (torch.randn(n, device=device, generator=g, dtype=torch.float32) * WEIGHT_STD).to(torch.bfloat16)


def router_bf16_torch(shape: MoEShape, layer: int, seed: int = 0, device: str = "cuda"):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(layer)) * 1009 + 977)
    return (torch.randn((shape.N, shape.H), device=device, generator=g, dtype=torch.float32) * WEIGHT_STD).to(torch.bfloat16)


def unpack_image_bf16(bits: np.ndarray, H: int, F: int):
    """uint16 image [3*H*F] -> (W1[F,H], W3[F,H], W2[H,F]) float32."""
    gu = bits[: 2 * F * H].reshape(F, 2, H)
    w2 = bits[2 * F * H:].reshape(H, F)
    return bf16_to_f32(gu[:, 0, :]), bf16_to_f32(gu[:, 1, :]), bf16_to_f32(w2)


# ----------------------------------------------------------------------------
# int4 images on the GPU (same storage format and row layout as the library's
# host-side packer; used where hundreds of experts have to be prepared)
# ----------------------------------------------------------------------------


def quantize_int4_g64_torch(w, levels=15):
    """torch version of `quantize_int4_g64` (same float32 arithmetic): float32
    [rows, cols] -> (codes uint8 [rows, cols], scale fp16 [rows, cols/64], zero fp16)."""
    import torch
    rows, cols = w.shape
    g = w.reshape(rows, cols // INT4_GROUP, INT4_GROUP).to(torch.float32)
    lo = g.amin(dim=2)
    hi = g.amax(dim=2)
    zero = lo.to(torch.float16)
    scale = ((hi - lo) / float(levels)).to(torch.float16)
    z32 = zero.to(torch.float32).unsqueeze(2)
    s32 = scale.to(torch.float32).unsqueeze(2)
    q = torch.round((g - z32) / s32)
    q = torch.where(s32 > 0, q, torch.zeros_like(q))
    q = q.clamp_(0.0, float(levels)).to(torch.uint8)
    return q.reshape(rows, cols), scale, zero


def _int4_rows_torch(q, scale, zero):
    """codes [rows, n] + scale/zero [rows, n/64] -> uint8 [rows, n/2 + n/16] in the streaming row
    format: blocks of up to 64 groups stored as [first 16 bytes of every group][second 16 bytes];
    inside a dword nibble s (s < 4) is element 2s and nibble s+4 is element 2s+1; then
    (scale, zero) per group."""
    import torch
    rows, n = q.shape
    G = n // INT4_GROUP
    e = q.reshape(rows, G, 2, 4, 8)                      # [row][group][half][dword][element]
    by = torch.stack([e[..., 0] | (e[..., 2] << 4), e[..., 4] | (e[..., 6] << 4),
                      e[..., 1] | (e[..., 3] << 4), e[..., 5] | (e[..., 7] << 4)], dim=-1)   # 4 bytes per dword
    by = by.reshape(rows, G, 2, 16)
    parts = []
    full = (G // 64) * 64
    if full:
        parts.append(by[:, :full].reshape(rows, full // 64, 64, 2, 16).permute(0, 1, 3, 2, 4).reshape(rows, -1))
    if G > full:
        parts.append(by[:, full:].permute(0, 2, 1, 3).reshape(rows, -1))
    sz = torch.stack([scale.view(torch.int16), zero.view(torch.int16)], dim=-1).contiguous().view(torch.uint8).reshape(rows, G * 4)
    return torch.cat(parts + [sz], dim=1)


def int4_image_from_weights_torch(w1, w3, w2):
    """float32 W1[F,H], W3[F,H], W2[H,F] (torch) -> uint8 image in the library's int4 layout
    (rows of W1 and W3 interleaved, then rows of W2)."""
    import torch
    r1 = _int4_rows_torch(*quantize_int4_g64_torch(w1))
    r3 = _int4_rows_torch(*quantize_int4_g64_torch(w3))
    r2 = _int4_rows_torch(*quantize_int4_g64_torch(w2))
    gu = torch.stack([r1, r3], dim=1).reshape(-1)
    return torch.cat([gu, r2.reshape(-1)])


def expert_image_int4_torch(shape: MoEShape, layer: int, expert: int, seed: int = 0, device: str = "cuda"):
    """int4 image of expert (layer, expert): bf16 N(0, 0.02^2) weights drawn on the device, quantised
    round-to-nearest per group of 64 and packed."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(layer)) * 1009 + int(expert))
    H, F = shape.H, shape.F
    mats = []
    for (r, c) in ((F, H), (F, H), (H, F)):
        w = (torch.randn((r, c), device=device, generator=g, dtype=torch.float32) * WEIGHT_STD).to(torch.bfloat16).to(torch.float32)
        mats.append(w)
    return int4_image_from_weights_torch(*mats)


def decode_int4_image(img: np.ndarray, H: int, F: int):
    """uint8 int4 image -> per matrix (codes [rows, n], scale fp16, zero fp16) for W1, W3, W2,
    reading the documented row format (the inverse of the packers; input preparation for the checker)."""
    def rows_of(buf, rows, n):
        G = n // INT4_GROUP
        rb = n // 2 + n // 16
        a = buf.reshape(rows, rb)
        codes = np.empty((rows, n), dtype=np.uint8)
        for blk in range((G + 63) // 64):
            nb = min(64, G - blk * 64)
            blkb = a[:, blk * 2048: blk * 2048 + nb * 32].reshape(rows, 2, nb, 4, 4)      # [half][group][dword][byte]
            # bytes of a dword: (e0|e2<<4), (e4|e6<<4), (e1|e3<<4), (e5|e7<<4)
            el = np.empty((rows, 2, nb, 4, 8), dtype=np.uint8)
            el[..., 0], el[..., 2] = blkb[..., 0] & 15, blkb[..., 0] >> 4
            el[..., 4], el[..., 6] = blkb[..., 1] & 15, blkb[..., 1] >> 4
            el[..., 1], el[..., 3] = blkb[..., 2] & 15, blkb[..., 2] >> 4
            el[..., 5], el[..., 7] = blkb[..., 3] & 15, blkb[..., 3] >> 4
            codes[:, blk * 4096: blk * 4096 + nb * 64] = el.transpose(0, 2, 1, 3, 4).reshape(rows, nb * 64)
        sz = np.ascontiguousarray(a[:, n // 2:]).view(np.uint16).reshape(rows, G, 2)
        return codes, sz[..., 0].copy().view(np.float16), sz[..., 1].copy().view(np.float16)

    rbH = H // 2 + H // 16
    gu = img[: 2 * F * rbH].reshape(F, 2, rbH)
    m1 = rows_of(np.ascontiguousarray(gu[:, 0]), F, H)
    m3 = rows_of(np.ascontiguousarray(gu[:, 1]), F, H)
    m2 = rows_of(img[2 * F * rbH:], H, F)
    return m1, m3, m2


# ----------------------------------------------------------------------------
# 2-bit images (same scheme, codes 0..3; a group's 64 codes are 16 bytes; in a dword field s of
# the low half is element 2s and field s of the high half is element 2s+1 of its 16 elements)
# ----------------------------------------------------------------------------


def _int2_rows_torch(q, scale, zero):
    """codes [rows, n] (0..3) + scale/zero [rows, n/64] -> uint8 [rows, n/4 + n/16]: per group 16
    bytes of codes (groups consecutive), then (scale, zero) per group."""
    import torch
    rows, n = q.shape
    G = n // INT4_GROUP
    e = q.reshape(rows, G, 4, 16)                        # [row][group][dword][element]
    def byte(a, b, c, d):
        return e[..., a] | (e[..., b] << 2) | (e[..., c] << 4) | (e[..., d] << 6)
    by = torch.stack([byte(0, 2, 4, 6), byte(8, 10, 12, 14), byte(1, 3, 5, 7), byte(9, 11, 13, 15)], dim=-1)
    sz = torch.stack([scale.view(torch.int16), zero.view(torch.int16)], dim=-1).contiguous().view(torch.uint8).reshape(rows, G * 4)
    return torch.cat([by.reshape(rows, G * 16), sz], dim=1)


def int2_image_from_weights_torch(w1, w3, w2):
    """float32 W1[F,H], W3[F,H], W2[H,F] (torch) -> uint8 image in the library's 2-bit layout."""
    import torch
    r1 = _int2_rows_torch(*quantize_int4_g64_torch(w1, levels=3))
    r3 = _int2_rows_torch(*quantize_int4_g64_torch(w3, levels=3))
    r2 = _int2_rows_torch(*quantize_int4_g64_torch(w2, levels=3))
    gu = torch.stack([r1, r3], dim=1).reshape(-1)
    return torch.cat([gu, r2.reshape(-1)])


def expert_image_int2_torch(shape: MoEShape, layer: int, expert: int, seed: int = 0, device: str = "cuda"):
    """2-bit image of expert (layer, expert): the same bf16 N(0, 0.02^2) weights as the int4 generator."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + int(layer)) * 1009 + int(expert))
    H, F = shape.H, shape.F
    mats = []
    for (r, c) in ((F, H), (F, H), (H, F)):
        w = (torch.randn((r, c), device=device, generator=g, dtype=torch.float32) * WEIGHT_STD).to(torch.bfloat16).to(torch.float32)
        mats.append(w)
    return int2_image_from_weights_torch(*mats)


def decode_int2_image(img: np.ndarray, H: int, F: int):
    """uint8 2-bit image -> per matrix (codes [rows, n], scale fp16, zero fp16) for W1, W3, W2."""
    def rows_of(buf, rows, n):
        G = n // INT4_GROUP
        rb = n // 4 + n // 16
        a = buf.reshape(rows, rb)
        by = a[:, : n // 4].reshape(rows, G, 4, 4)                      # [group][dword][byte]
        el = np.empty((rows, G, 4, 16), dtype=np.uint8)
        for b, first in enumerate((0, 8, 1, 9)):                        # byte b holds elements first, first+2, +4, +6
            for f in range(4):
                el[..., first + 2 * f] = (by[..., b] >> (2 * f)) & 3
        sz = np.ascontiguousarray(a[:, n // 4:]).view(np.uint16).reshape(rows, G, 2)
        return el.reshape(rows, n), sz[..., 0].copy().view(np.float16), sz[..., 1].copy().view(np.float16)

    rbH = H // 4 + H // 16
    gu = img[: 2 * F * rbH].reshape(F, 2, rbH)
    m1 = rows_of(np.ascontiguousarray(gu[:, 0]), F, H)
    m3 = rows_of(np.ascontiguousarray(gu[:, 1]), F, H)
    m2 = rows_of(img[2 * F * rbH:], H, F)
    return m1, m3, m2
