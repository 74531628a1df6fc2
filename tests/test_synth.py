"""Checks of the seeded input generators (no method arithmetic in them)."""
import numpy as np
import torch

from paper_2408_10284_amd import synth


def test_bf16_round_matches_torch_cpu():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(100000) * 10.0 ** rng.integers(-6, 6, 100000)).astype(np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(synth.bf16_round(a), ref)
    bits = synth.bf16_bits(a)
    np.testing.assert_array_equal(synth.bf16_to_f32(bits), ref)
    # exact ties round to even
    tie = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)
    np.testing.assert_array_equal(synth.bf16_round(tie), np.array([1.0, 1.0 + 2.0 ** -6], dtype=np.float32))


def test_generators_are_seeded_and_shaped():
    s = synth.MoEShape(H=64, F=128, N=4, L=2, dtype="bf16")
    w1, w3, w2 = synth.expert_weights(s, 1, 2)
    v1, v3, v2 = synth.expert_weights(s, 1, 2)
    assert w1.shape == (128, 64) and w3.shape == (128, 64) and w2.shape == (64, 128)
    np.testing.assert_array_equal(w1, v1)
    np.testing.assert_array_equal(w2, v2)
    assert not np.array_equal(w1, synth.expert_weights(s, 1, 3)[0])
    np.testing.assert_array_equal(w1, synth.bf16_round(w1))
    assert abs(w1.std() - 0.02) < 0.002
    wg = synth.router_weights(s, 0)
    assert wg.shape == (4, 64)


def test_ar1_statistics():
    x = synth.ar1_tokens(4000, 32, rho=0.8, seed=3, dtype="f32")
    assert abs(x.std() - 1.0) < 0.05
    c = np.mean(x[1:] * x[:-1])
    assert abs(c - 0.8) < 0.05


def test_int4_quantiser_error_bound():
    rng = np.random.default_rng(1)
    w = synth.bf16_round((rng.standard_normal((16, 256)) * 0.02).astype(np.float32))
    q, scale, zero = synth.quantize_int4_g64(w)
    assert q.dtype == np.uint8 and q.max() <= 15
    assert scale.shape == (16, 4) and scale.dtype == np.float16
    s = np.repeat(scale.astype(np.float32), 64, axis=1)
    z = np.repeat(zero.astype(np.float32), 64, axis=1)
    err = np.abs(q * s + z - w)
    # half a step, plus the fp16 rounding of zero and of 15*scale at the top of the range
    assert np.all(err <= 0.5 * s + 2.0 ** -11 * (np.abs(z) + 15 * s) + 1e-12)
    p = synth.pack_nibbles(q)
    assert p.shape == (16, 128)
    np.testing.assert_array_equal(p & 0xF, q[:, 0::2])
    np.testing.assert_array_equal(p >> 4, q[:, 1::2])
    # constant group: scale 0, codes 0
    q0, s0, z0 = synth.quantize_int4_g64(np.full((1, 64), 0.5, dtype=np.float32))
    assert np.all(q0 == 0) and s0[0, 0] == 0 and z0[0, 0] == np.float16(0.5)


def test_int2_quantiser_error_bound():
    rng = np.random.default_rng(2)
    w = synth.bf16_round((rng.standard_normal((8, 192)) * 0.02).astype(np.float32))
    q, scale, zero = synth.quantize_int2_g64(w)
    assert q.dtype == np.uint8 and q.max() == 3 and q.min() == 0
    s = np.repeat(scale.astype(np.float32), 64, axis=1)
    z = np.repeat(zero.astype(np.float32), 64, axis=1)
    err = np.abs(q * s + z - w)
    assert np.all(err <= 0.5 * s + 2.0 ** -11 * (np.abs(z) + 3 * s) + 1e-12)
    # every group uses both ends of its range
    g = q.reshape(8, 3, 64)
    assert np.all(g.min(axis=2) == 0) and np.all(g.max(axis=2) == 3)
