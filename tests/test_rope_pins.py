"""Pins for the rotary-embedding oracle (no GPU): the rotation is fixed to complex
multiplication written out in scalar Python, to closed forms and to the invariants that define
rotary embeddings; its rounding to the closed forms of fp16 / bf16 and to torch's casts.
(Paper Sec. 2.4 names rotary embeddings and their long-context rescaling without formulas; the
definition pinned here is the published one, every constant an input.)"""
import cmath
import math

import numpy as np
import pytest
import torch

from oracle.attention_oracle import attention_oracle
from oracle.rope_oracle import (attention_oracle_rope, attention_oracle_rope_rows, rope_rotate, rope_tables,
                                round_to_storage_type)


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_tables_closed_forms():
    cos, sin = rope_tables(50, 8, base=10000.0)
    assert cos.shape == sin.shape == (50, 4)
    assert np.all(cos[0] == 1.0) and np.all(sin[0] == 0.0)                 # position 0: identity
    assert cos[1, 0] == math.cos(1.0) and sin[1, 0] == math.sin(1.0)        # frequency 0 turns 1 rad per token
    assert np.isclose(cos[7, 3], math.cos(7 * 10000.0 ** (-6 / 8)), rtol=0, atol=1e-15)
    assert np.isclose(sin[49, 1], math.sin(49 * 10000.0 ** (-2 / 8)), rtol=0, atol=1e-13)
    assert np.allclose(cos ** 2 + sin ** 2, 1.0, rtol=0, atol=1e-15)
    # frequency rescaling and amplitude enter as given
    c2, s2 = rope_tables(50, 8, base=500.0, freq_scale=[1.0, 0.5, 0.25, 0.125], amplitude=1.25)
    assert np.isclose(c2[10, 2], 1.25 * math.cos(10 * 500.0 ** (-4 / 8) * 0.25), rtol=0, atol=1e-14)
    assert np.isclose(s2[3, 3], 1.25 * math.sin(3 * 500.0 ** (-6 / 8) * 0.125), rtol=0, atol=1e-14)


def test_rotation_is_complex_multiplication():
    """Scalar loop: the pair (x[f], x[f + D/2]) as a complex number times exp(i angle)."""
    N, D = 11, 6
    x = rand((2, 3, N, D), 1)
    cos, sin = rope_tables(N, D, base=77.0)
    got = rope_rotate(x, cos, sin)
    for b in range(2):
        for h in range(3):
            for i in range(N):
                for f in range(D // 2):
                    ang = i * 77.0 ** (-2.0 * f / D)
                    z = complex(x[b, h, i, f], x[b, h, i, f + D // 2]) * cmath.exp(1j * ang)
                    assert abs(got[b, h, i, f] - z.real) < 1e-12
                    assert abs(got[b, h, i, f + D // 2] - z.imag) < 1e-12


def test_norm_preserved_and_zero_angle_identity_and_angles_add():
    N, D = 9, 8
    x = rand((N, D), 2)
    cos, sin = rope_tables(N, D)
    y = rope_rotate(x, cos, sin)
    assert np.allclose((y ** 2).sum(-1), (x ** 2).sum(-1), rtol=1e-13)
    assert np.array_equal(rope_rotate(x, np.ones((N, D // 2)), np.zeros((N, D // 2))), x)
    # rotating by the angles of position a and then of position b = rotating by those of a + b
    ca, sa = cos[2:3].repeat(N, 0), sin[2:3].repeat(N, 0)
    cb, sb = cos[5:6].repeat(N, 0), sin[5:6].repeat(N, 0)
    c7, s7 = cos[7:8].repeat(N, 0), sin[7:8].repeat(N, 0)
    assert np.allclose(rope_rotate(rope_rotate(x, ca, sa), cb, sb), rope_rotate(x, c7, s7), rtol=0, atol=1e-13)


def test_scores_depend_on_relative_position_only():
    """The defining property: the same query vector at position i and key vector at position j
    give a dot product that depends on i - j alone."""
    N, D = 40, 16
    qv, kv = rand(D, 3), rand(D, 4)
    cos, sin = rope_tables(N, D, base=300.0)
    q = rope_rotate(np.tile(qv, (N, 1)), cos, sin)
    k = rope_rotate(np.tile(kv, (N, 1)), cos, sin)
    s = q @ k.T
    for delta in (-7, 0, 1, 13):
        diag = np.array([s[i, i - delta] for i in range(max(0, delta), min(N, N + delta))])
        assert np.allclose(diag, diag[0], rtol=0, atol=1e-12), delta
    assert not np.isclose(s[5, 3], s[5, 4])           # and does depend on it


def test_rounding_to_storage_types():
    x = np.concatenate([rand(5000, 5) * 3.0, rand(2000, 6) * 1e-3, [0.0, 1.0, -2.5, 65504.0, 1e-40, -3e-41]])
    # fp16: numpy's own cast; bf16: torch's cast (both round to nearest, ties to even, from fp64 -> via fp32
    # is exact here because the inputs are made fp32-representable first)
    x = x.astype(np.float32).astype(np.float64)
    assert np.array_equal(round_to_storage_type(x, "fp16"), x.astype(np.float16).astype(np.float64))
    t = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_to_storage_type(x, "bf16"), t)
    # ties go to even: 1 + 2^-8 is halfway between the bf16 neighbours 1 and 1 + 2^-7
    assert round_to_storage_type(np.array([1.0 + 2.0 ** -8]), "bf16")[0] == 1.0
    assert round_to_storage_type(np.array([1.0 + 3 * 2.0 ** -8]), "bf16")[0] == 1.0 + 2.0 ** -6
    assert round_to_storage_type(np.array([1.0 + 2.0 ** -11]), "fp16")[0] == 1.0


def test_attention_with_rotation_is_attention_of_rotated_rounded_inputs():
    B, H, N, D = 2, 2, 13, 8
    q, k, v = rand((B, H, N, D), 7), rand((B, H, N, D), 8), rand((B, H, N, D), 9)
    cos, sin = rope_tables(N, D, base=50.0)
    lens = (13, 9)
    for dtype in ("fp16", "bf16"):
        o, lse = attention_oracle_rope(q, k, v, cos, sin, dtype, lens, 0.3, 2, 3)
        # written out again here, element by element for q and k
        qr, kr = np.empty_like(q), np.empty_like(k)
        for i in range(N):
            for f in range(D // 2):
                c, s_ = cos[i, f], sin[i, f]
                for src, dst in ((q, qr), (k, kr)):
                    dst[..., i, f] = src[..., i, f] * c - src[..., i, f + D // 2] * s_
                    dst[..., i, f + D // 2] = src[..., i, f + D // 2] * c + src[..., i, f] * s_
        cast = (lambda a: a.astype(np.float16).astype(np.float64)) if dtype == "fp16" else \
            (lambda a: torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy())
        # (fp64 -> 16 bit in one step for fp16; torch rounds fp64 -> bf16 in one step as well)
        o2, lse2 = attention_oracle(cast(qr), cast(kr), v, lens, 0.3, 2, 3)
        assert np.array_equal(o, o2) and np.array_equal(lse, lse2)
        orow, lrow = attention_oracle_rope_rows(q, k, v, cos, sin, dtype, 1, 0, [0, 4, 8], 9, 0.3, 2, 3)
        assert np.array_equal(orow, o[1, 0, [0, 4, 8]]) and np.array_equal(lrow, lse[1, 0, [0, 4, 8]])


def test_rotation_changes_attention_unless_positions_are_equal():
    """With one token position repeated (all angles equal) the rotation cancels in q.k."""
    B, H, N, D = 1, 1, 6, 4
    q, k, v = rand((B, H, N, D), 10), rand((B, H, N, D), 11), rand((B, H, N, D), 12)
    cos, sin = rope_tables(N, D)
    same_c, same_s = cos[3:4].repeat(N, 0), sin[3:4].repeat(N, 0)
    o_plain, _ = attention_oracle(q, k, v)
    o_same, _ = attention_oracle(rope_rotate(q, same_c, same_s), rope_rotate(k, same_c, same_s), v)
    o_rot, _ = attention_oracle(rope_rotate(q, cos, sin), rope_rotate(k, cos, sin), v)
    assert np.allclose(o_same, o_plain, rtol=0, atol=1e-12)
    assert np.abs(o_rot - o_plain).max() > 1e-3
