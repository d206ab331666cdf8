"""fp64 CPU oracle for rotary position embedding applied to Q and K ahead of attention.
TEST INFRASTRUCTURE ONLY (same rules as attention_oracle.py: imported by tests/ only, shares
nothing with the product package).

What is computed.  The paper's classifier (Sec. 2.4 "ModernBERT") uses rotary position
embeddings, in a variant whose frequencies are rescaled to reach 32K tokens; the paper gives no
formula or constant for either, so this file follows the published definition of rotary
embeddings and takes every constant as an input:

    angle[i, f] = i * inv_freq[f],     i = token position, f = 0 .. D/2 - 1
    inv_freq[f] = base ** (-2 f / D) * freq_scale[f]            (freq_scale = 1: plain rotary)
    x'[i, f]       = x[i, f] cos(angle[i, f]) - x[i, f + D/2] sin(angle[i, f])
    x'[i, f + D/2] = x[i, f + D/2] cos(angle[i, f]) + x[i, f] sin(angle[i, f])

i.e. the pair (x[f], x[f + D/2]) is rotated by angle[i, f] (the half-split pairing), and the
scores become q'_i . k'_j, which depend on the positions only through i - j.  A frequency
rescaling (the long-context variant) enters through freq_scale and an optional constant
`amplitude` that multiplies cos and sin; the values the paper's model uses are not published:
PARITY OF THOSE CONSTANTS IS UNPINNED, the rotation itself is pinned (tests/test_rope_pins.py).

Readings (the paper is silent on all of them):
  * positions are absolute token indices 0, 1, 2, ... of the padded sequence;
  * half-split pairing (f, f + D/2), not interleaved (2f, 2f + 1);
  * the rotated q and k are ROUNDED TO THE STORAGE TYPE before the product, as an exported
    graph that applies the rotation as fp16 / bf16 tensor operations ahead of the attention
    node does, and as any kernel that feeds 16-bit matrix cores must; v is not rotated;
  * cos / sin come in as tables [N, D/2]; the oracle uses the table values it is given (the
    tests pass the same fp32-rounded tables to both sides), so table precision is not part of
    the comparison.
"""
from __future__ import annotations

import numpy as np

from oracle.attention_oracle import attention_oracle, attention_oracle_rows

__all__ = ["rope_tables", "rope_rotate", "round_to_storage_type", "attention_oracle_rope",
           "attention_oracle_rope_rows"]


def rope_tables(n_positions: int, head_dim: int, base: float = 10000.0, freq_scale=None, amplitude: float = 1.0):
    """cos, sin [n_positions, head_dim / 2] in fp64 for positions 0 .. n_positions - 1."""
    half = head_dim // 2
    f = np.arange(half, dtype=np.float64)
    inv_freq = base ** (-2.0 * f / head_dim)
    if freq_scale is not None:
        inv_freq = inv_freq * np.asarray(freq_scale, dtype=np.float64).reshape(half)
    angle = np.arange(n_positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    return amplitude * np.cos(angle), amplitude * np.sin(angle)


def rope_rotate(x, cos, sin):
    """x: [..., N, D]; cos, sin: [N, D/2].  Returns the rotated array in fp64."""
    x = np.asarray(x, dtype=np.float64)
    cos = np.asarray(cos, dtype=np.float64)
    sin = np.asarray(sin, dtype=np.float64)
    half = x.shape[-1] // 2
    lo, hi = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = lo * cos - hi * sin
    out[..., half:] = hi * cos + lo * sin
    return out


def round_to_storage_type(x, dtype: str):
    """Nearest fp16 / bf16 value, ties to even, returned as fp64 (the oracle's own rounding)."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == "fp16":
        return x.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        # fp64 -> fp32 first would round twice; bf16 keeps 8 significant bits, so do it directly:
        # scale each value to an integer significand of 8 bits and round that to even
        out = np.zeros_like(x)
        nz = np.isfinite(x) & (x != 0)
        m, e = np.frexp(x[nz])                    # x = m * 2**e, 0.5 <= |m| < 1
        e_min = -125                              # smallest normal bf16 exponent in frexp terms
        shift = np.maximum(e, e_min)              # subnormals keep the spacing of the smallest normal
        q = np.rint(np.ldexp(x[nz], 8 - shift))   # np.rint rounds half to even
        out[nz] = np.ldexp(q, shift - 8)
        out[~np.isfinite(x)] = x[~np.isfinite(x)]
        return out
    raise ValueError(f"unknown storage dtype {dtype!r}")


def _rotated(q, k, cos, sin, dtype):
    return (round_to_storage_type(rope_rotate(q, cos, sin), dtype),
            round_to_storage_type(rope_rotate(k, cos, sin), dtype))


def attention_oracle_rope(q, k, v, cos, sin, dtype, seq_lens=None, scale=1.0, left=-1, right=-1, key_bias=None):
    """Rotate q and k by position, round them to the storage type, then plain attention."""
    qr, kr = _rotated(q, k, cos, sin, dtype)
    return attention_oracle(qr, kr, v, seq_lens, scale, left, right, key_bias=key_bias)


def attention_oracle_rope_rows(q, k, v, cos, sin, dtype, b, h, rows, n_valid, scale=1.0, left=-1, right=-1):
    """Sampled query rows of one (batch, head) of the rotated problem."""
    q1 = np.asarray(q)[b:b + 1, h:h + 1]
    k1 = np.asarray(k)[b:b + 1, h:h + 1]
    v1 = np.asarray(v)[b:b + 1, h:h + 1]
    qr, kr = _rotated(q1, k1, cos, sin, dtype)
    return attention_oracle_rows(qr, kr, v1, 0, 0, rows, n_valid, scale, left, right)
