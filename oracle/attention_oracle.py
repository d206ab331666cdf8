"""fp64 CPU oracle for masked scaled-dot-product attention.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition that the GPU flash-attention forward is
checked against.  Only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import it; the product package never does, and this file
imports nothing from the product package.

What is computed (paper Sec. 2.2: softmax(Q K^T / sqrt(d_k)) V, a result that
flash attention reaches exactly, up to rounding order; Sec. 4.1.3: the operator's
inputs [Q, K, V, pad_bias] and attributes scale, window_size_left,
window_size_right; Eq. 1: the 1-D key-padding bias):

    for every batch b, head h and query row i < n_b
        s_j   = scale * sum_d Q[i,d] K[j,d]                for every key j < N
        s_j  += key_bias[b, j]   when an additive 1-D key bias is given (the operator's
                                 pad_bias input, Sec. 4.1.3 / Eq. 1: one value per key,
                                 shared by all heads and queries, NOT multiplied by scale)
        s_j   = -inf  where key j is not visible
        m     = max_j s_j,  e_j = exp(s_j - m),  l = sum_j e_j
        o[i]  = sum_j (e_j / l) V[j],   lse[i] = m + ln(l)
    rows i >= n_b (padding): o = 0, lse = -inf

Visibility of key j for query i in a sequence of valid length n_b:
    j < n_b                                   (key-padding mask, Eq. 1 read as exclusion)
    i - L <= j <= i + R   when the layer is local with window (L, R)
                          (Sec. 4.1.3 "ModernBERT Attention Mapping":
                           local layers L=63, R=64; global layers -1, -1)

The whole score row is formed and masked (no tiling, no running maximum, no
skipping); query rows are processed in blocks only to bound host memory, which
does not change any row's arithmetic because rows are independent.

Readings where the paper is silent (kept in step with the design notes):
  * mask = exclusion (-inf), not the finite -65504 bias of Eq. 1; the two agree
    exactly whenever a row has a visible key (`additive_bias_variant` below
    exists so a test can show that);
  * padding is a tail: keys/queries j >= n_b are padding;
  * padded query rows and rows with no visible key give o = 0, lse = -inf;
  * lse is the natural-log logsumexp of the scaled, masked scores;
  * window positions are absolute token indices, clipped at 0 and n_b;
  * a key bias of -inf excludes that key (an arbitrary, non-tail key mask); finite
    values are added literally, so the paper's -65504 on padded keys is also accepted.

Pins (tests/test_oracle_pins.py, no GPU): pure-Python brute force on tiny
inputs, scipy softmax/logsumexp and torch-CPU SDPA on special cases, closed
forms (Q = 0, L = R = 0, one-hot limit), invariants (rows of P sum to 1,
constant V, key permutation, masked keys have no effect, key shift,
split/merge identity); for the key bias: brute force, ln(w_j) bias = key j repeated
w_j times, constant bias shifts lse only, -inf bias = key removed, -65504 on the tail
= the literal form of Eq. 1.  Parity with the paper's trained-model activations is
unpinned: no weights or tensors are published with the paper.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "window_from_width",
    "visible_mask",
    "attention_oracle",
    "attention_oracle_rows",
    "additive_bias_variant",
]


def window_from_width(window: int) -> tuple[int, int]:
    """Map the single `window` argument of the C boundary to (L, R).

    window < 0  -> global layer, the paper's (-1, -1).
    window = W >= 1 -> L = (W - 1) // 2, R = W // 2, so W = 128 gives the paper's
    local-layer values 63 / 64 (Sec. 4.1.3) and exactly W visible keys for an
    interior row.
    """
    if window < 0:
        return (-1, -1)
    if window == 0:
        raise ValueError("window = 0 is not a legal width")
    return ((window - 1) // 2, window // 2)


def visible_mask(rows: np.ndarray, n_keys_total: int, n_valid: int, left: int, right: int) -> np.ndarray:
    """Boolean [len(rows), n_keys_total]: True where key j is visible to query rows[r].

    left < 0 means unbounded to the left, right < 0 unbounded to the right.
    """
    j = np.arange(n_keys_total, dtype=np.int64)[None, :]
    i = np.asarray(rows, dtype=np.int64)[:, None]
    vis = np.broadcast_to(j < n_valid, (i.shape[0], n_keys_total)).copy()
    if left >= 0:
        vis &= j >= i - left
    if right >= 0:
        vis &= j <= i + right
    return vis


def _rows_one_head(q, k, v, rows, n_valid, scale, left, right, want_p, key_bias=None):
    """Attention for the given query rows of one (batch, head). q,k,v: [N, D] float64;
    key_bias: None or [N] float64, added to the scaled scores."""
    n_total = k.shape[0]
    s = (q[rows] @ k.T) * scale                      # full score rows, [R, N]
    if key_bias is not None:
        s = s + key_bias[None, :]
    vis = visible_mask(rows, n_total, n_valid, left, right)
    s = np.where(vis, s, -np.inf)
    m = s.max(axis=1)                                # [R]
    has_key = np.isfinite(m)
    m_safe = np.where(has_key, m, 0.0)
    e = np.where(vis, np.exp(s - m_safe[:, None]), 0.0)
    l = e.sum(axis=1)
    l_safe = np.where(has_key, l, 1.0)
    p = e / l_safe[:, None]
    # p is exactly 0 on padded keys; summing over j < n_valid only keeps whatever
    # the caller left in the padded V rows (even NaN) out of 0 * V[j].
    o = p[:, :n_valid] @ v[:n_valid]
    with np.errstate(divide="ignore"):
        lse = np.where(has_key, m_safe + np.log(l_safe), -np.inf)
    return o, lse, (p if want_p else None)


def attention_oracle(q, k, v, seq_lens=None, scale=1.0, left=-1, right=-1,
                     row_block=256, return_p=False, key_bias=None):
    """Full oracle. q, k, v: [B, H, N, D] (any float dtype; converted exactly to fp64).
    key_bias: None or [B, N], one additive value per key (-inf excludes the key).

    seq_lens: None (every sequence has N valid tokens) or B integers; values are
    clamped into [0, N].  Returns (o [B,H,N,D] fp64, lse [B,H,N] fp64) and, when
    return_p is set, also P [B,H,N,N] (tiny inputs only).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, H, N, D = q.shape
    if seq_lens is None:
        seq_lens = [N] * B
    if key_bias is not None:
        key_bias = np.asarray(key_bias, dtype=np.float64).reshape(B, N)
    o = np.zeros((B, H, N, D), dtype=np.float64)
    lse = np.full((B, H, N), -np.inf, dtype=np.float64)
    P = np.zeros((B, H, N, N), dtype=np.float64) if return_p else None
    for b in range(B):
        n = int(min(max(int(seq_lens[b]), 0), N))
        for h in range(H):
            for r0 in range(0, n, row_block):
                rows = np.arange(r0, min(n, r0 + row_block))
                ob, lb, pb = _rows_one_head(q[b, h], k[b, h], v[b, h], rows, n,
                                            scale, left, right, return_p,
                                            None if key_bias is None else key_bias[b])
                o[b, h, rows] = ob
                lse[b, h, rows] = lb
                if return_p:
                    P[b, h, rows] = pb
    if return_p:
        return o, lse, P
    return o, lse


def attention_oracle_rows(q, k, v, b, h, rows, n_valid, scale=1.0, left=-1, right=-1, key_bias=None):
    """Oracle for selected query rows of one (b, h): used to sample large configs.
    key_bias: None or [B, N].

    q, k, v: [B, H, N, D] in any float dtype; only the (b, h) slice is converted.
    rows must all be < n_valid.  Returns (o [len(rows), D], lse [len(rows)]).
    """
    qh = np.asarray(q[b, h], dtype=np.float64)
    kh = np.asarray(k[b, h], dtype=np.float64)
    vh = np.asarray(v[b, h], dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    if rows.size and (rows.min() < 0 or rows.max() >= n_valid):
        raise ValueError("sampled rows must be valid query rows")
    kb = None if key_bias is None else np.asarray(key_bias, dtype=np.float64)[b]
    o, lse, _ = _rows_one_head(qh, kh, vh, rows, int(n_valid), scale, left, right, False, kb)
    return o, lse


def additive_bias_variant(q, k, v, seq_lens, scale=1.0, bias_value=-65504.0):
    """The paper's literal mask form for global layers (Eq. 1): scores get
    pad_bias[j] = bias_value * (1 - attention_mask[j]) added, then an ordinary
    softmax over ALL N keys.  Only valid query rows are returned meaningful;
    padded query rows are left at o = 0, lse = -inf to match `attention_oracle`.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, H, N, D = q.shape
    o = np.zeros((B, H, N, D), dtype=np.float64)
    lse = np.full((B, H, N), -np.inf, dtype=np.float64)
    for b in range(B):
        n = int(min(max(int(seq_lens[b]), 0), N))
        attention_mask = (np.arange(N) < n).astype(np.float64)
        pad_bias = bias_value * (1.0 - attention_mask)
        for h in range(H):
            s = (q[b, h, :n] @ k[b, h].T) * scale + pad_bias[None, :]
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            l = e.sum(axis=1, keepdims=True)
            o[b, h, :n] = (e / l) @ v[b, h]
            lse[b, h, :n] = (m + np.log(l))[:, 0]
    return o, lse
