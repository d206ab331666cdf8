"""Pins for the fp64 oracle (no GPU).  Each test fixes the oracle to something
other than itself: a brute-force scalar loop written here, a library routine on
a special case, a closed form, or an invariant of softmax attention
(paper Sec. 2.2 definition; Sec. 4.1.3 operator attributes; Eq. 1 mask)."""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle.attention_oracle import (additive_bias_variant, attention_oracle,
                                     attention_oracle_rows, visible_mask,
                                     window_from_width)


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# --------------------------------------------------------------------------
# brute force: pure-Python floats, written from the definition, no numpy math
# --------------------------------------------------------------------------
def brute(q, k, v, lens, scale, left, right, bias=None):
    B, H, N, D = q.shape
    o = [[[[0.0] * D for _ in range(N)] for _ in range(H)] for _ in range(B)]
    lse = [[[-math.inf] * N for _ in range(H)] for _ in range(B)]
    for b in range(B):
        n = max(0, min(int(lens[b]), N))
        for h in range(H):
            for i in range(n):
                terms = []
                for j in range(n):
                    if left >= 0 and j < i - left:
                        continue
                    if right >= 0 and j > i + right:
                        continue
                    dot = 0.0
                    for d in range(D):
                        dot += float(q[b, h, i, d]) * float(k[b, h, j, d])
                    extra = 0.0 if bias is None else float(bias[b][j])
                    if extra == -math.inf:
                        continue
                    terms.append((j, scale * dot + extra))
                if not terms:
                    continue
                big = max(t for _, t in terms)
                z = sum(math.exp(t - big) for _, t in terms)
                for j, t in terms:
                    w = math.exp(t - big) / z
                    for d in range(D):
                        o[b][h][i][d] += w * float(v[b, h, j, d])
                lse[b][h][i] = big + math.log(z)
    return np.array(o), np.array(lse)


@pytest.mark.parametrize("left,right", [(-1, -1), (0, 0), (1, 0), (0, 1), (1, 2), (2, 1), (3, 3), (7, 7), (20, 20), (-1, 1), (2, -1)])
@pytest.mark.parametrize("lens", [(7, 5), (1, 0), (8, 8), (3, 8)])
def test_brute_force_tiny(left, right, lens):
    B, H, N, D = 2, 2, 8, 4
    q, k, v = rand((B, H, N, D), 1), rand((B, H, N, D), 2), rand((B, H, N, D), 3)
    scale = 0.37
    o, lse = attention_oracle(q, k, v, lens, scale, left, right, row_block=3)
    ob, lb = brute(q, k, v, lens, scale, left, right)
    assert np.allclose(o, ob, rtol=0, atol=1e-12)
    fin = np.isfinite(lb)
    assert np.array_equal(fin, np.isfinite(lse))
    assert np.allclose(lse[fin], lb[fin], rtol=0, atol=1e-12)
    assert np.all(lse[~fin] == -np.inf)


def test_rows_api_matches_full():
    B, H, N, D = 2, 3, 37, 8
    q, k, v = rand((B, H, N, D), 4), rand((B, H, N, D), 5), rand((B, H, N, D), 6)
    lens = (30, 37)
    o, lse = attention_oracle(q, k, v, lens, 0.5, 4, 5)
    rows = [0, 3, 17, 29]
    orow, lrow = attention_oracle_rows(q, k, v, 0, 1, rows, 30, 0.5, 4, 5)
    assert np.array_equal(orow, o[0, 1, rows])
    assert np.array_equal(lrow, lse[0, 1, rows])
    with pytest.raises(ValueError):
        attention_oracle_rows(q, k, v, 0, 1, [30], 30, 0.5, 4, 5)


# --------------------------------------------------------------------------
# library special cases
# --------------------------------------------------------------------------
def test_global_unpadded_equals_scipy():
    B, H, N, D = 1, 2, 50, 16
    q, k, v = rand((B, H, N, D), 7), rand((B, H, N, D), 8), rand((B, H, N, D), 9)
    scale = 1 / math.sqrt(D)
    o, lse = attention_oracle(q, k, v, None, scale)
    for h in range(H):
        s = scale * q[0, h] @ k[0, h].T
        ref = scipy.special.softmax(s, axis=-1) @ v[0, h]
        assert np.allclose(o[0, h], ref, rtol=0, atol=1e-13)
        assert np.allclose(lse[0, h], scipy.special.logsumexp(s, axis=-1), rtol=0, atol=1e-13)


@pytest.mark.parametrize("left,right,n", [(-1, -1, 33), (5, 6, 40), (63, 64, 200), (0, 3, 17)])
def test_torch_sdpa_boolean_mask(left, right, n):
    B, H, N, D = 1, 2, 200, 8
    n = min(n, N)
    q, k, v = rand((B, H, N, D), 10), rand((B, H, N, D), 11), rand((B, H, N, D), 12)
    scale = 0.3
    o, _ = attention_oracle(q, k, v, (n,), scale, left, right)
    i = torch.arange(N)[:, None]
    j = torch.arange(N)[None, :]
    mask = (j < n).expand(N, N).clone()
    if left >= 0:
        mask &= j >= i - left
    if right >= 0:
        mask &= j <= i + right
    mask[n:, :] = True  # padded query rows: keep SDPA finite, they are not compared
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q), torch.from_numpy(k), torch.from_numpy(v),
        attn_mask=mask, scale=scale).numpy()
    assert np.allclose(o[0, :, :n], ref[0, :, :n], rtol=0, atol=1e-12)
    assert np.all(o[0, :, n:] == 0)


# --------------------------------------------------------------------------
# closed forms
# --------------------------------------------------------------------------
@pytest.mark.parametrize("n,N", [(300, 300), (260, 300)])
def test_zero_q_counts_visible_keys_paper_window(n, N):
    """Q = 0: o = mean of visible V rows and lse = ln(#visible).  With the local
    layer's (63, 64) an interior row sees exactly 128 keys, row 0 sees 65 and the
    last valid row sees 64 (Sec. 4.1.3 window values)."""
    H, D = 1, 4
    q = np.zeros((1, H, N, D))
    k, v = rand((1, H, N, D), 13), rand((1, H, N, D), 14)
    L, R = window_from_width(128)
    assert (L, R) == (63, 64)
    o, lse = attention_oracle(q, k, v, (n,), 0.7, L, R)
    count = np.exp(lse[0, 0, :n])
    expect = np.array([min(n - 1, i + R) - max(0, i - L) + 1 for i in range(n)], dtype=float)
    assert np.allclose(count, expect, rtol=1e-12)
    assert round(count[0]) == 65 and round(count[n - 1]) == 64 and round(count[100]) == 128
    for i in (0, 1, 100, n - 1):
        lo, hi = max(0, i - L), min(n - 1, i + R)
        assert np.allclose(o[0, 0, i], v[0, 0, lo:hi + 1].mean(axis=0), atol=1e-13)
    assert np.all(np.isneginf(lse[0, 0, n:])) and np.all(o[0, 0, n:] == 0)


def test_window_from_width_mapping():
    assert window_from_width(-1) == (-1, -1)
    assert window_from_width(-7) == (-1, -1)
    assert window_from_width(1) == (0, 0)
    assert window_from_width(2) == (0, 1)
    assert window_from_width(3) == (1, 1)
    assert window_from_width(128) == (63, 64)
    for W in range(1, 40):
        L, R = window_from_width(W)
        assert L + R + 1 == W
    with pytest.raises(ValueError):
        window_from_width(0)


def test_self_only_window():
    """L = R = 0: each query sees only itself: o[i] = V[i], lse[i] = scale q_i.k_i."""
    B, H, N, D = 1, 2, 19, 8
    q, k, v = rand((B, H, N, D), 15), rand((B, H, N, D), 16), rand((B, H, N, D), 17)
    o, lse = attention_oracle(q, k, v, (15,), 0.9, 0, 0)
    assert np.allclose(o[0, :, :15], v[0, :, :15], atol=1e-15)
    assert np.allclose(lse[0, :, :15], 0.9 * np.einsum("hnd,hnd->hn", q[0], k[0])[:, :15], atol=1e-13)


def test_wide_window_equals_global():
    B, H, N, D = 1, 1, 40, 8
    q, k, v = rand((B, H, N, D), 18), rand((B, H, N, D), 19), rand((B, H, N, D), 20)
    a = attention_oracle(q, k, v, (33,), 0.4, -1, -1)
    b = attention_oracle(q, k, v, (33,), 0.4, *window_from_width(2 * N))
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_one_hot_limit():
    """A huge scale makes the softmax pick the best-matching key."""
    N, D = 12, 6
    k = rand((1, 1, N, D), 21)
    v = rand((1, 1, N, D), 22)
    q = k.copy()[:, :, ::-1].copy()  # query i matches key N-1-i best (|k|^2 dominates)
    s = np.einsum("id,jd->ij", q[0, 0], k[0, 0])
    best = s.argmax(axis=1)
    o, lse = attention_oracle(q, k, v, None, 1e4)
    assert np.allclose(o[0, 0], v[0, 0, best], atol=1e-9)
    assert np.allclose(lse[0, 0], 1e4 * s.max(axis=1), rtol=1e-12)


def test_zero_scale_uniform():
    N, D = 9, 3
    q, k, v = rand((1, 1, N, D), 23), rand((1, 1, N, D), 24), rand((1, 1, N, D), 25)
    o, lse = attention_oracle(q, k, v, (7,), 0.0)
    assert np.allclose(o[0, 0, :7], np.broadcast_to(v[0, 0, :7].mean(axis=0), (7, D)), atol=1e-15)
    assert np.allclose(lse[0, 0, :7], math.log(7))


def test_transposed_operand_would_fail():
    """Known answer that separates Q.K^T from K.Q^T-style index mistakes:
    with K = one-hot rows, scores are columns of Q."""
    N, D = 4, 4
    q = np.arange(16, dtype=float).reshape(1, 1, N, D) / 10
    k = np.eye(4).reshape(1, 1, N, D)
    v = np.diag([1.0, 2.0, 3.0, 4.0]).reshape(1, 1, N, D)
    o, lse = attention_oracle(q, k, v, None, 1.0)
    for i in range(N):
        w = np.exp(q[0, 0, i]) / np.exp(q[0, 0, i]).sum()  # s_ij = q[i, j]
        assert np.allclose(o[0, 0, i], w * np.array([1, 2, 3, 4.0]), atol=1e-15)
        assert np.isclose(lse[0, 0, i], math.log(np.exp(q[0, 0, i]).sum()))


# --------------------------------------------------------------------------
# invariants
# --------------------------------------------------------------------------
def test_rows_of_p_sum_to_one_and_respect_mask():
    B, H, N, D = 2, 2, 23, 5
    q, k, v = rand((B, H, N, D), 26), rand((B, H, N, D), 27), rand((B, H, N, D), 28)
    lens = (23, 14)
    o, lse, P = attention_oracle(q, k, v, lens, 0.6, 3, 2, return_p=True)
    for b in range(B):
        n = lens[b]
        assert np.allclose(P[b, :, :n].sum(axis=-1), 1.0, atol=1e-14)
        vis = visible_mask(np.arange(n), N, n, 3, 2)
        assert np.all(P[b, :, :n][:, ~vis] == 0)
        assert np.all(P[b, :, :n][:, vis] > 0)
        assert np.all(P[b, :, n:] == 0)


def test_constant_v_gives_constant_output():
    B, H, N, D = 1, 2, 31, 4
    q, k = rand((B, H, N, D), 29), rand((B, H, N, D), 30)
    v = np.full((B, H, N, D), 2.5)
    v[..., 1] = -7.0
    o, _ = attention_oracle(q, k, v, (29,), 0.8, 5, 4)
    assert np.allclose(o[0, :, :29, 0], 2.5, atol=1e-15)
    assert np.allclose(o[0, :, :29, 1], -7.0, atol=1e-14)


def test_key_value_permutation_invariance_global():
    B, H, N, D = 1, 2, 27, 6
    q, k, v = rand((B, H, N, D), 31), rand((B, H, N, D), 32), rand((B, H, N, D), 33)
    perm = np.random.default_rng(0).permutation(N)
    a = attention_oracle(q, k, v, None, 0.5)
    b = attention_oracle(q, k[:, :, perm], v[:, :, perm], None, 0.5)
    assert np.allclose(a[0], b[0], atol=1e-14)
    assert np.allclose(a[1], b[1], atol=1e-14)


def test_masked_keys_have_no_effect_even_nan():
    B, H, N, D = 1, 2, 40, 4
    q, k, v = rand((B, H, N, D), 34), rand((B, H, N, D), 35), rand((B, H, N, D), 36)
    n = 25
    a = attention_oracle(q, k, v, (n,), 0.5, 6, 6)
    k2, v2, q2 = k.copy(), v.copy(), q.copy()
    k2[:, :, n:] = np.nan
    v2[:, :, n:] = np.inf
    q2[:, :, n:] = 1e300
    b = attention_oracle(q2, k2, v2, (n,), 0.5, 6, 6)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    # out-of-window but valid keys: changing them by a finite amount has no effect either
    k3, v3 = k.copy(), v.copy()
    k3[:, :, 0] = 1e3
    v3[:, :, 0] = -1e3
    c = attention_oracle(q, k3, v3, (n,), 0.5, 6, 6)
    assert np.array_equal(a[0][:, :, 7:n], c[0][:, :, 7:n])


def test_key_shift_identity():
    """Adding a vector c to every key leaves o unchanged and adds scale*q_i.c to lse."""
    B, H, N, D = 1, 1, 21, 5
    q, k, v = rand((B, H, N, D), 37), rand((B, H, N, D), 38), rand((B, H, N, D), 39)
    c = rand((D,), 40)
    a = attention_oracle(q, k, v, (18,), 0.45, 4, 9)
    b = attention_oracle(q, k + c, v, (18,), 0.45, 4, 9)
    assert np.allclose(a[0], b[0], atol=1e-13)
    assert np.allclose(b[1][0, 0, :18] - a[1][0, 0, :18], 0.45 * q[0, 0, :18] @ c, atol=1e-13)


def test_split_merge_identity():
    """Attention over keys A u B from the two partial results and their lse:
    the identity that makes tiled (flash) evaluation exact (Sec. 2.2)."""
    H, N, D = 2, 30, 6
    q, k, v = rand((1, H, N, D), 41), rand((1, H, N, D), 42), rand((1, H, N, D), 43)
    full_o, full_lse = attention_oracle(q, k, v, None, 0.5)
    cut = 11
    # the oracle is square (n queries, n keys): put each query in row 0 of a
    # problem whose keys are the chosen subset.
    def partial(ks, vs, nkeys):
        Nk = ks.shape[2]
        outs, lses = [], []
        for i in range(N):
            qq = np.zeros((1, H, Nk, D)); qq[:, :, 0] = q[:, :, i]
            # query row 0 with unbounded window over nkeys valid keys
            o_, l_ = attention_oracle(qq, ks, vs, (nkeys,), 0.5)
            outs.append(o_[0, :, 0]); lses.append(l_[0, :, 0])
        return np.stack(outs, 1), np.stack(lses, 1)
    oA, lA = partial(k, v, cut)
    oB, lB = partial(k[:, :, cut:], v[:, :, cut:], N - cut)
    wA, wB = np.exp(lA), np.exp(lB)
    merged = (wA[..., None] * oA + wB[..., None] * oB) / (wA + wB)[..., None]
    assert np.allclose(merged, full_o[0], atol=1e-13)
    assert np.allclose(np.log(wA + wB), full_lse[0], atol=1e-13)


def test_additive_bias_reading_equals_exclusion():
    """Eq. 1's finite bias (-65504 on padded keys) and true exclusion agree to
    rounding on every valid row at the workloads' score magnitudes."""
    B, H, N, D = 2, 2, 48, 8
    q, k, v = rand((B, H, N, D), 44), rand((B, H, N, D), 45), rand((B, H, N, D), 46)
    lens = (48, 31)
    a = attention_oracle(q, k, v, lens, 0.35)
    b = additive_bias_variant(q, k, v, lens, 0.35)
    assert np.allclose(a[0], b[0], rtol=0, atol=1e-15)
    assert np.allclose(a[1], b[1], rtol=0, atol=1e-13)


def test_seq_len_clamping_and_empty():
    B, H, N, D = 3, 1, 6, 2
    q, k, v = rand((B, H, N, D), 47), rand((B, H, N, D), 48), rand((B, H, N, D), 49)
    o, lse = attention_oracle(q, k, v, (0, -3, 99), 1.0)
    assert np.all(o[:2] == 0) and np.all(np.isneginf(lse[:2]))
    o_full, lse_full = attention_oracle(q[2:], k[2:], v[2:], None, 1.0)
    assert np.array_equal(o[2], o_full[0]) and np.array_equal(lse[2], lse_full[0])


# --------------------------------------------------------------------------
# additive 1-D key bias (the operator's pad_bias input, Sec. 4.1.3 / Eq. 1)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("left,right,lens", [(-1, -1, (7, 5)), (1, 2, (8, 3)), (0, 0, (8, 8)), (2, -1, (1, 6))])
def test_key_bias_brute_force(left, right, lens):
    B, H, N, D = 2, 2, 8, 4
    q, k, v = rand((B, H, N, D), 31), rand((B, H, N, D), 32), rand((B, H, N, D), 33)
    bias = rand((B, N), 34) * 2.0
    bias[0, 2] = -math.inf          # a masked key in the middle of the sequence
    bias[1, 0] = -65504.0
    o, lse = attention_oracle(q, k, v, lens, 0.41, left, right, row_block=3, key_bias=bias)
    ob, lb = brute(q, k, v, lens, 0.41, left, right, bias)
    fin = np.isfinite(lb)
    assert np.allclose(o, ob, rtol=0, atol=1e-12)
    assert np.array_equal(fin, np.isfinite(lse)) and np.allclose(lse[fin], lb[fin], rtol=0, atol=1e-12)


def test_rows_api_key_bias_brute_force():
    """The sampled-rows entry point with a bias: every batch element has its own bias row,
    and the rows it returns are pinned to the scalar loop (not to the full oracle), for the
    second batch element as well as the first."""
    B, H, N, D = 3, 2, 9, 4
    q, k, v = rand((B, H, N, D), 41), rand((B, H, N, D), 42), rand((B, H, N, D), 43)
    bias = rand((B, N), 44) * 2.0
    bias[1, 3] = -math.inf
    bias[2, 0] = -65504.0
    lens = (9, 7, 5)
    ob, lb = brute(q, k, v, lens, 0.37, 2, 3, bias)
    for b in range(B):
        rows = list(range(lens[b]))
        for h in range(H):
            orow, lrow = attention_oracle_rows(q, k, v, b, h, rows, lens[b], 0.37, 2, 3, key_bias=bias)
            assert np.allclose(orow, ob[b, h, rows], rtol=0, atol=1e-12), (b, h)
            assert np.allclose(lrow, lb[b, h, rows], rtol=0, atol=1e-12), (b, h)


def test_key_bias_log_weight_equals_repeated_keys():
    """bias_j = ln(w_j) with integer w_j is attention over a sequence in which key j (and
    its value) appears w_j times: fixes the sign of the bias and that scale does not touch it."""
    H, N, D = 2, 6, 4
    q, k, v = rand((1, H, N, D), 35), rand((1, H, N, D), 36), rand((1, H, N, D), 37)
    w = np.array([1, 3, 2, 1, 4, 2])
    o, lse = attention_oracle(q, k, v, None, 0.7, key_bias=np.log(w)[None, :])
    idx = np.repeat(np.arange(N), w)
    M = len(idx)
    q2 = np.zeros((1, H, M, D)); q2[:, :, :N] = q
    o2, lse2 = attention_oracle(q2, k[:, :, idx], v[:, :, idx], None, 0.7)
    assert np.allclose(o, o2[:, :, :N], rtol=0, atol=1e-13)
    assert np.allclose(lse, lse2[:, :, :N], rtol=0, atol=1e-13)


def test_key_bias_constant_shifts_lse_only():
    B, H, N, D = 2, 2, 9, 4
    q, k, v = rand((B, H, N, D), 38), rand((B, H, N, D), 39), rand((B, H, N, D), 40)
    lens = (9, 6)
    o0, l0 = attention_oracle(q, k, v, lens, 0.3, 2, 3)
    o1, l1 = attention_oracle(q, k, v, lens, 0.3, 2, 3, key_bias=np.full((B, N), 1.25))
    fin = np.isfinite(l0)
    assert np.allclose(o0, o1, rtol=0, atol=1e-13)
    assert np.allclose(l1[fin], l0[fin] + 1.25, rtol=0, atol=1e-13) and np.all(l1[~fin] == -np.inf)


def test_key_bias_minus_inf_removes_the_key():
    """A non-tail key mask: -inf on keys {1, 4} equals attention over the remaining keys."""
    H, N, D = 2, 7, 4
    q, k, v = rand((1, H, N, D), 41), rand((1, H, N, D), 42), rand((1, H, N, D), 43)
    bias = np.zeros((1, N)); bias[0, [1, 4]] = -np.inf
    o, lse = attention_oracle(q, k, v, None, 0.9, key_bias=bias)
    keep = [0, 2, 3, 5, 6]
    for h in range(H):
        sc = 0.9 * q[0, h] @ k[0, h, keep].T
        p = scipy.special.softmax(sc, axis=1)
        assert np.allclose(o[0, h], p @ v[0, h, keep], rtol=0, atol=1e-13)
        assert np.allclose(lse[0, h], scipy.special.logsumexp(sc, axis=1), rtol=0, atol=1e-13)
    # every key masked: same convention as a row with no visible key
    o2, lse2 = attention_oracle(q, k, v, None, 0.9, key_bias=np.full((1, N), -np.inf))
    assert np.all(o2 == 0) and np.all(lse2 == -np.inf)


def test_key_bias_literal_eq1_form():
    """-65504 on the padded tail with every key 'valid' is the literal Eq. 1 computation."""
    B, H, N, D = 2, 2, 10, 4
    q, k, v = rand((B, H, N, D), 44), rand((B, H, N, D), 45), rand((B, H, N, D), 46)
    lens = (10, 6)
    bias = np.where(np.arange(N)[None, :] < np.array(lens)[:, None], 0.0, -65504.0)
    o, lse = attention_oracle(q, k, v, None, 0.5, key_bias=bias)
    ov, lv = additive_bias_variant(q, k, v, lens, 0.5)
    for b, n in enumerate(lens):
        assert np.allclose(o[b, :, :n], ov[b, :, :n], rtol=0, atol=1e-13)
        assert np.allclose(lse[b, :, :n], lv[b, :, :n], rtol=0, atol=1e-13)
