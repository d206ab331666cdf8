"""GPU parity: the HIP flash-attention forward, called through the C boundary,
against the fp64 oracle on the same seeded inputs.

Tolerances (valid rows, against the unrounded fp64 oracle): fp16 max-abs <= 2e-3
and mean-abs <= 2e-4; bf16 max-abs <= 1e-2 and mean-abs <= 1e-3; logsumexp
within 1e-3.  Edge-case tests whose outputs can exceed 1 in magnitude (self-only
windows, one-hot softmax) scale the error by max(1, |reference|), because a
16-bit result cannot be closer than half an ulp of its own magnitude."""
import numpy as np
import pytest
import torch

import paper_2603_12646_amd as fa
from oracle.attention_oracle import attention_oracle, attention_oracle_rows, window_from_width
from workloads import ALL_CONFIGS, CONFIGS, draw, make_inputs, round_to_storage

from tests.gpu_util import (FA_DT, LSE_TOL, TOL, check_against, poison, run_ex, run_simple, to_dev)

pytestmark = pytest.mark.gpu

TUNINGS = {
    "auto": 0,
    "bm128_tr": fa.FA_TUNE_BM_128 | fa.FA_TUNE_V_LDS_TRANSPOSE | fa.FA_TUNE_MAP_LINEAR,
    "bm256_tr": fa.FA_TUNE_BM_256 | fa.FA_TUNE_V_LDS_TRANSPOSE | fa.FA_TUNE_MAP_LINEAR,
    "bm128_scalar_xcd": fa.FA_TUNE_BM_128 | fa.FA_TUNE_V_SCALAR | fa.FA_TUNE_MAP_XCD,
    "bm256_scalar_xcd": fa.FA_TUNE_BM_256 | fa.FA_TUNE_V_SCALAR | fa.FA_TUNE_MAP_XCD,
    "bm32_linear": fa.FA_TUNE_BM_32 | fa.FA_TUNE_MAP_LINEAR,
    "bm32_xcd": fa.FA_TUNE_BM_32 | fa.FA_TUNE_MAP_XCD,
    "bm384_linear": fa.FA_TUNE_BM_384 | fa.FA_TUNE_MAP_LINEAR,
    "bm512_xcd": fa.FA_TUNE_BM_512 | fa.FA_TUNE_MAP_XCD,
    "win_pipelined": fa.FA_TUNE_WIN_PIPELINED,
    "win_two_phase": fa.FA_TUNE_WIN_TWO_PHASE,
    "win_two_phase_linear": fa.FA_TUNE_WIN_TWO_PHASE | fa.FA_TUNE_MAP_LINEAR,
    "mixed_linear": fa.FA_TUNE_BM_MIXED | fa.FA_TUNE_MAP_LINEAR,
    "mixed_xcd": fa.FA_TUNE_BM_MIXED | fa.FA_TUNE_MAP_XCD,
}
# Small global calls take the key-split kernel by themselves (at most 256 blocks of 32 query
# rows, more than 128 tokens); the small-shape tests below therefore run three times: the
# library's choice, the pipelined kernel forced, the key-split kernel forced; and with the
# 12- and 8-wavefront shapes of the pipelined kernel (384 and 512 rows per workgroup).
GLOBAL_KERNELS = {"auto": 0, "bm128": fa.FA_TUNE_BM_128, "bm32": fa.FA_TUNE_BM_32,
                  "bm384": fa.FA_TUNE_BM_384, "bm512": fa.FA_TUNE_BM_512, "mixed": fa.FA_TUNE_BM_MIXED}


# ------------------------------------------------------------------ small shapes, full compare
@pytest.mark.parametrize("tuning", sorted(TUNINGS))
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("left,right", [(-1, -1), (63, 64), (0, 0), (3, 3), (0, 5), (70, -1), (-1, 9), (200, 130)])
def test_small_ragged_all_windows(dtype, left, right, tuning):
    """Several 64-key tiles plus a ragged tail (333 = 5*64 + 13), two lengths, padding
    in the middle of a tile, every window form."""
    B, H, N, D = 2, 3, 333, 64
    _, q, k, v = draw(100, B, H, N, D, dtype)
    lens = [333, 201]
    o_ref, lse_ref = attention_oracle(q, k, v, lens, 0.125, left, right)
    o, lse = run_ex(q, k, v, lens, dtype, 0.125, left, right, TUNINGS[tuning])
    check_against(o, lse, o_ref, lse_ref, lens, dtype, relative=True, label=f"{dtype} {left},{right} {tuning}")


@pytest.mark.parametrize("kern", sorted(GLOBAL_KERNELS))
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("N", [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 257, 640])
def test_lengths_around_tile_edges(dtype, N, kern):
    B, H, D = 1, 2, 64
    _, q, k, v = draw(200 + N, B, H, N, D, dtype)
    for window in ((-1, 128, 2) if kern == "auto" else (-1,)):
        L, R = window_from_width(window)
        o_ref, lse_ref = attention_oracle(q, k, v, None, 0.125, L, R)
        o, lse = run_simple(q, k, v, None, dtype, 0.125, window, tuning=GLOBAL_KERNELS[kern])
        check_against(o, lse, o_ref, lse_ref, None, dtype, relative=True, label=f"N={N} w={window} {kern}")


@pytest.mark.parametrize("kern", sorted(GLOBAL_KERNELS))
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_seq_lens_degenerate_values(dtype, kern):
    """n_b = 0, negative, above max_len (clamped), 1, and exactly a tile edge."""
    B, H, N, D = 6, 2, 192, 64
    _, q, k, v = draw(300, B, H, N, D, dtype)
    lens = [0, -5, 1000, 1, 128, 191]
    for window in ((-1, 128) if kern == "auto" else (-1,)):
        L, R = window_from_width(window)
        o_ref, lse_ref = attention_oracle(q, k, v, lens, 0.125, L, R)
        o, lse = run_simple(q, k, v, lens, dtype, 0.125, window, tuning=GLOBAL_KERNELS[kern])
        check_against(o, lse, o_ref, lse_ref, lens, dtype, relative=True, label=f"w={window} {kern}")


WINDOW_KERNELS = {"pipelined": fa.FA_TUNE_WIN_PIPELINED, "two_phase": fa.FA_TUNE_WIN_TWO_PHASE}


@pytest.mark.parametrize("kern", sorted(WINDOW_KERNELS))
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("D", [32, 64, 128])
def test_window_kernels_tile_edges_degenerate_lengths_and_garbage_padding(D, dtype, kern):
    """Both families of window kernels (small calls take the pipelined ones by themselves) on the
    paper's 63/64 window and two narrower ones: lengths around tile edges, degenerate sequence
    lengths, and NaN / inf in the padded rows (valid rows must not change by a bit)."""
    tun = WINDOW_KERNELS[kern]
    scale = 1.0 / np.sqrt(D)
    for N in (1, 31, 33, 64, 65, 127, 129, 257, 640):
        _, q, k, v = draw(250 + N, 1, 2, N, D, dtype)
        for left, right in ((63, 64), (0, 0), (31, 32)):
            o_ref, lse_ref = attention_oracle(q, k, v, None, scale, left, right)
            o, lse = run_ex(q, k, v, None, dtype, scale, left, right, tuning=tun)
            check_against(o, lse, o_ref, lse_ref, None, dtype, relative=True, label=f"N={N} ({left},{right}) D{D} {kern}")
    B, H, N = 6, 2, 192
    _, q, k, v = draw(350, B, H, N, D, dtype)
    lens = [0, -5, 1000, 1, 128, 191]
    o_ref, lse_ref = attention_oracle(q, k, v, lens, scale, 63, 64)
    o, lse = run_ex(q, k, v, lens, dtype, scale, 63, 64, tuning=tun)
    check_against(o, lse, o_ref, lse_ref, lens, dtype, relative=True, label=f"degenerate D{D} {kern}")
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for b, n in enumerate(lens):
        n = min(max(n, 0), N)
        q2[b, :, n:] = np.inf
        k2[b, :, n:] = np.nan
        v2[b, :, n:] = -np.inf
    o2, lse2 = run_ex(q2, k2, v2, lens, dtype, scale, 63, 64, tuning=tun)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)


@pytest.mark.parametrize("kern", sorted(GLOBAL_KERNELS))
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_padded_rows_may_hold_anything(dtype, kern):
    """NaN / inf / huge values in padded Q, K, V rows leave valid rows bit-identical."""
    B, H, N, D = 2, 2, 300, 64
    _, q, k, v = draw(301, B, H, N, D, dtype)
    lens = [170, 255]
    tun = GLOBAL_KERNELS[kern]
    for window in ((-1, 128) if kern == "auto" else (-1,)):
        a_o, a_lse = run_simple(q, k, v, lens, dtype, 0.125, window, tuning=tun)
        q2, k2, v2 = q.copy(), k.copy(), v.copy()
        for b, n in enumerate(lens):
            q2[b, :, n:] = np.inf
            k2[b, :, n:] = np.nan
            v2[b, :, n:] = np.nan
            v2[b, :, n::2] = -np.inf
        b_o, b_lse = run_simple(q2, k2, v2, lens, dtype, 0.125, window, tuning=tun)
        assert np.array_equal(a_o, b_o) and np.array_equal(a_lse, b_lse)
        L, R = window_from_width(window)
        o_ref, lse_ref = attention_oracle(q, k, v, lens, 0.125, L, R)
        check_against(b_o, b_lse, o_ref, lse_ref, lens, dtype, label=f"poisoned w={window}")


@pytest.mark.parametrize("kern", sorted(GLOBAL_KERNELS))
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("scale", [0.0, -0.125, 1.0, 0.3, 8.0])
def test_scales(dtype, scale, kern):
    """scale = 0 (uniform attention), negative, not a power of two, and large
    (near one-hot softmax, running maximum far from zero)."""
    B, H, N, D = 1, 2, 200, 64
    _, q, k, v = draw(302, B, H, N, D, dtype)
    lens = [187]
    o_ref, lse_ref = attention_oracle(q, k, v, lens, scale)
    o, lse = run_simple(q, k, v, lens, dtype, scale, tuning=GLOBAL_KERNELS[kern])
    check_against(o, lse, o_ref, lse_ref, lens, dtype, relative=True, label=f"scale={scale} {kern}")


@pytest.mark.parametrize("kern", sorted(GLOBAL_KERNELS))
def test_increasing_scores_force_many_rescales(kern):
    """Keys ordered so every tile's maximum beats the previous one by a wide margin:
    the reference maximum must be refreshed tile after tile."""
    tun = GLOBAL_KERNELS[kern]
    N, D = 512, 64
    rng = np.random.default_rng(7)
    q = np.zeros((1, 1, N, D), np.float32); q[..., 0] = 1.0
    k = np.zeros((1, 1, N, D), np.float32); k[0, 0, :, 0] = np.arange(N) * 0.25
    v0 = rng.standard_normal((1, 1, N, D)).astype(np.float32)
    k0 = k
    for dtype in ("fp16", "bf16"):
        k, v = round_to_storage(k0, dtype), round_to_storage(v0, dtype)
        o_ref, lse_ref = attention_oracle(q, k, v, None, 1.0)
        o, lse = run_simple(q, k, v, None, dtype, 1.0, tuning=tun)
        check_against(o, lse, o_ref, lse_ref, None, dtype, relative=True, label="ramp")
        o_ref, lse_ref = attention_oracle(q, k[:, :, ::-1].copy(), v, None, 1.0)
        o, lse = run_simple(q, k[:, :, ::-1].copy(), v, None, dtype, 1.0, tuning=tun)
        check_against(o, lse, o_ref, lse_ref, None, dtype, relative=True, label="ramp down")
        # steeper ramps: a block's probabilities against the stale reference overflow the
        # storage type (scale 8) and even fp32 (scale 40) before the refresh catches them
        for scale in (8.0, 40.0):
            o_ref, lse_ref = attention_oracle(q, k, v, None, scale)
            o, lse = run_simple(q, k, v, None, dtype, scale, tuning=tun)
            check_against(o, lse, o_ref, lse_ref, None, dtype, relative=True, label=f"steep ramp {scale}")


def test_constant_v_and_zero_q_closed_forms():
    """Q = 0: lse = ln(#visible keys) pins the window edges on the GPU as well."""
    N, D = 400, 64
    _, q, k, v = draw(303, 1, 1, N, D, "fp16")
    q0 = np.zeros_like(q)
    o, lse = run_simple(q0, k, v, [390], "fp16", 0.125, 128)
    count = np.exp(lse[0, 0, :390])
    expect = np.array([min(389, i + 64) - max(0, i - 63) + 1 for i in range(390)], float)
    assert np.allclose(count, expect, rtol=1e-5)
    vc = np.full_like(v, 0.75)
    o, _ = run_simple(q, k, vc, [390], "fp16", 0.125, -1)
    assert np.allclose(o[0, 0, :390], 0.75, atol=1e-3)


def test_lse_null_and_other_stream_and_determinism():
    B, H, N, D = 2, 2, 260, 64
    _, q, k, v = draw(304, B, H, N, D, "fp16")
    lens = [260, 100]
    o1, lse1 = run_simple(q, k, v, lens, "fp16", 0.125, -1)
    o2, none = run_simple(q, k, v, lens, "fp16", 0.125, -1, want_lse=False)
    assert none is None and np.array_equal(o1, o2)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        o3, lse3 = run_simple(q, k, v, lens, "fp16", 0.125, -1, stream=s)
    assert np.array_equal(o1, o3) and np.array_equal(lse1, lse3)
    for _ in range(3):
        o4, lse4 = run_simple(q, k, v, lens, "fp16", 0.125, -1)
        assert np.array_equal(o1, o4) and np.array_equal(lse1, lse4)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_strided_inputs_bshd_and_packed_qkv(dtype):
    """[batch, len, 3, heads, dim] packed QKV read in place, output written as
    [batch, len, heads, dim]."""
    B, H, N, D = 2, 3, 150, 64
    _, q, k, v = draw(305, B, H, N, D, dtype)
    lens = [150, 99]
    o_ref, lse_ref = attention_oracle(q, k, v, lens, 0.125, 10, 20)
    packed = np.stack([q, k, v], axis=0).transpose(1, 3, 0, 2, 4).copy()  # B, N, 3, H, D
    dev = to_dev(packed, dtype)
    o = poison((B, N, H, D), dtype)
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    sl = torch.tensor(lens, dtype=torch.int32).cuda()
    st = (N * 3 * H * D, D, 3 * H * D)
    fa.fa_fwd_ex(dtype=FA_DT[dtype], q=dev[:, :, 0].data_ptr(), k=dev[:, :, 1].data_ptr(),
                 v=dev[:, :, 2].data_ptr(), o=o, lse=lse, seq_lens=sl, batch=B, heads=H, max_len=N,
                 scale=0.125, window_left=10, window_right=20, q_strides=st, k_strides=st,
                 v_strides=st, o_strides=(N * H * D, D, H * D))
    torch.cuda.synchronize()
    o_np = o.double().cpu().numpy().transpose(0, 2, 1, 3)
    check_against(o_np, lse.double().cpu().numpy(), o_ref, lse_ref, lens, dtype, relative=True, label="strided")


@pytest.mark.parametrize("kern", sorted(GLOBAL_KERNELS))
def test_strided_inputs_global_layer(kern):
    """Packed QKV read in place by both global-layer kernels of head_dim 64."""
    B, H, N, D = 2, 3, 300, 64
    _, q, k, v = draw(306, B, H, N, D, "fp16")
    lens = [300, 211]
    o_ref, lse_ref = attention_oracle(q, k, v, lens, 0.125)
    packed = np.stack([q, k, v], axis=0).transpose(1, 3, 0, 2, 4).copy()  # B, N, 3, H, D
    dev = to_dev(packed, "fp16")
    o = poison((B, N, H, D), "fp16")
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    sl = torch.tensor(lens, dtype=torch.int32).cuda()
    st = (N * 3 * H * D, D, 3 * H * D)
    fa.fa_fwd_ex(dtype=FA_DT["fp16"], q=dev[:, :, 0].data_ptr(), k=dev[:, :, 1].data_ptr(),
                 v=dev[:, :, 2].data_ptr(), o=o, lse=lse, seq_lens=sl, batch=B, heads=H, max_len=N,
                 scale=0.125, q_strides=st, k_strides=st, v_strides=st, o_strides=(N * H * D, D, H * D),
                 tuning=GLOBAL_KERNELS[kern])
    torch.cuda.synchronize()
    o_np = o.double().cpu().numpy().transpose(0, 2, 1, 3)
    check_against(o_np, lse.double().cpu().numpy(), o_ref, lse_ref, lens, "fp16", relative=True, label=f"strided {kern}")


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("B,H,N,lens", [
    (1, 1, 2100, [2049]),       # 17 blocks per wavefront: the ring of four slots is refilled many times
    (1, 2, 700, [40]),          # first ring requested from max_len, sequence far shorter: blocks fetched and dropped
    (2, 1, 640, [97, 640]),     # wavefront 3 has one partial block / five full ones
    (1, 3, 130, [65]),          # wavefront 3 (and 2 for most rows) has no block at all
    (1, 1, 4128, [4128]),       # exactly 129 blocks
    (3, 1, 513, [0, 513, 1]),   # empty sequence, one key
])
def test_key_split_kernel_ring_and_ragged_ends(dtype, B, H, N, lens):
    """The key-split kernel forced on shapes that exercise its private ring, the early
    request of blocks past the sequence end, wavefronts without work, and the merge of
    partial results when some of them are empty; padded rows hold NaN."""
    _, q, k, v = draw(1400 + N, B, H, N, 64, dtype)
    o_ref, lse_ref = attention_oracle(q, k, v, lens, 0.125)
    for b, n in enumerate(lens):
        k[b, :, n:] = np.nan
        v[b, :, n:] = np.nan
    o, lse = run_simple(q, k, v, lens, dtype, 0.125, tuning=fa.FA_TUNE_BM_32)
    check_against(o, lse, o_ref, lse_ref, lens, dtype, relative=True, label=f"key split {B}x{H}x{N}")
    o2, lse2 = run_simple(q, k, v, lens, dtype, 0.125, tuning=fa.FA_TUNE_BM_32 | fa.FA_TUNE_MAP_LINEAR)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("H,N,n", [(12, 8192, 7900), (12, 8192, 8192), (12, 8192, 5500), (12, 8192, 5376),
                                   (12, 8192, 3000), (12, 8192, 0), (5, 16384, 16001), (7, 8192, 8191),
                                   (48, 2048, 1999), (96, 1024, 1024), (200, 384, 383),
                                   # beyond 1024 tiles: rounds of 256-row pairs, then 128-row workgroups / pairs / 256-row
                                   (12, 16384, 16384), (12, 16384, 12288), (12, 16384, 14000), (12, 16384, 10100),
                                   (16, 16384, 16384), (24, 8192, 6000), (20, 8192, 8000), (13, 12288, 11000),
                                   (255, 1024, 1000), (3, 32768, 30000), (12, 20000, 19999)])
def test_mixed_shape_launch_covers_every_row(dtype, H, N, n):
    """One sequence, 256-row and 128-row workgroups in one launch, split on the device from the
    length: every row must come out exactly as the 128-row kernel computes it (the per-row
    arithmetic is the same, so bit for bit; a tile that no workgroup took would leave NaNs),
    with both workgroup-to-tile mappings; sampled rows also against the oracle."""
    _, q, k, v = draw(4200 + H, 1, H, N, 64, dtype)
    o1, lse1 = run_simple(q, k, v, [n], dtype, 0.125, tuning=fa.FA_TUNE_BM_128)
    for mapping in (fa.FA_TUNE_MAP_XCD, fa.FA_TUNE_MAP_LINEAR):
        o2, lse2 = run_simple(q, k, v, [n], dtype, 0.125, tuning=fa.FA_TUNE_BM_MIXED | mapping)
        assert np.array_equal(o1, o2) and np.array_equal(lse1, lse2)
    if n > 0:
        rng = np.random.default_rng(H)
        for h in (0, H // 2, H - 1):
            rows = np.unique(np.concatenate([rng.integers(0, n, 24), [0, n - 1]]))
            o_ref, lse_ref = attention_oracle_rows(q, k, v, 0, h, rows, n, 0.125)
            assert np.abs(o2[0, h, rows] - o_ref).max() <= TOL[dtype]["max_abs"]
            assert np.abs(lse2[0, h, rows] - lse_ref).max() <= LSE_TOL


@pytest.mark.parametrize("H,N,n", [(12, 8192, 7000), (10, 16384, 12345)])
def test_mixed_shape_launch_reads_packed_qkv_and_writes_bshd(H, N, n):
    """The mixed launch on [len, 3, heads, dim] packed inputs and a [len, heads, dim] output: bit
    for bit what the 128-row kernel produces from dense copies, padded rows (whole tiles of them
    are filled by the launch's spare workgroup ids) included."""
    D, dtype = 64, "fp16"
    _, q, k, v = draw(4300 + H, 1, H, N, D, dtype)
    o_ref, lse_ref = run_simple(q, k, v, [n], dtype, 0.125, tuning=fa.FA_TUNE_BM_128)
    packed = np.stack([q, k, v], axis=0).transpose(1, 3, 0, 2, 4).copy()  # 1, N, 3, H, D
    dev = to_dev(packed, dtype)
    o = poison((1, N, H, D), dtype)
    lse = torch.full((1, H, N), float("nan"), dtype=torch.float32, device="cuda")
    sl = torch.tensor([n], dtype=torch.int32).cuda()
    st = (N * 3 * H * D, D, 3 * H * D)
    fa.fa_fwd_ex(dtype=FA_DT[dtype], q=dev[:, :, 0].data_ptr(), k=dev[:, :, 1].data_ptr(), v=dev[:, :, 2].data_ptr(),
                 o=o, lse=lse, seq_lens=sl, batch=1, heads=H, max_len=N, scale=0.125, q_strides=st, k_strides=st,
                 v_strides=st, o_strides=(N * H * D, D, H * D), tuning=fa.FA_TUNE_BM_MIXED)
    torch.cuda.synchronize()
    assert np.array_equal(o.double().cpu().numpy().transpose(0, 2, 1, 3), o_ref)
    assert np.array_equal(lse.double().cpu().numpy(), lse_ref)
    assert np.all(o_ref[0, :, n:] == 0) and np.all(np.isneginf(lse_ref[0, :, n:]))


def test_key_split_merge_with_far_apart_maxima():
    """Each wavefront's share of the keys has its own score level (key block j scores about
    6 * (j % 4) higher): the merge has to scale three of the four partial results far down."""
    N, D = 512, 64
    rng = np.random.default_rng(11)
    q = np.zeros((1, 1, N, D), np.float32); q[..., 0] = 1.0
    k0 = rng.standard_normal((1, 1, N, D)).astype(np.float32) * 0.1
    k0[0, 0, :, 0] = 6.0 * ((np.arange(N) // 32) % 4)
    v0 = rng.standard_normal((1, 1, N, D)).astype(np.float32)
    for dtype in ("fp16", "bf16"):
        k, v = round_to_storage(k0, dtype), round_to_storage(v0, dtype)
        for scale in (1.0, 4.0):
            o_ref, lse_ref = attention_oracle(q, k, v, None, scale)
            o, lse = run_simple(q, k, v, None, dtype, scale, tuning=fa.FA_TUNE_BM_32)
            check_against(o, lse, o_ref, lse_ref, None, dtype, relative=True, label=f"merge {dtype} {scale}")


@pytest.mark.parametrize("D,left,right", [(128, -1, -1), (128, 10, 20), (32, -1, -1)])
def test_strided_inputs_other_head_dims(D, left, right):
    """Packed QKV read in place for head_dim 128 (pipelined global kernel and masked kernel)
    and head_dim 32."""
    B, H, N = 2, 2, 260
    _, q, k, v = draw(307 + D, B, H, N, D, "bf16")
    lens = [260, 77]
    scale = 1.0 / np.sqrt(D)
    o_ref, lse_ref = attention_oracle(q, k, v, lens, scale, left, right)
    packed = np.stack([q, k, v], axis=0).transpose(1, 3, 0, 2, 4).copy()  # B, N, 3, H, D
    dev = to_dev(packed, "bf16")
    o = poison((B, N, H, D), "bf16")
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    sl = torch.tensor(lens, dtype=torch.int32).cuda()
    st = (N * 3 * H * D, D, 3 * H * D)
    fa.fa_fwd_ex(dtype=FA_DT["bf16"], q=dev[:, :, 0].data_ptr(), k=dev[:, :, 1].data_ptr(),
                 v=dev[:, :, 2].data_ptr(), o=o, lse=lse, seq_lens=sl, batch=B, heads=H, max_len=N,
                 head_dim=D, scale=scale, window_left=left, window_right=right, q_strides=st,
                 k_strides=st, v_strides=st, o_strides=(N * H * D, D, H * D))
    torch.cuda.synchronize()
    o_np = o.double().cpu().numpy().transpose(0, 2, 1, 3)
    check_against(o_np, lse.double().cpu().numpy(), o_ref, lse_ref, lens, "bf16", relative=True, label=f"strided D={D}")


def test_valid_call_returns_zero_and_bad_call_leaves_output_untouched():
    B, H, N, D = 1, 1, 64, 64
    _, q, k, v = draw(306, B, H, N, D, "fp16")
    qd, kd, vd = to_dev(q, "fp16"), to_dev(k, "fp16"), to_dev(v, "fp16")
    o = poison((B, H, N, D), "fp16")
    assert fa.fa_fwd(qd, kd, vd, o, None, B, H, None, N, D, 0.125, -1, check=False) == 0
    torch.cuda.synchronize()
    assert torch.isfinite(o).all()
    o2 = poison((B, H, N, D), "fp16")
    assert fa.fa_fwd(qd, kd, vd, o2, None, B, H, None, N, 48, 0.125, -1, check=False) == -3
    assert fa.fa_fwd(qd, kd, vd, o2, None, B, H, None, N, D, 0.125, 0, check=False) == -5
    torch.cuda.synchronize()
    assert torch.isnan(o2).all()


# ------------------------------------------------------------------ head_dim 32 and 128
HD_TUNINGS = {"auto": 0, "scalar_linear": fa.FA_TUNE_V_SCALAR | fa.FA_TUNE_MAP_LINEAR,
              "bm256_where_it_exists": fa.FA_TUNE_BM_256, "win_pipelined": fa.FA_TUNE_WIN_PIPELINED,
              "win_two_phase": fa.FA_TUNE_WIN_TWO_PHASE}


@pytest.mark.parametrize("tuning", sorted(HD_TUNINGS))
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("D", [32, 128])
@pytest.mark.parametrize("left,right", [(-1, -1), (63, 64), (0, 0), (0, 5), (70, -1), (-1, 9)])
def test_head_dims_small_ragged_all_windows(D, dtype, left, right, tuning):
    """The operator's other two head sizes (paper Sec. 4.1.3 dispatches on 32, 64, 128):
    several key tiles, a ragged tail, padding inside a tile, a fully padded query tile."""
    B, H, N = 2, 2, 333
    _, q, k, v = draw(400 + D, B, H, N, D, dtype)
    lens = [333, 120]
    scale = 1.0 / np.sqrt(D)
    o_ref, lse_ref = attention_oracle(q, k, v, lens, scale, left, right)
    o, lse = run_ex(q, k, v, lens, dtype, scale, left, right, HD_TUNINGS[tuning])
    check_against(o, lse, o_ref, lse_ref, lens, dtype, relative=True, label=f"D={D} {dtype} {left},{right} {tuning}")


@pytest.mark.parametrize("D", [32, 128])
@pytest.mark.parametrize("N", [1, 31, 33, 64, 65, 129, 257])
def test_head_dims_lengths_around_tile_edges(D, N):
    B, H = 1, 2
    for dtype in ("fp16", "bf16"):
        _, q, k, v = draw(500 + N + D, B, H, N, D, dtype)
        for window in (-1, 128, 2):
            L, R = window_from_width(window)
            o_ref, lse_ref = attention_oracle(q, k, v, None, 0.2, L, R)
            o, lse = run_simple(q, k, v, None, dtype, 0.2, window)
            check_against(o, lse, o_ref, lse_ref, None, dtype, relative=True, label=f"D={D} N={N} w={window}")


@pytest.mark.parametrize("D", [32, 128])
def test_head_dims_closed_forms_and_padding(D):
    """Q = 0: o = mean of the visible V rows and lse = ln(#visible) exactly as counted from
    the window and the length; garbage (NaN, Inf) in the padded rows changes nothing."""
    B, H, N = 2, 2, 200
    _, q, k, v = draw(600 + D, B, H, N, D, "fp16")
    lens = [200, 77]
    q0 = np.zeros_like(q)
    o, lse = run_simple(q0, k, v, lens, "fp16", 0.125, 128)
    for b, n in enumerate(lens):
        for i in (0, 1, 63, 64, n // 2, n - 1):
            lo, hi = max(0, i - 63), min(n - 1, i + 64)
            assert abs(lse[b, 0, i] - np.log(hi - lo + 1)) <= 1e-3
            assert np.abs(o[b, 1, i] - v[b, 1, lo:hi + 1].astype(np.float64).mean(axis=0)).max() <= 2e-3
    o1, lse1 = run_simple(q, k, v, lens, "fp16", 0.125, -1)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for x, val in ((q2, np.nan), (k2, np.inf), (v2, np.nan)):
        x[1, :, 77:] = val
    o2, lse2 = run_simple(q2, k2, v2, lens, "fp16", 0.125, -1)
    assert np.array_equal(o1, o2) and np.array_equal(lse1, lse2)


@pytest.mark.parametrize("D", [32, 128])
def test_head_dims_longer_sequence_sampled_rows(D):
    """2K tokens, two lengths, global and local: sampled rows against the oracle."""
    B, H, N = 2, 4, 2048
    lens = [2048, 1500]
    # peaked scores (gain 1.5) on both legs.  A peaked softmax over the few keys of a window
    # gives outputs beyond 2 in magnitude, where a bf16 number is by itself up to 7.8e-3 off:
    # the output error is scaled by max(1, |reference|) as for every test whose outputs leave
    # [-1, 1]; lse keeps its absolute bound.
    for dtype, window, gain in (("fp16", -1, 1.5), ("bf16", 128, 1.5)):
        _, q, k, v = draw(700 + D, B, H, N, D, dtype, qk_gain=gain)
        scale = 1.0 / np.sqrt(D)
        o, lse = run_simple(q, k, v, lens, dtype, scale, window)
        L, R = window_from_width(window)
        rows = np.array([0, 1, 63, 64, 127, 128, 777, 1499, 1500, 2047])
        for b in range(B):
            n = lens[b]
            rr = rows[rows < n]
            for h in (0, H - 1):
                o_ref, lse_ref = attention_oracle_rows(q, k, v, b, h, rr, n, scale, L, R)
                d = np.abs(o[b, h, rr] - o_ref) / np.maximum(1.0, np.abs(o_ref))
                assert d.max() <= TOL[dtype]["max_abs"], (dtype, b, h, d.max())
                assert np.abs(lse[b, h, rr] - lse_ref).max() <= LSE_TOL
            assert np.all(o[b, :, n:] == 0) and np.all(np.isneginf(lse[b, :, n:]))


def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """The library allocates nothing, never synchronises and launches on the caller's stream,
    so a global and a local call can be recorded into a graph; every replay (with eager work
    and fresh inputs in between) must reproduce the eager result bit for bit."""
    B, H, N, D = 2, 3, 600, 64
    lens = [600, 333]
    sl = torch.tensor(lens, dtype=torch.int32).cuda()
    qd = torch.zeros((B, H, N, D), dtype=torch.float16, device="cuda")
    kd, vd = torch.zeros_like(qd), torch.zeros_like(qd)
    o_g, o_l = poison((B, H, N, D), "fp16"), poison((B, H, N, D), "fp16")
    lse_g = torch.zeros((B, H, N), dtype=torch.float32, device="cuda")
    lse_l = torch.zeros_like(lse_g)

    def calls():
        fa.fa_fwd(qd, kd, vd, o_g, lse_g, B, H, sl, N, D, 0.125, -1)
        fa.fa_fwd(qd, kd, vd, o_l, lse_l, B, H, sl, N, D, 0.125, 128)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        calls()                     # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls()
    for rep in range(3):
        _, q, k, v = draw(900 + rep, B, H, N, D, "fp16")
        qd.copy_(to_dev(q, "fp16")); kd.copy_(to_dev(k, "fp16")); vd.copy_(to_dev(v, "fp16"))
        o_g.fill_(float("nan")); o_l.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [x.clone() for x in (o_g, lse_g, o_l, lse_l)]
        o_g.fill_(float("nan")); o_l.fill_(float("nan"))
        calls()
        torch.cuda.synchronize()
        for a_, b_ in zip(got, (o_g, lse_g, o_l, lse_l)):
            assert torch.equal(a_, b_), f"replay {rep} differs from the eager call"
        o_ref, lse_ref = attention_oracle(q, k, v, lens, 0.125)
        check_against(got[0].double().cpu().numpy(), got[1].double().cpu().numpy(), o_ref, lse_ref, lens, "fp16",
                      label=f"graph replay {rep}")


def test_concurrent_callers_on_their_own_streams():
    """The paper's deployment runs several classifier sessions and many requests side by side
    (Sec. 4.1.1, Sec. 5 concurrency table): eight host threads, each with its own stream, shape,
    mask form and data, call the library at the same time, twenty times each.  The library
    keeps no state between calls, so every thread's last output must match the oracle and
    its first output bit for bit."""
    import threading

    cases = [  # (seed, B, H, N, lens, dtype, window)
        (1200, 1, 12, 512, [512], "fp16", -1),
        (1201, 1, 12, 512, [470], "bf16", 128),
        (1202, 2, 4, 300, [300, 77], "fp16", -1),
        (1203, 1, 3, 1000, [901], "bf16", -1),
        (1204, 3, 2, 260, [260, 1, 130], "fp16", 64),
        (1205, 1, 12, 512, [333], "fp16", 128),
        (1206, 1, 2, 2048, [2048], "bf16", -1),
        (1207, 2, 2, 640, [640, 639], "fp16", 256),
    ]
    work = []
    for seed, B, H, N, lens, dtype, window in cases:
        _, q, k, v = draw(seed, B, H, N, 64, dtype)
        work.append(dict(q=to_dev(q, dtype), k=to_dev(k, dtype), v=to_dev(v, dtype), o=poison((B, H, N, 64), dtype),
                         lse=torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda"),
                         sl=torch.tensor(lens, dtype=torch.int32).cuda(), stream=torch.cuda.Stream(),
                         host=(q, k, v), first=None, error=None))
    torch.cuda.synchronize()
    gate = threading.Barrier(len(cases))

    def caller(i):
        seed, B, H, N, lens, dtype, window = cases[i]
        w = work[i]
        fn = fa.fa_fwd if dtype == "fp16" else fa.fa_fwd_bf16
        try:
            gate.wait(timeout=60)
            for rep in range(20):
                fn(w["q"], w["k"], w["v"], w["o"], w["lse"], B, H, w["sl"], N, 64, 0.125, window, stream=w["stream"])
                if rep == 0:
                    w["stream"].synchronize()
                    w["first"] = (w["o"].clone(), w["lse"].clone())
                    with torch.cuda.stream(w["stream"]):
                        w["o"].fill_(float("nan"))
            w["stream"].synchronize()
        except Exception as e:  # reported by the main thread
            w["error"] = e

    threads = [threading.Thread(target=caller, args=(i,)) for i in range(len(cases))]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
        assert not t.is_alive()
    torch.cuda.synchronize()
    for i, (seed, B, H, N, lens, dtype, window) in enumerate(cases):
        w = work[i]
        assert w["error"] is None, f"caller {i}: {w['error']}"
        assert torch.equal(w["first"][0], w["o"]) and torch.equal(w["first"][1], w["lse"]), f"caller {i}: calls differ"
        L, R = window_from_width(window)
        o_ref, lse_ref = attention_oracle(*w["host"], lens, 0.125, L, R)
        check_against(w["o"].double().cpu().numpy(), w["lse"].double().cpu().numpy(), o_ref, lse_ref, lens, dtype,
                      label=f"concurrent caller {i}")


def test_call_on_a_stream_limited_to_half_the_compute_units():
    """Co-location with another tenant (paper Sec. 1, Sec. 4.1.1): the caller hands over a stream
    that may only use 128 of the 256 compute units.  Nothing in the kernels depends on how
    many units run them, so global and local layers must give the same bits as on the
    default stream, and match the oracle."""
    from paper_2603_12646_amd.cu_mask import CuMaskedStream, first_units

    B, H, N = 2, 6, 1500
    lens = [1500, 1111]
    _, q, k, v = draw(1300, B, H, N, 64, "bf16")
    qd, kd, vd = (to_dev(x, "bf16") for x in (q, k, v))
    sl = torch.tensor(lens, dtype=torch.int32).cuda()
    torch.cuda.synchronize()
    with CuMaskedStream(first_units(128)) as ms:
        for window in (-1, 128):
            o_m, o_d = poison((B, H, N, 64), "bf16"), poison((B, H, N, 64), "bf16")
            lse_m = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
            lse_d = lse_m.clone()
            torch.cuda.synchronize()
            fa.fa_fwd_bf16(qd, kd, vd, o_m, lse_m, B, H, sl, N, 64, 0.125, window, stream=ms.handle)
            ms.synchronize()
            fa.fa_fwd_bf16(qd, kd, vd, o_d, lse_d, B, H, sl, N, 64, 0.125, window)
            torch.cuda.synchronize()
            assert torch.equal(o_m, o_d) and torch.equal(lse_m, lse_d)
            L, R = window_from_width(window)
            o_ref, lse_ref = attention_oracle(q, k, v, lens, 0.125, L, R)
            check_against(o_m.double().cpu().numpy(), lse_m.double().cpu().numpy(), o_ref, lse_ref, lens, "bf16",
                          label=f"half the compute units, window {window}")


# ------------------------------------------------------------------ additive key bias
def _random_bias(seed, B, N, dtype, holes=True, gain=2.0):
    rng = np.random.default_rng(seed)
    bias = round_to_storage((rng.standard_normal((B, N)) * gain).astype(np.float32), dtype)
    if holes:   # non-tail key mask: about one key in five excluded
        bias[rng.random((B, N)) < 0.2] = -np.inf
    return bias


@pytest.mark.parametrize("tuning", [0, fa.FA_TUNE_BM_256, fa.FA_TUNE_V_SCALAR])
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("D", [32, 64, 128])
@pytest.mark.parametrize("left,right", [(-1, -1), (63, 64), (0, 5), (70, -1)])
def test_key_bias_random_values_and_holes(D, dtype, left, right, tuning):
    """The operator's pad_bias input (paper Sec. 4.1.3, Eq. 1) with arbitrary values and
    -inf holes, on top of sequence lengths and windows.  Global layers of head_dim 64 / 128
    take the pipelined kernel (128- and 256-row tiles), everything else the masked kernel."""
    B, H, N = 2, 2, 333
    _, q, k, v = draw(800 + D, B, H, N, D, dtype)
    lens = [333, 150]
    bias = _random_bias(801 + D, B, N, dtype)
    scale = 1.0 / np.sqrt(D)
    o_ref, lse_ref = attention_oracle(q, k, v, lens, scale, left, right, key_bias=bias)
    o, lse = run_ex(q, k, v, lens, dtype, scale, left, right, tuning=tuning, key_bias=bias)
    check_against(o, lse, o_ref, lse_ref, lens, dtype, relative=True, label=f"bias D={D} {dtype} {left},{right} {tuning}")


@pytest.mark.parametrize("N", [1, 31, 33, 64, 65, 127, 129, 257, 640])
@pytest.mark.parametrize("D", [64, 128])
def test_key_bias_global_lengths_around_tile_edges(D, N):
    """Pipelined kernel with a bias: prologue only, tail only, several tiles plus a tail;
    negative scale and scale 0 as well (scale 0 falls back to the masked kernel)."""
    B, H = 2, 2
    for dtype in ("fp16", "bf16"):
        _, q, k, v = draw(820 + N + D, B, H, N, D, dtype)
        # bf16: a milder bias, so that outputs stay well below 1 in magnitude (a bf16 output of
        # magnitude 1 is by itself 1e-3 away from the exact value on average)
        bias = _random_bias(821 + N, B, N, dtype, holes=N > 4, gain=2.0 if dtype == "fp16" else 0.5)
        lens = [N, max(1, N - 7)]
        for scale in (0.11, -0.2, 0.0):
            o_ref, lse_ref = attention_oracle(q, k, v, lens, scale, key_bias=bias)
            o, lse = run_ex(q, k, v, lens, dtype, scale, key_bias=bias)
            check_against(o, lse, o_ref, lse_ref, lens, dtype, relative=True,
                          label=f"bias {dtype} D={D} N={N} scale={scale}")


def test_key_bias_8k_sampled_rows():
    """The 8K workload with a random key mask (one key in ten excluded) and small biases."""
    w = CONFIGS["c3_8k"]
    lens, q, k, v = make_inputs(w)
    rng = np.random.default_rng(5)
    bias = round_to_storage((rng.standard_normal((w.batch, w.max_len)) * 0.5).astype(np.float32), w.dtype)
    bias[rng.random((w.batch, w.max_len)) < 0.1] = -np.inf
    o, lse = run_ex(q, k, v, lens, w.dtype, w.scale, key_bias=bias)
    n = int(lens[0])
    assert np.all(o[0, :, n:] == 0) and np.all(np.isneginf(lse[0, :, n:]))
    for h in (0, 5, 11):
        rows = sample_rows(n, rng, 200)
        o_ref, lse_ref = attention_oracle_rows(q, k, v, 0, h, rows, n, w.scale, key_bias=bias)
        assert np.abs(o[0, h, rows] - o_ref).max() <= TOL[w.dtype]["max_abs"]
        assert np.abs(lse[0, h, rows] - lse_ref).max() <= LSE_TOL


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_key_bias_batch_of_two_sampled_rows(dtype):
    """Two sequences of different lengths, each with its OWN bias row (a different random key
    mask and different values per batch element): sampled rows of both against the oracle, so
    that a bias row taken from the wrong batch element cannot pass."""
    B, H, N, D = 2, 3, 3000, 64
    lens = [3000, 2300]
    _, q, k, v = draw(5150, B, H, N, D, dtype)
    rng = np.random.default_rng(51)
    bias = round_to_storage(rng.standard_normal((B, N)).astype(np.float32), dtype)
    bias[rng.random((B, N)) < 0.15] = -np.inf
    assert not np.array_equal(bias[0], bias[1])
    o, lse = run_ex(q, k, v, lens, dtype, 0.125, key_bias=bias)
    for b in range(B):
        n = lens[b]
        assert np.all(o[b, :, n:] == 0) and np.all(np.isneginf(lse[b, :, n:]))
        for h in (0, H - 1):
            rows = sample_rows(n, rng, 100)
            o_ref, lse_ref = attention_oracle_rows(q, k, v, b, h, rows, n, 0.125, key_bias=bias)
            assert np.abs(o[b, h, rows] - o_ref).max() <= TOL[dtype]["max_abs"], (dtype, b, h)
            assert np.abs(lse[b, h, rows] - lse_ref).max() <= LSE_TOL, (dtype, b, h)


def test_key_bias_paper_padding_form_equals_seq_lens():
    """-65504 on the padded keys and no seq_lens (the paper's own input form) gives, on the
    valid rows, the result of the seq_lens form; a zero bias changes nothing."""
    B, H, N, D = 2, 3, 200, 64
    _, q, k, v = draw(810, B, H, N, D, "fp16")
    lens = [200, 131]
    bias = np.where(np.arange(N)[None, :] < np.array(lens)[:, None], 0.0, -65504.0).astype(np.float32)
    o_ref, lse_ref = attention_oracle(q, k, v, lens, 0.125)
    o, lse = run_ex(q, k, v, None, "fp16", 0.125, key_bias=bias)
    for b, n in enumerate(lens):
        assert np.abs(o[b, :, :n] - o_ref[b, :, :n]).max() <= TOL["fp16"]["max_abs"]
        assert np.abs(lse[b, :, :n] - lse_ref[b, :, :n]).max() <= LSE_TOL
    o0, lse0 = run_ex(q, k, v, lens, "fp16", 0.125, key_bias=np.zeros((B, N), dtype=np.float32))
    o1, lse1 = run_ex(q, k, v, lens, "fp16", 0.125, tuning=fa.FA_TUNE_BM_128)
    check_against(o0, lse0, o_ref, lse_ref, lens, "fp16", label="zero bias")
    assert np.abs(o0 - o1).max() <= 1e-3 and np.abs(lse0[:, :, :131] - lse1[:, :, :131]).max() <= 1e-3


def test_key_bias_all_keys_excluded_and_large_values():
    """Every key at -inf: o = 0, lse = -inf, no NaN.  Large biases force reference refreshes."""
    B, H, N, D = 1, 2, 130, 64
    _, q, k, v = draw(811, B, H, N, D, "fp16")
    o, lse = run_ex(q, k, v, None, "fp16", 0.125, key_bias=np.full((B, N), -np.inf, dtype=np.float32))
    assert np.all(o == 0) and np.all(np.isneginf(lse))
    bias = round_to_storage((np.arange(N, dtype=np.float32) * 3.0)[None, :], "fp16")   # rising: a refresh per block
    o_ref, lse_ref = attention_oracle(q, k, v, None, 0.125, key_bias=bias)
    o, lse = run_ex(q, k, v, None, "fp16", 0.125, key_bias=bias)
    check_against(o, lse, o_ref, lse_ref, None, "fp16", relative=True, label="rising bias")


# ------------------------------------------------------------------ the five named workloads
@pytest.mark.parametrize("name", ["c1_512", "c2_batch32"])
def test_named_small_configs_full_compare(name):
    w = CONFIGS[name]
    lens, q, k, v = make_inputs(w)
    L, R = window_from_width(w.window)
    o_ref, lse_ref = attention_oracle(q, k, v, lens, w.scale, L, R)
    o, lse = run_simple(q, k, v, lens, w.dtype, w.scale, w.window)
    mx, mean = check_against(o, lse, o_ref, lse_ref, lens, w.dtype, label=name)
    print(f"{name}: max-abs {mx:.3e} mean-abs {mean:.3e}")


def sample_rows(n, rng, count):
    edge = set(range(min(130, n))) | set(range(max(0, n - 130), n))
    rest = rng.choice(n, size=min(count, n), replace=False).tolist()
    return np.array(sorted(edge | set(rest)), dtype=np.int64)


@pytest.mark.parametrize("name", ["c3_8k", "c4_16k_x3", "c5a_32k_global", "c5b_32k_local", "d128_8k", "d128_32k",
                                  "d128_32k_local", "d32_8k", "d32_32k", "d32_32k_local"])
def test_named_large_configs_sampled_rows(name):
    """Full-size launch, as bench.py times it; the oracle recomputes sampled query
    rows (the first and last 130 valid rows of every (batch, head) plus random ones)
    one by one against the full key range.  Padded rows are checked exhaustively."""
    w = ALL_CONFIGS[name]
    lens, q, k, v = make_inputs(w)
    L, R = window_from_width(w.window)
    o, lse = run_simple(q, k, v, lens, w.dtype, w.scale, w.window)
    rng = np.random.default_rng(11)
    tol = TOL[w.dtype]
    worst, total, count = 0.0, 0.0, 0
    for b in range(w.batch):
        n = int(lens[b])
        assert np.all(o[b, :, n:] == 0) and np.all(np.isneginf(lse[b, :, n:]))
        for h in range(w.heads):
            rows = sample_rows(n, rng, 384)
            o_ref, lse_ref = attention_oracle_rows(q, k, v, b, h, rows, n, w.scale, L, R)
            d = np.abs(o[b, h, rows] - o_ref)
            assert np.all(np.isfinite(o[b, h, rows]))
            worst = max(worst, float(d.max())); total += float(d.sum()); count += d.size
            assert np.abs(lse[b, h, rows] - lse_ref).max() <= LSE_TOL, (name, b, h)
    print(f"{name}: max-abs {worst:.3e} mean-abs {total / count:.3e} over {count} sampled outputs")
    assert worst <= tol["max_abs"] and total / count <= tol["mean_abs"]


@pytest.mark.parametrize("dtype,window,tuning", [("bf16", -1, 0), ("fp16", 128, 0), ("fp16", -1, fa.FA_TUNE_BM_32),
                                                 ("bf16", 700, 0)])
def test_quarter_million_tokens_sampled_rows(dtype, window, tuning):
    """Eight times the longest named workload: one head of 262 144 tokens (a key-padding tail
    of 1 000), where row offsets pass 2^24 bytes and a row's sum runs over 261 144 keys.
    Global (pipelined and key-split kernels), the 128-key window and a 700-key window (ring
    kernel); sampled rows against the oracle, padded rows exhaustively."""
    B, H, N, D = 1, 1, 262144, 64
    n = N - 1000
    _, q, k, v = draw(1500, B, H, N, D, dtype)
    L, R = window_from_width(window)
    o, lse = run_simple(q, k, v, [n], dtype, 0.125, window, tuning=tuning)
    assert np.all(o[0, :, n:] == 0) and np.all(np.isneginf(lse[0, :, n:]))
    rows = sample_rows(n, np.random.default_rng(12), 160)
    o_ref, lse_ref = attention_oracle_rows(q, k, v, 0, 0, rows, n, 0.125, L, R)
    d = np.abs(o[0, 0, rows] - o_ref)
    assert np.all(np.isfinite(o[0, 0, rows]))
    assert d.max() <= TOL[dtype]["max_abs"] and d.mean() <= TOL[dtype]["mean_abs"], (d.max(), d.mean())
    assert np.abs(lse[0, 0, rows] - lse_ref).max() <= LSE_TOL


@pytest.mark.parametrize("window", [-1, 16])
def test_thousands_of_tiny_sequences(window):
    """3 000 sequences of 0 to 40 tokens, 3 heads: the grid is almost all batch index, most
    tiles are ragged or empty, and every XCD's share of a batch element is a fraction of a tile
    row.  Full compare, both tile orders."""
    B, H, N, D = 3000, 3, 40, 64
    rng = np.random.default_rng(13)
    lens = rng.integers(0, N + 1, size=B).tolist()
    _, q, k, v = draw(1600, B, H, N, D, "fp16")
    L, R = window_from_width(window)
    o_ref, lse_ref = attention_oracle(q, k, v, lens, 0.125, L, R)
    for tuning in (fa.FA_TUNE_MAP_XCD, fa.FA_TUNE_MAP_LINEAR):
        o, lse = run_ex(q, k, v, lens, "fp16", 0.125, L, R, tuning=tuning)
        check_against(o, lse, o_ref, lse_ref, lens, "fp16", relative=True, label=f"tiny sequences {window} {tuning:#x}")


# ------------------------------------------------------------------ measurement helper program
def test_ceilings_program_reports_plausible_numbers():
    """The standalone program bench.py runs for its `ceilings` block: matrix-core rate with
    zero and with random operands, the kernels' instruction mix without memory traffic, and a
    1 GiB copy."""
    import json
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(fa.LIB_PATH), "fa_ceilings")
    assert os.path.exists(exe), "fa_ceilings not built (python -m paper_2603_12646_amd.build)"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
    d = json.loads(r.stdout.strip().splitlines()[-1])
    for key in ("mfma_f16_zero_tflops", "mfma_f16_random_tflops", "mfma_bf16_zero_tflops",
                "mfma_bf16_random_tflops", "copy_gbs"):
        assert d[key] > 0
    assert 500 < d["mfma_f16_random_tflops"] <= d["mfma_f16_zero_tflops"] * 1.05 < 2500 * 1.1
    assert 1000 < d["copy_gbs"] < 8000
    # the attention instruction mix: below the matrix-core-only rate, and head_dim 128 (twice the
    # matrix work per exponential) above head_dim 64
    for t in ("f16", "bf16"):
        assert 300 < d[f"mix_{t}_d32_tflops"] < d[f"mix_{t}_d64_tflops"] < d[f"mix_{t}_d128_tflops"] < d[f"mfma_{t}_zero_tflops"] * 1.05
        assert d[f"softmax_valu_only_{t}_d64_tflops"] > d[f"mix_{t}_d64_tflops"] * 0.8
