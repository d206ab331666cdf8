"""GPU parity of the rotary-embedding path (rotation of q and k inside the call) against the
fp64 oracle of oracle/rope_oracle.py on the same seeded inputs and the same fp32 tables.
Tolerances as for every other parity test (fp16 2e-3 / 2e-4, bf16 1e-2 / 1e-3, lse 1e-3)."""
import numpy as np
import pytest
import torch

import paper_2603_12646_amd as fa
from oracle.rope_oracle import attention_oracle_rope, attention_oracle_rope_rows, rope_tables
from workloads import ALL_CONFIGS, draw, make_inputs, round_to_storage

from tests.gpu_util import FA_DT, LSE_TOL, TOL, check_against, poison, to_dev

pytestmark = pytest.mark.gpu


def tables(N, D, base=10000.0, freq_scale=None, amplitude=1.0):
    """fp32 tables for the device and the same values widened to fp64 for the oracle."""
    cos, sin = rope_tables(N, D, base, freq_scale, amplitude)
    c32, s32 = cos.astype(np.float32), sin.astype(np.float32)
    return c32, s32, c32.astype(np.float64), s32.astype(np.float64)


def run_rope(q32, k32, v32, lens, dtype, scale, c32, s32, left=-1, right=-1, tuning=0, key_bias=None, rope_stride=0,
             scratch_bytes=0, **extra):
    B, H, N, D = q32.shape
    q, k, v = to_dev(q32, dtype), to_dev(k32, dtype), to_dev(v32, dtype)
    o = poison((B, H, N, D), dtype)
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    sl = None if lens is None else torch.as_tensor(np.asarray(lens), dtype=torch.int32).cuda()
    cd, sd = torch.from_numpy(np.ascontiguousarray(c32)).cuda(), torch.from_numpy(np.ascontiguousarray(s32)).cuda()
    kb = None if key_bias is None else to_dev(np.ascontiguousarray(key_bias, dtype=np.float32), dtype)
    # lent scratch: poisoned, so that anything read from it that the call did not write shows up
    scratch = torch.full((scratch_bytes,), 0xFF, dtype=torch.uint8, device="cuda") if scratch_bytes else None
    fa.fa_fwd_ex(dtype=FA_DT[dtype], q=q, k=k, v=v, o=o, lse=lse, seq_lens=sl, batch=B, heads=H, max_len=N,
                 head_dim=D, scale=scale, window_left=left, window_right=right, tuning=tuning, key_bias=kb,
                 rope_cos=cd, rope_sin=sd, rope_stride=rope_stride, scratch=scratch, scratch_bytes=scratch_bytes, **extra)
    torch.cuda.synchronize()
    return o.double().cpu().numpy(), lse.double().cpu().numpy()


ROPE_TUNINGS = {"auto": 0, "bm256": fa.FA_TUNE_BM_256, "bm128_linear": fa.FA_TUNE_BM_128 | fa.FA_TUNE_MAP_LINEAR,
                "masked_kernel": fa.FA_TUNE_V_SCALAR, "win_pipelined": fa.FA_TUNE_WIN_PIPELINED}


@pytest.mark.parametrize("tuning", sorted(ROPE_TUNINGS))
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("D", [32, 64, 128])
@pytest.mark.parametrize("left,right", [(-1, -1), (63, 64), (0, 5), (70, -1), (200, 130)])
def test_rope_small_ragged(D, dtype, left, right, tuning):
    B, H, N = 2, 2, 300
    lens = [300, 171]
    _, q, k, v = draw(9000 + D, B, H, N, D, dtype)
    c32, s32, c64, s64 = tables(N, D, base=10000.0)
    scale = 1.0 / np.sqrt(D)
    o_ref, lse_ref = attention_oracle_rope(q, k, v, c64, s64, dtype, lens, scale, left, right)
    o, lse = run_rope(q, k, v, lens, dtype, scale, c32, s32, left, right, ROPE_TUNINGS[tuning])
    check_against(o, lse, o_ref, lse_ref, lens, dtype, label=f"rope D{D} {dtype} ({left},{right}) {tuning}")


@pytest.mark.parametrize("D", [32, 64, 128])
@pytest.mark.parametrize("N", [1, 31, 33, 64, 65, 127, 129, 257, 640])
def test_rope_lengths_around_tile_edges(D, N):
    for dtype, window in (("fp16", -1), ("bf16", 128)):
        _, q, k, v = draw(9100 + N, 1, 3, N, D, dtype)
        c32, s32, c64, s64 = tables(N, D, base=500.0)
        L, R = (-1, -1) if window < 0 else (63, 64)
        o_ref, lse_ref = attention_oracle_rope(q, k, v, c64, s64, dtype, None, 0.125, L, R)
        o, lse = run_rope(q, k, v, None, dtype, 0.125, c32, s32, L, R)
        check_against(o, lse, o_ref, lse_ref, None, dtype, label=f"rope N{N} D{D} {dtype}")


def test_rope_rescaled_frequencies_amplitude_and_padded_table():
    """The long-context variant's inputs: per-frequency factors and an amplitude (values here are
    arbitrary: the paper publishes none), and a table whose rows are wider than head_dim / 2."""
    B, H, N, D = 1, 4, 700, 64
    _, q, k, v = draw(9200, B, H, N, D, "fp16")
    fs = np.linspace(1.0, 0.03, D // 2)
    c32, s32, c64, s64 = tables(N, D, base=160000.0, freq_scale=fs, amplitude=1.07)
    wide_c = np.full((N, 40), 7.0, np.float32); wide_c[:, :32] = c32
    wide_s = np.full((N, 40), -7.0, np.float32); wide_s[:, :32] = s32
    o_ref, lse_ref = attention_oracle_rope(q, k, v, c64, s64, "fp16", [650], 0.125)
    o, lse = run_rope(q, k, v, [650], "fp16", 0.125, wide_c, wide_s, rope_stride=40)
    check_against(o, lse, o_ref, lse_ref, [650], "fp16", label="rope rescaled")


def test_rope_zero_angles_leave_the_result_bit_identical():
    B, H, N, D = 2, 3, 500, 64
    lens = [500, 333]
    _, q, k, v = draw(9300, B, H, N, D, "bf16")
    ones, zeros = np.ones((N, D // 2), np.float32), np.zeros((N, D // 2), np.float32)
    # (the same kernel on both sides: a call this small without a rotation would otherwise take the
    # key-split / resident pipelined kernels, whose summation order differs)
    for left, right, tuning in ((-1, -1, fa.FA_TUNE_BM_128), (63, 64, fa.FA_TUNE_WIN_TWO_PHASE), (70, -1, fa.FA_TUNE_V_SCALAR)):
        o1, lse1 = run_rope(q, k, v, lens, "bf16", 0.125, ones, zeros, left, right, tuning)
        qd, kd, vd = to_dev(q, "bf16"), to_dev(k, "bf16"), to_dev(v, "bf16")
        o2 = poison((B, H, N, D), "bf16")
        lse2 = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
        fa.fa_fwd_ex(dtype=fa.FA_DTYPE_BF16, q=qd, k=kd, v=vd, o=o2, lse=lse2, seq_lens=torch.tensor(lens, dtype=torch.int32).cuda(),
                     batch=B, heads=H, max_len=N, head_dim=D, scale=0.125, window_left=left, window_right=right, tuning=tuning)
        torch.cuda.synchronize()
        assert np.array_equal(o1, o2.double().cpu().numpy()) and np.array_equal(lse1, lse2.double().cpu().numpy())


def test_rope_with_key_bias():
    B, H, N, D = 2, 2, 400, 64
    lens = [400, 250]
    rng = np.random.default_rng(94)
    for dtype in ("fp16", "bf16"):
        _, q, k, v = draw(9400, B, H, N, D, dtype)
        bias = round_to_storage(rng.standard_normal((B, N)).astype(np.float32), dtype)
        bias[rng.random((B, N)) < 0.1] = -np.inf
        c32, s32, c64, s64 = tables(N, D)
        for left, right in ((-1, -1), (63, 64)):
            o_ref, lse_ref = attention_oracle_rope(q, k, v, c64, s64, dtype, lens, 0.125, left, right, key_bias=bias)
            o, lse = run_rope(q, k, v, lens, dtype, 0.125, c32, s32, left, right, key_bias=bias)
            # a biased softmax over the few keys of a window is peaked: outputs leave [-1, 1], so the
            # output error is scaled by max(1, |reference|) as in the key-bias tests without a rotation
            check_against(o, lse, o_ref, lse_ref, lens, dtype, relative=True, label=f"rope+bias {dtype} ({left},{right})")


@pytest.mark.parametrize("name", ["c3_8k", "c5b_32k_local", "c4_16k_x3"])
def test_rope_named_workloads_sampled_rows(name):
    """Full-size launches of the 8K global, 32K local and 3 x 16K workloads with a rotation
    (base 160000 on global layers, 10000 on local ones); sampled rows against the oracle."""
    w = ALL_CONFIGS[name]
    lens, q, k, v = make_inputs(w)
    L, R = (-1, -1) if w.window < 0 else ((w.window - 1) // 2, w.window // 2)
    c32, s32, c64, s64 = tables(w.max_len, w.head_dim, base=160000.0 if w.window < 0 else 10000.0)
    o, lse = run_rope(q, k, v, lens, w.dtype, w.scale, c32, s32, L, R)
    rng = np.random.default_rng(95)
    for b in range(w.batch):
        n = int(lens[b])
        assert np.all(o[b, :, n:] == 0) and np.all(np.isneginf(lse[b, :, n:]))
        for h in (0, w.heads - 1):
            rows = np.unique(np.concatenate([rng.integers(0, n, 96), np.arange(0, 70), np.arange(n - 70, n)]))
            o_ref, lse_ref = attention_oracle_rope_rows(q, k, v, c64, s64, w.dtype, b, h, rows, n, w.scale, L, R)
            assert np.abs(o[b, h, rows] - o_ref).max() <= TOL[w.dtype]["max_abs"], (name, b, h)
            assert np.abs(lse[b, h, rows] - lse_ref).max() <= LSE_TOL, (name, b, h)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("D,B,H,N,lens", [(64, 2, 3, 700, [700, 333]), (32, 1, 2, 513, [500]), (128, 1, 2, 300, [300]),
                                          (64, 1, 12, 8192, [7900])])
def test_rope_rotation_ahead_of_the_call_with_lent_scratch(D, B, H, N, lens, dtype):
    """A global layer with a rotation and enough lent scratch rotates q and k once, ahead of the
    attention kernel: the same bits as the in-call rotation (the same rotation arithmetic and
    rounding, and a row's attention arithmetic does not depend on the tile shape), with and
    without a key bias, and from strided (packed) inputs; a scratch one byte short is ignored."""
    _, q, k, v = draw(9600 + D, B, H, N, D, dtype)
    c32, s32, c64, s64 = tables(N, D, base=160000.0)
    scale = 1.0 / np.sqrt(D)
    need = fa.fa_rope_scratch_bytes(B, H, N, D)
    assert need == 2 * B * H * N * D * 2
    # the pipelined kernel on both sides (a small plain call would take the key-split kernel, whose
    # summation order differs); the 8K case is left to the library: mixed shapes against 128 rows
    tun = fa.FA_TUNE_BM_128 if N <= 1024 else 0
    o_in, lse_in = run_rope(q, k, v, lens, dtype, scale, c32, s32, tuning=tun)
    o_sc, lse_sc = run_rope(q, k, v, lens, dtype, scale, c32, s32, tuning=tun, scratch_bytes=need)
    assert np.array_equal(o_in, o_sc) and np.array_equal(lse_in, lse_sc)
    o_short, lse_short = run_rope(q, k, v, lens, dtype, scale, c32, s32, tuning=tun, scratch_bytes=need - 1)
    assert np.array_equal(o_in, o_short) and np.array_equal(lse_in, lse_short)
    if N <= 1024:
        o_ref, lse_ref = attention_oracle_rope(q, k, v, c64, s64, dtype, lens, scale)
        check_against(o_sc, lse_sc, o_ref, lse_ref, lens, dtype, label=f"rope scratch D{D} {dtype}")
        rng = np.random.default_rng(96)
        bias = round_to_storage(rng.standard_normal((B, N)).astype(np.float32) * 0.5, dtype)
        bias[rng.random((B, N)) < 0.1] = -np.inf
        o_b, lse_b = run_rope(q, k, v, lens, dtype, scale, c32, s32, key_bias=bias, scratch_bytes=need)
        o_bref, lse_bref = attention_oracle_rope(q, k, v, c64, s64, dtype, lens, scale, key_bias=bias)
        check_against(o_b, lse_b, o_bref, lse_bref, lens, dtype, relative=True, label=f"rope scratch + bias D{D} {dtype}")
        # packed [B, N, 3, H, D] input: q and k are strided views
        qkv = np.stack([q.transpose(0, 2, 1, 3), k.transpose(0, 2, 1, 3), v.transpose(0, 2, 1, 3)], axis=2)   # [B, N, 3, H, D]
        dev = to_dev(np.ascontiguousarray(qkv), dtype)
        strides = (N * 3 * H * D, D, 3 * H * D)
        o = poison((B, H, N, D), dtype)
        lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
        scratch = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")
        fa.fa_fwd_ex(dtype=FA_DT[dtype], q=dev[:, :, 0], k=dev[:, :, 1], v=dev[:, :, 2], o=o, lse=lse,
                     seq_lens=torch.tensor(lens, dtype=torch.int32).cuda(), batch=B, heads=H, max_len=N, head_dim=D,
                     scale=scale, q_strides=strides, k_strides=strides, v_strides=strides,
                     rope_cos=torch.from_numpy(c32).cuda(), rope_sin=torch.from_numpy(s32).cuda(),
                     scratch=scratch, scratch_bytes=need, tuning=tun)
        torch.cuda.synchronize()
        assert np.array_equal(o.double().cpu().numpy(), o_sc) and np.array_equal(lse.double().cpu().numpy(), lse_sc)
