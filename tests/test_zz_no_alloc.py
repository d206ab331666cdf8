"""fa_fwd_ex_static_scratch (the entry point for callers that cannot allocate: its scratch is an
array inside the library's device image) against fa_fwd_ex with scratch lent by the caller, through
the C boundary: two calls in a row, the second with a smaller input; then the refusals."""
import numpy as np
import pytest
import torch

import paper_2603_12646_amd as fa
from oracle.rope_oracle import attention_oracle_rope_rows, rope_tables
from workloads import draw

from tests.gpu_util import FA_DT, LSE_TOL, TOL, poison, to_dev

pytestmark = pytest.mark.gpu


def call(q32, k32, v32, n, dtype, c32, s32, static, left=-1, right=-1):
    B, H, N, D = q32.shape
    q, k, v = to_dev(q32, dtype), to_dev(k32, dtype), to_dev(v32, dtype)
    o = poison((B, H, N, D), dtype)
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    sl = torch.tensor([n] * B, dtype=torch.int32).cuda()
    cd, sd = torch.from_numpy(c32).cuda(), torch.from_numpy(s32).cuda()
    need = fa.fa_rope_scratch_bytes(B, H, N, D)
    lent = None if static else torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")
    rc = fa.fa_fwd_ex(dtype=FA_DT[dtype], q=q, k=k, v=v, o=o, lse=lse, seq_lens=sl, batch=B, heads=H, max_len=N,
                      head_dim=D, scale=1.0 / np.sqrt(D), window_left=left, window_right=right, rope_cos=cd, rope_sin=sd,
                      scratch=lent, scratch_bytes=0 if static else need, static_scratch=static, check=False)
    torch.cuda.synchronize()
    return rc, o.double().cpu().numpy(), lse.double().cpu().numpy()


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_static_scratch_entry_point_matches_lent_scratch_on_two_calls_in_a_row(dtype):
    # first call: 8K tokens x 12 heads (25 MB of the 64 MB array); second: a smaller input, which
    # leaves most of what the first call wrote in the array untouched
    for (H, N, n, D, seed) in ((12, 8192, 7900, 64, 9700), (5, 1300, 1201, 128, 9701)):
        _, q, k, v = draw(seed, 1, H, N, D, dtype)
        cos, sin = rope_tables(N, D, base=160000.0)
        c32, s32 = cos.astype(np.float32), sin.astype(np.float32)
        rc_s, o_s, lse_s = call(q, k, v, n, dtype, c32, s32, static=True)
        rc_l, o_l, lse_l = call(q, k, v, n, dtype, c32, s32, static=False)
        assert rc_s == 0 and rc_l == 0
        assert np.array_equal(o_s, o_l) and np.array_equal(lse_s, lse_l)       # same kernels, same bits
        assert np.all(o_s[0, :, n:] == 0) and np.all(np.isneginf(lse_s[0, :, n:]))
        rows = np.unique(np.concatenate([np.random.default_rng(seed).integers(0, n, 40), [0, n - 1]]))
        for h in (0, H - 1):
            o_ref, lse_ref = attention_oracle_rope_rows(q, k, v, c32.astype(np.float64), s32.astype(np.float64), dtype,
                                                        0, h, rows, n, 1.0 / np.sqrt(D))
            assert np.abs(o_s[0, h, rows] - o_ref).max() <= TOL[dtype]["max_abs"]
            assert np.abs(lse_s[0, h, rows] - lse_ref).max() <= LSE_TOL


def test_static_scratch_entry_point_refuses_what_does_not_fit_and_ignores_what_needs_none():
    # 32K tokens x 12 heads x 64 would need 100 MB of scratch: refused, nothing enqueued, output untouched
    H, N, D = 12, 32768, 64
    assert fa.fa_rope_scratch_bytes(1, H, N, D) > fa.FA_STATIC_SCRATCH_BYTES
    q = torch.zeros((1, H, N, D), dtype=torch.float16, device="cuda")
    o = torch.full((1, H, N, D), float("nan"), dtype=torch.float16, device="cuda")
    tab = torch.ones((N, D // 2), dtype=torch.float32, device="cuda")
    rc = fa.fa_fwd_ex(dtype=fa.FA_DTYPE_F16, q=q, k=q, v=q, o=o, batch=1, heads=H, max_len=N, head_dim=D, scale=0.125,
                      rope_cos=tab, rope_sin=tab, static_scratch=True, check=False)
    torch.cuda.synchronize()
    assert rc == -10 and "scratch" in fa.fa_strerror(rc)
    assert bool(torch.isnan(o).all())
    # a local layer rotates inside the call and a call without a rotation has nothing to rotate: no scratch
    # is used, whatever the size, and the results are those of fa_fwd_ex
    _, q32, k32, v32 = draw(9702, 1, 12, 32768, 64, "bf16")
    cos, sin = rope_tables(32768, 64)
    c32, s32 = cos.astype(np.float32), sin.astype(np.float32)
    rc_s, o_s, lse_s = call(q32, k32, v32, 32768, "bf16", c32, s32, static=True, left=63, right=64)
    rc_l, o_l, lse_l = call(q32, k32, v32, 32768, "bf16", c32, s32, static=False, left=63, right=64)
    assert rc_s == 0 and rc_l == 0 and np.array_equal(o_s, o_l) and np.array_equal(lse_s, lse_l)


def test_static_scratch_call_recorded_into_a_hip_graph_and_replayed():
    """What the entry point is for: the rotation kernel and the attention kernel of a call that
    lends nothing, recorded into a HIP graph (the scratch address was looked up by the eager
    warm-up call on this GPU) and replayed with fresh inputs and eager work in between; every
    replay must reproduce the eager fa_fwd_ex result with lent scratch bit for bit."""
    H, N, n, D, dtype = 6, 2048, 1999, 64, "bf16"
    cos, sin = rope_tables(N, D, base=160000.0)
    cd, sd = torch.from_numpy(cos.astype(np.float32)).cuda(), torch.from_numpy(sin.astype(np.float32)).cuda()
    sl = torch.tensor([n], dtype=torch.int32).cuda()
    qd = torch.zeros((1, H, N, D), dtype=torch.bfloat16, device="cuda")
    kd, vd = torch.zeros_like(qd), torch.zeros_like(qd)
    o = poison((1, H, N, D), dtype)
    lse = torch.zeros((1, H, N), dtype=torch.float32, device="cuda")
    need = fa.fa_rope_scratch_bytes(1, H, N, D)
    lent = torch.empty(need, dtype=torch.uint8, device="cuda")

    def static_call(out, out_lse):
        fa.fa_fwd_ex(dtype=fa.FA_DTYPE_BF16, q=qd, k=kd, v=vd, o=out, lse=out_lse, seq_lens=sl, batch=1, heads=H, max_len=N,
                     head_dim=D, scale=0.125, rope_cos=cd, rope_sin=sd, static_scratch=True)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        static_call(o, lse)                     # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        static_call(o, lse)
    for rep in range(3):
        _, q, k, v = draw(9800 + rep, 1, H, N, D, dtype)
        qd.copy_(to_dev(q, dtype)); kd.copy_(to_dev(k, dtype)); vd.copy_(to_dev(v, dtype))
        o.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got_o, got_lse = o.clone(), lse.clone()
        o2, lse2 = poison((1, H, N, D), dtype), torch.zeros_like(lse)
        fa.fa_fwd_ex(dtype=fa.FA_DTYPE_BF16, q=qd, k=kd, v=vd, o=o2, lse=lse2, seq_lens=sl, batch=1, heads=H, max_len=N,
                     head_dim=D, scale=0.125, rope_cos=cd, rope_sin=sd, scratch=lent, scratch_bytes=need)
        torch.cuda.synchronize()
        assert torch.equal(got_o, o2) and torch.equal(got_lse, lse2), f"replay {rep} differs from the eager call"
