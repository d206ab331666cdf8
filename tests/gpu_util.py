"""Helpers for the GPU parity tests: move seeded inputs to the device, call the
C boundary through the binding, bring results back as float64."""
import numpy as np
import torch

import paper_2603_12646_amd as fa

TORCH_DT = {"fp16": torch.float16, "bf16": torch.bfloat16}
FA_DT = {"fp16": fa.FA_DTYPE_F16, "bf16": fa.FA_DTYPE_BF16}

# spec tolerances against the fp64 oracle, valid rows only
TOL = {"fp16": dict(max_abs=2e-3, mean_abs=2e-4), "bf16": dict(max_abs=1e-2, mean_abs=1e-3)}
LSE_TOL = 1e-3


def lse_tol(lse_ref):
    """Allowed |lse - reference|: 1e-3 absolute.  lse is an fp32 number, so where the
    reference is so large that 1e-3 is below eight fp32 spacings at its magnitude (|lse| in
    the thousands: ramps of huge scores) the bound is eight spacings instead; for the
    |lse| of ordinary workloads (below 1000) this is 1e-3 exactly."""
    a = np.abs(np.asarray(lse_ref, dtype=np.float64))
    spacing = np.spacing(a.astype(np.float32)).astype(np.float64)
    return np.maximum(LSE_TOL, 8.0 * spacing)


def to_dev(x32, dtype):
    """float32 numpy array of storage-representable values -> device tensor (exact)."""
    return torch.from_numpy(x32).to(TORCH_DT[dtype]).cuda()


def poison(shape, dtype):
    """Output buffers start as NaN so rows the kernel forgets to write are noticed."""
    return torch.full(shape, float("nan"), dtype=TORCH_DT[dtype], device="cuda")


def run_simple(q32, k32, v32, lens, dtype, scale, window=-1, want_lse=True, stream=None, tuning=0):
    """The plain entry points; with a nonzero `tuning` the same call goes through fa_fwd_ex
    (window width mapped to left/right as the plain entry points do) so that a kernel shape
    can be forced."""
    B, H, N, D = q32.shape
    q, k, v = to_dev(q32, dtype), to_dev(k32, dtype), to_dev(v32, dtype)
    o = poison((B, H, N, D), dtype)
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    sl = None if lens is None else torch.as_tensor(np.asarray(lens), dtype=torch.int32).cuda()
    if tuning:
        left, right = (-1, -1) if window < 0 else ((window - 1) // 2, window // 2)
        fa.fa_fwd_ex(dtype=FA_DT[dtype], q=q, k=k, v=v, o=o, lse=lse, seq_lens=sl, batch=B, heads=H, max_len=N,
                     head_dim=D, scale=scale, window_left=left, window_right=right, tuning=tuning, stream=stream)
    else:
        fn = fa.fa_fwd if dtype == "fp16" else fa.fa_fwd_bf16
        fn(q, k, v, o, lse, B, H, sl, N, D, scale, window, stream=stream)
    torch.cuda.synchronize()
    return o.double().cpu().numpy(), (None if lse is None else lse.double().cpu().numpy())


def run_ex(q32, k32, v32, lens, dtype, scale, left=-1, right=-1, tuning=0, want_lse=True, key_bias=None):
    """key_bias: None or float32 [B, N] of storage-representable values (inf allowed)."""
    B, H, N, D = q32.shape
    q, k, v = to_dev(q32, dtype), to_dev(k32, dtype), to_dev(v32, dtype)
    o = poison((B, H, N, D), dtype)
    lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    sl = None if lens is None else torch.as_tensor(np.asarray(lens), dtype=torch.int32).cuda()
    kb = None if key_bias is None else to_dev(np.ascontiguousarray(key_bias, dtype=np.float32), dtype)
    fa.fa_fwd_ex(dtype=FA_DT[dtype], q=q, k=k, v=v, o=o, lse=lse, seq_lens=sl, batch=B, heads=H,
                 max_len=N, head_dim=D, scale=scale, window_left=left, window_right=right,
                 tuning=tuning, key_bias=kb)
    torch.cuda.synchronize()
    return o.double().cpu().numpy(), (None if lse is None else lse.double().cpu().numpy())


def check_against(o_gpu, lse_gpu, o_ref, lse_ref, lens, dtype, relative=False, label=""):
    """Element-by-element comparison on valid rows; exact zeros / -inf on padded rows."""
    B, H, N, D = o_ref.shape
    tol = TOL[dtype]
    errs = []
    for b in range(B):
        n = N if lens is None else int(min(max(int(lens[b]), 0), N))
        if n < N:
            assert np.all(o_gpu[b, :, n:] == 0), f"{label}: padded rows of o not zero (b={b})"
            if lse_gpu is not None:
                assert np.all(np.isneginf(lse_gpu[b, :, n:])), f"{label}: padded lse not -inf (b={b})"
        if n == 0:
            continue
        d = np.abs(o_gpu[b, :, :n] - o_ref[b, :, :n])
        if relative:
            d = d / np.maximum(1.0, np.abs(o_ref[b, :, :n]))
        assert np.all(np.isfinite(o_gpu[b, :, :n])), f"{label}: non-finite output (b={b})"
        errs.append(d.ravel())
        if lse_gpu is not None:
            fin = np.isfinite(lse_ref[b, :, :n])
            assert np.array_equal(fin, np.isfinite(lse_gpu[b, :, :n])), f"{label}: lse finiteness (b={b})"
            # lse is fp32: absolute bound whatever `relative` says (see lse_tol)
            dl = np.abs(lse_gpu[b, :, :n][fin] - lse_ref[b, :, :n][fin])
            excess = dl - lse_tol(lse_ref[b, :, :n][fin])
            assert dl.size == 0 or excess.max() <= 0, f"{label}: lse err {dl.max():.3e} (b={b})"
    if errs:
        e = np.concatenate(errs)
        assert e.max() <= tol["max_abs"], f"{label}: max-abs {e.max():.3e} > {tol['max_abs']}"
        assert e.mean() <= tol["mean_abs"], f"{label}: mean-abs {e.mean():.3e} > {tol['mean_abs']}"
        return float(e.max()), float(e.mean())
    return 0.0, 0.0
