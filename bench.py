#!/usr/bin/env python3
"""Benchmark of the flash-attention forward hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu] [--no-others]

A step is one fa_fwd call (tile schedule, QK^T, mask, online softmax, PV,
epilogue: the whole path) over one synthetic batch already resident in HBM.
Prints ONE JSON line.  `value` is algorithmic TFLOP/s: 4 * head_dim * heads *
(number of visible (query, key) pairs) per call, padded and out-of-window pairs
counting as zero work.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense fp16 / bf16 matrix peak
HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
HEADLINE = "c3_8k"


def visible_pairs(lens, left, right):
    """Number of (query, key) pairs the mask leaves visible, summed over the batch (per head)."""
    total = 0
    for n in lens:
        n = int(n)
        if n <= 0:
            continue
        i = np.arange(n, dtype=np.int64)
        lo = np.zeros(n, np.int64) if left < 0 else np.maximum(0, i - left)
        hi = np.full(n, n - 1, np.int64) if right < 0 else np.minimum(n - 1, i + right)
        total += int((hi - lo + 1).sum())
    return total


def window_lr(window):
    return (-1, -1) if window < 0 else ((window - 1) // 2, window // 2)


def algorithmic_work(w, lens):
    L, R = window_lr(w.window)
    pairs = visible_pairs(lens, L, R)
    flops = 4.0 * w.head_dim * w.heads * pairs
    rows = int(sum(max(0, int(n)) for n in lens))
    nbytes = 2 * 4 * w.heads * w.head_dim * rows + 4 * w.heads * rows
    return flops, nbytes


def read_traffic(name):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if present."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split("#")[0].split()
        if len(parts) >= 3 and parts[0] == name:
            return float(parts[1]) + float(parts[2])
    return None


PRECONDITION_MS = 60.0      # untimed calls of the same workload before the warm-up calls


def gpu_time(w, lens, q, k, v, steps, warmup, tuning=0, precondition_ms=PRECONDITION_MS):
    """Times exactly `steps` calls after `warmup` untimed ones.  Before the warm-up calls the same
    call is repeated, untimed, for about precondition_ms of wall time: a GPU that has idled for
    a few milliseconds (loading inputs, the host-side oracle leg) sits at a low clock and needs
    some 25 launches of this size to come back up (measured: the first 20 calls after an idle
    half-second take 0.25-0.26 ms each, every later hundred 0.220 ms), so a figure taken right
    after 5 warm-up calls measures the ramp, not the kernel."""
    import torch
    import paper_2603_12646_amd as fa

    tdt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
    qd, kd, vd = (torch.from_numpy(x).to(tdt).cuda() for x in (q, k, v))
    o = torch.empty_like(qd)
    lse = torch.empty((w.batch, w.heads, w.max_len), dtype=torch.float32, device="cuda")
    sl = torch.from_numpy(np.asarray(lens, dtype=np.int32)).cuda()
    fn = fa.fa_fwd if w.dtype == "fp16" else fa.fa_fwd_bf16

    L, R = window_lr(w.window)
    dt = fa.FA_DTYPE_F16 if w.dtype == "fp16" else fa.FA_DTYPE_BF16

    def step():
        if tuning:   # sweeps only: force a kernel shape through the superset entry point
            fa.fa_fwd_ex(dtype=dt, q=qd, k=kd, v=vd, o=o, lse=lse, seq_lens=sl, batch=w.batch,
                         heads=w.heads, max_len=w.max_len, head_dim=w.head_dim, scale=w.scale,
                         window_left=L, window_right=R, tuning=tuning)
        else:
            fn(qd, kd, vd, o, lse, w.batch, w.heads, sl, w.max_len, w.head_dim, w.scale, w.window)

    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < precondition_ms:
        for _ in range(8):
            step()
        torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    start.record()          # same stream the kernels are launched on (torch's current stream)
    for _ in range(steps):
        step()
    stop.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = start.elapsed_time(stop)
    del qd, kd, vd, o, lse
    return wall_ms / steps, ev_ms / steps


def per_call_times(w, lens, q, k, v, calls=50, warmup=10, flush_cache=False):
    """One HIP event pair per call, on the stream the kernel is launched on.  Returns (median ms,
    min ms).  flush_cache: between calls a 1 GiB buffer is overwritten, which evicts the
    tensors from the 256 MB last-level cache, so every call reads its inputs from HBM."""
    import torch
    import paper_2603_12646_amd as fa

    tdt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
    qd, kd, vd = (torch.from_numpy(x).to(tdt).cuda() for x in (q, k, v))
    o = torch.empty_like(qd)
    lse = torch.empty((w.batch, w.heads, w.max_len), dtype=torch.float32, device="cuda")
    sl = torch.from_numpy(np.asarray(lens, dtype=np.int32)).cuda()
    fn = fa.fa_fwd if w.dtype == "fp16" else fa.fa_fwd_bf16
    junk = torch.empty(1 << 30, dtype=torch.uint8, device="cuda") if flush_cache else None
    times = []
    for i in range(warmup + calls):
        if junk is not None:
            junk.fill_(i & 0xFF)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        fn(qd, kd, vd, o, lse, w.batch, w.heads, sl, w.max_len, w.head_dim, w.scale, w.window)
        stop.record()
        stop.synchronize()
        if i >= warmup:
            times.append(start.elapsed_time(stop))
    del qd, kd, vd, o, lse, junk
    return float(np.median(times)), float(np.min(times))


def cold_cache_times(w, lens, q, k, v, reps=20):
    """The bandwidth-bound local layer with the last-level cache emptied before every call.
    Two ways of emptying it, both timed as a loop of (flush, call) pairs minus the same loop of
    flushes alone, all on one stream with no host synchronisation inside the loops:
      * "read": a reduction over 1 GiB reads the cache full of CLEAN lines, so the call's
        inputs come from HBM and evicting costs nothing -- the kernel's own cold-cache time;
      * "write": a fill of 1 GiB leaves the cache full of DIRTY lines, so the call also pays
        for writing 256 MB of somebody else's data back to HBM while it reads its inputs.
    Returns {"read": ms, "write": ms}."""
    import torch
    import paper_2603_12646_amd as fa

    tdt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
    qd, kd, vd = (torch.from_numpy(x).to(tdt).cuda() for x in (q, k, v))
    o = torch.empty_like(qd)
    lse = torch.empty((w.batch, w.heads, w.max_len), dtype=torch.float32, device="cuda")
    sl = torch.from_numpy(np.asarray(lens, dtype=np.int32)).cuda()
    fn = fa.fa_fwd if w.dtype == "fp16" else fa.fa_fwd_bf16
    junk = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")

    def call(i):
        fn(qd, kd, vd, o, lse, w.batch, w.heads, sl, w.max_len, w.head_dim, w.scale, w.window)

    def loop_ms(body):
        torch.cuda.synchronize()
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for i in range(reps):
            body(i)
        stop.record()
        torch.cuda.synchronize()
        return start.elapsed_time(stop) / reps

    out = {}
    for mode, flush in (("read", lambda i: torch.sum(junk, dim=0, keepdim=True, out=sink)),
                        ("write", lambda i: junk.fill_(float(i)))):
        loop_ms(flush)                                     # untimed: first use of the flush kernel
        loop_ms(lambda i: (flush(i), call(i)))
        diffs = []
        for _ in range(5):
            alone = loop_ms(flush)
            both = loop_ms(lambda i: (flush(i), call(i)))
            diffs.append(both - alone)
        out[mode] = float(np.median(diffs))
    del qd, kd, vd, o, lse, junk
    return out


def layer_sequence_time(w, lens, q, k, v, layers=22, every=3, window=128, reps=5):
    """Attention calls of one pass through a ModernBERT-shaped encoder (paper Sec. 2.4 and
    4.1.3: local layers with a 128-token window, every third layer global): `layers` calls
    back to back on the workload's tensors, global when layer % every == 0.  Returns
    (ms per pass launched call by call, ms per pass replayed from a HIP graph, number of
    global layers)."""
    import torch
    import paper_2603_12646_amd as fa

    tdt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
    qd, kd, vd = (torch.from_numpy(x).to(tdt).cuda() for x in (q, k, v))
    o = torch.empty_like(qd)
    lse = torch.empty((w.batch, w.heads, w.max_len), dtype=torch.float32, device="cuda")
    sl = torch.from_numpy(np.asarray(lens, dtype=np.int32)).cuda()
    fn = fa.fa_fwd if w.dtype == "fp16" else fa.fa_fwd_bf16
    n_global = len([l for l in range(layers) if l % every == 0])

    def one_pass():
        for layer in range(layers):
            fn(qd, kd, vd, o, lse, w.batch, w.heads, sl, w.max_len, w.head_dim, w.scale,
               -1 if layer % every == 0 else window)

    one_pass()
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(reps):
        one_pass()
    stop.record()
    torch.cuda.synchronize()
    eager_ms = start.elapsed_time(stop) / reps

    # the same 22 launches recorded once into a HIP graph and replayed: no host work between
    # the kernels (the library allocates nothing and never synchronises, so it can be captured)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_pass()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_pass()
    graph.replay()
    torch.cuda.synchronize()
    start.record()
    for _ in range(reps):
        graph.replay()
    stop.record()
    torch.cuda.synchronize()
    graph_ms = start.elapsed_time(stop) / reps
    del graph
    return eager_ms, graph_ms, n_global


def three_sessions_time(reps=10):
    """The paper deploys three classifier sessions side by side (Sec. 4.1.1, 4.1.3): the three
    sequences of the 16K workload as three independent calls on three streams, against the
    same three sequences as one batched call.  Returns (ms concurrent, ms batched)."""
    import torch
    import paper_2603_12646_amd as fa
    from workloads import ALL_CONFIGS, make_inputs

    w = ALL_CONFIGS["c4_16k_x3"]
    lens, q, k, v = make_inputs(w)
    tdt = torch.bfloat16
    qd, kd, vd = (torch.from_numpy(x).to(tdt).cuda() for x in (q, k, v))
    o = torch.empty_like(qd)
    lse = torch.empty((w.batch, w.heads, w.max_len), dtype=torch.float32, device="cuda")
    sl = torch.from_numpy(np.asarray(lens, dtype=np.int32)).cuda()
    streams = [torch.cuda.Stream() for _ in range(w.batch)]     # default priority

    def concurrent():
        for b, st in enumerate(streams):
            with torch.cuda.stream(st):
                fa.fa_fwd_bf16(qd[b:b + 1], kd[b:b + 1], vd[b:b + 1], o[b:b + 1], lse[b:b + 1], 1, w.heads,
                               sl[b:b + 1], w.max_len, w.head_dim, w.scale, w.window)

    def batched():
        fa.fa_fwd_bf16(qd, kd, vd, o, lse, w.batch, w.heads, sl, w.max_len, w.head_dim, w.scale, w.window)

    out = []
    for fn, multi in ((concurrent, True), (batched, False)):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        out.append((time.perf_counter() - t0) * 1e3 / reps)
    return out[0], out[1]


def concurrent_requests_time(levels=(10, 20), reps=20):
    """The paper's steady state after prompt compression is many 512-token requests in flight
    at once (Sec. 5, concurrency table: C = 10 and 20): C independent calls of the 512-token
    workload's shape, (a) each on a stream of its own, (b) back to back on one stream, (c) as
    one batched call.  Host launch time is part of all three.  Returns {C: {...ms}}."""
    import torch
    import paper_2603_12646_amd as fa
    from workloads import ALL_CONFIGS, make_inputs

    w = ALL_CONFIGS["c1_512"]
    _, q, k, v = make_inputs(w)
    out = {}
    for c in levels:
        tdt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
        fn = fa.fa_fwd if w.dtype == "fp16" else fa.fa_fwd_bf16
        qd, kd, vd = (torch.from_numpy(np.repeat(x, c, axis=0)).to(tdt).cuda() for x in (q, k, v))
        o = torch.empty_like(qd)
        lse = torch.empty((c, w.heads, w.max_len), dtype=torch.float32, device="cuda")
        sl = torch.full((c,), w.max_len, dtype=torch.int32, device="cuda")
        streams = [torch.cuda.Stream() for _ in range(c)]   # default priority

        views = [(qd[b:b + 1], kd[b:b + 1], vd[b:b + 1], o[b:b + 1], lse[b:b + 1], sl[b:b + 1]) for b in range(c)]

        def one(b, stream=None):
            qb, kb, vb, ob, lb, sb = views[b]
            fn(qb, kb, vb, ob, lb, 1, w.heads, sb, w.max_len, w.head_dim, w.scale, w.window, stream=stream)

        def own_streams():
            for b, st in enumerate(streams):
                one(b, st)

        def one_stream():
            for b in range(c):
                one(b)

        def batched():
            fn(qd, kd, vd, o, lse, c, w.heads, sl, w.max_len, w.head_dim, w.scale, w.window)

        res = {}
        for name, f in (("own_streams_ms", own_streams), ("one_stream_ms", one_stream), ("one_batched_call_ms", batched)):
            f()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                f()
            torch.cuda.synchronize()
            res[name] = round((time.perf_counter() - t0) * 1e3 / reps, 4)
        out[str(c)] = res
        del qd, kd, vd, o, lse
    return out


def co_location_time(reps=30):
    """The router shares its GPU with the LLM serving instances (paper Sec. 1, Sec. 4.1.1): the
    8K workload on a stream that may use all 256 compute units, and on one limited to 128.
    Returns {units: ms per call}, host launch time included."""
    import torch
    import paper_2603_12646_amd as fa
    from paper_2603_12646_amd.cu_mask import CuMaskedStream, first_units
    from workloads import ALL_CONFIGS, make_inputs

    w = ALL_CONFIGS["c3_8k"]
    lens, q, k, v = make_inputs(w)
    qd, kd, vd = (torch.from_numpy(x).to(torch.float16).cuda() for x in (q, k, v))
    o = torch.empty_like(qd)
    lse = torch.empty((w.batch, w.heads, w.max_len), dtype=torch.float32, device="cuda")
    sl = torch.from_numpy(np.asarray(lens, dtype=np.int32)).cuda()
    torch.cuda.synchronize()
    out = {}
    for units in (256, 128):
        with CuMaskedStream(first_units(units)) as ms:
            def call():
                fa.fa_fwd(qd, kd, vd, o, lse, w.batch, w.heads, sl, w.max_len, w.head_dim, w.scale, w.window,
                          stream=ms.handle)
            for _ in range(3):
                call()
            ms.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                call()
            ms.synchronize()
            out[str(units)] = round((time.perf_counter() - t0) * 1e3 / reps, 4)
    return out


def rotary_time(names=("c3_8k", "c5a_32k_global", "c5b_32k_local"), reps=30):
    """The same launches with the rotary position embedding of q and k done inside the call (the
    paper's encoder uses rotary embeddings, Sec. 2.4): ms per call with and without the rotation.
    Angles: base 160000 on global layers, 10000 on local ones, no rescaling (the paper gives no
    constants; the cost does not depend on them)."""
    import torch
    import paper_2603_12646_amd as fa
    from workloads import ALL_CONFIGS, make_inputs

    out = {}
    for name in names:
        w = ALL_CONFIGS[name]
        lens, q, k, v = make_inputs(w)
        tdt = torch.float16 if w.dtype == "fp16" else torch.bfloat16
        qd, kd, vd = (torch.from_numpy(x).to(tdt).cuda() for x in (q, k, v))
        o = torch.empty_like(qd)
        lse = torch.empty((w.batch, w.heads, w.max_len), dtype=torch.float32, device="cuda")
        sl = torch.from_numpy(np.asarray(lens, dtype=np.int32)).cuda()
        half = w.head_dim // 2
        inv_freq = (160000.0 if w.window < 0 else 10000.0) ** (-2.0 * np.arange(half) / w.head_dim)
        ang = np.arange(w.max_len)[:, None] * inv_freq[None, :]
        cos = torch.from_numpy(np.cos(ang).astype(np.float32)).cuda()
        sin = torch.from_numpy(np.sin(ang).astype(np.float32)).cuda()
        L, R = window_lr(w.window)
        dt = fa.FA_DTYPE_F16 if w.dtype == "fp16" else fa.FA_DTYPE_BF16
        res = {}
        need = fa.fa_rope_scratch_bytes(w.batch, w.heads, w.max_len, w.head_dim)
        scratch = torch.empty(need, dtype=torch.uint8, device="cuda") if w.window < 0 else None
        legs = [("ms_plain", (None, None), None), ("ms_with_rotation", (cos, sin), None)]
        if scratch is not None:     # global layer: q and k rotated once ahead of the call, in lent scratch
            legs.append(("ms_with_rotation_ahead_in_lent_scratch", (cos, sin), scratch))
        for label, tables, scr in legs:
            def call():
                fa.fa_fwd_ex(dtype=dt, q=qd, k=kd, v=vd, o=o, lse=lse, seq_lens=sl, batch=w.batch, heads=w.heads,
                             max_len=w.max_len, head_dim=w.head_dim, scale=w.scale, window_left=L, window_right=R,
                             rope_cos=tables[0], rope_sin=tables[1], scratch=scr, scratch_bytes=need if scr is not None else 0)
            t_pre = time.perf_counter()
            while (time.perf_counter() - t_pre) * 1e3 < PRECONDITION_MS:     # as in gpu_time
                for _ in range(8):
                    call()
                torch.cuda.synchronize()
            start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            start.record()
            for _ in range(reps):
                call()
            stop.record()
            torch.cuda.synchronize()
            res[label] = round(start.elapsed_time(stop) / reps, 4)
        out[name] = res
        del qd, kd, vd, o, lse, cos, sin, scratch
    return out


def measured_ceilings():
    """What this machine sustains with nothing but matrix-core instructions (zero and random
    operands) and with a plain copy: the program built from csrc/ceilings.hip, run as a child
    process.  Context for roofline.frac, which is quoted against the published peaks."""
    import subprocess
    exe = os.path.join(ROOT, "paper_2603_12646_amd", "fa_ceilings")
    if not os.path.exists(exe):
        return None
    try:
        r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
        return json.loads(r.stdout.strip().splitlines()[-1]) if r.returncode == 0 else None
    except Exception:
        return None


def cpu_baseline(w, lens, q, k, v, budget_s=15.0):
    """The fp64 oracle as it stands, timed on this host on whole (batch, head) slices
    until about budget_s seconds have been spent."""
    from oracle.attention_oracle import attention_oracle_rows
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    L, R = window_lr(w.window)
    done_pairs, t_used, slices = 0, 0.0, 0
    rows_per_slice = 8192
    for b in range(w.batch):
        n = int(lens[b])
        if n <= 0:
            continue
        for h in range(w.heads):
            rows = np.arange(0, min(n, rows_per_slice))
            t0 = time.perf_counter()
            for r0 in range(0, len(rows), 256):
                attention_oracle_rows(q, k, v, b, h, rows[r0:r0 + 256], n, w.scale, L, R)
            t_used += time.perf_counter() - t0
            i = rows
            lo = np.zeros_like(i) if L < 0 else np.maximum(0, i - L)
            hi = np.full_like(i, n - 1) if R < 0 else np.minimum(n - 1, i + R)
            done_pairs += int((hi - lo + 1).sum())
            slices += 1
            if t_used >= budget_s:
                break
        if t_used >= budget_s:
            break
    flops = 4.0 * w.head_dim * done_pairs
    cpu_model = ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                cpu_model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {
        "value": flops / t_used / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
        "os_cpu_count": os.cpu_count(), "cpu_model": cpu_model,
        "sample": f"first min(n, {rows_per_slice}) query rows of {slices} (batch, head) slices of {w.name}, "
                  f"full key range, {t_used:.1f} s of oracle time; algorithmic flops of those rows / time",
        "seconds": t_used,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-others", action="store_true", help="time only the named workload")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured matrix-core / copy ceilings (a child process of about a second)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise copy of 256 MiB three times, so a rocprofv3 "
                         "--pmc run of this command has a kernel of known traffic to scale against")
    ap.add_argument("--precondition-ms", type=float, default=PRECONDITION_MS,
                    help="untimed calls of the workload for this long before the warm-up calls "
                         "(0 for short profiler runs that should hold few dispatches)")
    ap.add_argument("--tuning", type=lambda x: int(x, 0), default=0,
                    help="FA_TUNE_* bits forwarded to fa_fwd_ex (sweeps); 0 = library's choice")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(the path would shard by (batch, head) with no exchange)", file=sys.stderr)
        sys.exit(2)

    import torch
    from workloads import ALL_CONFIGS, make_inputs
    import paper_2603_12646_amd as fa

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        sys.exit(3)
    fa.load_library()
    torch.cuda.set_device(0)

    w = ALL_CONFIGS[args.workload]
    lens, q, k, v = make_inputs(w)
    flops, nbytes = algorithmic_work(w, lens)
    wall_ms, ev_ms = gpu_time(w, lens, q, k, v, args.steps, args.warmup, args.tuning, args.precondition_ms)
    # the reported rate is taken from the HIP-event time of the timed region (the host's wall
    # clock around the same region, which adds the final synchronisation, is reported beside it)
    tflops = flops / (ev_ms * 1e-3) / 1e12
    hbm_bound = w.window >= 0
    if hbm_bound:
        roof = {"bound": "hbm", "achieved": nbytes / (ev_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": flops / (ev_ms * 1e-3) / 1e12, "peak": MFMA_PEAK_TFLOPS,
                "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = read_traffic(w.name)
    roof["kernel_ms"] = ev_ms
    med_ms, min_ms = per_call_times(w, lens, q, k, v)
    roof["kernel_ms_median_of_single_calls"] = med_ms   # one event pair per call: includes launch gaps
    roof["kernel_ms_min_of_single_calls"] = min_ms
    roof["algorithmic_flops"] = flops
    roof["algorithmic_bytes"] = nbytes

    out = {
        "metric": "attention fwd TFLOP/s (algorithmic flops; % of MFMA peak in roofline.frac); ms per call in ms_per_step",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ev_ms, "ms_per_step_host_wall_clock": wall_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "heads": w.heads, "max_len": w.max_len,
                   "head_dim": w.head_dim, "seq_lens": [int(x) for x in lens][:8], "window": w.window,
                   "scale": w.scale, "qk_gain": w.qk_gain, "tuning": args.tuning,
                   "preconditioning_ms": args.precondition_ms},
        "roofline": roof,
    }

    if not args.no_ceilings:
        ceil = measured_ceilings()
        if ceil is not None and not hbm_bound:
            # the same launches on all-zero tensors: identical instruction stream, but no operand
            # bits toggle, so the chip holds a higher clock -- what the kernel's structure sustains
            # when power is not the limit (context only; never the reported value)
            z = np.zeros_like(q)
            _, zms = gpu_time(w, lens, z, z, z, max(10, args.steps // 4), 3, args.tuning)
            ceil["same_kernel_zero_data_tflops"] = flops / (zms * 1e-3) / 1e12
            del z
        out["ceilings"] = ceil
        if ceil and not hbm_bound:
            key = "mfma_f16_random_tflops" if w.dtype == "fp16" else "mfma_bf16_random_tflops"
            roof["frac_of_measured_random_data_ceiling"] = roof["achieved"] / ceil[key]
            # the kernels' own instruction mix (matrix products + softmax vector work, operands
            # in registers, no memory traffic) as the same program measured it
            mkey = f"mix_{'f16' if w.dtype == 'fp16' else 'bf16'}_d{w.head_dim}_tflops"
            if ceil.get(mkey):
                roof["frac_of_measured_mix_ceiling"] = roof["achieved"] / ceil[mkey]
        elif ceil:
            roof["frac_of_measured_copy"] = roof["achieved"] / ceil["copy_gbs"]

    if args.calibrate_copy:
        src = torch.ones(128 * 1024 * 1024, dtype=torch.float16, device="cuda")   # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)        # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        out["config"]["calibrate_copy_bytes_each_way"] = src.numel() * 2
        del src, dst

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, lens, q, k, v)
    del q, k, v

    if not args.no_others:
        others = {}
        for name, ow in ALL_CONFIGS.items():
            if name == w.name:
                continue
            ol, oq, ok_, ov = make_inputs(ow)
            of, ob = algorithmic_work(ow, ol)
            steps = max(10, min(args.steps, 100))
            wms, ems = gpu_time(ow, ol, oq, ok_, ov, steps, max(3, min(args.warmup, 10)), args.tuning)
            others[name] = {"ms_per_call": ems, "tflops": of / (ems * 1e-3) / 1e12,
                            "frac_mfma_peak": of / (ems * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                            "algorithmic_gbs": ob / (ems * 1e-3) / 1e9, "dtype": ow.dtype, "head_dim": ow.head_dim}
            if ow.window >= 0:
                # bandwidth-bound layer: back-to-back calls find part of their 200 MB in the
                # last-level cache; also time it with the cache emptied before every call
                cold = cold_cache_times(ow, ol, oq, ok_, ov)
                others[name]["ms_per_call_cold_cache_clean"] = cold["read"]
                others[name]["algorithmic_gbs_cold_cache_clean"] = ob / (cold["read"] * 1e-3) / 1e9
                others[name]["ms_per_call_cold_cache_dirty"] = cold["write"]
                others[name]["algorithmic_gbs_cold_cache_dirty"] = ob / (cold["write"] * 1e-3) / 1e9
            del oq, ok_, ov
        out["config"]["other_workloads"] = others
        # one encoder pass worth of attention calls (22 layers, every third global) at 8K and 32K
        seqs = {}
        for name in ("c1_512", "c3_8k", "c5a_32k_global"):
            lw = ALL_CONFIGS[name]
            ll, lq, lk, lv = make_inputs(lw)
            ms, graph_ms, n_global = layer_sequence_time(lw, ll, lq, lk, lv)
            seqs[name] = {"layers": 22, "global_layers": n_global, "local_window": 128, "ms_per_pass": ms,
                          "ms_per_pass_hip_graph": graph_ms}
            del lq, lk, lv
        out["config"]["layer_sequence"] = seqs
        conc_ms, batch_ms = three_sessions_time()
        out["config"]["three_sessions_16k"] = {"three_streams_ms": conc_ms, "one_batched_call_ms": batch_ms}
        out["config"]["concurrent_requests_512"] = concurrent_requests_time()
        out["config"]["co_location_8k_ms_by_compute_units"] = co_location_time()
        out["config"]["rotary_embedding_in_call"] = rotary_time()

    print(json.dumps(out))


if __name__ == "__main__":
    main()
