"""GPU parity on randomly drawn (but seeded, always valid) argument combinations: head_dim,
storage type, batch, heads, length, sequence lengths, window form, scale sign, tuning word
and an optional key bias with excluded keys, each against the fp64 oracle."""
import numpy as np
import pytest

from oracle.attention_oracle import attention_oracle
from workloads import draw, round_to_storage

from tests.gpu_util import check_against, run_ex

pytestmark = pytest.mark.gpu


def draw_case(rng, case):
    D = int(rng.choice([32, 64, 64, 64, 128]))
    dtype = str(rng.choice(["fp16", "bf16"]))
    B, H = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    N = int(rng.choice([rng.integers(1, 70), rng.integers(70, 300), rng.integers(300, 900)]))
    lens = [int(rng.integers(0, N + 1)) if rng.random() < 0.7 else N for _ in range(B)]
    if rng.random() < 0.3:
        lens = None
    mode = rng.random()
    if mode < 0.4:
        left, right = -1, -1
    elif mode < 0.6:
        left, right = 63, 64
    elif mode < 0.8:
        left, right = int(rng.integers(0, 200)), int(rng.integers(0, 200))
    elif mode < 0.9:
        left, right = int(rng.integers(0, 100)), -1
    else:
        left, right = -1, int(rng.integers(0, 100))
    scale = float(rng.choice([1.0 / np.sqrt(D), 0.3, -0.1, 0.02]))
    tuning = int(rng.choice([0, 0, 0x1, 0x2, 0x3, 0x20, 0x100, 0x201, 0x103]))
    bias = None
    if rng.random() < 0.4:
        # bf16 gets a milder bias so that outputs stay below 1 in magnitude
        bias = round_to_storage((rng.standard_normal((B, N)) * (1.0 if dtype == "fp16" else 0.4)).astype(np.float32), dtype)
        if rng.random() < 0.5:
            bias[rng.random((B, N)) < 0.15] = -np.inf
    gain = 1.0 if dtype == "bf16" else float(rng.choice([1.0, 1.5]))
    _, q, k, v = draw(10000 + case, B, H, N, D, dtype, qk_gain=gain)
    label = (f"case {case}: D={D} {dtype} B={B} H={H} N={N} lens={lens} window=({left},{right}) scale={scale:.3f} "
             f"tuning={tuning:#x} bias={'yes' if bias is not None else 'no'}")
    return dict(q=q, k=k, v=v, lens=lens, dtype=dtype, scale=scale, left=left, right=right, tuning=tuning,
                bias=bias, label=label)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_argument_combinations(seed):
    rng = np.random.default_rng(seed)
    for case in range(40):
        c = draw_case(rng, 100 * seed + case)
        o_ref, lse_ref = attention_oracle(c["q"], c["k"], c["v"], c["lens"], c["scale"], c["left"], c["right"],
                                          key_bias=c["bias"])
        o, lse = run_ex(c["q"], c["k"], c["v"], c["lens"], c["dtype"], c["scale"], c["left"], c["right"],
                        tuning=c["tuning"], key_bias=c["bias"])
        check_against(o, lse, o_ref, lse_ref, c["lens"], c["dtype"], relative=True, label=c["label"])
