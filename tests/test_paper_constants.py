"""The few numbers the paper prints about the attention operator, checked
against the oracle's conventions and the workload shapes."""
import pathlib

import numpy as np

from oracle.attention_oracle import attention_oracle, additive_bias_variant, window_from_width
from workloads import CONFIGS


def load():
    out = {}
    for line in (pathlib.Path(__file__).parent / "golden" / "paper_constants.txt").read_text().splitlines():
        line = line.split("#")[0].strip()
        if line:
            key, val = line.split()
            out[key] = float(val)
    return out


def test_window_constants():
    c = load()
    L, R = window_from_width(int(c["local_window_width"]))
    assert (L, R) == (c["local_window_left"], c["local_window_right"])
    assert window_from_width(-1) == (c["global_window_left"], c["global_window_right"])
    assert CONFIGS["c5b_32k_local"].window == c["local_window_width"]
    # an interior row of a local layer sees exactly `width` keys
    N = 300
    q = np.zeros((1, 1, N, 2)); kv = np.ones((1, 1, N, 2))
    _, lse = attention_oracle(q, kv, kv, None, 1.0, L, R)
    assert round(float(np.exp(lse[0, 0, 150]))) == c["local_window_width"]


def test_mask_memory_implies_twelve_heads_fp16():
    """1.5 / 6 / 24 GB of SDPA mask at 8K / 16K / 32K equal heads * S^2 * 2 bytes
    with 12 heads: the head count and head_dim the workloads use."""
    c = load()
    for S, key in ((8192, "sdpa_mask_gb_at_8k"), (16384, "sdpa_mask_gb_at_16k"), (32768, "sdpa_mask_gb_at_32k")):
        assert 12 * S * S * 2 / 2 ** 30 == c[key]
    for w in CONFIGS.values():
        assert w.heads == 12 and w.head_dim == c["head_dim"]


def test_pad_bias_constant_is_fp16_lowest():
    c = load()
    assert c["pad_bias_value"] == float(np.finfo(np.float16).min)
    rng = np.random.default_rng(5)
    q, k, v = (rng.standard_normal((1, 1, 20, 4)) for _ in range(3))
    a = attention_oracle(q, k, v, (13,), 0.5)
    b = additive_bias_variant(q, k, v, (13,), 0.5, bias_value=c["pad_bias_value"])
    assert np.allclose(a[0], b[0], atol=1e-15)
