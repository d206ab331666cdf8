"""Input recipes: rounding to storage types and the five named workloads."""
import numpy as np
import torch

from workloads import CONFIGS, draw, make_inputs, round_to_storage


def test_round_to_storage_matches_torch_casts():
    x = np.random.default_rng(0).standard_normal(200000).astype(np.float32) * 3
    x[:5] = [0.0, -0.0, 1.0, 65504.0, 1e-8]
    for name, tdt in (("fp16", torch.float16), ("bf16", torch.bfloat16)):
        ours = round_to_storage(x, name)
        ref = torch.from_numpy(x).to(tdt).to(torch.float32).numpy()
        assert np.array_equal(ours.view(np.uint32), ref.view(np.uint32))
        # idempotent: already-representable values survive a second rounding
        assert np.array_equal(round_to_storage(ours, name), ours)


def test_bf16_ties_to_even():
    # 1 + 2^-8 is exactly half way between bf16 neighbours 1.0 and 1.0078125
    x = np.array([1.0 + 2.0 ** -8, 1.0078125 + 2.0 ** -8], dtype=np.float32)
    r = round_to_storage(x, "bf16")
    assert r[0] == 1.0 and r[1] == 1.015625


def test_draw_is_seeded_and_ordered():
    a = draw(3, 2, 2, 16, 8, "fp16", random_lens=(4, 16))
    b = draw(3, 2, 2, 16, 8, "fp16", random_lens=(4, 16))
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    c = draw(4, 2, 2, 16, 8, "fp16", random_lens=(4, 16))
    assert not np.array_equal(a[1], c[1])
    assert a[0].dtype == np.int32 and a[0].min() >= 4 and a[0].max() <= 16


def test_named_configs_shapes():
    w = CONFIGS["c1_512"]
    lens, q, k, v = make_inputs(w)
    assert q.shape == (1, 12, 512, 64) and lens.tolist() == [512]
    assert abs(float(q.std()) - 1.0) < 0.01
    w2 = CONFIGS["c2_batch32"]
    lens2, q2, _, _ = make_inputs(w2)
    assert q2.shape == (32, 12, 512, 64)
    assert lens2.min() >= 256 and lens2.max() <= 512 and len(set(lens2.tolist())) > 8
    assert CONFIGS["c3_8k"].seq_lens == (7900,) and CONFIGS["c3_8k"].qk_gain == 1.5
    assert CONFIGS["c4_16k_x3"].seq_lens == (16384, 12000, 9000)
    assert CONFIGS["c5b_32k_local"].window == 128 and CONFIGS["c5a_32k_global"].window < 0
    assert [CONFIGS[n].seed for n in ("c1_512", "c2_batch32", "c3_8k", "c4_16k_x3", "c5a_32k_global")] == [0, 1, 2, 3, 4]
