"""The work bench.py divides by its timings (no GPU): algorithmic flops = 4 * head_dim *
heads * visible (query, key) pairs over valid lengths and the window band only; bytes =
q, k, v read and o written once over valid rows, plus lse."""
import numpy as np

import bench
from oracle.attention_oracle import visible_mask
from workloads import ALL_CONFIGS, CONFIGS, make_inputs


def lens_of(w):
    if w.random_lens is not None:
        lens, _, _, _ = make_inputs(w)
        return lens
    if w.seq_lens is not None:
        return np.asarray(w.seq_lens)
    return np.full((w.batch,), w.max_len)


def test_visible_pairs_closed_forms():
    assert bench.visible_pairs([512], -1, -1) == 512 * 512
    assert bench.visible_pairs([7900], -1, -1) == 62_410_000
    # 128-wide band clipped at both ends: 32768 * 128 - (63 * 64 / 2) - (64 * 65 / 2)
    assert bench.visible_pairs([32768], 63, 64) == 32768 * 128 - 2016 - 2080 == 4_190_208
    assert bench.visible_pairs([16384, 12000, 9000], -1, -1) == 16384 ** 2 + 12000 ** 2 + 9000 ** 2


def test_visible_pairs_matches_the_oracle_mask_by_counting():
    for n, left, right in [(37, -1, -1), (37, 3, 5), (50, 0, 0), (64, 63, 64), (20, 30, 2), (33, -1, 4), (33, 6, -1)]:
        vis = visible_mask(np.arange(n), n, n, left, right)
        assert bench.visible_pairs([n], left, right) == int(vis.sum()), (n, left, right)


def test_flops_and_bytes_of_the_named_workloads():
    expect_gflop = {"c1_512": 0.805, "c3_8k": 191.7, "c4_16k_x3": 1515.8, "c5a_32k_global": 3298.5,
                    "c5b_32k_local": 12.87}
    for name, gf in expect_gflop.items():
        w = CONFIGS[name]
        flops, nbytes = bench.algorithmic_work(w, lens_of(w))
        assert abs(flops / 1e9 - gf) <= 0.05 * max(1.0, gf / 100), (name, flops)
        rows = int(sum(lens_of(w)))
        assert nbytes == 2 * 4 * w.heads * w.head_dim * rows + 4 * w.heads * rows
    w = CONFIGS["c2_batch32"]
    lens = lens_of(w)
    flops, _ = bench.algorithmic_work(w, lens)
    assert flops == 4.0 * 64 * 12 * float(sum(int(n) ** 2 for n in lens))
    w = ALL_CONFIGS["d128_8k"]
    assert bench.algorithmic_work(w, lens_of(w))[0] == 4.0 * 128 * 8 * 7900 ** 2


def test_multi_gpu_request_is_refused(monkeypatch, capsys):
    import sys
    import pytest
    monkeypatch.setattr(sys, "argv", ["bench.py", "--gpus", "2"])
    with pytest.raises(SystemExit) as e:
        bench.main()
    assert e.value.code == 2 and "ONE GPU" in capsys.readouterr().err
