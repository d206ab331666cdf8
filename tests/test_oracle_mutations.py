"""Show that the pins bite: plant plausible mistakes in a copy of the oracle's
source (on the CPU) and check that the pin battery rejects every one."""
import importlib
import pathlib
import types

import pytest

import tests.test_oracle_pins as pins

SRC = pathlib.Path(__file__).resolve().parent.parent / "oracle" / "attention_oracle.py"

MUTATIONS = {
    "dropped scale": ("(q[rows] @ k.T) * scale", "(q[rows] @ k.T)"),
    "transposed score operand": ("(q[rows] @ k.T) * scale", "(k[rows] @ q.T) * scale"),
    "left edge off by one": ("vis &= j >= i - left", "vis &= j > i - left"),
    "right edge off by one": ("vis &= j <= i + right", "vis &= j < i + right"),
    "left/right swapped": ("vis &= j >= i - left", "vis &= j >= i - right"),
    "padding boundary off by one": ("vis = np.broadcast_to(j < n_valid", "vis = np.broadcast_to(j <= n_valid"),
    "no key padding mask": ("vis = np.broadcast_to(j < n_valid", "vis = np.broadcast_to(j < n_keys_total"),
    "lse without max": ("m_safe + np.log(l_safe)", "np.log(l_safe)"),
    "lse base 2": ("m_safe + np.log(l_safe)", "m_safe + np.log2(l_safe)"),
    "unnormalised": ("p = e / l_safe[:, None]", "p = e"),
    "wrong sign in exp": ("np.exp(s - m_safe[:, None])", "np.exp(m_safe[:, None] - s)"),
    "window width mapping": ("return ((window - 1) // 2, window // 2)", "return (window // 2, window // 2)"),
    "window halves swapped": ("return ((window - 1) // 2, window // 2)", "return (window // 2, (window - 1) // 2)"),
    "key bias dropped": ("s = s + key_bias[None, :]", "s = s"),
    "key bias subtracted": ("s = s + key_bias[None, :]", "s = s - key_bias[None, :]"),
    "key bias multiplied by scale": ("s = s + key_bias[None, :]", "s = s + key_bias[None, :] * scale"),
    "key bias of another batch element": ("None if key_bias is None else key_bias[b])", "None if key_bias is None else key_bias[0])"),
    "sampled rows: key bias of another batch element": ("np.asarray(key_bias, dtype=np.float64)[b]", "np.asarray(key_bias, dtype=np.float64)[0]"),
    "sampled rows: key bias dropped": ("scale, left, right, False, kb)", "scale, left, right, False, None)"),
    "padded rows computed": ("for r0 in range(0, n, row_block):\n                rows = np.arange(r0, min(n, r0 + row_block))",
                             "for r0 in range(0, N, row_block):\n                rows = np.arange(r0, min(N, r0 + row_block))"),
}

BATTERY = [
    (pins.test_brute_force_tiny, [(l, r, lens) for (l, r) in [(-1, -1), (1, 2), (2, 1), (0, 0)] for lens in [(7, 5), (1, 0)]]),
    (pins.test_global_unpadded_equals_scipy, [()]),
    (pins.test_torch_sdpa_boolean_mask, [(5, 6, 40), (-1, -1, 33)]),
    (pins.test_zero_q_counts_visible_keys_paper_window, [(300, 300), (260, 300)]),
    (pins.test_window_from_width_mapping, [()]),
    (pins.test_self_only_window, [()]),
    (pins.test_one_hot_limit, [()]),
    (pins.test_transposed_operand_would_fail, [()]),
    (pins.test_rows_of_p_sum_to_one_and_respect_mask, [()]),
    (pins.test_key_shift_identity, [()]),
    (pins.test_split_merge_identity, [()]),
    (pins.test_masked_keys_have_no_effect_even_nan, [()]),
    (pins.test_seq_len_clamping_and_empty, [()]),
    (pins.test_key_bias_brute_force, [(-1, -1, (7, 5)), (1, 2, (8, 3))]),
    (pins.test_rows_api_key_bias_brute_force, [()]),
    (pins.test_key_bias_log_weight_equals_repeated_keys, [()]),
    (pins.test_key_bias_constant_shifts_lse_only, [()]),
    (pins.test_key_bias_minus_inf_removes_the_key, [()]),
]

NAMES = ["attention_oracle", "attention_oracle_rows", "additive_bias_variant", "visible_mask", "window_from_width"]


def run_battery():
    for fn, argsets in BATTERY:
        for args in argsets:
            fn(*args)


def test_battery_passes_on_the_real_oracle():
    run_battery()


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, monkeypatch):
    old, new = MUTATIONS[name]
    src = SRC.read_text()
    assert src.count(old) == 1, f"mutation anchor for {name!r} not unique"
    mod = types.ModuleType("mutated_oracle")
    exec(compile(src.replace(old, new), "mutated_oracle", "exec"), mod.__dict__)
    for n in NAMES:
        monkeypatch.setattr(pins, n, getattr(mod, n))
    with pytest.raises((AssertionError, ValueError, IndexError, FloatingPointError)):
        run_battery()
