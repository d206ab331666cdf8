"""The rotary-embedding pins bite: plausible mistakes planted in a copy of the oracle's source
(on the CPU) are each rejected by the pin battery."""
import pathlib
import types

import pytest

import tests.test_rope_pins as pins

SRC = pathlib.Path(__file__).resolve().parent.parent / "oracle" / "rope_oracle.py"

MUTATIONS = {
    "sine sign flipped": ("out[..., :half] = lo * cos - hi * sin", "out[..., :half] = lo * cos + hi * sin"),
    "second half rotates the other way": ("out[..., half:] = hi * cos + lo * sin", "out[..., half:] = hi * cos - lo * sin"),
    "halves swapped": ("lo, hi = x[..., :half], x[..., half:]", "hi, lo = x[..., :half], x[..., half:]"),
    "interleaved pairing": ("lo, hi = x[..., :half], x[..., half:]", "lo, hi = x[..., 0::2], x[..., 1::2]"),
    "exponent f / D": ("base ** (-2.0 * f / head_dim)", "base ** (-1.0 * f / head_dim)"),
    "positions start at 1": ("np.arange(n_positions, dtype=np.float64)[:, None]", "np.arange(1, n_positions + 1, dtype=np.float64)[:, None]"),
    "frequency scale ignored": ("inv_freq = inv_freq * np.asarray(freq_scale", "inv_freq = inv_freq * 1.0 + 0.0 * np.asarray(freq_scale"),
    "amplitude ignored": ("return amplitude * np.cos(angle), amplitude * np.sin(angle)", "return np.cos(angle), np.sin(angle)"),
    "keys not rotated": ("round_to_storage_type(rope_rotate(k, cos, sin), dtype))", "round_to_storage_type(k, dtype))"),
    "rotated inputs not rounded": ("return (round_to_storage_type(rope_rotate(q, cos, sin), dtype),", "return (rope_rotate(q, cos, sin),"),
    "bf16 keeps 9 bits": ("q = np.rint(np.ldexp(x[nz], 8 - shift))", "q = np.rint(np.ldexp(x[nz], 9 - shift))"),
    "bf16 truncates": ("q = np.rint(np.ldexp(x[nz], 8 - shift))", "q = np.trunc(np.ldexp(x[nz], 8 - shift))"),
}

BATTERY = [pins.test_tables_closed_forms, pins.test_rotation_is_complex_multiplication,
           pins.test_norm_preserved_and_zero_angle_identity_and_angles_add,
           pins.test_scores_depend_on_relative_position_only, pins.test_rounding_to_storage_types,
           pins.test_attention_with_rotation_is_attention_of_rotated_rounded_inputs,
           pins.test_rotation_changes_attention_unless_positions_are_equal]
NAMES = ["attention_oracle_rope", "attention_oracle_rope_rows", "rope_rotate", "rope_tables", "round_to_storage_type"]


def test_battery_passes_on_the_real_oracle():
    for fn in BATTERY:
        fn()


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, monkeypatch):
    old, new = MUTATIONS[name]
    src = SRC.read_text()
    assert src.count(old) == 1, f"mutation anchor for {name!r} not unique"
    mod = types.ModuleType("mutated_rope_oracle")
    exec(compile(src.replace(old, new), "mutated_rope_oracle", "exec"), mod.__dict__)
    for n in NAMES:
        monkeypatch.setattr(pins, n, getattr(mod, n))
    with pytest.raises((AssertionError, ValueError, IndexError, FloatingPointError)):
        for fn in BATTERY:
            fn()
