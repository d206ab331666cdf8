"""Host-only checks of the C boundary: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching a device."""
import ctypes
import math
import pathlib
import re

import pytest

import paper_2603_12646_amd as fa

ROOT = pathlib.Path(__file__).resolve().parent.parent
HEADER = (ROOT / "include" / "fa.h").read_text()


def declared_functions():
    body = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    return sorted(set(re.findall(r"\b(fa_[a-z0-9_]+)\s*\(", body)))


def test_header_declares_the_expected_entry_points():
    assert declared_functions() == ["fa_fwd", "fa_fwd_bf16", "fa_fwd_ex", "fa_strerror",
                                    "fa_version", "fa_workspace_bytes"]


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(fa.LIB_PATH)
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_version_and_struct_size_match_header():
    m = re.search(r"#define FA_VERSION (\d+)", HEADER)
    assert fa.fa_version() == int(m.group(1))
    # the binding's struct must have the size the library checks against
    p = fa.FaParams()
    p.struct_size = ctypes.sizeof(fa.FaParams) + 8
    assert fa.load_library().fa_fwd_ex(ctypes.byref(p)) == -8


def test_error_enum_values_in_header_match_strerror():
    codes = dict((name, int(val)) for name, val in re.findall(r"(FA_ERR_[A-Z_]+) = (-\d+)", HEADER))
    assert len(codes) == 9 and sorted(codes.values()) == list(range(-9, 0))
    seen = set()
    for name, code in codes.items():
        msg = fa.fa_strerror(code)
        assert msg and msg != "unknown error code" and msg not in seen
        seen.add(msg)
    assert fa.fa_strerror(0) == "success"
    assert fa.fa_strerror(-99) == "unknown error code"
    assert fa.fa_strerror(700) == "HIP runtime error"


def test_workspace_is_zero_for_every_shape():
    for shape in [(1, 12, 512, 64), (32, 12, 512, 64), (1, 12, 32768, 64), (3, 12, 16384, 64)]:
        assert fa.fa_workspace_bytes(*shape) == 0


P = 0x1000  # a non-null, 16-byte aligned address that is never dereferenced on these paths


def call(fn=fa.fa_fwd, q=P, k=P, v=P, o=P, lse=P, batch=1, heads=1, seq_lens=P, max_len=8,
         head_dim=64, scale=0.125, window=-1):
    return fn(q, k, v, o, lse, batch, heads, seq_lens, max_len, head_dim, scale, window,
              stream=0, check=False)


@pytest.mark.parametrize("fn", [fa.fa_fwd, fa.fa_fwd_bf16])
def test_simple_entry_points_reject_bad_arguments(fn):
    assert call(fn, q=0) == -1 and call(fn, k=0) == -1 and call(fn, v=0) == -1 and call(fn, o=0) == -1
    assert call(fn, batch=0) == -2 and call(fn, heads=-1) == -2 and call(fn, max_len=0) == -2
    # supported: 32, 64, 128 (valid calls would launch, so only the rejections are tried here)
    assert all(call(fn, head_dim=d) == -3 for d in (0, -64, 16, 48, 96, 256))
    assert call(fn, scale=math.nan) == -4 and call(fn, scale=math.inf) == -4 and call(fn, scale=-math.inf) == -4
    assert call(fn, window=0) == -5
    assert call(fn, q=P + 2) == -6 and call(fn, o=P + 8) == -6 and call(fn, lse=P + 2) == -6
    # too many workgroups for one grid
    assert call(fn, batch=1 << 20, heads=1 << 10, max_len=1 << 20) == -2


def test_ex_entry_point_rejects_bad_arguments():
    base = dict(dtype=fa.FA_DTYPE_F16, q=P, k=P, v=P, o=P, batch=1, heads=1, max_len=8, scale=1.0,
                stream=0, check=False)
    assert fa.fa_fwd_ex(**{**base, "dtype": 7}) == -7
    assert fa.fa_fwd_ex(**{**base, "tuning": 0x4000}) == -9
    assert fa.fa_fwd_ex(**{**base, "tuning": 0x7}) == -9 and fa.fa_fwd_ex(**{**base, "tuning": 0x8}) == -9
    # output rows that would overlap: zero / negative batch or head stride, rows inside each other
    two = {**base, "batch": 2, "heads": 2}
    assert fa.fa_fwd_ex(**{**two, "o_strides": (0, 512, 64)}) == -2
    assert fa.fa_fwd_ex(**{**two, "o_strides": (1024, -512, 64)}) == -2
    assert fa.fa_fwd_ex(**{**two, "o_strides": (1024, 64, 64)}) == -2        # heads 64 apart, 8 rows of 64 each
    assert fa.fa_fwd_ex(**{**two, "o_strides": (512, 512, 64)}) == -2        # batch stride = head stride
    assert fa.fa_fwd_ex(**{**base, "q_strides": (512, 64, 65)}) == -6
    assert fa.fa_fwd_ex(**{**base, "k_strides": (512, 64, 32)}) == -2
    assert fa.fa_fwd_ex(**{**base, "key_bias": P + 1}) == -6
    assert fa.fa_fwd_ex(**{**base, "key_bias": P, "key_bias_stride": 4}) == -2     # shorter than max_len
    assert fa.fa_fwd_ex(**{**base, "key_bias_stride": -8}) == -2
    # rotation tables: both or neither, 16-byte aligned, rows of at least head_dim / 2 floats in fours
    assert fa.fa_fwd_ex(**{**base, "rope_cos": P}) == -1 and fa.fa_fwd_ex(**{**base, "rope_sin": P}) == -1
    assert fa.fa_fwd_ex(**{**base, "rope_cos": P + 4, "rope_sin": P}) == -6
    assert fa.fa_fwd_ex(**{**base, "rope_cos": P, "rope_sin": P, "rope_stride": 34}) == -6
    assert fa.fa_fwd_ex(**{**base, "rope_cos": P, "rope_sin": P, "rope_stride": 16}) == -2
    assert fa.fa_fwd_ex(**{**base, "rope_stride": -4}) == -2
    assert fa.load_library().fa_fwd_ex(None) == -1
    with pytest.raises(fa.FaError) as e:
        fa.fa_fwd_ex(**{**base, "head_dim": 48, "check": True})
    assert e.value.code == -3


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(fa, "_lib", None)
    monkeypatch.setattr(fa, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        fa.fa_version()


def test_product_package_does_not_import_the_oracle():
    for path in (ROOT / "paper_2603_12646_amd").rglob("*"):
        if path.suffix in (".py", ".cpp", ".hip", ".h"):
            text = path.read_text()
            assert "oracle" not in text.lower().replace("no cpu or pytorch fallback", ""), path


def test_cu_mask_words():
    """Mask words for a stream limited to the first compute units (host arithmetic only)."""
    from paper_2603_12646_amd.cu_mask import first_units
    import pytest as _pytest

    assert first_units(256) == [0xFFFFFFFF] * 8
    assert first_units(128) == [0xFFFFFFFF] * 4 + [0] * 4
    assert first_units(40) == [0xFFFFFFFF, 0xFF, 0, 0, 0, 0, 0, 0]
    assert first_units(1, 32) == [1]
    assert sum(bin(w).count("1") for w in first_units(97)) == 97
    for bad in (0, 257):
        with _pytest.raises(ValueError):
            first_units(bad)


C_CALLER = r"""
#include <stddef.h>
#include <stdio.h>
#include <string.h>
#include "fa.h"

int main(void) {
  fa_params p;
  memset(&p, 0, sizeof p);
  p.struct_size = (uint32_t)sizeof p;
  printf("%d %u %u %u %u %u %d %d %d %s\n", fa_version(), (unsigned)sizeof(fa_params),
         (unsigned)offsetof(fa_params, q_strides), (unsigned)offsetof(fa_params, stream),
         (unsigned)offsetof(fa_params, tuning), (unsigned)offsetof(fa_params, key_bias),
         fa_fwd(NULL, NULL, NULL, NULL, NULL, 1, 1, NULL, 8, 64, 1.0f, -1, NULL),
         fa_fwd_ex(&p), (int)fa_workspace_bytes(1, 12, 512, 64), fa_strerror(0));
  return 0;
}
"""


def test_header_is_plain_c_and_its_struct_layout_is_the_bindings(tmp_path):
    """A C99 caller compiled with gcc -pedantic against include/fa.h and linked to the built
    library: the header needs nothing but <stdint.h>/<stddef.h>, the error paths answer
    without a device, and the struct the C compiler lays out is the one the Python binding
    fills."""
    import shutil
    import subprocess

    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "caller.c"
    src.write_text(C_CALLER)
    exe = tmp_path / "caller"
    libdir = str(pathlib.Path(fa.LIB_PATH).parent)
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", str(ROOT / "include"),
                    str(src), "-o", str(exe), fa.LIB_PATH, f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib",
                    "-Wl,--allow-shlib-undefined"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(None, 9)
    m = re.search(r"#define FA_VERSION (\d+)", HEADER)
    assert int(out[0]) == int(m.group(1))
    assert int(out[1]) == ctypes.sizeof(fa.FaParams)
    assert int(out[2]) == fa.FaParams.q_strides.offset
    assert int(out[3]) == fa.FaParams.stream.offset
    assert int(out[4]) == fa.FaParams.tuning.offset
    assert int(out[5]) == fa.FaParams.key_bias.offset
    assert int(out[6]) < 0 and int(out[7]) < 0      # null pointers: rejected on the host
    assert int(out[8]) == 0
    assert out[9].strip() == fa.fa_strerror(0)
