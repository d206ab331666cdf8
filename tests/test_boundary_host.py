"""Host-only checks of the C boundary: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching a device."""
import ctypes
import math
import os
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
    assert declared_functions() == ["fa_fwd", "fa_fwd_bf16", "fa_fwd_ex", "fa_fwd_ex_static_scratch",
                                    "fa_rope_scratch_bytes", "fa_strerror", "fa_version", "fa_workspace_bytes"]


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
    assert len(codes) == 10 and sorted(codes.values()) == list(range(-10, 0))
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
    assert fa.fa_fwd_ex(**{**base, "tuning": 0x4000}) == -9 and fa.fa_fwd_ex(**{**base, "tuning": 0x3000}) == -9
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


SANITIZER_DRIVER = r"""
// Host side of the boundary under AddressSanitizer / UBSan: fa_api.cpp compiled by the host
// compiler against stub launchers (no HIP, no device), driven through rejections and through
// calls that reach the launcher with every tile shape and stride form.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>
#include "fa.h"
#include "fa_args.h"

static FaKernelArgs last;
static int last_bm = -7, launches = 0;
int fa_launch_f16(const FaKernelArgs& a, int bm, int, int, void*) { last = a; last_bm = bm; ++launches; return 0; }
int fa_launch_bf16(const FaKernelArgs& a, int bm, int, int, void*) { last = a; last_bm = bm; ++launches; return 0; }
static FaRopeArgs last_rot;
static int rotations = 0;
int fa_launch_rope_rotate(const FaRopeArgs& r, int, void*) { last_rot = r; ++rotations; return 0; }
alignas(16) static char static_array[16];
static int lookups = 0;
int fa_static_scratch(void** ptr) { *ptr = static_array; ++lookups; return 0; }

#define EXPECT(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main() {
  alignas(16) static char buf[64];
  void* P = buf;
  fa_params p;
  std::memset(&p, 0, sizeof p);
  p.struct_size = sizeof p;
  p.q = p.k = p.v = P; p.o = P;
  p.batch = 1; p.heads = 12; p.max_len = 8192; p.head_dim = 64; p.scale = 0.125f;
  p.window_left = p.window_right = -1;
  EXPECT(fa_fwd_ex(&p) == 0 && launches == 1 && last_bm == 0);            // one 8K sequence: the mixed launch
  p.heads = 16; EXPECT(fa_fwd_ex(&p) == 0 && last_bm == 512);
  p.heads = 24; EXPECT(fa_fwd_ex(&p) == 0 && last_bm == 0 && last.mix_ids_a == 768);   // 1536 tiles: 768 of 256 rows
  p.batch = 2; EXPECT(fa_fwd_ex(&p) == 0 && last_bm == 256 && last.mix_ids_a == 0); p.batch = 1;
  p.heads = 12; p.max_len = 512; EXPECT(fa_fwd_ex(&p) == 0 && last_bm == 32);
  p.batch = 32; EXPECT(fa_fwd_ex(&p) == 0 && last_bm == 128);
  p.batch = 1; p.max_len = 32768; p.window_left = 63; p.window_right = 64;
  EXPECT(fa_fwd_ex(&p) == 0 && last_bm == 128 && last.wl == 63 && last.wr == 64);
  p.window_left = 40000; p.window_right = -1; EXPECT(fa_fwd_ex(&p) == 0 && last.wl == -1 && last.wr == -1);
  for (int d : {32, 64, 128})
    for (unsigned t = 0; t <= 6; ++t) {
      p.head_dim = d; p.tuning = t; p.window_left = p.window_right = -1;
      EXPECT(fa_fwd_ex(&p) == 0);
      EXPECT(last.total_tiles > 0 && last.n_qtiles > 0 && last.xcd_per > 0);
    }
  p.tuning = 0;
  // head_dim 32 never takes the mixed launch: 256 rows where the fill model says so
  p.head_dim = 32; p.heads = 24; p.max_len = 8192; EXPECT(fa_fwd_ex(&p) == 0 && last_bm == 256);
  p.heads = 12; EXPECT(fa_fwd_ex(&p) == 0 && last_bm == 128);
  p.head_dim = 64; p.max_len = 32768;
  // strides: [batch, len, heads, dim] passes, interleaved output rows do not
  const int64_t bshd[3] = {(int64_t)32768 * 12 * 64, 64, 12 * 64};
  std::memcpy(p.q_strides, bshd, sizeof bshd); std::memcpy(p.o_strides, bshd, sizeof bshd);
  EXPECT(fa_fwd_ex(&p) == 0 && last.qs[2] == 12 * 64 && last.os[1] == 64);
  p.o_strides[1] = 0; EXPECT(fa_fwd_ex(&p) == FA_ERR_BAD_SHAPE);
  std::memset(p.o_strides, 0, sizeof p.o_strides);
  // extremes: sizes that overflow a grid or an int64 element count are refused, not wrapped
  p.batch = 1 << 30; p.heads = 1 << 30; p.max_len = 1 << 30; EXPECT(fa_fwd_ex(&p) == FA_ERR_BAD_SHAPE);
  p.batch = 1; p.heads = 1; p.max_len = (1 << 30) + 1; EXPECT(fa_fwd_ex(&p) == FA_ERR_BAD_SHAPE);
  p.max_len = 1; EXPECT(fa_fwd_ex(&p) == 0);
  p.scale = 0.0f; EXPECT(fa_fwd_ex(&p) == 0 && last.tau_raw > 1e30f);
  p.scale = -3.0f; EXPECT(fa_fwd_ex(&p) == 0 && last.negate_q == 1 && last.c > 0.f);
  // a rotation on a global layer: in the call without scratch, ahead of it (on dense copies) with enough
  alignas(16) static float table[64];
  alignas(16) static char lent[64];
  p.batch = 1; p.heads = 12; p.max_len = 8192; p.head_dim = 64; p.scale = 0.125f; p.window_left = p.window_right = -1;
  p.rope_cos = p.rope_sin = table;
  EXPECT(fa_fwd_ex(&p) == 0 && rotations == 0 && last.rope_cos == table && last_bm != 0 && last.q == P);
  p.max_len = 32768; EXPECT(fa_fwd_ex(&p) == 0 && rotations == 0 && last_bm == 256);       // rotation in the call: never the mixed launch
  p.max_len = 8192;
  p.scratch = lent; p.scratch_bytes = fa_rope_scratch_bytes(1, 12, 8192, 64) - 1;
  EXPECT(fa_fwd_ex(&p) == 0 && rotations == 0 && last.rope_cos == table);                    // too small: ignored
  p.scratch_bytes += 1;
  EXPECT(fa_rope_scratch_bytes(1, 12, 8192, 64) == (size_t)2 * 12 * 8192 * 64 * 2);
  EXPECT(fa_fwd_ex(&p) == 0 && rotations == 1 && last.rope_cos == nullptr && last.q == lent && last_bm == 0);
  EXPECT(last_rot.q == P && last_rot.k_out == lent + 12 * 8192 * 64 * 2 && last.k == last_rot.k_out && last.ks[2] == 64);
  p.scratch = lent + 4; EXPECT(fa_fwd_ex(&p) == FA_ERR_MISALIGNED && rotations == 1);
  p.scratch = lent; p.window_left = 63; p.window_right = 64;
  EXPECT(fa_fwd_ex(&p) == 0 && rotations == 1 && last.rope_cos == table);                    // local layer: in the call
  p.window_left = p.window_right = -1; p.tuning = 0x7;
  EXPECT(fa_fwd_ex(&p) == FA_ERR_BAD_TUNING && rotations == 1);                              // refused: nothing enqueued
  // the entry point with the library's own scratch: the array instead of the lent buffer, refusal beyond its size
  p.tuning = 0; p.scratch = lent; p.scratch_bytes = 1u << 30;
  EXPECT(fa_fwd_ex_static_scratch(&p) == 0 && rotations == 2 && lookups == 1 && last.q == static_array && last_rot.q_out == static_array);
  p.max_len = 32768;
  EXPECT(fa_rope_scratch_bytes(1, 12, 32768, 64) > FA_STATIC_SCRATCH_BYTES);
  EXPECT(fa_fwd_ex_static_scratch(&p) == FA_ERR_SCRATCH && rotations == 2);
  p.window_left = 63; p.window_right = 64;
  EXPECT(fa_fwd_ex_static_scratch(&p) == 0 && rotations == 2 && lookups == 2 && last.rope_cos == table);   // local layer: no scratch used
  p.window_left = p.window_right = -1; p.rope_cos = p.rope_sin = nullptr;
  EXPECT(fa_fwd_ex_static_scratch(&p) == 0 && rotations == 2 && lookups == 2 && last.q == P);               // no rotation: plain call
  EXPECT(fa_fwd_ex_static_scratch(nullptr) == FA_ERR_NULL_POINTER);
  p.max_len = 8192; p.scratch = nullptr; p.scratch_bytes = 0;
  // the plain entry points and the queries
  EXPECT(fa_fwd(P, P, P, P, nullptr, 2, 3, nullptr, 100, 64, 1.0f, 128, nullptr) == 0 && last.wl == 63 && last.wr == 64);
  EXPECT(fa_fwd_bf16(P, P, P, P, nullptr, 2, 3, nullptr, 100, 64, 1.0f, 0, nullptr) == FA_ERR_BAD_WINDOW);
  EXPECT(fa_workspace_bytes(4, 12, 32768, 64) == 0);
  for (int code = -12; code <= 3; ++code) EXPECT(std::strlen(fa_strerror(code)) > 0);
  EXPECT(std::strstr(fa_strerror(FA_ERR_SCRATCH), "scratch") != nullptr);
  printf("ok %d launches\n", launches);
  return 0;
}
"""


def test_host_boundary_under_address_and_undefined_sanitizers(tmp_path):
    """fa_api.cpp built by g++ with -fsanitize=address,undefined against stub launchers: the
    validation, stride, overflow and tile-shape arithmetic runs clean, and the kernel-shape
    choices reach the launcher as documented."""
    import shutil
    import subprocess

    if shutil.which("g++") is None:
        pytest.skip("no g++")
    src = tmp_path / "driver.cpp"
    src.write_text(SANITIZER_DRIVER)
    exe = tmp_path / "driver"
    csrc = ROOT / "paper_2603_12646_amd" / "csrc"
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-I", str(ROOT / "include"), "-I", str(csrc), str(src), str(csrc / "fa_api.cpp"), "-o", str(exe)],
                   check=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok ") and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


MIX_MAP_DRIVER = r"""
// Every workgroup id of the mixed-shape launch walked on the CPU: for each (heads, max_len, n,
// id order) the 256-row and 128-row tiles handed out must cover rows [0, 128 T) of every head
// exactly once and stay inside them, and the spare ids must be numbered 0 .. spares-1 once each.
#include <cstdio>
#include <vector>
#include "fa_mix_map.h"

static long cases = 0;

static int check(int H, int max_len, int n, bool map_xcd) {
  const int tmax = (max_len + 127) / 128, tiles = (n + 127) / 128;
  const int ids_a = fa_mix_ids(tmax, H);
  if (ids_a < 0 || ids_a % 8) { printf("ids_a %d for H %d tmax %d\n", ids_a, H, tmax); return 1; }
  std::vector<int> cover((size_t)H * tiles, 0);
  std::vector<int> spare_seen;
  int spares = -1, n_a = 0, n_b = 0;
  for (int bid = 0; bid < ids_a + kMixIdsB; ++bid) {
    const FaMixTile m = fa_mix_locate(bid, map_xcd, ids_a, kMixIdsB, H, tiles);
    if (m.kind == 0) continue;
    if (m.kind == 3) {
      if (spares < 0) { spares = m.spares; spare_seen.assign(spares, 0); }
      if (m.spares != spares || m.spare < 0 || m.spare >= spares || spare_seen[m.spare]++) { printf("spare id %d\n", bid); return 1; }
      continue;
    }
    const int rows = m.kind == 1 ? 256 : 128;
    if (m.kind == 1 && bid >= ids_a) { printf("256-row tile on id %d of the 128-row range\n", bid); return 1; }
    if (m.kind == 2 && bid < ids_a) { printf("128-row tile on id %d of the 256-row range\n", bid); return 1; }
    if (m.head < 0 || m.head >= H || m.q0 < 0 || m.q0 % 128 || m.q0 + rows > 128 * tiles) {
      printf("H %d max_len %d n %d xcd %d id %d: kind %d head %d q0 %d\n", H, max_len, n, (int)map_xcd, bid, m.kind, m.head, m.q0);
      return 1;
    }
    for (int t = m.q0 / 128; t < (m.q0 + rows) / 128; ++t) ++cover[(size_t)m.head * tiles + t];
    (m.kind == 1 ? n_a : n_b)++;
  }
  for (size_t i = 0; i < cover.size(); ++i)
    if (cover[i] != 1) { printf("H %d max_len %d n %d xcd %d: head %zu tile %zu covered %d times\n", H, max_len, n, (int)map_xcd, i / tiles, i % tiles, cover[i]); return 1; }
  if (spares >= 0) for (int s : spare_seen) if (s != 1) { printf("spare numbering\n"); return 1; }
  if (tiles < tmax && spares <= 0) { printf("H %d max_len %d n %d: padding tiles but no spare id\n", H, max_len, n); return 1; }
  if (n_a != fa_mix_a_total(tiles, H) || 2 * n_a + n_b != tiles * H) { printf("totals\n"); return 1; }
  ++cases;
  return 0;
}

int main() {
  // the split itself: the documented regimes
  if (fa_mix_a_total(64, 12) != 256 || fa_mix_a_total(128, 12) != 768 || fa_mix_a_total(192, 12) != 1024 || fa_mix_a_total(256, 12) != 1536 ||
      fa_mix_a_total(32, 12) != 0 || fa_mix_a_total(1, 1000) != 0 || fa_mix_a_total(96, 12) != 512 ||
      fa_mix_a_total(3, 400) != 400) { printf("split rule\n"); return 1; }
  const int heads[] = {1, 2, 3, 5, 7, 8, 12, 13, 16, 24, 32, 64, 100, 255, 256};
  const int lens[] = {1, 127, 128, 129, 300, 1000, 2048, 4097, 7900, 8192, 10000, 12288, 16384, 20000, 24576, 28672, 32768, 40000, 65536};
  for (int H : heads)
    for (int N : lens)
      for (int xcd = 0; xcd < 2; ++xcd) {
        // n = N, a few lengths inside every regime below it, and the empty sequence
        const int ns[] = {N, N - 1, N - 127, N - 128, N / 2, N / 3, (int)(N * 0.8), 129, 1, 0};
        for (int n : ns) {
          if (n < 0) continue;
          if (check(H, N, n, xcd != 0)) return 1;
        }
      }
  // every length of one 12-head and one 5-head call
  for (int n = 0; n <= 16384; n += 97) if (check(12, 16384, n, true) || check(5, 16384, n, false)) return 1;
  printf("ok %ld cases\n", cases);
  return 0;
}
"""


def test_mixed_launch_covers_every_tile_exactly_once(tmp_path):
    """The id -> tile arithmetic the mixed-shape kernel evaluates on the device (fa_mix_map.h),
    compiled for the host and walked id by id under the sanitizers."""
    import shutil
    import subprocess

    if shutil.which("g++") is None:
        pytest.skip("no g++")
    src = tmp_path / "mixmap.cpp"
    src.write_text(MIX_MAP_DRIVER)
    exe = tmp_path / "mixmap"
    csrc = ROOT / "paper_2603_12646_amd" / "csrc"
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-I", str(csrc), str(src), "-o", str(exe)], check=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok ") and "runtime error" not in r.stderr
