// Argument block passed by value from the host entry points to the gfx950 kernels.
#pragma once
#include <stdint.h>

struct FaKernelArgs {
  const void* q;
  const void* k;
  const void* v;
  void* o;
  float* lse;               // may be null
  const int32_t* seq_lens;  // device, may be null
  const void* key_bias;     // device, [batch][kb_stride] 16-bit values, may be null
  int64_t kb_stride;        // elements between batch rows of key_bias
  float inv_abs_scale;      // 1 / |scale| (0 when scale is 0): key bias in raw-score units
  const float* rope_cos;    // device, [max_len][rope_stride] fp32 tables, or null: q and k are rotated
  const float* rope_sin;    // by position (pairs (f, f + head_dim/2)) and rounded to 16 bits first
  int64_t rope_stride;      // floats between table rows (>= head_dim / 2, multiple of 4)
  int32_t batch, heads, max_len;
  int32_t head_dim;         // 32, 64 or 128
  int64_t qs[3], ks[3], vs[3], os[3];  // element strides: batch, head, row
  float c;          // |scale| * log2(e): scores are handled in the log2 domain
  int32_t negate_q; // scale < 0: q's sign bits are flipped on load, c stays positive
  float tau_raw;    // a row's reference maximum is refreshed only when a tile's maximum
                    // exceeds it by more than this (raw score units)
  int32_t wl, wr;   // window extents, < 0 = unbounded (already clamped to max_len)
  int32_t n_qtiles; // ceil(max_len / BM)
  int32_t total_tiles;  // batch * heads * n_qtiles
  int32_t map_xcd;  // nonzero: each XCD owns a contiguous eighth of every batch element's tiles
  int32_t xcd_per;  // ceil(heads * n_qtiles / 8)
  int32_t mix_ids_a; // mixed-shape kernel: workgroup ids reserved for 256-row workgroups (fa_mix_map.h)
};

// Rotation of q and k ahead of a global layer (rows of both tensors rotated by position and
// written, rounded to the storage type, to dense [batch, heads, max_len, head_dim] copies).
struct FaRopeArgs {
  const void* q;
  const void* k;
  void* q_out;
  void* k_out;
  int64_t qs[3], ks[3];     // element strides of the inputs: batch, head, row
  const float* rope_cos;
  const float* rope_sin;
  int64_t rope_stride;
  int32_t batch, heads, max_len, head_dim;
};
int fa_launch_rope_rotate(const FaRopeArgs& r, int is_bf16, void* stream);
// Address, on the current device, of the library's static scratch array of FA_STATIC_SCRATCH_BYTES
// (looked up once per device).  Returns hipError_t as int.
int fa_static_scratch(void** ptr);

// Host-side launchers implemented in fa_kernels.hip.  Return hipError_t as int.
// bm: query rows per workgroup: 32 (key-split kernel), 128, 256, 384 (12 wavefronts), 512 (8
// wavefronts), or 0 = 256-row and 128-row workgroups mixed (one sequence, a.mix_ids_a set); v_path: 0 = LDS
// transpose reads, 1 = 16-bit reads.
// win_kernel: 0 = library's choice among the window kernels, 1 = never the two-phase kernel, 2 = the
// two-phase kernel wherever it applies.
int fa_launch_f16(const FaKernelArgs& a, int bm, int v_path, int win_kernel, void* stream);
int fa_launch_bf16(const FaKernelArgs& a, int bm, int v_path, int win_kernel, void* stream);
