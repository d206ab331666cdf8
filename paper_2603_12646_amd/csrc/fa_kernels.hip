// Flash-attention forward for gfx950 (MI355X): head_dim 64 (also 32 and 128), fp16 / bf16
// storage, fp32 accumulation, key-padding mask by sequence length, optional local window.
//
// The operation is softmax(scale * Q K^T + mask) V per (batch, head), evaluated
// one key block at a time with a running row maximum and row sum so that no
// n x n matrix is ever formed (paper Sec. 2.2; operator attributes scale,
// window_size_left/right and the 1-D padding mask from Sec. 4.1.3 and Eq. 1).
//
// Work decomposition (one workgroup = 4 wavefronts = 256 threads):
//   * a workgroup owns BM = 4*32*NQB query rows of one (batch, head); each
//     wavefront owns NQB blocks of 32 query rows and keeps their Q fragments,
//     running maximum / sum and the head_dim-wide output accumulator in registers;
//   * K and V are streamed through LDS, fetched from HBM/L2 ahead of the arithmetic
//     (in the main kernels with direct global->LDS loads into an unpadded, XOR-swizzled
//     tile; in the reference masked kernel through registers into a padded tile).
//
// Matrix-core mapping (v_mfma_f32_32x32x16_{f16,bf16}, D = A * B + C with
// A: 32 x 16, B: 16 x 32, C: 32 x 32; lane l holds A[l%32][8*(l/32)..+7],
// B[8*(l/32)..+7][l%32] and C[8*(r/4) + 4*(l/32) + r%4][l%32] for r = 0..15):
//   * scores are computed TRANSPOSED, S^T = K * Q^T, so that a lane's 16
//     accumulator values all belong to ONE query (column l%32) and 16 different
//     keys.  Row maxima and sums are then in-lane reductions plus a single
//     exchange between lane l and lane l^32;
//   * the same accumulator registers, rounded to 16 bits and packed, are exactly a
//     B operand of the second product O^T = V^T * P^T once the summation index is
//     ordered as the accumulator orders it (the k index of an MFMA is a dummy
//     index, so any order works if A and B agree).  P never goes through LDS;
//   * the A operand of the second product is V^T: four consecutive keys for one
//     output column d per 64-bit piece.  V sits in LDS as [key][d] (as it is in
//     HBM) and is fetched with the LDS transpose read ds_read_b64_tr_b16.
//
// Softmax (log2 domain, c = scale*log2(e)):  p = exp2(s*c - m*c).  The reference
// maximum m of a row is only refreshed when a block's maximum exceeds it by more
// than a threshold (2^8 in p); rescaling the accumulator is then rare, and the
// result is unchanged because numerator and denominator share the reference.
//
// Kernels:
//   fa_fwd_global_kernel  global layers (no window), head_dim 64 or 128.  Full 64-key tiles run in a
//       software pipeline over 32-key x 32-query units: while the vector ALU turns unit
//       w's scores into probabilities, the matrix cores compute unit w+1's scores and
//       accumulate unit w-1's P.V.  The ragged last tile takes the masked block.
//   fa_fwd_window_resident_kernel  local layers whose key range per query tile fits in
//       LDS (the paper's 63/64 window): everything is requested at once, then each
//       wavefront runs the same pipeline over the blocks its queries can see.
//   fa_fwd_window_kernel  wider or one-sided windows: ring of 32-key stages.
//   fa_fwd_keysplit_kernel  global layers of head_dim 64 with so few query tiles that the
//       other kernels would leave most of the chip idle (one 512-token sequence): a
//       workgroup owns 32 query rows, its four wavefronts split the KEYS, and the four
//       partial results are merged through LDS.
//   fa_fwd_masked_kernel  general path (register staging, padded tiles, optional 16-bit V
//       reads) for head_dim 32, 64, 128: the production path of head_dim 32 and of the local
//       layers of head_dim 128, and at head_dim 64 an independent implementation for the tests.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <type_traits>

#include "fa.h"
#include "fa_args.h"
#include "fa_mix_map.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf2v __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));

constexpr int kD = 64;        // head_dim of the pipelined kernels (the masked kernel takes 32, 64, 128)
constexpr int kBN = 64;       // keys per LDS tile
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
// Row strides of the PADDED LDS tiles in 16-bit elements, for head_dim D.  K is read with
// 16-byte accesses by 32 rows at once (a row stride of D/2 + 4 dwords puts 16 consecutive
// rows on 16 different 16-byte bank groups for D = 32, 64, 128); V is read by the
// transpose load, 4 rows x 32 bytes per 16 lanes.
constexpr int stride_k(int D) { return D + 8; }
constexpr int stride_v(int D) { return D + 16; }
constexpr float kLn2 = 0.693147180559945309f;
// A lane's 16 probabilities of one block may sum to at most this (against the row's
// current reference) before the reference is refreshed.  2^14 keeps every single p
// inside fp16 range (max 65504) with room to spare and makes refreshes very rare.
constexpr float kPLimit = 16384.f;

struct F16 {
  typedef half8 v8;
  static constexpr bool kSumRounded = true;
  static __device__ __forceinline__ floatx16 mfma(v8 a, v8 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {  // round to nearest even
    half2v h = __builtin_convertvector((floatx2){a, b}, half2v);
    return __builtin_bit_cast(uint32_t, h);
  }
  // acc + lo + hi of a packed pair, accumulated in fp32
  static __device__ __forceinline__ float sum2(uint32_t pk, float acc) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2v, pk), (half2v){1, 1}, acc, false);
  }
  // lo + hi of a packed pair: the three-operand form with a constant zero addend, so that a
  // chain of sums needs no register zeroed first (the compiler, given the builtin with a zero
  // accumulator, moves 0 into a register and uses the accumulating two-operand form)
  static __device__ __forceinline__ float sum2_first(uint32_t pk) {
    float d;
    asm("v_dot2_f32_f16 %0, %1, %2, 0" : "=v"(d) : "v"(pk), "s"(0x3c003c00u));
    return d;
  }
  static __device__ __forceinline__ float to_float(uint16_t x) { return (float)__builtin_bit_cast(_Float16, x); }
};

struct BF16 {
  typedef bf8 v8;
  static constexpr bool kSumRounded = false;
  static __device__ __forceinline__ floatx16 mfma(v8 a, v8 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {
    bf2v h = __builtin_convertvector((floatx2){a, b}, bf2v);
    return __builtin_bit_cast(uint32_t, h);
  }
  static __device__ __forceinline__ float sum2(uint32_t pk, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2v, pk),
                                           (bf2v){(__bf16)1.0f, (__bf16)1.0f}, acc, false);
  }
  static __device__ __forceinline__ float sum2_first(uint32_t pk) { return sum2(pk, 0.f); }  // unused: bf16 sums fp32 values
  static __device__ __forceinline__ float to_float(uint16_t x) { return __builtin_bit_cast(float, (uint32_t)x << 16); }
};

// Exchange between the two lanes (l, l ^ 32) that hold the same query: afterwards
// a = x of the lower lane of the pair and b = x of the upper one, in both lanes.
// v_permlane32_swap exchanges lanes 32..63 of its first register with lanes 0..31 of
// its second.  Written as asm because the compiler folds the builtin's two results
// into one when both inputs are the same value; the s_nops cover the VALU-write ->
// permlane-read hazards the compiler cannot see inside an asm block.
__device__ __forceinline__ void swap_halves(float x, float& a, float& b) {
  a = x;
  asm("s_nop 1\n\tv_mov_b32 %1, %0\n\ts_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "=&v"(b));
}
__device__ __forceinline__ float max_xor32(float x) {
  float a, b;
  swap_halves(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float sum_xor32(float x) {
  float a, b;
  swap_halves(x, a, b);
  return a + b;
}

// 16 bytes per lane from global memory straight into LDS: lane L's data lands at
// lds_dst + 16*L (lds_dst wavefront-uniform), the global address is gbase (uniform, scalar
// registers) + a per-lane byte offset.  Written as asm: the compiler would make every
// later LDS read wait for such a load (it cannot tell that the stage being filled and the
// stage being read are disjoint), which would serialise the prefetch.  The caller waits
// with wait_direct_loads() before the barrier that publishes the stage.  M0 holds the LDS
// address: M0 is a reserved register for inline asm (the compiler rejects it on a clobber list
// with a warning that such a clobber "may lead to undefined behaviour") and is rewritten by the
// compiler before every use of its own, so nothing of its contents is assumed after the asm.
__device__ __forceinline__ void load16_to_lds(const void* gbase, uint32_t lane_off_bytes, void* lds_dst) {
  typedef __attribute__((address_space(3))) void lds_void;
  const uint32_t l = (uint32_t)(size_t)(lds_void*)lds_dst;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(l), "v"(lane_off_bytes), "s"(gbase)
               : "memory");
}
// s_waitcnt immediate that waits for vmcnt <= N only (expcnt and lgkmcnt fields at their
// maxima): vmcnt is bits 3:0 plus bits 15:14 of the immediate.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_direct_loads() { wait_vmcnt<0>(); }

template <class T>
__device__ __forceinline__ typename T::v8 as_v8(uint4 u) {
  return __builtin_bit_cast(typename T::v8, u);
}

// A operand of S^T = K Q^T for one k-step: K[row l%32][16*ks + 8*(l/32) .. +7]
template <class T, int D = kD>
__device__ __forceinline__ typename T::v8 load_k_frag(const uint16_t* kblk, int l32, int hh, int ks) {
  return as_v8<T>(*(const uint4*)&kblk[l32 * stride_k(D) + ks * 16 + hh * 8]);
}

// A operand of O^T = V^T P^T: column d = 32*db + l%32 of V, summation slots
// (hh, e) = keys 16*ks2 + (e < 4 ? 4*hh + e : 8 + 4*hh + e - 4) of the 32-key block.
// Within 16 lanes, lane p fetches 4 consecutive d of key row p/4; the transpose
// read hands lane i the 4 keys of column i.
template <class T, int D = kD>
__device__ __forceinline__ typename T::v8 load_vt_frag(const uint16_t* vblk, int lane, int ks2, int db) {
  constexpr int SV = stride_v(D);
  const int hh = lane >> 5, p16 = lane & 15;
  const int row = ks2 * 16 + 4 * hh + (p16 >> 2);
  const int col = db * 32 + 16 * ((lane >> 4) & 1) + 4 * (p16 & 3);
  typedef __attribute__((address_space(3))) shortx4 lds_s4;
  const shortx4 x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)&vblk[row * SV + col]);
  const shortx4 x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)&vblk[(row + 8) * SV + col]);
  shortx8 x;
  x[0] = x0[0]; x[1] = x0[1]; x[2] = x0[2]; x[3] = x0[3];
  x[4] = x1[0]; x[5] = x1[1]; x[6] = x1[2]; x[7] = x1[3];
  return __builtin_bit_cast(typename T::v8, x);
}

// Same operand through plain 16-bit LDS reads (slow; kept as an independent path).
template <class T, int D = kD>
__device__ __forceinline__ typename T::v8 load_vt_frag_scalar(const uint16_t* vblk, int lane, int ks2, int db) {
  const int hh = lane >> 5, l32 = lane & 31;
  shortx8 x;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int row = ks2 * 16 + (e < 4 ? 4 * hh + e : 8 + 4 * hh + e - 4);
    x[e] = (short)vblk[row * stride_v(D) + db * 32 + l32];
  }
  return __builtin_bit_cast(typename T::v8, x);
}

// The same two operands from an UNPADDED, swizzled tile (64 halves = 128 bytes per row),
// the layout that direct global->LDS loads produce: 16-byte chunk position c' of row r
// holds logical chunk c' ^ k_swz(r) for K and c' ^ v_swz(r) for V.  LDS has 64 four-byte
// banks, so two consecutive rows cover all banks once and the row's parity already picks
// the half; the swizzles spread what remains.
//   K: the 16-byte operand read of a k-step touches rows 0..15 at one chunk (lanes 0..15)
//      and the neighbouring chunk of the same rows (lanes 32..47): rows of equal parity
//      must land on 8 different chunk positions, whichever 16 lanes are served together.
//   V: a transpose read touches 4 rows x 4 chunks (or 8 rows x 2 chunks) per 32 lanes.
// Measured on gfx950: 246 B/clk per CU for the K reads and 199 B/clk for the V reads,
// the same as conflict-free linear addresses.  kblk / vblk must start at a row that is a
// multiple of 16.
__device__ __forceinline__ int k_swz(int r) { return 2 * ((r >> 1) & 3) + ((r >> 3) & 1); }
__device__ __forceinline__ int v_swz(int r) { return 4 * ((r >> 1) & 1) + 2 * ((r >> 2) & 1); }
// head_dim 128: a 256-byte row covers all 64 banks by itself and has 16 chunk positions.
//   K: rows 0..15 at one chunk need 16 different positions, rows 0..7 at a chunk pair too.
//   V: 4 rows x 4 chunks, or 8 rows x 2 chunks, per 32 lanes.
__device__ __forceinline__ int k_swz128(int r) { return 2 * (r & 7) + ((r >> 3) & 1); }
__device__ __forceinline__ int v_swz128(int r) { return 4 * (r & 3) + 2 * ((r >> 2) & 1); }
// head_dim 32: a 64-byte row has 4 chunk positions and four rows cover the banks once.
//   K: rows r, r+4, r+8, r+12 share their banks, so at one chunk they need four different
//      positions, and rows r, r+4 at a chunk pair (2 ks, 2 ks + 1) two disjoint pairs.
//   V: 4 rows x 4 chunks per 32 lanes is 256 contiguous bytes: no swizzle needed.
__device__ __forceinline__ int k_swz32(int r) { return 2 * ((r >> 2) & 1) + ((r >> 3) & 1); }
template <int D>
__device__ __forceinline__ int k_swz_d(int r) { return D == 128 ? k_swz128(r) : (D == 32 ? k_swz32(r) : k_swz(r)); }
template <int D>
__device__ __forceinline__ int v_swz_d(int r) { return D == 128 ? v_swz128(r) : (D == 32 ? 0 : v_swz(r)); }
// Operand fragments out of a swizzled 32-row block of any head_dim (row = D elements).
template <class T, int D>
__device__ __forceinline__ typename T::v8 load_k_frag_swz_d(const uint16_t* kblk, int l32, int hh, int ks) {
  return as_v8<T>(*(const uint4*)&kblk[l32 * D + (((2 * ks + hh) ^ k_swz_d<D>(l32)) * 8)]);
}
template <class T, int D>
__device__ __forceinline__ typename T::v8 load_vt_frag_swz_d(const uint16_t* vblk, int lane, int ks2, int db) {
  const int hh = lane >> 5, p16 = lane & 15, g = (lane >> 4) & 1;
  const int row = ks2 * 16 + 4 * hh + (p16 >> 2);  // (rows row and row + 8 have the same swizzle)
  const int off = (((4 * db + 2 * g + ((p16 & 3) >> 1)) ^ v_swz_d<D>(row)) * 8) + (p16 & 1) * 4;
  typedef __attribute__((address_space(3))) shortx4 lds_s4;
  const shortx4 x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)&vblk[row * D + off]);
  const shortx4 x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)&vblk[(row + 8) * D + off]);
  shortx8 x;
  x[0] = x0[0]; x[1] = x0[1]; x[2] = x0[2]; x[3] = x0[3];
  x[4] = x1[0]; x[5] = x1[1]; x[6] = x1[2]; x[7] = x1[3];
  return __builtin_bit_cast(typename T::v8, x);
}

template <class T>
__device__ __forceinline__ typename T::v8 load_k_frag_swz(const uint16_t* kblk, int l32, int hh, int ks) {
  return as_v8<T>(*(const uint4*)&kblk[l32 * kD + (((2 * ks + hh) ^ k_swz(l32)) * 8)]);
}
template <class T>
__device__ __forceinline__ typename T::v8 load_vt_frag_swz(const uint16_t* vblk, int lane, int ks2, int db) {
  const int hh = lane >> 5, p16 = lane & 15, g = (lane >> 4) & 1;
  const int row = ks2 * 16 + 4 * hh + (p16 >> 2);
  const int off = (((4 * db + 2 * g + ((p16 & 3) >> 1)) ^ v_swz(row)) * 8) + (p16 & 1) * 4;
  typedef __attribute__((address_space(3))) shortx4 lds_s4;
  const shortx4 x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)&vblk[row * kD + off]);
  const shortx4 x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)&vblk[(row + 8) * kD + off]);
  shortx8 x;
  x[0] = x0[0]; x[1] = x0[1]; x[2] = x0[2]; x[3] = x0[3];
  x[4] = x1[0]; x[5] = x1[1]; x[6] = x1[2]; x[7] = x1[3];
  return __builtin_bit_cast(typename T::v8, x);
}

template <int NQB, int D = kD>
struct RowState {
  floatx16 oacc[NQB][D / 32];  // O^T: [qb][d block], rows d = 32*db + 8*(r/4) + 4*hh + r%4
  float m_ref[NQB];       // reference maximum (raw score units), -inf before the first key
  float mc[NQB];          // m_ref * c, 0 while m_ref = -inf
  float lsum[NQB];        // this lane's share of the row sum
};

// Refresh the reference of rows whose block maximum ran away from it.  Each lane
// decides on its own row's evidence only, so a row's arithmetic never depends on
// which other rows share its wavefront.
template <int NQB, int D>
__device__ __forceinline__ void rescale_rows(RowState<NQB, D>& st, int qb, bool refresh, float tmax, float c) {
  const float m_new = refresh ? tmax : st.m_ref[qb];
  const float mc_new = (m_new == -INFINITY) ? 0.f : m_new * c;
  // nothing has been accumulated while the old reference is -inf: keep 0 * alpha out of
  // reach of an infinite alpha
  const float alpha = (st.m_ref[qb] == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(st.mc[qb] - mc_new);
  st.m_ref[qb] = m_new;
  st.mc[qb] = mc_new;
  st.lsum[qb] *= alpha;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) st.oacc[qb][db][r] *= alpha;
}

// Selection by bit r of a visibility word without a compare: the bit, sign-extended, is an
// all-ones or all-zeros word (one v_bfe_i32), and one more bitwise instruction keeps the value or
// replaces it (a test, a compare and a select would be three).
__device__ __forceinline__ uint32_t bit_to_word(uint32_t vis, int r) { return (uint32_t)__builtin_amdgcn_sbfe((int)vis, r, 1); }
__device__ __forceinline__ float keep_or_zero(float x, uint32_t vis, int r) {
  return __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, x) & bit_to_word(vis, r));
}
__device__ __forceinline__ float keep_or_neg_inf(float x, uint32_t vis, int r) {
  const uint32_t m = bit_to_word(vis, r);
  return __builtin_bit_cast(float, (__builtin_bit_cast(uint32_t, x) & m) | (0xFF800000u & ~m));
}

// Probabilities of one 32 x 32 block against the row's current reference, rounded and
// packed as the B operand of the P.V product, plus the lane's share of their row sum.
// fp16: the sum is taken over the ROUNDED probabilities (the numbers the matrix product
// uses), two per v_dot2c instruction.  bf16: the unrounded fp32 values are summed; with
// 8 mantissa bits the rounded sum would cost lse up to ~2e-3 when a row sees only a
// handful of keys.  vis: bit r set = accumulator element r is a visible key.
template <class T, bool MASKED>
__device__ __forceinline__ void prob_block(const floatx16& sv, float c, float mcq, uint32_t vis,
                                           uint32_t (&pk)[8], float& blk) {
  const float nmc = -mcq;
  float l0 = 0.f, l1 = 0.f;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[2 * r], c, nmc));
    float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[2 * r + 1], c, nmc));
    if (MASKED) {
      e0 = keep_or_zero(e0, vis, 2 * r);
      e1 = keep_or_zero(e1, vis, 2 * r + 1);
    }
    pk[r] = T::pack2(e0, e1);
    if (!T::kSumRounded) {
      l0 += e0;
      l1 += e1;
    }
  }
  if (T::kSumRounded) {
    l0 = T::sum2_first(pk[0]);
    l1 = T::sum2_first(pk[1]);
#pragma unroll
    for (int r = 2; r < 8; r += 2) {
      l0 = T::sum2(pk[r], l0);
      l1 = T::sum2(pk[r + 1], l1);
    }
  }
  blk = l0 + l1;
}

// Visibility bits of a lane's 16 accumulator elements for the block starting at key kb0:
// bit r is set iff jlo <= kb0 + 8*(r/4) + 4*hh + r%4 <= jhi.  Built from one 32-bit range
// mask (bit k = key kb0 + 4*hh + k visible) whose nibbles 0, 2, 4, 6 are the lane's keys.
__device__ __forceinline__ uint32_t visible_bits(int kb0, int hh, int jlo, int jhi) {
  int lo = jlo - kb0 - 4 * hh, hi = jhi - kb0 - 4 * hh;
  lo = lo < 0 ? 0 : lo;
  hi = hi > 31 ? 31 : hi;
  const bool none = hi < lo;                          // also covers hi < 0 and lo > 31
  const int lo_s = lo > 31 ? 31 : lo, hi_s = hi < 0 ? 0 : hi;  // shift counts stay in 0..31
  const uint32_t m = none ? 0u : ((0xFFFFFFFFu >> (31 - hi_s)) & (0xFFFFFFFFu << lo_s));
  return (m & 0xFu) | ((m >> 4) & 0xF0u) | ((m >> 8) & 0xF00u) | ((m >> 12) & 0xF000u);
}

// One 32-key block, scores to accumulator, with per-element masking if MASKED.
// kblk / vblk: LDS rows of the block; kb0: its first key index; [jlo, jhi] per lane
// is the visible key range of the lane's query.  FRAG selects how operands come out of
// LDS: 0 padded tile + transpose read, 1 padded tile + 16-bit reads, 2 swizzled tile +
// transpose read.
//
// bias2 (optional): 32 floats in LDS, the block's additive key bias times log2(e).  With a
// bias the row state is kept in the log2 domain (m_ref = mc = reference of s*c + bias2).
// bias_raw (optional, instead of bias2): 32 floats in LDS, the bias divided by |scale|; it
// is simply added to the raw scores and everything else stays in raw-score units.
template <class T, int NQB, bool MASKED, int FRAG, int D>
__device__ __forceinline__ void simple_block(RowState<NQB, D>& st, const typename T::v8 (&qreg)[NQB][D / 16],
                                             const uint16_t* kblk, const uint16_t* vblk, int kb0,
                                             const int (&jlo)[NQB], const int (&jhi)[NQB], int lane,
                                             float c, float tau_raw, const float* bias2 = nullptr,
                                             const float* bias_raw = nullptr) {
  const int l32 = lane & 31, hh = lane >> 5;
  floatx16 sacc[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[qb][r] = 0.f;
  static_assert(FRAG != 2 || D == kD, "swizzled tiles exist for head_dim 64 only");
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    const typename T::v8 ka = FRAG == 2 ? load_k_frag_swz<T>(kblk, l32, hh, ks) : load_k_frag<T, D>(kblk, l32, hh, ks);
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) sacc[qb] = T::mfma(ka, qreg[qb][ks], sacc[qb]);
  }
  if (bias_raw) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 b4 = *(const float4*)&bias_raw[8 * g + 4 * hh];
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        sacc[qb][4 * g + 0] += b4.x;
        sacc[qb][4 * g + 1] += b4.y;
        sacc[qb][4 * g + 2] += b4.z;
        sacc[qb][4 * g + 3] += b4.w;
      }
    }
  }
  uint32_t pk[NQB][8];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const uint32_t vis = MASKED ? visible_bits(kb0, hh, jlo[qb], jhi[qb]) : 0xFFFFu;
    float p[16];
    float ls;  // read after a possible rescale of the row state
    if (bias2) {
      // scores in the log2 domain, bias included; the reference lives in the same domain
      float t[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 b4 = *(const float4*)&bias2[8 * g + 4 * hh];
        t[4 * g + 0] = __builtin_fmaf(sacc[qb][4 * g + 0], c, b4.x);
        t[4 * g + 1] = __builtin_fmaf(sacc[qb][4 * g + 1], c, b4.y);
        t[4 * g + 2] = __builtin_fmaf(sacc[qb][4 * g + 2], c, b4.z);
        t[4 * g + 3] = __builtin_fmaf(sacc[qb][4 * g + 3], c, b4.w);
      }
      float tmax = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (MASKED) t[r] = keep_or_neg_inf(t[r], vis, r);
        tmax = fmaxf(tmax, t[r]);
      }
      tmax = max_xor32(tmax);
      const bool refresh = (tmax - st.m_ref[qb]) > 8.0f;
      if (__any(refresh)) rescale_rows(st, qb, refresh, tmax, 1.0f);
      const float mcq = st.mc[qb];
      ls = st.lsum[qb];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float e = __builtin_amdgcn_exp2f(t[r] - mcq);
        if (MASKED) e = keep_or_zero(e, vis, r);
        p[r] = e;
        ls += e;
      }
    } else {
      float tmax = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float sv = MASKED ? keep_or_neg_inf(sacc[qb][r], vis, r) : sacc[qb][r];
        tmax = fmaxf(tmax, sv);
      }
      tmax = max_xor32(tmax);
      const bool refresh = (tmax - st.m_ref[qb]) > tau_raw;
      if (__any(refresh)) rescale_rows(st, qb, refresh, tmax, c);
      const float nmc = -st.mc[qb];
      ls = st.lsum[qb];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float e = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[qb][r], c, nmc));
        if (MASKED) e = keep_or_zero(e, vis, r);
        p[r] = e;
        ls += e;
      }
    }
    st.lsum[qb] = ls;
#pragma unroll
    for (int r = 0; r < 8; ++r) pk[qb][r] = T::pack2(p[2 * r], p[2 * r + 1]);
  }
#pragma unroll
  for (int ks2 = 0; ks2 < 2; ++ks2) {
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
      const typename T::v8 va = FRAG == 2   ? load_vt_frag_swz<T>(vblk, lane, ks2, db)
                                : FRAG == 0 ? load_vt_frag<T, D>(vblk, lane, ks2, db)
                                            : load_vt_frag_scalar<T, D>(vblk, lane, ks2, db);
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const uint4 pu = make_uint4(pk[qb][ks2 * 4 + 0], pk[qb][ks2 * 4 + 1], pk[qb][ks2 * 4 + 2],
                                    pk[qb][ks2 * 4 + 3]);
        st.oacc[qb][db] = T::mfma(va, as_v8<T>(pu), st.oacc[qb][db]);
      }
    }
  }
}

// ---- pieces shared by both kernels ----------------------------------------------------
struct TileCoord {
  int b, h, qt, n, q0;
};

// CLAMP = false leaves tc.n as loaded (the caller clamps it into [0, max_len] when it first
// needs it, so that the wait for the load can come after other work).
template <int BM, bool CLAMP = true>
__device__ __forceinline__ bool locate_tile(const FaKernelArgs& a, TileCoord& tc) {
  if (a.map_xcd) {
    // Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2.  Tiles of
    // one (batch, head) read the same K/V, so every XCD takes one contiguous eighth of each
    // batch element's (head, query tile) range: K/V re-reads stay in that XCD's L2, and
    // the eighths are equal work whatever the sequence lengths are.
    const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int per = a.xcd_per;                // ceil(heads * n_qtiles / 8)
    tc.b = j / per;
    const int t = x * per + (j - tc.b * per);
    if (tc.b >= a.batch || t >= a.heads * a.n_qtiles) return false;
    tc.h = t / a.n_qtiles;
    tc.qt = t - tc.h * a.n_qtiles;
  } else {
    const int tile = blockIdx.x;
    if (tile >= a.total_tiles) return false;
    tc.qt = tile % a.n_qtiles;
    const int bh = tile / a.n_qtiles;
    tc.h = bh % a.heads;
    tc.b = bh / a.heads;
  }
  int n = a.max_len;
  if (a.seq_lens) {
    n = a.seq_lens[tc.b];
    if (CLAMP) n = n < 0 ? 0 : (n > a.max_len ? a.max_len : n);
  }
  tc.n = n;
  tc.q0 = tc.qt * BM;
  return true;
}

// Workgroup entirely in the padding: o = 0, lse = -inf.
template <int BM, int D = kD, int THREADS = kThreads>
__device__ __forceinline__ void zero_fill(const FaKernelArgs& a, const TileCoord& tc, uint16_t* op, float* lsep) {
  const int tid = threadIdx.x, N = a.max_len;
  constexpr int CH = D / 8;  // 16-byte chunks per row
  const int r = tid / CH, c16 = tid % CH;
  for (int row = tc.q0 + r; row < tc.q0 + BM && row < N; row += THREADS / CH)
    *(uint4*)(op + row * a.os[2] + c16 * 8) = make_uint4(0, 0, 0, 0);
  if (lsep)
    for (int row = tc.q0 + tid; row < tc.q0 + BM && row < N; row += THREADS) lsep[row] = -INFINITY;
}

// ---- rotary position embedding (optional) ----------------------------------------------
// Eight pairs (lo[e], hi[e]) = elements (f + e, f + e + head_dim/2) of one row are rotated by
// the row's angles: lo' = lo cos - hi sin, hi' = hi cos + lo sin, in fp32, and rounded to the
// storage type (nearest even).  cs / sn point at the row's table entries f .. f + 7.
template <class T>
__device__ __forceinline__ void rotate8(uint4& lo, uint4& hi, const float* cs, const float* sn) {
  const float4 c0 = *(const float4*)cs, c1 = *(const float4*)(cs + 4);
  const float4 s0 = *(const float4*)sn, s1 = *(const float4*)(sn + 4);
  const float cc[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
  const float ss[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
  const uint32_t lw[4] = {lo.x, lo.y, lo.z, lo.w}, hw[4] = {hi.x, hi.y, hi.z, hi.w};
  uint32_t lo_out[4], hi_out[4];
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    float l[2], h[2], lr[2], hr[2];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      l[x] = T::to_float((uint16_t)(lw[w] >> (16 * x)));
      h[x] = T::to_float((uint16_t)(hw[w] >> (16 * x)));
      lr[x] = __builtin_fmaf(l[x], cc[2 * w + x], -(h[x] * ss[2 * w + x]));
      hr[x] = __builtin_fmaf(h[x], cc[2 * w + x], l[x] * ss[2 * w + x]);
    }
    lo_out[w] = T::pack2(lr[0], lr[1]);
    hi_out[w] = T::pack2(hr[0], hr[1]);
  }
  lo = make_uint4(lo_out[0], lo_out[1], lo_out[2], lo_out[3]);
  hi = make_uint4(hi_out[0], hi_out[1], hi_out[2], hi_out[3]);
}

// Rotates `rows` rows of K in place in LDS (all threads of the workgroup take part; the caller
// puts barriers around the call).  Element e of tile row r lives at
// tile[r * stride + (((e / 8) ^ swizzle(r & 31)) * 8) + e % 8], swizzle = k_swz_d<D> for tiles
// written by direct loads (SWIZZLED) and 0 for padded tiles; tile row r is key key0 + r
// (clamped into the tensor: rows outside it are never used unmasked).
template <class T, int D, bool SWIZZLED>
__device__ __forceinline__ void rope_rows_in_lds(const FaKernelArgs& a, uint16_t* tile, int stride, int rows, int key0,
                                                 int tid, int nthreads, int key32 = -1) {
  // key32 >= 0: tile rows 32 .. 63 are keys key32 .. key32 + 31 instead of key0 + 32 ... (the
  // two 32-row halves of a pipeline stage are fetched from separately clamped row bases)
  constexpr int HALF = D / 16;  // 16-byte chunks per half row
  for (int u = tid; u < rows * HALF; u += nthreads) {
    const int r = u / HALF, c = u % HALF;
    int key = (key32 >= 0 && r >= 32) ? key32 + r - 32 : key0 + r;
    key = key < 0 ? 0 : (key < a.max_len ? key : a.max_len - 1);
    const int sw = SWIZZLED ? k_swz_d<D>(r & 31) : 0;
    uint4* plo = (uint4*)&tile[r * stride + ((c ^ sw) * 8)];
    uint4* phi = (uint4*)&tile[r * stride + (((c + HALF) ^ sw) * 8)];
    uint4 lo = *plo, hi = *phi;
    rotate8<T>(lo, hi, a.rope_cos + (int64_t)key * a.rope_stride + 8 * c, a.rope_sin + (int64_t)key * a.rope_stride + 8 * c);
    *plo = lo;
    *phi = hi;
  }
}

// ROPE = false: the kernel is never launched with a rotation (no code for it).
template <class T, int NQB, int KS, bool ROPE = true>
__device__ __forceinline__ void load_q(const FaKernelArgs& a, const uint16_t* qp, int qw0, int lane,
                                       typename T::v8 (&qreg)[NQB][KS]) {
  const int l32 = lane & 31, hh = lane >> 5, N = a.max_len;
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    int row = qw0 + qb * 32 + l32;
    row = row < N ? row : N - 1;
    const uint16_t* src = qp + row * a.qs[2] + hh * 8;
    uint4 u[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) u[ks] = *(const uint4*)(src + ks * 16);
    if (ROPE && a.rope_cos) {
      // the lane holds columns 16 ks + 8 hh + e: chunk ks pairs with chunk ks + KS/2
#pragma unroll
      for (int ks = 0; ks < KS / 2; ++ks) {
        const int64_t t = (int64_t)row * a.rope_stride + 16 * ks + 8 * hh;
        rotate8<T>(u[ks], u[ks + KS / 2], a.rope_cos + t, a.rope_sin + t);
      }
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (a.negate_q) {
        u[ks].x ^= 0x80008000u; u[ks].y ^= 0x80008000u; u[ks].z ^= 0x80008000u; u[ks].w ^= 0x80008000u;
      }
      qreg[qb][ks] = as_v8<T>(u[ks]);
    }
  }
}

template <int NQB, int D>
__device__ __forceinline__ void init_state(RowState<NQB, D>& st) {
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    st.m_ref[qb] = -INFINITY;
    st.mc[qb] = 0.f;
    st.lsum[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.oacc[qb][db][r] = 0.f;
  }
}

// Epilogue: o = O / l, cast, store; lse.  A lane holds one output ROW in pieces of four
// columns, so storing from registers would scatter 8-byte pieces over 32 rows per
// instruction.  Each wavefront instead transposes its 32 x 64 block through a private
// LDS patch (rows padded by 16 bytes) and stores whole rows, 16 bytes per lane.
// wave_patch: epi_patch(D) 16-bit elements of LDS owned by this wavefront; the caller has
// made sure (barrier) that nobody still reads tiles from that memory.
constexpr int epi_stride(int D) { return D + 8; }
constexpr int epi_patch(int D) { return 32 * epi_stride(D); }
constexpr int kEpiPatch = epi_patch(kD);

template <class T, int NQB, int D>
__device__ __forceinline__ void epilogue(const FaKernelArgs& a, RowState<NQB, D>& st, uint16_t* op, float* lsep,
                                         int qw0, int n, int lane, uint16_t* wave_patch) {
  constexpr int kEpiStride = epi_stride(D);
  constexpr int CH = D / 8;         // 16-byte chunks per output row
  constexpr int RPP = 64 / CH;      // rows stored per pass
  const int l32 = lane & 31, hh = lane >> 5, N = a.max_len;
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int ig = qw0 + qb * 32 + l32;
    const float ltot = sum_xor32(st.lsum[qb]);
    const bool live = (ig < n) && (ltot > 0.f);
    const float inv = live ? 1.0f / ltot : 0.f;
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = T::pack2(st.oacc[qb][db][4 * g + 0] * inv, st.oacc[qb][db][4 * g + 1] * inv);
        w.y = T::pack2(st.oacc[qb][db][4 * g + 2] * inv, st.oacc[qb][db][4 * g + 3] * inv);
        if (!live) w = make_uint2(0, 0);  // padded rows and rows with no visible key
        *(uint2*)&wave_patch[l32 * kEpiStride + db * 32 + 8 * g + 4 * hh] = w;
      }
    }
    // same wavefront writes and reads the patch: program order is enough
#pragma unroll
    for (int pass = 0; pass < 32 / RPP; ++pass) {
      const int r = pass * RPP + lane / CH;
      const uint4 v = *(const uint4*)&wave_patch[r * kEpiStride + (lane % CH) * 8];
      const int row = qw0 + qb * 32 + r;
      if (row < N) *(uint4*)(op + row * a.os[2] + (lane % CH) * 8) = v;
    }
    if (lsep && hh == 0 && ig < N)
      lsep[ig] = live ? (st.mc[qb] + __builtin_amdgcn_logf(ltot)) * kLn2 : -INFINITY;
  }
}

// One unit of the resident pipelines (head_dim 64, one query block per wavefront, K/V
// blocks as swizzled 32 x 64 tiles in LDS): probabilities of the current block from s_cur;
// meanwhile the matrix cores form the NEXT block's scores (s_nxt, from k_next, started from
// init(s_nxt): zero or a bias) and add the PREVIOUS block's P.V (p_prev, v_prev).
// kb0: first key of the current block; interior: every valid query of the wavefront sees all
// 32 keys, so no mask work; otherwise [jlo, jhi] is the lane's visible key range.
// alive: the lane's query row exists.
// EDGE = false is the straight-line form for the common unit - interior block, every existing
// row already has a reference - whose only branch is the rare overflow redo at the end, so
// that the compiler can interleave the vector work with the matrix products of the same
// wavefront (with the mask and adoption branches in between it cannot); the caller checks
// both conditions.  EDGE = true handles everything.
template <class T, bool EDGE, class Init>
__device__ __forceinline__ void resident_unit(RowState<1>& st, const typename T::v8 (&qreg)[1][4], floatx16& s_cur,
                                              floatx16& s_nxt, typename T::v8 (&p_prev)[2],
                                              typename T::v8 (&p_cur)[2], const uint16_t* k_next,
                                              const uint16_t* v_prev, Init init, int kb0, bool interior, int jlo,
                                              int jhi, bool alive, float c, int lane) {
  const int l32 = lane & 31, hh = lane >> 5;
  typename T::v8 ka[4], va[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) ka[ks] = load_k_frag_swz<T>(k_next, l32, hh, ks);
#pragma unroll
  for (int i = 0; i < 4; ++i) va[i] = load_vt_frag_swz<T>(v_prev, lane, i >> 1, i & 1);
  init(s_nxt);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    s_nxt = T::mfma(ka[ks], qreg[0][ks], s_nxt);
    st.oacc[0][ks & 1] = T::mfma(va[ks], p_prev[ks >> 1], st.oacc[0][ks & 1]);
  }
  uint32_t pk[8];
  float blk;
  uint32_t vis = 0xFFFFu;
  if (EDGE && !interior) vis = visible_bits(kb0, hh, jlo, jhi);
  // Rows that have not seen a key yet (the wavefront's first block, and the odd row whose
  // window starts a block later) adopt this block's maximum as their reference.  Nothing
  // has been accumulated for such a row, so there is nothing to rescale.
  if (EDGE && __any(alive && st.m_ref[0] == -INFINITY)) {
    float t0 = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) t0 = fmaxf(t0, keep_or_neg_inf(s_cur[r], vis, r));
    const float tmax = max_xor32(t0);
    if (st.m_ref[0] == -INFINITY) {
      st.m_ref[0] = tmax;
      st.mc[0] = tmax == -INFINITY ? 0.f : tmax * c;
    }
  }
  if (!EDGE || interior) prob_block<T, false>(s_cur, c, st.mc[0], vis, pk, blk);
  else prob_block<T, true>(s_cur, c, st.mc[0], vis, pk, blk);
  // !(blk <= limit) also catches a NaN sum
  const bool trig = alive && !(blk <= kPLimit);
  if (__any(trig)) {
    // a row refreshes iff one of ITS two lanes tripped: no dependence on other rows
    const bool row_trig = sum_xor32(trig ? 1.f : 0.f) > 0.f;
    float t0 = -INFINITY;
#pragma unroll
    for (int r = 0; r < 16; ++r) t0 = fmaxf(t0, keep_or_neg_inf(s_cur[r], vis, r));
    const float tmax = max_xor32(t0);
    rescale_rows(st, 0, row_trig, tmax, c);
    if (EDGE) prob_block<T, true>(s_cur, c, st.mc[0], vis, pk, blk);
    else prob_block<T, false>(s_cur, c, st.mc[0], vis, pk, blk);
  }
  st.lsum[0] += blk;
  p_cur[0] = as_v8<T>(make_uint4(pk[0], pk[1], pk[2], pk[3]));
  p_cur[1] = as_v8<T>(make_uint4(pk[4], pk[5], pk[6], pk[7]));
}

// ======================================================================================
// Masked kernel: windows (and any tile that needs per-element masks)
// ======================================================================================
template <class T, int D, int NQB, bool V_TR, bool BIAS = false>
// (two wavefronts per SIMD asked for where the compiler would otherwise settle for one)
__global__ __launch_bounds__(kThreads, ((D == 128 && !BIAS) || NQB == 2) ? 2 : 1) void fa_fwd_masked_kernel(const FaKernelArgs a) {
  constexpr int BM = kWaves * 32 * NQB;
  constexpr int SK = stride_k(D), SV = stride_v(D);
  static_assert(2 * kBN * SK >= kWaves * epi_patch(D), "the K stages double as the epilogue patches");
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[2][kBN * SK];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[2][kBN * SV];
  __shared__ __attribute__((aligned(16))) float lds_b[2][BIAS ? kBN : 4];  // key bias * log2(e) of the tile

  TileCoord tc;
  if (!locate_tile<BM>(a, tc)) return;
  const int N = a.max_len, n = tc.n, q0 = tc.q0;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31;

  const uint16_t* qp = (const uint16_t*)a.q + tc.b * a.qs[0] + tc.h * a.qs[1];
  const uint16_t* kp = (const uint16_t*)a.k + tc.b * a.ks[0] + tc.h * a.ks[1];
  const uint16_t* vp = (const uint16_t*)a.v + tc.b * a.vs[0] + tc.h * a.vs[1];
  uint16_t* op = (uint16_t*)a.o + tc.b * a.os[0] + tc.h * a.os[1];
  float* lsep = a.lse ? a.lse + ((int64_t)tc.b * a.heads + tc.h) * N : nullptr;

  if (q0 >= n) {
    zero_fill<BM, D>(a, tc, op, lsep);
    return;
  }

  // key range of this workgroup
  const int q_last = (q0 + BM < n ? q0 + BM : n) - 1;
  int lo = 0, hi = n;
  if (a.wl >= 0) lo = q0 - a.wl > 0 ? q0 - a.wl : 0;
  if (a.wr >= 0) hi = q_last + a.wr + 1 < n ? q_last + a.wr + 1 : n;
  const int t_lo = lo / kBN;
  const int t_hi = (hi + kBN - 1) / kBN;

  // this wavefront's queries
  const int qw0 = q0 + wave * 32 * NQB;
  const int qw_last = (qw0 + 32 * NQB < n ? qw0 + 32 * NQB : n) - 1;  // < qw0: all padding
  const bool wave_has_rows = qw_last >= qw0;

  typename T::v8 qreg[NQB][D / 16];
  load_q<T, NQB>(a, qp, qw0, lane, qreg);
  RowState<NQB, D> st;
  init_state(st);
  int jlo[NQB], jhi[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int ig = qw0 + qb * 32 + l32;
    jlo[qb] = 0;
    jhi[qb] = n - 1;
    if (a.wl >= 0 && ig - a.wl > jlo[qb]) jlo[qb] = ig - a.wl;
    if (a.wr >= 0 && ig + a.wr < jhi[qb]) jhi[qb] = ig + a.wr;
  }

  // staging: a 64-key tile is 64 rows of D/8 16-byte chunks; thread t moves chunk t % (D/8)
  // of rows t / (D/8) + i * RS, i = 0 .. NST-1 (named registers, not an array: an array
  // captured by the lambdas ends up in scratch memory)
  constexpr int CH = D / 8, RS = kThreads / CH, NST = kBN / RS;  // NST = 1, 2, 4 for D = 32, 64, 128
  const int st_r = tid / CH, st_c = (tid % CH) * 8;
  uint4 kst0, kst1, kst2, kst3, vst0, vst1, vst2, vst3;
  auto fetch_row = [&](int jg, uint4& kk, uint4& vv) {
    const int jc = jg < N ? jg : N - 1;
    kk = *(const uint4*)(kp + jc * a.ks[2] + st_c);
    vv = *(const uint4*)(vp + jc * a.vs[2] + st_c);
    // padded V rows are replaced by zeros: 0 * (whatever is stored there) must be 0
    if (jg >= n) vv = make_uint4(0, 0, 0, 0);
  };
  const uint16_t* bp = BIAS ? (const uint16_t*)a.key_bias + tc.b * a.kb_stride : nullptr;
  float bst = 0.f;  // threads 0..63: the bias of key t*64 + tid
  auto fetch = [&](int t) {
    fetch_row(t * kBN + st_r, kst0, vst0);
    if (NST > 1) fetch_row(t * kBN + RS + st_r, kst1, vst1);
    if (NST > 2) {
      fetch_row(t * kBN + 2 * RS + st_r, kst2, vst2);
      fetch_row(t * kBN + 3 * RS + st_r, kst3, vst3);
    }
    if (BIAS && tid < kBN) {
      const int jg = t * kBN + tid;
      bst = T::to_float(bp[jg < N ? jg : N - 1]) * 1.44269504088896340736f;
    }
  };
  auto stash = [&](int buf) {
    if (BIAS && tid < kBN) lds_b[buf][tid] = bst;
    *(uint4*)&lds_k[buf][st_r * SK + st_c] = kst0;
    *(uint4*)&lds_v[buf][st_r * SV + st_c] = vst0;
    if (NST > 1) {
      *(uint4*)&lds_k[buf][(RS + st_r) * SK + st_c] = kst1;
      *(uint4*)&lds_v[buf][(RS + st_r) * SV + st_c] = vst1;
    }
    if (NST > 2) {
      *(uint4*)&lds_k[buf][(2 * RS + st_r) * SK + st_c] = kst2;
      *(uint4*)&lds_v[buf][(2 * RS + st_r) * SV + st_c] = vst2;
      *(uint4*)&lds_k[buf][(3 * RS + st_r) * SK + st_c] = kst3;
      *(uint4*)&lds_v[buf][(3 * RS + st_r) * SV + st_c] = vst3;
    }
  };

  fetch(t_lo);
  stash(0);
  __syncthreads();
  // rotary embedding: a staged K tile is rotated in place before anybody reads it
  if (a.rope_cos) {
    rope_rows_in_lds<T, D, false>(a, lds_k[0], SK, kBN, t_lo * kBN, tid, kThreads);
    __syncthreads();
  }

  int buf = 0;
  for (int t = t_lo; t < t_hi; ++t) {
    if (t + 1 < t_hi) fetch(t + 1);
    if (wave_has_rows) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const int kb0 = t * kBN + kb * 32;
        // wavefront-uniform: skip key blocks no query of this wavefront sees
        if (kb0 >= n) continue;
        if (a.wl >= 0 && kb0 + 31 < qw0 - a.wl) continue;
        if (a.wr >= 0 && kb0 > qw_last + a.wr) continue;
        simple_block<T, NQB, true, V_TR ? 0 : 1>(st, qreg, &lds_k[buf][kb * 32 * SK], &lds_v[buf][kb * 32 * SV],
                                                 kb0, jlo, jhi, lane, a.c, a.tau_raw,
                                                 BIAS ? &lds_b[buf][kb * 32] : nullptr);
      }
    }
    if (t + 1 < t_hi) stash(buf ^ 1);
    __syncthreads();
    buf ^= 1;
    if (a.rope_cos && t + 1 < t_hi) {
      rope_rows_in_lds<T, D, false>(a, lds_k[buf], SK, kBN, (t + 1) * kBN, tid, kThreads);
      __syncthreads();
    }
  }
  // the loop ended with a barrier: the K stages are free
  epilogue<T, NQB>(a, st, op, lsep, qw0, n, lane, &lds_k[0][0] + wave * epi_patch(D));
}

// ======================================================================================
// Window kernel: local layers.  The key range of a 128-row query tile is only a few
// hundred keys, so the work is bound by getting K/V (and Q, O) through HBM once and by
// latency: K/V move in 32-key blocks through a ring of kWinStages LDS stages filled by
// direct global->LDS loads, kWinStages - 1 blocks ahead of the arithmetic (small stages
// keep several workgroups per compute unit AND several blocks per workgroup in flight).
// A wavefront multiplies only the blocks its own 32 queries can see; blocks it sees
// completely skip the mask work.  One barrier per block.
// ======================================================================================
constexpr int kWinStages = 4;
constexpr int kWinBN = 32;  // keys per stage

template <class T>
__global__ __launch_bounds__(kThreads, 2) void fa_fwd_window_kernel(const FaKernelArgs a) {
  constexpr int BM = kWaves * 32;
  // at least the four 32 x 72 epilogue patches must fit in lds_k
  constexpr int kStageElems = kWinBN * kD;
  constexpr int kKElems = kWinStages * kStageElems > kWaves * kEpiPatch ? kWinStages * kStageElems : kWaves * kEpiPatch;
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[kKElems];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[kWinStages * kStageElems];

  TileCoord tc;
  if (!locate_tile<BM>(a, tc)) return;
  const int N = a.max_len, n = tc.n, q0 = tc.q0;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31;

  const uint16_t* qp = (const uint16_t*)a.q + tc.b * a.qs[0] + tc.h * a.qs[1];
  const uint16_t* kp = (const uint16_t*)a.k + tc.b * a.ks[0] + tc.h * a.ks[1];
  const uint16_t* vp = (const uint16_t*)a.v + tc.b * a.vs[0] + tc.h * a.vs[1];
  uint16_t* op = (uint16_t*)a.o + tc.b * a.os[0] + tc.h * a.os[1];
  float* lsep = a.lse ? a.lse + ((int64_t)tc.b * a.heads + tc.h) * N : nullptr;

  if (q0 >= n) {
    zero_fill<BM>(a, tc, op, lsep);
    return;
  }

  // key range of this workgroup, in 32-key blocks
  const int q_last = (q0 + BM < n ? q0 + BM : n) - 1;
  int lo = 0, hi = n;
  if (a.wl >= 0) lo = q0 - a.wl > 0 ? q0 - a.wl : 0;
  if (a.wr >= 0) hi = q_last + a.wr + 1 < n ? q_last + a.wr + 1 : n;
  const int t_lo = lo / kWinBN;
  const int t_hi = (hi + kWinBN - 1) / kWinBN;

  // Block t goes to stage t % kWinStages.  Wavefront w moves rows 8w..8w+7 of the block
  // (one 1 KB load each for K and V); a lane's row is clamped to the last row of the
  // tensor (rows >= n are masked or zeroed below), so its global offset is a per-lane
  // 32-bit byte offset from the (batch, head) slice.
  const int dl_r = 8 * wave + (lane >> 3);
  const uint32_t kchunk = 2u * (uint32_t)(((lane & 7) ^ k_swz(dl_r)) * 8);
  const uint32_t vchunk = 2u * (uint32_t)(((lane & 7) ^ v_swz(dl_r)) * 8);
  const uint32_t krow_b = 2u * (uint32_t)a.ks[2], vrow_b = 2u * (uint32_t)a.vs[2];
  auto issue_block = [&](int t) {
    const int stage = t % kWinStages;
    const int jg = t * kWinBN + dl_r;
    const uint32_t jc = (uint32_t)(jg < N ? jg : N - 1);
    load16_to_lds(kp, jc * krow_b + kchunk, &lds_k[stage * kStageElems + 8 * wave * kD]);
    load16_to_lds(vp, jc * vrow_b + vchunk, &lds_v[stage * kStageElems + 8 * wave * kD]);
  };
  // After a block has landed: V rows at or beyond n are overwritten with zeros by the
  // lanes that fetched them (0 * whatever is stored in the padding must be 0).
  auto scrub_block = [&](int t) {
    if (t * kWinBN + kWinBN <= n) return;
    if (t * kWinBN + dl_r >= n)
      *(uint4*)&lds_v[(t % kWinStages) * kStageElems + dl_r * kD + (lane & 7) * 8] = make_uint4(0, 0, 0, 0);
  };

  // prologue: kWinStages - 1 blocks in flight before anything else
#pragma unroll
  for (int i = 0; i < kWinStages - 1; ++i)
    if (t_lo + i < t_hi) issue_block(t_lo + i);

  const int qw0 = q0 + wave * 32;
  const int qw_last = (qw0 + 32 < n ? qw0 + 32 : n) - 1;  // < qw0: all padding
  const bool wave_has_rows = qw_last >= qw0;
  typename T::v8 qreg[1][4];
  load_q<T, 1, 4, false>(a, qp, qw0, lane, qreg);
  RowState<1> st;
  init_state(st);
  int jlo[1], jhi[1];
  {
    const int ig = qw0 + l32;
    jlo[0] = 0;
    jhi[0] = n - 1;
    if (a.wl >= 0 && ig - a.wl > jlo[0]) jlo[0] = ig - a.wl;
    if (a.wr >= 0 && ig + a.wr < jhi[0]) jhi[0] = ig + a.wr;
  }

  for (int t = t_lo; t < t_hi; ++t) {
    // Each block is 2 loads per wavefront, and loads complete in order: block t has landed
    // once at most 2 * (number of younger blocks in flight) loads are outstanding.
    const int younger = (t_hi - 1 - t < kWinStages - 2 ? t_hi - 1 - t : kWinStages - 2);
    if (younger >= 2) wait_vmcnt<4>();
    else if (younger == 1) wait_vmcnt<2>();
    else wait_vmcnt<0>();
    scrub_block(t);
    __syncthreads();
    // stage (t-1) % kWinStages is free now: every wavefront finished block t-1 before this barrier
    if (t + kWinStages - 1 < t_hi) issue_block(t + kWinStages - 1);
    const int kb0 = t * kWinBN;
    // wavefront-uniform: skip key blocks no query of this wavefront sees
    if (!wave_has_rows || kb0 >= n) continue;
    if (a.wl >= 0 && kb0 + 31 < qw0 - a.wl) continue;
    if (a.wr >= 0 && kb0 > qw_last + a.wr) continue;
    // blocks every valid query of the wavefront sees completely need no mask work
    const bool interior = kb0 + 32 <= n && (a.wl < 0 || kb0 >= qw_last - a.wl) &&
                          (a.wr < 0 || kb0 + 31 <= qw0 + a.wr);
    const uint16_t* kblk = &lds_k[(t % kWinStages) * kStageElems];
    const uint16_t* vblk = &lds_v[(t % kWinStages) * kStageElems];
    if (interior) simple_block<T, 1, false, 2>(st, qreg, kblk, vblk, kb0, jlo, jhi, lane, a.c, a.tau_raw);
    else simple_block<T, 1, true, 2>(st, qreg, kblk, vblk, kb0, jlo, jhi, lane, a.c, a.tau_raw);
  }
  __syncthreads();  // all blocks consumed: the K stages become the epilogue patches
  epilogue<T, 1>(a, st, op, lsep, qw0, n, lane, lds_k + wave * kEpiPatch);
}

// ======================================================================================
// Resident window kernel: local layers whose whole key range per 128-row query tile fits
// in kResBlocks 32-key blocks of LDS (the paper's 63/64 window needs exactly 8).  All of
// the tile's K/V is requested at once with direct global->LDS loads, one barrier
// publishes it, and then every wavefront runs the same software pipeline as the global
// kernel over just the blocks its own 32 queries can see - next block's scores and the
// previous block's P.V on the matrix cores while the vector ALU forms this block's
// probabilities - with mask work only on the blocks that are cut by the window or the
// sequence end.  No further barriers until the epilogue.
// ======================================================================================
constexpr int kResBlocks = 8;

template <class T, bool BIAS = false>
__global__ __launch_bounds__(kThreads, 2) void fa_fwd_window_resident_kernel(const FaKernelArgs a) {
  constexpr int BM = kWaves * 32;
  constexpr int kBlk = 32 * kD;  // elements per block
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[kResBlocks * kBlk];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[kResBlocks * kBlk];
  // BIAS: additive key bias / |scale| of every resident key; it enters the scores as the C
  // operand of each block's first MFMA
  __shared__ __attribute__((aligned(16))) float lds_bias[BIAS ? kResBlocks * 32 : 4];

  TileCoord tc;
  if (!locate_tile<BM, false>(a, tc)) return;  // tc.n still as loaded: see below
  const int N = a.max_len, q0 = tc.q0;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;

  const uint16_t* qp = (const uint16_t*)a.q + tc.b * a.qs[0] + tc.h * a.qs[1];
  const uint16_t* kp = (const uint16_t*)a.k + tc.b * a.ks[0] + tc.h * a.ks[1];
  const uint16_t* vp = (const uint16_t*)a.v + tc.b * a.vs[0] + tc.h * a.vs[1];
  uint16_t* op = (uint16_t*)a.o + tc.b * a.os[0] + tc.h * a.os[1];
  float* lsep = a.lse ? a.lse + ((int64_t)tc.b * a.heads + tc.h) * N : nullptr;

  // Key blocks this tile can touch, from the tile position and the tensor length alone: the
  // loads below are issued BEFORE the sequence length is looked at, so that the latency of
  // reading it (it sits in device memory) overlaps theirs instead of preceding it - a
  // workgroup that is alone on its compute unit (short sequences) has nothing else to hide
  // it behind.  Block b lives in slot b - b_lo; blocks past the sequence end are fetched and
  // never read.
  const int lo = q0 - a.wl > 0 ? q0 - a.wl : 0;
  const int b_lo = lo >> 5;
  int b_hi_ld = (q0 + BM + a.wr + 31) >> 5;
  b_hi_ld = b_hi_ld < ((N + 31) >> 5) ? b_hi_ld : ((N + 31) >> 5);
  if (b_hi_ld > b_lo + kResBlocks) b_hi_ld = b_lo + kResBlocks;  // never true for the windows the host routes here

  // Wavefront w moves rows 8w..8w+7 of every block (one 1 KB load each for K and V).  A
  // lane's row is clamped to the last row of the tensor (rows >= n are masked or zeroed
  // below), so its global offset is a per-lane 32-bit byte offset from the slice.
  const int dl_r = 8 * wave + (lane >> 3);
  {
    const int b_hi = b_hi_ld;
    const uint32_t kchunk = 2u * (uint32_t)(((lane & 7) ^ k_swz(dl_r)) * 8);
    const uint32_t vchunk = 2u * (uint32_t)(((lane & 7) ^ v_swz(dl_r)) * 8);
    const uint32_t krow_b = 2u * (uint32_t)a.ks[2], vrow_b = 2u * (uint32_t)a.vs[2];
    if (b_hi * 32 <= N) {
      // every row exists: one per-lane offset, the block base advances in scalar registers
      const uint32_t klane = (uint32_t)dl_r * krow_b + kchunk, vlane = (uint32_t)dl_r * vrow_b + vchunk;
      const uint16_t* kg = kp + (int64_t)b_lo * 32 * a.ks[2];
      const uint16_t* vg = vp + (int64_t)b_lo * 32 * a.vs[2];
#pragma unroll
      for (int i = 0; i < kResBlocks; ++i) {
        if (b_lo + i < b_hi) {
          load16_to_lds(kg, klane, &lds_k[i * kBlk + 8 * wave * kD]);
          load16_to_lds(vg, vlane, &lds_v[i * kBlk + 8 * wave * kD]);
          kg += 32 * a.ks[2];
          vg += 32 * a.vs[2];
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < kResBlocks; ++i) {
        if (b_lo + i < b_hi) {
          const int jg = (b_lo + i) * 32 + dl_r;
          const uint32_t jc = (uint32_t)(jg < N ? jg : N - 1);
          load16_to_lds(kp, jc * krow_b + kchunk, &lds_k[i * kBlk + 8 * wave * kD]);
          load16_to_lds(vp, jc * vrow_b + vchunk, &lds_v[i * kBlk + 8 * wave * kD]);
        }
      }
    }
  }

  if (BIAS) {
    // one value per thread: key b_lo*32 + tid (256 resident keys, 256 threads)
    const uint16_t* bp = (const uint16_t*)a.key_bias + tc.b * a.kb_stride;
    const int jg = b_lo * 32 + tid;
    lds_bias[tid] = T::to_float(bp[jg < N ? jg : N - 1]) * a.inv_abs_scale;
  }

  const int qw0 = q0 + wave * 32;
  typename T::v8 qreg[1][4];
  load_q<T, 1, 4, false>(a, qp, qw0, lane, qreg);

  // only now the sequence length
  const int n = tc.n < 0 ? 0 : (tc.n > N ? N : tc.n);
  tc.n = n;
  if (q0 >= n) {
    wait_direct_loads();  // the loads write this workgroup's LDS: they must land before it ends
    zero_fill<BM>(a, tc, op, lsep);
    return;
  }
  const int q_last = (q0 + BM < n ? q0 + BM : n) - 1;
  const int hi = q_last + a.wr + 1 < n ? q_last + a.wr + 1 : n;
  int b_hi = (hi + 31) >> 5;  // blocks [b_lo, b_hi) hold visible keys
  if (b_hi > b_hi_ld) b_hi = b_hi_ld;
  const int qw_last = (qw0 + 32 < n ? qw0 + 32 : n) - 1;  // < qw0: all padding
  const bool wave_has_rows = qw_last >= qw0;
  RowState<1> st;
  init_state(st);
  const int ig = qw0 + l32;
  const bool alive = ig < n;
  int jlo = ig - a.wl > 0 ? ig - a.wl : 0;
  int jhi = ig + a.wr < n - 1 ? ig + a.wr : n - 1;
  const float c = a.c;

  wait_direct_loads();
  // V rows at or beyond n are overwritten with zeros by the lanes that fetched them
  // (0 * whatever is stored in the padding must be 0); only the last block can have any
  {
    const int i = b_hi - 1 - b_lo;
    if ((b_hi - 1) * 32 + dl_r >= n) *(uint4*)&lds_v[i * kBlk + dl_r * kD + (lane & 7) * 8] = make_uint4(0, 0, 0, 0);
  }
  __syncthreads();

  if (wave_has_rows) {
    // blocks this wavefront's queries can see
    int fb = (qw0 - a.wl) >> 5;
    fb = fb < b_lo ? b_lo : fb;
    int lb = (qw_last + a.wr) >> 5;
    lb = lb > b_hi - 1 ? b_hi - 1 : lb;

    floatx16 sA, sB;
    typename T::v8 pA[2], pB[2];
    pA[0] = pA[1] = as_v8<T>(make_uint4(0, 0, 0, 0));
    // accumulator input of a block's score product: its bias, or zero
    auto score_init = [&](floatx16& sv, int slot) {
      if (BIAS) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 b4 = *(const float4*)&lds_bias[slot * 32 + 8 * g + 4 * hh];
          sv[4 * g + 0] = b4.x;
          sv[4 * g + 1] = b4.y;
          sv[4 * g + 2] = b4.z;
          sv[4 * g + 3] = b4.w;
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) sv[r] = 0.f;
      }
    };
    score_init(sA, fb - b_lo);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      sA = T::mfma(load_k_frag_swz<T>(&lds_k[(fb - b_lo) * kBlk], l32, hh, ks), qreg[0][ks], sA);

    // One unit of the pipeline: probabilities of block u; scores of block u+1; P.V of
    // block u-1.  At the two ends the neighbour slot is clamped: its product is unused
    // (scores) or multiplied by zero probabilities (P.V).
    auto unit = [&](floatx16& s_cur, floatx16& s_nxt, typename T::v8 (&p_prev)[2], typename T::v8 (&p_cur)[2], int u) {
      const int un = u + 1 > b_hi - 1 ? b_hi - 1 : u + 1;
      const int up = u - 1 < b_lo ? b_lo : u - 1;
      // blocks every valid query of the wavefront sees completely need no mask work
      const int kb0 = u * 32;
      const bool interior = kb0 + 32 <= n && kb0 >= qw_last - a.wl && kb0 + 31 <= qw0 + a.wr;
      // (the straight-line form of the unit measured no faster here: two wavefronts per SIMD
      // already overlap each other's matrix and vector work)
      resident_unit<T, true>(st, qreg, s_cur, s_nxt, p_prev, p_cur, &lds_k[(un - b_lo) * kBlk],
                             &lds_v[(up - b_lo) * kBlk], [&](floatx16& sv) { score_init(sv, un - b_lo); }, kb0,
                             interior, jlo, jhi, alive, c, lane);
    };
    auto drain = [&](typename T::v8 (&p_last)[2], int u) {
      const uint16_t* vblk = &lds_v[(u - b_lo) * kBlk];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        st.oacc[0][i & 1] = T::mfma(load_vt_frag_swz<T>(vblk, lane, i >> 1, i & 1), p_last[i >> 1], st.oacc[0][i & 1]);
    };
    int u = fb;
    for (; u + 1 <= lb; u += 2) {
      unit(sA, sB, pA, pB, u);
      unit(sB, sA, pB, pA, u + 1);
    }
    if (u <= lb) {
      unit(sA, sB, pA, pB, u);
      drain(pB, u);
    } else {
      drain(pA, lb);
    }
  }
  __syncthreads();  // all blocks consumed: the K storage becomes the epilogue patches
  epilogue<T, 1>(a, st, op, lsep, qw0, n, lane, lds_k + wave * kEpiPatch);
}

// ======================================================================================
// Two-phase window kernel: local layers of head_dim 64 in which a wavefront's 32 queries see at
// most kTwoPhaseBlocks 32-key blocks (the paper's 63/64 window: five) and a 128-row tile at
// most kResBlocks.  Such a layer is bound by memory traffic (64 flop per byte), and what
// decides its speed is how many workgroups a compute unit holds at once: workgroups load,
// compute and store one after the other, so the more of them are resident, the more of the
// time the memory system has requests in flight.  With K and V both resident in LDS (64 KB,
// the kernel above) that is two workgroups per unit.  Here ONE 32 KB region holds the K
// blocks first and the V blocks afterwards, which allows four workgroups per unit:
//   phase 1: K blocks arrive by direct loads; every wavefront forms the scores of ALL its
//            visible blocks (up to 5 x 16 accumulator registers per lane: a whole window row
//            fits in registers), barrier;
//   phase 2: the V blocks are requested into the same region, and while they travel the
//            wavefront turns its scores into probabilities - an ordinary softmax over the
//            whole row: exact maximum, no running reference, nothing to rescale;
//   phase 3: V has landed (barrier): O^T = sum over blocks of V^T P^T, epilogue.
// No software pipeline inside a wavefront: the four wavefronts a SIMD holds are in different
// phases and fill each other's gaps.  (Touching V's cache lines at the start, so that the
// phase-2 request finds them in cache, measured 8 % slower on a cold cache: not done.)
// ======================================================================================
constexpr int kTwoPhaseBlocks = 5;

template <class T, int D>
__global__ __launch_bounds__(kThreads, D == 128 ? 2 : 4) void fa_fwd_window_twophase_kernel(const FaKernelArgs a) {
  constexpr int BM = kWaves * 32;
  constexpr int KS = D / 16, DB = D / 32;
  constexpr int kBlk = 32 * D;  // elements per block
  static_assert(kResBlocks * kBlk >= kWaves * epi_patch(D), "the region doubles as the epilogue patches");
  __shared__ __attribute__((aligned(16))) uint16_t lds[kResBlocks * kBlk];

  TileCoord tc;
  if (!locate_tile<BM, false>(a, tc)) return;  // tc.n still as loaded: see below
  const int N = a.max_len, q0 = tc.q0;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;

  const uint16_t* qp = (const uint16_t*)a.q + tc.b * a.qs[0] + tc.h * a.qs[1];
  const uint16_t* kp = (const uint16_t*)a.k + tc.b * a.ks[0] + tc.h * a.ks[1];
  const uint16_t* vp = (const uint16_t*)a.v + tc.b * a.vs[0] + tc.h * a.vs[1];
  uint16_t* op = (uint16_t*)a.o + tc.b * a.os[0] + tc.h * a.os[1];
  float* lsep = a.lse ? a.lse + ((int64_t)tc.b * a.heads + tc.h) * N : nullptr;

  // Key blocks this tile can touch, from the tile position and the tensor length alone (the
  // sequence length is looked at only after the loads are on their way).  Block b lives in
  // slot b - b_lo; blocks past the sequence end are fetched and never read.
  const int lo = q0 - a.wl > 0 ? q0 - a.wl : 0;
  const int b_lo = lo >> 5;
  int b_hi_ld = (q0 + BM + a.wr + 31) >> 5;
  b_hi_ld = b_hi_ld < ((N + 31) >> 5) ? b_hi_ld : ((N + 31) >> 5);
  if (b_hi_ld > b_lo + kResBlocks) b_hi_ld = b_lo + kResBlocks;  // never true for the windows the host routes here

  // A direct load moves 1 KB = RPL rows of a block (lane L: row L / CH, chunk position L % CH of
  // the load), so a block is LPB loads; the loads of all blocks, numbered block * LPB + part,
  // are dealt round-robin to the four wavefronts: wavefront w issues loads w, w + 4, w + 8, ...
  //   head_dim 64 (LPB 4): load x of the wavefront is block x, part w;
  //   head_dim 128 (LPB 8): block x / 2, part w + 4 (x % 2);
  //   head_dim 32 (LPB 2): block 2 x + w / 2, part w % 2.
  // So a wavefront has NPART (1 or 2) distinct parts, whose per-lane offsets are computed once,
  // and its blocks advance by a fixed step: the scalar base moves by a 64-bit add per block.
  // A lane's row is clamped to the last row of the tensor where the tile reaches past it (rows
  // >= n are masked or zeroed below); its global offset is then a per-lane 32-bit byte offset
  // from the slice.
  constexpr int CH = D / 8, RPL = 64 / CH, LPB = 32 / RPL;   // D = 32: 4, 16, 2;  64: 8, 8, 4;  128: 16, 4, 8
  constexpr int kLoadsPerWave = kResBlocks * LPB / kWaves;
  constexpr int NPART = LPB > kWaves ? LPB / kWaves : 1;
  constexpr int BSTEP = LPB < kWaves ? kWaves / LPB : 1;     // blocks between consecutive loads of one part
  const int blk0 = LPB < kWaves ? wave / LPB : 0;            // the wavefront's first block
  const bool all_rows_exist = b_hi_ld * 32 <= N;   // workgroup-uniform
  auto request_blocks = [&](const uint16_t* base, int64_t row_elems, bool is_k) {
    const uint32_t row_bytes = 2u * (uint32_t)row_elems;
    int row_of[NPART];            // row within a block that this lane fetches, per part
    uint32_t chunk_bytes[NPART];  // byte offset of its (swizzled) 16-byte chunk within the row
    uint32_t lds_part[NPART];     // element offset of the part within a block's LDS slot
#pragma unroll
    for (int pi = 0; pi < NPART; ++pi) {
      const int part = LPB >= kWaves ? wave + kWaves * pi : wave % LPB;
      row_of[pi] = part * RPL + lane / CH;
      const int swz = is_k ? k_swz_d<D>(row_of[pi]) : v_swz_d<D>(row_of[pi]);
      chunk_bytes[pi] = 2u * (uint32_t)(((lane % CH) ^ swz) * 8);
      lds_part[pi] = (uint32_t)(part * RPL * D);
    }
    if (all_rows_exist) {
      uint32_t lane_off[NPART];
#pragma unroll
      for (int pi = 0; pi < NPART; ++pi) lane_off[pi] = (uint32_t)row_of[pi] * row_bytes + chunk_bytes[pi];
      const int64_t blk_elems = 32 * row_elems;
      const uint16_t* g = base + (int64_t)(b_lo + blk0) * blk_elems;
#pragma unroll
      for (int x = 0; x < kLoadsPerWave; ++x) {
        const int pi = x % NPART;
        const int i = blk0 + (x / NPART) * BSTEP;   // wavefront-uniform
        if (b_lo + i < b_hi_ld) load16_to_lds(g, lane_off[pi], &lds[i * kBlk + lds_part[pi]]);
        if (pi == NPART - 1) g += BSTEP * blk_elems;
      }
    } else {
#pragma unroll
      for (int x = 0; x < kLoadsPerWave; ++x) {
        const int pi = x % NPART;
        const int i = blk0 + (x / NPART) * BSTEP;
        if (b_lo + i < b_hi_ld) {
          const int jg = (b_lo + i) * 32 + row_of[pi];
          const uint32_t jc = (uint32_t)(jg < N ? jg : N - 1);
          load16_to_lds(base, jc * row_bytes + chunk_bytes[pi], &lds[i * kBlk + lds_part[pi]]);
        }
      }
    }
  };
  request_blocks(kp, a.ks[2], true);

  const int qw0 = q0 + wave * 32;
  typename T::v8 qreg[1][KS];
  load_q<T, 1>(a, qp, qw0, lane, qreg);

  // only now the sequence length
  const int n = tc.n < 0 ? 0 : (tc.n > N ? N : tc.n);
  tc.n = n;
  if (q0 >= n) {
    wait_direct_loads();  // the loads write this workgroup's LDS: they must land before it ends
    zero_fill<BM, D>(a, tc, op, lsep);
    return;
  }
  const int q_last = (q0 + BM < n ? q0 + BM : n) - 1;
  const int hi = q_last + a.wr + 1 < n ? q_last + a.wr + 1 : n;
  int b_hi = (hi + 31) >> 5;  // blocks [b_lo, b_hi) hold visible keys
  if (b_hi > b_hi_ld) b_hi = b_hi_ld;
  const int qw_last = (qw0 + 32 < n ? qw0 + 32 : n) - 1;  // < qw0: all padding
  const bool wave_has_rows = qw_last >= qw0;
  const int ig = qw0 + l32;
  const int jlo = ig - a.wl > 0 ? ig - a.wl : 0;
  const int jhi = ig + a.wr < n - 1 ? ig + a.wr : n - 1;
  const float c = a.c;
  // blocks this wavefront's queries can see: fb .. fb + cnt - 1, cnt <= kTwoPhaseBlocks
  int fb = (qw0 - a.wl) >> 5;
  fb = fb < b_lo ? b_lo : fb;
  int lb = (qw_last + a.wr) >> 5;
  lb = lb > b_hi - 1 ? b_hi - 1 : lb;
  int cnt = wave_has_rows ? lb - fb + 1 : 0;
  cnt = cnt > kTwoPhaseBlocks ? kTwoPhaseBlocks : cnt;  // (the host routes no wider window here)

  // ---- phase 1: scores of every visible block
  wait_direct_loads();
  __syncthreads();
  if (a.rope_cos) {
    // rotary embedding: the K blocks are rotated in place, once for the four wavefronts
    rope_rows_in_lds<T, D, true>(a, lds, D, (b_hi - b_lo) * 32, b_lo * 32, tid, kThreads);
    __syncthreads();
  }
  floatx16 sc[kTwoPhaseBlocks];   // sc[i] is set and used for i < cnt only
#pragma unroll
  for (int i = 0; i < kTwoPhaseBlocks; ++i) {
    if (i < cnt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[i][r] = 0.f;
      const uint16_t* kblk = &lds[(fb + i - b_lo) * kBlk];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) sc[i] = T::mfma(load_k_frag_swz_d<T, D>(kblk, l32, hh, ks), qreg[0][ks], sc[i]);
    }
  }
  __syncthreads();  // every wavefront has its K fragments out of the region

  // ---- phase 2: request V into the same region; softmax meanwhile
  request_blocks(vp, a.vs[2], false);
  // The paper's window (63 left, 64 right) away from the ends of the sequence: the wavefront's 32
  // queries see five blocks, the middle three completely, and of the outer two query t (0..31)
  // sees keys t+1..31 of the first and keys 0..t of the last: between them exactly one block's
  // worth of keys per query.  The last block's scores are merged into the first's (element by
  // element, the one the query sees), the merged block takes the unmasked path like the middle
  // three, and its probabilities are dealt back to the two blocks for the P.V products.  A
  // masked block costs three times the vector instructions of an unmasked one.
  const bool merged_ends = a.wl == 63 && a.wr == 64 && qw0 >= 64 && qw0 + 96 <= n;   // wavefront-uniform; implies cnt == 5
  if (merged_ends) {
    // accumulator element r is key offset 8 (r / 4) + 4 hh + r % 4 of its block
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[0][r] = 8 * (r >> 2) + (r & 3) <= l32 - 4 * hh ? sc[4][r] : sc[0][r];
  }
  const int cnt2 = merged_ends ? 4 : cnt;   // blocks that go through the softmax
  uint32_t vis[kTwoPhaseBlocks];
  float t0 = -INFINITY;
#pragma unroll
  for (int i = 0; i < kTwoPhaseBlocks; ++i) {
    vis[i] = 0;
    if (i < cnt2) {
      const int kb0 = (fb + i) * 32;
      // blocks every valid query of the wavefront sees completely need no mask work
      const bool interior = (kb0 + 32 <= n && kb0 >= qw_last - a.wl && kb0 + 31 <= qw0 + a.wr) || (i == 0 && merged_ends);
      if (interior) {
        vis[i] = 0xFFFFu;
#pragma unroll
        for (int r = 0; r < 16; r += 2) t0 = fmaxf(fmaxf(t0, sc[i][r]), sc[i][r + 1]);
      } else {
        vis[i] = visible_bits(kb0, hh, jlo, jhi);
#pragma unroll
        for (int r = 0; r < 16; ++r) t0 = fmaxf(t0, keep_or_neg_inf(sc[i][r], vis[i], r));
      }
    }
  }
  RowState<1, D> st;
  init_state(st);
  const float tmax = max_xor32(t0);
  st.m_ref[0] = tmax;
  st.mc[0] = tmax == -INFINITY ? 0.f : tmax * c;   // a row without a visible key: every p is masked to 0
  typename T::v8 pr[kTwoPhaseBlocks][2];
#pragma unroll
  for (int i = 0; i < kTwoPhaseBlocks; ++i) {
    if (i < cnt2) {
      uint32_t pk[8];
      float blk;
      if (vis[i] == 0xFFFFu) prob_block<T, false>(sc[i], c, st.mc[0], vis[i], pk, blk);
      else prob_block<T, true>(sc[i], c, st.mc[0], vis[i], pk, blk);
      st.lsum[0] += blk;
      pr[i][0] = as_v8<T>(make_uint4(pk[0], pk[1], pk[2], pk[3]));
      pr[i][1] = as_v8<T>(make_uint4(pk[4], pk[5], pk[6], pk[7]));
    } else {
      pr[i][0] = pr[i][1] = as_v8<T>(make_uint4(0, 0, 0, 0));
    }
  }
  if (merged_ends) {
    // the merged block's probabilities back to their blocks: pair r holds key offsets k0, k0 + 1
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
      const uint4 u = __builtin_bit_cast(uint4, pr[0][h2]);
      const uint32_t w[4] = {u.x, u.y, u.z, u.w};
      uint32_t first[4], last[4];
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const int r = 4 * h2 + x, k0 = 8 * (r >> 1) + 2 * (r & 1), thr = l32 - 4 * hh;
        const uint32_t m = (k0 <= thr ? 0x0000FFFFu : 0u) | (k0 + 1 <= thr ? 0xFFFF0000u : 0u);
        last[x] = w[x] & m;
        first[x] = w[x] & ~m;
      }
      pr[0][h2] = as_v8<T>(make_uint4(first[0], first[1], first[2], first[3]));
      pr[4][h2] = as_v8<T>(make_uint4(last[0], last[1], last[2], last[3]));
    }
  }

  // ---- phase 3: V has landed
  wait_direct_loads();
  // V rows at or beyond n are overwritten with zeros by the lanes that fetched them
  // (0 * whatever is stored in the padding must be 0); only the last block can have any
  {
    const int i = b_hi - 1 - b_lo;
#pragma unroll
    for (int x = 0; x < kLoadsPerWave; ++x) {
      const int j = wave + kWaves * x;
      if (j / LPB == i) {
        const int r = (j % LPB) * RPL + lane / CH;
        if ((b_hi - 1) * 32 + r >= n) *(uint4*)&lds[i * kBlk + r * D + (lane % CH) * 8] = make_uint4(0, 0, 0, 0);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kTwoPhaseBlocks; ++i) {
    if (i < cnt) {
      const uint16_t* vblk = &lds[(fb + i - b_lo) * kBlk];
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
        for (int db = 0; db < DB; ++db)
          st.oacc[0][db] = T::mfma(load_vt_frag_swz_d<T, D>(vblk, lane, ks2, db), pr[i][ks2], st.oacc[0][db]);
    }
  }
  __syncthreads();  // all blocks consumed: the region becomes the epilogue patches
  epilogue<T, 1, D>(a, st, op, lsep, qw0, n, lane, lds + wave * epi_patch(D));
}

// ======================================================================================
// Key-split kernel: global layers with very few query tiles (a single short sequence).
// With 128-row tiles one 512-token sequence of 12 heads is 48 workgroups on 256 compute
// units, one wavefront per SIMD walking 16 key blocks one after the other.  Here a
// workgroup owns ONE 32-row query block and its four wavefronts split the keys: wavefront w
// takes the 32-key blocks w, w+4, w+8, ...  Nothing is shared between wavefronts until the
// end, so each stages its own blocks in a private ring of kSplitRing LDS slots (direct
// global->LDS loads, no barriers; up to 512 keys everything is requested at once).  The
// four partial (reference, sum, accumulator) states are then merged through LDS with the
// split/merge identity of the online softmax, and wavefront 0 runs the common epilogue.
// ======================================================================================
constexpr int kSplitRing = 4;

template <class T>
__global__ __launch_bounds__(kThreads, 1) void fa_fwd_keysplit_kernel(const FaKernelArgs a) {
  constexpr int BM = 32;
  constexpr int kBlk = 32 * kD;  // elements per 32-key block
  constexpr int kMergeVals = 35; // 32 accumulator values, reference, reference * c, sum share
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[kWaves * kSplitRing * kBlk];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[kWaves * kSplitRing * kBlk];
  __shared__ float mbuf[(kWaves - 1) * kMergeVals * 64];  // [wavefront 1..3][value][lane]
  static_assert(kSplitRing * kBlk >= kEpiPatch, "wavefront 0's V ring doubles as its epilogue patch");

  TileCoord tc;
  if (!locate_tile<BM, false>(a, tc)) return;  // tc.n still as loaded: see below
  const int N = a.max_len, q0 = tc.q0;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;

  const uint16_t* qp = (const uint16_t*)a.q + tc.b * a.qs[0] + tc.h * a.qs[1];
  const uint16_t* kp = (const uint16_t*)a.k + tc.b * a.ks[0] + tc.h * a.ks[1];
  const uint16_t* vp = (const uint16_t*)a.v + tc.b * a.vs[0] + tc.h * a.vs[1];
  uint16_t* op = (uint16_t*)a.o + tc.b * a.os[0] + tc.h * a.os[1];
  float* lsep = a.lse ? a.lse + ((int64_t)tc.b * a.heads + tc.h) * N : nullptr;

  uint16_t* my_k = &lds_k[wave * kSplitRing * kBlk];
  uint16_t* my_v = &lds_v[wave * kSplitRing * kBlk];

  // Block i of this wavefront is key block wave + 4 i and lives in ring slot i % kSplitRing.
  // A block is 4 + 4 loads of 8 rows each (1 KB per load).  A lane's row is clamped to the
  // last row of the tensor (rows >= n are masked or zeroed below), so its global offset is a
  // per-lane 32-bit byte offset from the (batch, head) slice.
  const int r8 = lane >> 3;
  const uint32_t krow_b = 2u * (uint32_t)a.ks[2], vrow_b = 2u * (uint32_t)a.vs[2];
  auto issue_block = [&](int i) {
    const int j = wave + kWaves * i, slot = i % kSplitRing;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int r = 8 * g + r8;  // row within the block
      const int jg = 32 * j + r;
      const uint32_t jc = (uint32_t)(jg < N ? jg : N - 1);
      load16_to_lds(kp, jc * krow_b + 2u * (uint32_t)(((lane & 7) ^ k_swz(r)) * 8), &my_k[slot * kBlk + 8 * g * kD]);
      load16_to_lds(vp, jc * vrow_b + 2u * (uint32_t)(((lane & 7) ^ v_swz(r)) * 8), &my_v[slot * kBlk + 8 * g * kD]);
    }
  };
  // The first ring of blocks is requested from the tensor length alone, BEFORE the sequence
  // length is looked at: reading it (device memory) then overlaps the loads instead of
  // preceding them.  Blocks past the sequence end are fetched and never read.
  const int nb_max = (N + 31) >> 5;
  const int cnt_max = nb_max > wave ? (nb_max - wave + kWaves - 1) / kWaves : 0;
  int issued = cnt_max < kSplitRing ? cnt_max : kSplitRing;  // blocks 0 .. issued-1 are requested
#pragma unroll
  for (int i = 0; i < kSplitRing; ++i)
    if (i < issued) issue_block(i);

  typename T::v8 qreg[1][4];
  load_q<T, 1, 4, false>(a, qp, q0, lane, qreg);  // every wavefront holds the same 32 query rows

  // only now the sequence length
  const int n = tc.n < 0 ? 0 : (tc.n > N ? N : tc.n);
  tc.n = n;
  if (q0 >= n) {
    wait_direct_loads();  // the loads write this workgroup's LDS: they must land before it ends
    zero_fill<BM>(a, tc, op, lsep);
    return;
  }
  const int nb = (n + 31) >> 5;
  const int cnt = nb > wave ? (nb - wave + kWaves - 1) / kWaves : 0;  // this wavefront's blocks; <= cnt_max

  RowState<1> st;
  init_state(st);
  const bool alive = q0 + l32 < n;

  // loads complete in order, 8 per block: block i has landed once at most 8 * (blocks
  // requested after it) loads are outstanding
  auto wait_for = [&](int i) {
    const int younger = issued - 1 - i;
    if (younger >= 3) wait_vmcnt<24>();
    else if (younger == 2) wait_vmcnt<16>();
    else if (younger == 1) wait_vmcnt<8>();
    else wait_vmcnt<0>();
  };
  // V rows at or beyond n are overwritten with zeros by the lanes that fetched them (0 *
  // whatever is stored in the padding must be 0); the slot is this wavefront's own
  auto scrub = [&](int i) {
    const int kb0 = 32 * (wave + kWaves * i);
    if (kb0 + 32 <= n) return;
    uint16_t* vblk = &my_v[(i % kSplitRing) * kBlk];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      if (kb0 + 8 * g + r8 >= n) *(uint4*)&vblk[(8 * g + r8) * kD + (lane & 7) * 8] = make_uint4(0, 0, 0, 0);
  };

  if (cnt > 0) {
    // the same software pipeline as the resident window kernel, over this wavefront's blocks
    floatx16 sA, sB;
    typename T::v8 pA[2], pB[2];
    pA[0] = pA[1] = as_v8<T>(make_uint4(0, 0, 0, 0));
    auto zero_scores = [](floatx16& sv) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sv[r] = 0.f;
    };
    wait_for(0);
    scrub(0);
    zero_scores(sA);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) sA = T::mfma(load_k_frag_swz<T>(my_k, l32, hh, ks), qreg[0][ks], sA);
    // A global layer shows every existing row at least one key of the wavefront's first block:
    // the rows take its maximum as their reference here, once, so that every full block can
    // run the straight-line unit (nothing is accumulated yet, so there is nothing to rescale).
    {
      const int kb0 = 32 * wave;
      const uint32_t vis = kb0 + 32 <= n ? 0xFFFFu : visible_bits(kb0, hh, 0, n - 1);
      float t0 = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) t0 = fmaxf(t0, keep_or_neg_inf(sA[r], vis, r));
      const float tmax = max_xor32(t0);
      st.m_ref[0] = tmax;
      st.mc[0] = tmax == -INFINITY ? 0.f : tmax * a.c;
    }

    // Unit i: probabilities of block i; scores of block i+1; P.V of block i-1.  At the two
    // ends the neighbour is clamped: its product is unused (scores) or multiplied by zero
    // probabilities (P.V).
    auto unit = [&](floatx16& s_cur, floatx16& s_nxt, typename T::v8 (&p_prev)[2], typename T::v8 (&p_cur)[2], int i) {
      const int in = i + 1 < cnt ? i + 1 : cnt - 1;
      const int ip = i > 0 ? i - 1 : 0;
      if (i + 1 < cnt) {
        wait_for(i + 1);
        scrub(i + 1);
      }
      const int kb0 = 32 * (wave + kWaves * i);
      if (kb0 + 32 <= n)
        resident_unit<T, false>(st, qreg, s_cur, s_nxt, p_prev, p_cur, &my_k[(in % kSplitRing) * kBlk],
                                &my_v[(ip % kSplitRing) * kBlk], zero_scores, kb0, true, 0, n - 1, alive, a.c, lane);
      else
        resident_unit<T, true>(st, qreg, s_cur, s_nxt, p_prev, p_cur, &my_k[(in % kSplitRing) * kBlk],
                               &my_v[(ip % kSplitRing) * kBlk], zero_scores, kb0, kb0 + 32 <= n, 0, n - 1, alive, a.c,
                               lane);
      // block i-1 is consumed (its fragments are in registers): refill its slot.  Only
      // sequences beyond kSplitRing blocks per wavefront (512 keys) get here.
      if (i >= 1 && i - 1 + kSplitRing < cnt) {
        issue_block(i - 1 + kSplitRing);
        issued = i + kSplitRing;
      }
    };
    auto drain = [&](typename T::v8 (&p_last)[2], int i) {
      const uint16_t* vblk = &my_v[(i % kSplitRing) * kBlk];
#pragma unroll
      for (int x = 0; x < 4; ++x)
        st.oacc[0][x & 1] = T::mfma(load_vt_frag_swz<T>(vblk, lane, x >> 1, x & 1), p_last[x >> 1], st.oacc[0][x & 1]);
    };
    int i = 0;
    for (; i + 1 < cnt; i += 2) {
      unit(sA, sB, pA, pB, i);
      unit(sB, sA, pB, pA, i + 1);
    }
    if (i < cnt) {
      unit(sA, sB, pA, pB, i);
      drain(pB, i);
    } else {
      drain(pA, cnt - 1);
    }
  }
  // blocks requested beyond this wavefront's share of [0, n) may still be landing in its ring
  wait_direct_loads();

  // ---- merge the four partial results (same lane <-> (row, column) mapping in every wavefront)
  if (wave > 0) {
    float* dst = mbuf + (wave - 1) * kMergeVals * 64 + lane;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) dst[(16 * db + r) * 64] = st.oacc[0][db][r];
    dst[32 * 64] = st.m_ref[0];
    dst[33 * 64] = st.mc[0];
    dst[34 * 64] = st.lsum[0];
  }
  __syncthreads();
  if (wave != 0) return;
  {
    float m_new = st.m_ref[0];
#pragma unroll
    for (int w = 0; w < kWaves - 1; ++w) m_new = fmaxf(m_new, mbuf[w * kMergeVals * 64 + 32 * 64 + lane]);
    const float mc_new = (m_new == -INFINITY) ? 0.f : m_new * a.c;
    // a wavefront that saw no key has nothing accumulated: factor 0, kept away from exp2(+inf)
    const float f0 = (st.m_ref[0] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(st.mc[0] - mc_new);
    st.lsum[0] *= f0;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.oacc[0][db][r] *= f0;
#pragma unroll
    for (int w = 0; w < kWaves - 1; ++w) {
      const float* src = mbuf + w * kMergeVals * 64 + lane;
      const float f = (src[32 * 64] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(src[33 * 64] - mc_new);
      st.lsum[0] = __builtin_fmaf(f, src[34 * 64], st.lsum[0]);
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          st.oacc[0][db][r] = __builtin_fmaf(f, src[(16 * db + r) * 64], st.oacc[0][db][r]);
    }
    st.m_ref[0] = m_new;
    st.mc[0] = mc_new;
  }
  epilogue<T, 1, kD>(a, st, op, lsep, q0, n, lane, lds_v);
}

// ======================================================================================
// Global kernel: software pipeline over the full tiles + masked ragged tail
// ======================================================================================
// BIAS: the additive key bias rides on the score product: the bias of a key block, divided
// by |scale|, is the C operand of the block's first MFMA, so the scores arrive with the bias
// already in them and the vector work is unchanged.  Bias values are staged per K tile
// through a register of wavefront 0 into a small LDS array with the tile's two stages.
// NW: wavefronts per workgroup (4, 8 or 12).  All of them share ONE pair of K/V stages, so the
// tile traffic from L2 into LDS per flop falls with NW; a workgroup of 8 or 12 wavefronts
// is meant to be alone on its compute unit (2 or 3 wavefronts per SIMD).
//
// The body is a device function over LDS storage owned by the kernel that calls it, so that one
// kernel can hold two shapes of it (see fa_fwd_global_mixed_kernel).
template <int D, int NW>
struct GlobalLds {
  static constexpr int SK = stride_k(D), SV = stride_v(D);
  // Two stages of 64 unpadded rows during the pipeline; the ragged tail reuses the same
  // storage with padded rows (K 64 rows, V 96 rows), which is why these arrays are sized by
  // the padded strides; the epilogue needs one patch per wavefront in the K storage.
  static constexpr int kKElems = 2 * kBN * SK > NW * epi_patch(D) ? 2 * kBN * SK : NW * epi_patch(D);
  static constexpr int kVElems = 2 * kBN * SV;
  static_assert(2 * kBN * SV >= 96 * SV, "the tail reuses the V stages");
};

// tc: the workgroup's tile (tc.n already clamped into [0, max_len]).
// ROPE: q and k are rotated by position (a.rope_cos / a.rope_sin are set): a compile-time
// variant, so that the kernels without a rotation carry none of its code in their loops.
template <class T, int D, int NQB, int NW, bool BIAS, bool ROTATE = true, bool ROPE = false>
__device__ __forceinline__ void global_body(const FaKernelArgs& a, const TileCoord& tc, uint16_t* lds_k,
                                            uint16_t* lds_v, float* lds_bias) {
  static_assert(D == 32 || D == 64 || D == 128, "pipelined kernel: head_dim 32, 64 or 128");
  static_assert(NW == 4 || NW == 8 || NW == 12, "4, 8 or 12 wavefronts");
  constexpr int THREADS = NW * 64;
  constexpr int BM = NW * 32 * NQB;
  constexpr int KS = D / 16;  // k-steps of a score block
  constexpr int DB = D / 32;  // 32-row blocks of O^T
  constexpr int SK = stride_k(D), SV = stride_v(D);

  const int N = a.max_len, n = tc.n, q0 = tc.q0;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, hh = lane >> 5;

  const uint16_t* qp = (const uint16_t*)a.q + tc.b * a.qs[0] + tc.h * a.qs[1];
  const uint16_t* kp = (const uint16_t*)a.k + tc.b * a.ks[0] + tc.h * a.ks[1];
  const uint16_t* vp = (const uint16_t*)a.v + tc.b * a.vs[0] + tc.h * a.vs[1];
  uint16_t* op = (uint16_t*)a.o + tc.b * a.os[0] + tc.h * a.os[1];
  float* lsep = a.lse ? a.lse + ((int64_t)tc.b * a.heads + tc.h) * N : nullptr;
  const uint16_t* bp = BIAS ? (const uint16_t*)a.key_bias + tc.b * a.kb_stride : nullptr;
  // bias of key j in raw-score units (index clamped: keys outside [0, n) are never used unmasked)
  auto bias_of = [&](int j) {
    j = j < 0 ? 0 : (j < N ? j : N - 1);
    return T::to_float(bp[j]) * a.inv_abs_scale;
  };

  if (q0 >= n) {
    zero_fill<BM, D, THREADS>(a, tc, op, lsep);
    return;
  }

  const int qw0 = q0 + wave * 32 * NQB;
  const int qw_last = (qw0 + 32 * NQB < n ? qw0 + 32 * NQB : n) - 1;
  const bool wave_has_rows = qw_last >= qw0;

  typename T::v8 qreg[NQB][KS];
  load_q<T, NQB, KS, ROPE>(a, qp, qw0, lane, qreg);
  RowState<NQB, D> st;
  init_state(st);

  const int nf = n / kBN;  // full tiles: every key visible to every valid query
  const float c = a.c, tau_raw = a.tau_raw;

  // The pipeline advances in UNITS: one unit = one 32-key block u against one of the
  // wavefront's 32-query blocks qb, in the order (u,0) .. (u,NQB-1), (u+1,0) ...
  // During a unit the vector ALU turns the unit's scores into probabilities while the
  // matrix cores compute the NEXT unit's scores and add the PREVIOUS unit's P.V.
  // K fragments of a key block are read from LDS once and serve all NQB query blocks;
  // likewise the V^T fragments.
  //
  // Iteration t covers key blocks 2t, 2t+1.  It reads K of blocks 2t+1, 2t+2 (next
  // unit's scores) and V of blocks 2t-1, 2t (NQB = 1) or 2t, 2t+1 (NQB = 2): the LDS
  // "tile" of iteration t is K rows [64t+32, 64t+96) and V rows [64t+kVShift, +64).
  constexpr int kVShift = NQB == 1 ? -32 : 0;
  // Pipeline tiles go from HBM/L2 straight into LDS (global_load_lds, 16 bytes per lane):
  // a wavefront's load fills 1 KB of LDS in lane order, i.e. RPI = 8 rows of 128 bytes
  // (head_dim 64) or 4 rows of 256 bytes (head_dim 128), so the LDS tile is unpadded
  // [64 rows][D/8 chunks of 16 bytes] and bank conflicts are avoided by choosing WHICH
  // global chunk each lane fetches: chunk position c' of row r holds global chunk
  // c' ^ k_swz(r) for K and c' ^ v_swz(r) for V.  Wavefront w moves rows 8w..8w+7 of each
  // 32-row half in NI = 8 / RPI loads.  Row bases are wavefront-uniform; each lane adds a
  // fixed offset.  Halves whose rows would leave [0, N) are only ever the unused ends of
  // the pipeline (V before block 0, K after the last full block): their base is clamped,
  // their contents unused.
  // With 8 or 12 wavefronts, wavefronts 0..7 move one half each: wavefront w rows
  // 8 (w % 4) .. + 7 of half w / 4; the others move nothing.
  // head_dim 32 (64-byte rows): a load is 16 rows, a half two loads, and wavefront w moves half
  // w of the four (K first, K second, V first, V second) by itself.
  constexpr int CH = D / 8, RPI = 64 / CH, NI = D == 32 ? 2 : 8 / RPI;
  static_assert(D != 32 || NW == 4, "head_dim 32: four wavefronts");
  const int fw = wave & 3;  // row group within a half
  uint32_t koff[NI], voff[NI];  // bytes (head_dim 32: koff holds the wavefront's own half's offsets)
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    if (D == 32) {
      const int dl_r = 16 * i + lane / CH;
      const bool is_k = wave < 2;  // wavefront-uniform
      koff[i] = 2u * (uint32_t)(dl_r * (is_k ? a.ks[2] : a.vs[2]) +
                                (((lane % CH) ^ (is_k ? k_swz_d<D>(dl_r) : v_swz_d<D>(dl_r))) * 8));
      voff[i] = 0;
    } else {
      const int dl_r = 8 * fw + i * RPI + lane / CH;  // row within a 32-row half
      koff[i] = 2u * (uint32_t)(dl_r * a.ks[2] + (((lane % CH) ^ k_swz_d<D>(dl_r)) * 8));
      voff[i] = 2u * (uint32_t)(dl_r * a.vs[2] + (((lane % CH) ^ v_swz_d<D>(dl_r)) * 8));
    }
  }
  // the four 32-row halves of a tile: global row bases kg / vg, LDS halves kdst / vdst
  auto fetch_halves = [&](const uint16_t* kga, const uint16_t* kgb, const uint16_t* vga, const uint16_t* vgb,
                          uint16_t* kstage, uint16_t* vstage) {
    uint16_t* kdst = kstage + 8 * fw * D;
    uint16_t* vdst = vstage + 8 * fw * D;
    if (D == 32) {
      const uint16_t* g = wave == 0 ? kga : (wave == 1 ? kgb : (wave == 2 ? vga : vgb));
      uint16_t* dst = (wave < 2 ? kstage : vstage) + (wave & 1) * 32 * D;
#pragma unroll
      for (int i = 0; i < NI; ++i) load16_to_lds(g, koff[i], dst + i * 16 * D);
    } else if (NW == 4) {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        load16_to_lds(kga, koff[i], kdst + i * RPI * D);
        load16_to_lds(kgb, koff[i], kdst + 32 * D + i * RPI * D);
        load16_to_lds(vga, voff[i], vdst + i * RPI * D);
        load16_to_lds(vgb, voff[i], vdst + 32 * D + i * RPI * D);
      }
    } else if (wave < 8) {
      const bool second = wave >= 4;  // wavefront-uniform
      const uint16_t* kg = second ? kgb : kga;
      const uint16_t* vg = second ? vgb : vga;
      kdst += second ? 32 * D : 0;
      vdst += second ? 32 * D : 0;
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        load16_to_lds(kg, koff[i], kdst + i * RPI * D);
        load16_to_lds(vg, voff[i], vdst + i * RPI * D);
      }
    }
  };
  auto fetch = [&](int t, uint16_t* kstage, uint16_t* vstage) {
    const int k0r = t * kBN + 32 < 0 ? 0 : t * kBN + 32;
    const int k1r = t * kBN + 64 > N - 32 ? N - 32 : t * kBN + 64;
    const int v0r = t * kBN + kVShift < 0 ? 0 : t * kBN + kVShift;
    const int v1r = t * kBN + kVShift + 32 < 0 ? 0 : t * kBN + kVShift + 32;
    fetch_halves(kp + (int64_t)k0r * a.ks[2], kp + (int64_t)k1r * a.ks[2], vp + (int64_t)v0r * a.vs[2],
                 vp + (int64_t)v1r * a.vs[2], kstage, vstage);
  };
  // Inside the pipeline loop the four row bases just advance by one tile per iteration
  // (scalar 64-bit adds); only the very last tile's second K half can need the clamp.
  const uint16_t* kg0 = kp + (int64_t)(kBN + 32) * a.ks[2];
  const uint16_t* kg1 = kp + (int64_t)(kBN + 64) * a.ks[2];
  const uint16_t* vg0 = vp + (int64_t)(kBN + kVShift) * a.vs[2];
  const uint16_t* vg1 = vp + (int64_t)(kBN + kVShift + 32) * a.vs[2];
  const int k1_last_row = n / kBN * kBN > N - 32 ? N - 32 : n / kBN * kBN;  // tile nf-1: min(64 nf, N-32)
  const uint16_t* kg1_last = kp + (int64_t)k1_last_row * a.ks[2];
  auto fetch_next = [&](bool last, uint16_t* kstage, uint16_t* vstage) {
    fetch_halves(kg0, last ? kg1_last : kg1, vg0, vg1, kstage, vstage);
    kg0 += kBN * a.ks[2];
    kg1 += kBN * a.ks[2];
    vg0 += kBN * a.vs[2];
    vg1 += kBN * a.vs[2];
  };
  // per-lane fragment offsets (16-bit elements) into a 32-row block of a swizzled tile
  uint32_t kfo[KS], vfo[DB];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) kfo[ks] = l32 * D + (((2 * ks + hh) ^ k_swz_d<D>(l32)) * 8);
  {
    const int p16 = lane & 15, g = (lane >> 4) & 1;
#pragma unroll
    for (int db = 0; db < DB; ++db)
      vfo[db] = (4 * hh + (p16 >> 2)) * D +
                (((4 * db + 2 * g + ((p16 & 3) >> 1)) ^ v_swz_d<D>(4 * hh + (p16 >> 2))) * 8) +
                (p16 & 1) * 4;
  }
  auto k_frag = [&](const uint16_t* kblk, int ks) { return as_v8<T>(*(const uint4*)&kblk[kfo[ks]]); };
  auto vt_frag = [&](const uint16_t* vblk, int ks2, int db) {
    typedef __attribute__((address_space(3))) shortx4 lds_s4;
    const shortx4 x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)&vblk[vfo[db] + ks2 * 16 * D]);
    const shortx4 x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)&vblk[vfo[db] + (ks2 * 16 + 8) * D]);
    shortx8 x;
    x[0] = x0[0]; x[1] = x0[1]; x[2] = x0[2]; x[3] = x0[3];
    x[4] = x1[0]; x[5] = x1[1]; x[6] = x1[2]; x[7] = x1[3];
    return __builtin_bit_cast(typename T::v8, x);
  };

  // pipeline registers: scores of the current / next unit, packed probabilities of the
  // previous / current unit, operand fragments of the key block in flight
  floatx16 sA, sB;
  floatx16 bcur;  // BIAS: the bias of the key block whose K fragments are in ka (C layout)
#pragma unroll
  for (int r = 0; r < 16; ++r) bcur[r] = 0.f;
  auto bias_frag = [&](const float* bblk) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 b4 = *(const float4*)&bblk[8 * g + 4 * hh];
      bcur[4 * g + 0] = b4.x;
      bcur[4 * g + 1] = b4.y;
      bcur[4 * g + 2] = b4.z;
      bcur[4 * g + 3] = b4.w;
    }
  };
  float bst = 0.f;  // BIAS: wavefront 0 carries the next tile's bias from its load to its LDS write
  typename T::v8 pA[2], pB[2], ka[KS], va[2][DB];
  pA[0] = pA[1] = as_v8<T>(make_uint4(0, 0, 0, 0));
#pragma unroll
  for (int i = 0; i < 2 * DB; ++i) va[i / DB][i % DB] = as_v8<T>(make_uint4(0, 0, 0, 0));

  // Long sequences with one query block per wavefront put three wavefronts of three different
  // workgroups on a SIMD, and the hardware serves the oldest first: one workgroup races ahead,
  // finishes early and leaves the SIMD to two wavefronts, then one, which use it less well.
  // Rotating the wave priorities by hardware wave slot, one step per iteration, keeps the
  // three abreast to the end (per-wavefront stamps at 8K: finish times within 5 % of each
  // other instead of 35 %; 1-2 % off the call).
  const bool rotate_prio = ROTATE && NQB == 1 && nf >= 64;
  int wslot = 0;
  if (rotate_prio) {
    unsigned hw_id;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw_id));
    wslot = (int)(hw_id & 15u);  // wave slot within the SIMD
  }
  if (nf > 0) {
    // prologue: unit (0,0)'s scores need K rows [0, 32): tile "-1" (rows [-32, 32), clamped)
    fetch(-1, &lds_k[kBN * D], &lds_v[kBN * D]);
    fetch(0, lds_k, lds_v);
    if (BIAS && wave == 0) {
      // tile -1 (keys -32..31) into stage 1, tile 0 (keys 32..95) into stage 0
      lds_bias[kBN + lane] = bias_of(lane - 32);
      lds_bias[lane] = bias_of(lane + 32);
    }
    wait_direct_loads();
    __syncthreads();
    if (ROPE) {
      // rotary embedding: every K stage is rotated in place once it has landed (stage 1 holds
      // keys 0..31 in its second half, stage 0 keys 32..63 and min(64, N - 32) ...)
      rope_rows_in_lds<T, D, true>(a, &lds_k[kBN * D + 32 * D], D, 32, 0, tid, THREADS);
      rope_rows_in_lds<T, D, true>(a, lds_k, D, 64, 32, tid, THREADS, kBN > N - 32 ? N - 32 : kBN);
      __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) sA[r] = 0.f;
    if (BIAS) {
      bias_frag(&lds_bias[kBN + 32]);
      sA = bcur;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      ka[ks] = k_frag(&lds_k[kBN * D + 32 * D], ks);
      sA = T::mfma(ka[ks], qreg[0][ks], sA);
    }
    if (!BIAS) {
      // Every query block takes the maximum of its scores against key block 0 as its first
      // reference, here, once (nothing is accumulated yet, so there is nothing to rescale): the
      // units then need no "has this row a reference yet" test.  With a key bias block 0 can be
      // masked out entirely, so those kernels keep the test.
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        floatx16 s0 = sA;
        if (qb > 0) {
#pragma unroll
          for (int r = 0; r < 16; ++r) s0[r] = 0.f;
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) s0 = T::mfma(ka[ks], qreg[qb][ks], s0);
        }
        float t0 = fmaxf(s0[0], s0[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) t0 = fmaxf(fmaxf(t0, s0[r]), s0[r + 1]);
        const float tmax = max_xor32(t0);
        st.m_ref[qb] = tmax;
        st.mc[qb] = tmax == -INFINITY ? 0.f : tmax * c;
      }
    }
    __syncthreads();  // stage 1 is refilled during iteration 0

    // The probabilities are formed against the row's current reference right away; the
    // lane's share of the block's row sum doubles as the overflow sentinel (any p beyond
    // kPLimit, an infinity included, pushes it over).  Only then - rarely - is the exact
    // block maximum computed, the reference refreshed and the block redone.
    auto softmax_block = [&](const floatx16& sv, float mcq, uint32_t (&pk)[8], float& blk) {
      prob_block<T, false>(sv, c, mcq, 0xFFFFu, pk, blk);
    };
    // One unit.  QB: query block of the current scores; NQ: query block of the next
    // unit; PQ: query block of the previous unit; LOAD: this unit starts a new key block
    // for both matrix products (fragments come from kblk / vblk), otherwise the
    // fragments already in registers are reused.
    auto unit = [&](auto QBc, auto NQc, auto PQc, auto LOADc, floatx16& s_cur, floatx16& s_nxt,
                    typename T::v8 (&p_prev)[2], typename T::v8 (&p_cur)[2], const uint16_t* kblk,
                    const uint16_t* vblk, const float* bblk) {
      constexpr int QB = decltype(QBc)::value, NQ = decltype(NQc)::value, PQ = decltype(PQc)::value;
      constexpr bool LOAD = decltype(LOADc)::value;
      if (LOAD) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) ka[ks] = k_frag(kblk, ks);
#pragma unroll
        for (int i = 0; i < 2 * DB; ++i) va[i / DB][i % DB] = vt_frag(vblk, i / DB, i % DB);
        if (BIAS) bias_frag(bblk);
      }
      // the first product of the score block takes the bias (or zero) as its C operand
      if (BIAS) {
        s_nxt = bcur;
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) s_nxt[r] = 0.f;
      }
      // dependent products (the k-steps of a score block, the two of an output block)
      // alternate with independent ones
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        s_nxt = T::mfma(ka[ks], qreg[NQ][ks], s_nxt);
        st.oacc[PQ][ks % DB] = T::mfma(va[ks / DB][ks % DB], p_prev[ks / DB], st.oacc[PQ][ks % DB]);
      }
      uint32_t pk[8];
      float blk;
      softmax_block(s_cur, st.mc[QB], pk, blk);
      // !(blk <= limit) also catches a NaN sum; no reference yet = first block
      const bool trig = !(blk <= kPLimit) || (BIAS && st.m_ref[QB] == -INFINITY);
      if (__any(trig)) {
        // a row refreshes iff one of ITS two lanes tripped: no dependence on other rows
        const bool row_trig = sum_xor32(trig ? 1.f : 0.f) > 0.f;
        float t0 = fmaxf(s_cur[0], s_cur[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) t0 = fmaxf(fmaxf(t0, s_cur[r]), s_cur[r + 1]);
        const float tmax = max_xor32(t0);
        // the accumulator of this query block already holds P.V of all earlier key blocks
        rescale_rows(st, QB, row_trig, tmax, c);
        softmax_block(s_cur, st.mc[QB], pk, blk);
      }
      st.lsum[QB] += blk;
      p_cur[0] = as_v8<T>(make_uint4(pk[0], pk[1], pk[2], pk[3]));
      p_cur[1] = as_v8<T>(make_uint4(pk[4], pk[5], pk[6], pk[7]));
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    // One iteration on LDS stage STAGE (a compile-time constant, so every LDS address is a
    // per-lane register plus an immediate); the other stage is being filled meanwhile.
    auto iter = [&](auto STAGEc, int t) {
      constexpr int STAGE = decltype(STAGEc)::value;
      const uint16_t* kt = &lds_k[STAGE * kBN * D];
      const uint16_t* vt = &lds_v[STAGE * kBN * D];
      const float* bt = &lds_bias[BIAS ? STAGE * kBN : 0];
      if (rotate_prio) {
        const int ph = (t + wslot) % 3;
        if (ph == 0) __builtin_amdgcn_s_setprio(2);
        else if (ph == 1) __builtin_amdgcn_s_setprio(1);
        else __builtin_amdgcn_s_setprio(0);
      }
      // the stage being filled was last read in iteration t-1; every wavefront is past
      // that iteration's barrier
      if (t + 1 < nf) {
        fetch_next(t + 2 == nf, &lds_k[(STAGE ^ 1) * kBN * D], &lds_v[(STAGE ^ 1) * kBN * D]);
        if (BIAS && wave == 0) bst = bias_of((t + 1) * kBN + 32 + lane);
      }
      if (wave_has_rows) {
        if constexpr (NQB == 1) {
          unit(I0{}, I0{}, I0{}, std::true_type{}, sA, sB, pA, pB, kt, vt, bt);
          unit(I0{}, I0{}, I0{}, std::true_type{}, sB, sA, pB, pA, kt + 32 * D, vt + 32 * D, bt + 32);
        } else {
          unit(I0{}, I1{}, I1{}, std::false_type{}, sA, sB, pA, pB, kt, vt, bt);
          unit(I1{}, I0{}, I0{}, std::true_type{}, sB, sA, pB, pA, kt, vt, bt);
          unit(I0{}, I1{}, I1{}, std::false_type{}, sA, sB, pA, pB, kt, vt, bt);
          unit(I1{}, I0{}, I0{}, std::true_type{}, sB, sA, pB, pA, kt + 32 * D, vt + 32 * D, bt + 32);
        }
      }
      // the other bias stage was last read in iteration t-1
      if (BIAS && wave == 0 && t + 1 < nf) lds_bias[(STAGE ^ 1) * kBN + lane] = bst;
      wait_direct_loads();  // this wavefront's share of the next tile has landed
      __syncthreads();
      if (ROPE && t + 1 < nf) {
        rope_rows_in_lds<T, D, true>(a, &lds_k[(STAGE ^ 1) * kBN * D], D, 64, (t + 1) * kBN + 32, tid, THREADS,
                                     t + 2 == nf ? k1_last_row : (t + 1) * kBN + 64);
        __syncthreads();
      }
    };
    int t = 0;
    for (; t + 1 < nf; t += 2) {
      iter(I0{}, t);
      iter(I1{}, t + 1);
    }
    if (t < nf) iter(I0{}, t);
    if (rotate_prio) __builtin_amdgcn_s_setprio(0);
  }

  // ---- drain + ragged tail -------------------------------------------------------------
  // lds_v rows 0..31: V of the last full block (its P.V is still pending);
  // lds_v rows 32..95 and lds_k rows 0..63: the partial tile [64 nf, 64 nf + 64).
  const int tail = n - nf * kBN;
  {
    const int base = nf * kBN;
    for (int i = tid; i < 96 * CH; i += THREADS) {
      const int row = i / CH, c8 = (i % CH) * 8;
      const int jg = base - 32 + row;
      const int jc = jg < 0 ? 0 : (jg < N ? jg : N - 1);
      uint4 vv = *(const uint4*)(vp + jc * a.vs[2] + c8);
      if (jg >= n) vv = make_uint4(0, 0, 0, 0);  // 0 * (anything stored in the padding) must be 0
      *(uint4*)&lds_v[row * SV + c8] = vv;
    }
    if (tail > 0) {
      for (int i = tid; i < 64 * CH; i += THREADS) {
        const int row = i / CH, c8 = (i % CH) * 8;
        const int jg = base + row;
        const int jc = jg < N ? jg : N - 1;
        *(uint4*)&lds_k[row * SK + c8] = *(const uint4*)(kp + jc * a.ks[2] + c8);
      }
      if (BIAS && wave == 0) lds_bias[lane] = bias_of(base + lane);  // every stage is free after the loop
    }
  }
  __syncthreads();
  if (ROPE && tail > 0) {
    rope_rows_in_lds<T, D, false>(a, lds_k, SK, 64, nf * kBN, tid, THREADS);
    __syncthreads();
  }
  if (wave_has_rows) {
    if (nf > 0) {
      // after an even number of units the pending probabilities sit in pA; they belong
      // to the last full key block and the wavefront's last query block
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const typename T::v8 vf = load_vt_frag<T, D>(lds_v, lane, ks2, db);
          st.oacc[NQB - 1][db] = T::mfma(vf, pA[ks2], st.oacc[NQB - 1][db]);
        }
    }
    if (tail > 0) {
      int jlo[NQB], jhi[NQB];
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        jlo[qb] = 0;
        jhi[qb] = n - 1;
      }
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const int kb0 = nf * kBN + kb * 32;
        if (kb0 >= n) continue;
        simple_block<T, NQB, true, 0>(st, qreg, &lds_k[kb * 32 * SK], &lds_v[(32 + kb * 32) * SV], kb0,
                                      jlo, jhi, lane, c, tau_raw, nullptr, BIAS ? &lds_bias[kb * 32] : nullptr);
      }
    }
  }
  __syncthreads();  // tail consumed: the K storage becomes the epilogue patches
  epilogue<T, NQB>(a, st, op, lsep, qw0, n, lane, lds_k + wave * epi_patch(D));
}

template <class T, int D, int NQB, int NW, bool BIAS = false, bool ROPE = false>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void fa_fwd_global_kernel(const FaKernelArgs a) {
  typedef GlobalLds<D, NW> L;
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[L::kKElems];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[L::kVElems];
  __shared__ __attribute__((aligned(16))) float lds_bias[BIAS ? 2 * kBN : 4];  // [stage][tile row], bias / |scale|
  TileCoord tc;
  if (!locate_tile<NW * 32 * NQB>(a, tc)) return;
  global_body<T, D, NQB, NW, BIAS, true, ROPE>(a, tc, lds_k, lds_v, lds_bias);
}

// ======================================================================================
// Mixed-shape global kernel (head_dim 64, ONE sequence): 256-row and 128-row workgroups in one
// launch.  A launch of 256-row workgroups alone ends, unless their number is a multiple of 512,
// with a round in which units hold one workgroup (a single wavefront per SIMD overlaps its own
// matrix and vector work badly and runs at less than half the rate) or none; the 128-row shape
// alone moves twice the K/V tile traffic per flop.  Here full rounds of 256-row pairs are
// followed by 128-row workgroups, or by pairs of one of each, on the rows that remain (one
// 8K-token sequence of 12 heads: 248 pairs on 256 units; one 16K-token sequence: 512 + 512).
// The split is made ON THE DEVICE from the sequence length, which the host does not know; the
// id -> tile arithmetic and its rules are in fa_mix_map.h.  The host launches mix_ids_a +
// kMixIdsB ids, enough for every length up to max_len.  Ids without a tile zero-fill the tiles
// that lie entirely in the padding (rows at or beyond 128 T), or exit.
// ======================================================================================
template <class T>
__global__ __launch_bounds__(kThreads, 2) void fa_fwd_global_mixed_kernel(const FaKernelArgs a) {
  typedef GlobalLds<kD, 4> L;
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[L::kKElems];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[L::kVElems];
  __shared__ __attribute__((aligned(16))) float lds_bias[4];
  const int N = a.max_len, H = a.heads;
  int n = N;
  if (a.seq_lens) {
    n = a.seq_lens[0];
    n = n < 0 ? 0 : (n > N ? N : n);
  }
  const int tiles = (n + 127) >> 7;
  const FaMixTile m = fa_mix_locate((int)blockIdx.x, a.map_xcd != 0, a.mix_ids_a, kMixIdsB, H, tiles);
  TileCoord tc;
  tc.b = 0;
  tc.n = n;
  // (wavefront-uniform by construction; said explicitly so that the addresses derived from
  // them stay in scalar registers)
  tc.h = __builtin_amdgcn_readfirstlane(m.head);
  tc.q0 = __builtin_amdgcn_readfirstlane(m.q0);
  if (m.kind == 1) {
    tc.qt = m.q0 >> 8;
    global_body<T, kD, 2, 4, false, false>(a, tc, lds_k, lds_v, lds_bias);
  } else if (m.kind == 2) {
    tc.qt = m.q0 >> 7;
    global_body<T, kD, 1, 4, false, false>(a, tc, lds_k, lds_v, lds_bias);
  } else if (m.kind == 3) {
    // tiles T .. ceil(max_len / 128) - 1 of every head are padding only: o = 0, lse = -inf.
    // The spare ids share them out in a strided loop (there are normally more ids than tiles).
    const int pad = ((N + 127) >> 7) - tiles;
    for (int z = m.spare; z < pad * H; z += m.spares) {
      tc.h = z / pad;
      tc.qt = tiles + z % pad;
      tc.q0 = 128 * tc.qt;
      zero_fill<128, kD, kThreads>(a, tc, (uint16_t*)a.o + tc.h * a.os[1], a.lse ? a.lse + (int64_t)tc.h * N : nullptr);
    }
  }
}

// ======================================================================================
// Rotation of q and k ahead of a global layer.  A global layer that rotates K inside the call
// rotates every K tile once per query tile; when the caller lends scratch memory, q and k are
// rotated once here instead (the same rotate8, the same rounding: the attention kernel then
// sees bit for bit what the in-call rotation would have produced) and the plain kernels run on
// the copies.  One thread rotates eight pairs of one row; blockIdx.z < batch: q, else k.
// ======================================================================================
template <class T>
__global__ __launch_bounds__(256) void fa_rope_rotate_kernel(const FaRopeArgs r) {
  const int half = r.head_dim / 16;                      // 16-byte chunks per half row: 2, 4 or 8
  const int rows_per_block = 256 / half;
  const int row = blockIdx.x * rows_per_block + (int)threadIdx.x / half, c = (int)threadIdx.x % half;
  if (row >= r.max_len) return;
  const int h = blockIdx.y;
  const bool is_k = (int)blockIdx.z >= r.batch;
  const int b = is_k ? (int)blockIdx.z - r.batch : (int)blockIdx.z;
  const int64_t* st = is_k ? r.ks : r.qs;
  const uint16_t* src = (const uint16_t*)(is_k ? r.k : r.q) + b * st[0] + h * st[1] + row * st[2];
  uint16_t* dst = (uint16_t*)(is_k ? r.k_out : r.q_out) + (((int64_t)b * r.heads + h) * r.max_len + row) * r.head_dim;
  uint4 lo = *(const uint4*)(src + 8 * c), hi = *(const uint4*)(src + r.head_dim / 2 + 8 * c);
  const int64_t t = (int64_t)row * r.rope_stride + 8 * c;
  rotate8<T>(lo, hi, r.rope_cos + t, r.rope_sin + t);
  *(uint4*)(dst + 8 * c) = lo;
  *(uint4*)(dst + r.head_dim / 2 + 8 * c) = hi;
}

// Scratch for callers that cannot allocate (fa_fwd_ex_static_scratch): one array per GPU, held
// until the process ends.  The name below is a host-side stand-in for the symbol; the device
// address is looked up once per device and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char fa_static_scratch_array[FA_STATIC_SCRATCH_BYTES];

template <class T>
int launch(const FaKernelArgs& a, int bm, int v_path, int win_kernel, void* stream) {
  typedef void (*Kernel)(const FaKernelArgs);
  unsigned grid = (unsigned)a.total_tiles;
  if (a.map_xcd) grid = 8u * (unsigned)a.xcd_per * (unsigned)a.batch;
  if (bm == 0) grid = a.mix_ids_a + kMixIdsB;
  const bool global = a.wl < 0 && a.wr < 0;
  // per-lane 32-bit byte offsets into a (batch, head) slice
  const bool slice_fits_32bit = (double)a.max_len * (double)(a.ks[2] > a.vs[2] ? a.ks[2] : a.vs[2]) * 2.0 < 4.0e9;
  // 32-key blocks a 128-row query tile of a two-sided window can touch (tiles start at multiples of 128)
  const int win_blocks = (a.wl >= 0 && a.wr >= 0) ? (127 + a.wr) / 32 + (a.wl + 31) / 32 + 1 : 1 << 30;
  // 32-key blocks the 32 queries of one wavefront can see (they start at a multiple of 32)
  const int wave_blocks = (a.wl >= 0 && a.wr >= 0) ? (31 + a.wr) / 32 + (a.wl + 31) / 32 + 1 : 1 << 30;
  Kernel kern = nullptr;
  unsigned threads = kThreads;
  // rotary embedding is applied by the two-phase window kernel, the pipelined global kernel
  // (four-wavefront shapes) and the masked kernel
  const bool rope = a.rope_cos != nullptr;
  // Calls of at most 1.5 tiles per compute unit are bound by one workgroup's latency, not by
  // bandwidth: there the pipelined kernel with K and V resident (ONE memory round trip per
  // workgroup instead of two) is as fast or a little faster (measured, 12 heads: 2K tokens 7.4
  // against 7.8 us, 4K equal, 8K 17.3 against 14.9 us, 32K 43 against 37 us); it exists for
  // head_dim 64 only.
  const bool latency_bound = a.head_dim == kD && a.total_tiles <= 384;
  if (!a.key_bias && !global && v_path == 0 && bm == 128 && slice_fits_32bit && win_blocks <= kResBlocks &&
      wave_blocks <= kTwoPhaseBlocks && win_kernel != 1 && !(latency_bound && !rope && win_kernel != 2)) {
    // local layer with a narrow two-sided window (the paper's 63/64), any head_dim
    kern = a.head_dim == 32 ? fa_fwd_window_twophase_kernel<T, 32>
                            : (a.head_dim == 64 ? fa_fwd_window_twophase_kernel<T, 64> : fa_fwd_window_twophase_kernel<T, 128>);
  } else if (a.key_bias && !rope && !global && v_path == 0 && a.c > 0.f && a.head_dim == kD && bm == 128 && slice_fits_32bit &&
      win_blocks <= kResBlocks) {
    // additive key bias on a local layer whose key range stays resident in LDS
    kern = fa_fwd_window_resident_kernel<T, true>;
  } else if (a.key_bias && !rope && global && v_path == 0 && a.c > 0.f && (a.head_dim == 64 || a.head_dim == 128)) {
    // additive key bias on a global layer: the pipelined kernel with the bias as MFMA C operand
    if (a.head_dim == 128) kern = fa_fwd_global_kernel<T, 128, 1, 4, true>;
    else if (bm == 256) kern = fa_fwd_global_kernel<T, 64, 2, 4, true>;
    else kern = fa_fwd_global_kernel<T, 64, 1, 4, true>;
  } else if (a.key_bias) {
    // additive key bias otherwise: the masked kernel, 128-row tiles, any head_dim and window
    if (a.head_dim == 32) kern = fa_fwd_masked_kernel<T, 32, 1, true, true>;
    else if (a.head_dim == 64) kern = fa_fwd_masked_kernel<T, 64, 1, true, true>;
    else kern = fa_fwd_masked_kernel<T, 128, 1, true, true>;
  } else if (rope && global && v_path == 0) {
    // rotation on a global layer: the pipelined kernel's four-wavefront shapes
    if (a.head_dim == 128) kern = fa_fwd_global_kernel<T, 128, 1, 4, false, true>;
    else if (a.head_dim == 32) kern = bm == 256 ? fa_fwd_global_kernel<T, 32, 2, 4, false, true> : fa_fwd_global_kernel<T, 32, 1, 4, false, true>;
    else kern = bm == 256 ? fa_fwd_global_kernel<T, 64, 2, 4, false, true> : fa_fwd_global_kernel<T, 64, 1, 4, false, true>;
  } else if (a.head_dim == 128 && global && v_path == 0) {
    if (bm == 256) {
      kern = fa_fwd_global_kernel<T, 128, 1, 8>;   // eight wavefronts on one pair of K/V stages
      threads = 512;
    } else {
      kern = fa_fwd_global_kernel<T, 128, 1, 4>;
    }
  } else if (a.head_dim == 32 && global && v_path == 0) {
    kern = bm == 256 ? fa_fwd_global_kernel<T, 32, 2, 4> : fa_fwd_global_kernel<T, 32, 1, 4>;
  } else if (a.head_dim != kD) {
    // wide or one-sided windows of head_dim 32 / 128 (and the 16-bit V-read path): the masked
    // kernel covers every mask; bm is 128 here
    if (a.head_dim == 32) kern = v_path == 0 ? fa_fwd_masked_kernel<T, 32, 1, true> : fa_fwd_masked_kernel<T, 32, 1, false>;
    else kern = v_path == 0 ? fa_fwd_masked_kernel<T, 128, 1, true> : fa_fwd_masked_kernel<T, 128, 1, false>;
  } else if (bm == 32) {
    // the host asks for 32-row tiles only for global layers of head_dim 64 without a bias
    kern = fa_fwd_keysplit_kernel<T>;
  } else if (global && v_path == 0) {
    if (bm == 0) {
      kern = fa_fwd_global_mixed_kernel<T>;
    } else if (bm == 512) {
      kern = fa_fwd_global_kernel<T, 64, 2, 8>;
      threads = 512;
    } else if (bm == 384) {
      kern = fa_fwd_global_kernel<T, 64, 1, 12>;
      threads = 768;
    } else if (bm == 256) {
      kern = fa_fwd_global_kernel<T, 64, 2, 4>;
    } else {
      kern = fa_fwd_global_kernel<T, 64, 1, 4>;
    }
  } else if (!global && !rope && v_path == 0 && bm == 128 && slice_fits_32bit) {
    kern = win_blocks <= kResBlocks ? fa_fwd_window_resident_kernel<T> : fa_fwd_window_kernel<T>;
  } else if (bm == 256) {
    kern = v_path == 0 ? fa_fwd_masked_kernel<T, 64, 2, true> : fa_fwd_masked_kernel<T, 64, 2, false>;
  } else {
    kern = v_path == 0 ? fa_fwd_masked_kernel<T, 64, 1, true> : fa_fwd_masked_kernel<T, 64, 1, false>;
  }
  // hipLaunchKernel returns THIS launch's status; an error left by the caller's earlier HIP
  // work stays where it is (neither reported as ours nor cleared)
  FaKernelArgs args = a;
  void* argv[] = {&args};
  return (int)hipLaunchKernel((const void*)kern, dim3(grid), dim3(threads), argv, 0, (hipStream_t)stream);
}

}  // namespace

int fa_launch_rope_rotate(const FaRopeArgs& r, int is_bf16, void* stream) {
  const int rows_per_block = 256 / (r.head_dim / 16);
  const dim3 grid((unsigned)((r.max_len + rows_per_block - 1) / rows_per_block), (unsigned)r.heads, 2u * (unsigned)r.batch);
  FaRopeArgs args = r;
  void* argv[] = {&args};
  const void* kern = is_bf16 ? (const void*)fa_rope_rotate_kernel<BF16> : (const void*)fa_rope_rotate_kernel<F16>;
  return (int)hipLaunchKernel(kern, grid, dim3(256), argv, 0, (hipStream_t)stream);
}

int fa_static_scratch(void** ptr) {
  constexpr int kMaxDevices = 64;
  static void* per_device[kMaxDevices] = {};   // each GPU holds its own copy of the array at its own address
  static std::mutex lock;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> guard(lock);
  if (!per_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(fa_static_scratch_array));
    if (e != hipSuccess) return (int)e;
    per_device[dev] = p;
  }
  *ptr = per_device[dev];
  return 0;
}

int fa_launch_f16(const FaKernelArgs& a, int bm, int v_path, int win_kernel, void* stream) {
  return launch<F16>(a, bm, v_path, win_kernel, stream);
}
int fa_launch_bf16(const FaKernelArgs& a, int bm, int v_path, int win_kernel, void* stream) {
  return launch<BF16>(a, bm, v_path, win_kernel, stream);
}
