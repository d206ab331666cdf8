// Flash-attention forward for gfx950 (MI355X): head_dim 64, fp16 / bf16 storage,
// fp32 accumulation, key-padding mask by sequence length, optional local window.
//
// The operation is softmax(scale * Q K^T + mask) V per (batch, head), evaluated
// one key tile at a time with a running row maximum and row sum so that no
// n x n matrix is ever formed (paper Sec. 2.2; operator attributes scale,
// window_size_left/right and the 1-D padding mask from Sec. 4.1.3 and Eq. 1).
//
// Work decomposition (one workgroup = 4 wavefronts = 256 threads):
//   * a workgroup owns BM = 4*32*NQB query rows of one (batch, head); each
//     wavefront owns NQB blocks of 32 query rows and keeps their Q fragments,
//     running maximum / sum and the 64-wide output accumulator in registers;
//   * K and V are streamed through LDS in tiles of BN = 64 keys, double buffered,
//     fetched from HBM/L2 with 16-byte loads one tile ahead of the arithmetic.
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
// maximum m of a row is only refreshed when a tile's maximum exceeds it by more
// than a threshold (2^8 in p); rescaling the accumulator is then rare, and the
// result is unchanged because numerator and denominator share the reference.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "fa_args.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf2v __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));

constexpr int kD = 64;        // head_dim
constexpr int kBN = 64;       // keys per LDS tile
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kSK = kD + 8;   // LDS row stride of the K tile, in 16-bit elements
constexpr int kSV = kD + 8;   // LDS row stride of the V tile
constexpr float kLn2 = 0.693147180559945309f;

struct F16 {
  typedef half8 v8;
  static __device__ __forceinline__ floatx16 mfma(v8 a, v8 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {  // round to nearest even
    half2v h = __builtin_convertvector((floatx2){a, b}, half2v);
    return __builtin_bit_cast(uint32_t, h);
  }
};

struct BF16 {
  typedef bf8 v8;
  static __device__ __forceinline__ floatx16 mfma(v8 a, v8 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {
    bf2v h = __builtin_convertvector((floatx2){a, b}, bf2v);
    return __builtin_bit_cast(uint32_t, h);
  }
};

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

template <class T>
__device__ __forceinline__ typename T::v8 as_v8(uint4 u) {
  return __builtin_bit_cast(typename T::v8, u);
}

template <class T, int NQB, bool V_TR>
__global__ __launch_bounds__(kThreads) void fa_fwd_kernel(const FaKernelArgs a) {
  constexpr int BM = kWaves * 32 * NQB;
  __shared__ __attribute__((aligned(16))) uint16_t lds_k[2][kBN * kSK];
  __shared__ __attribute__((aligned(16))) uint16_t lds_v[2][kBN * kSV];

  // ---- which tile ------------------------------------------------------------
  int tile = blockIdx.x;
  if (a.map_xcd) {
    // Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a contiguous
    // run of tiles so neighbours that share K/V share an L2.
    const int per = (a.total_tiles + 7) >> 3;
    tile = (tile & 7) * per + (tile >> 3);
  }
  if (tile >= a.total_tiles) return;
  const int qt = tile % a.n_qtiles;
  const int bh = tile / a.n_qtiles;
  const int h = bh % a.heads;
  const int b = bh / a.heads;
  const int N = a.max_len;

  int n = N;
  if (a.seq_lens) {
    n = a.seq_lens[b];
    n = n < 0 ? 0 : (n > N ? N : n);
  }
  const int q0 = qt * BM;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: lets key-block skips be scalar branches
  const int l32 = lane & 31;
  const int hh = lane >> 5;

  const uint16_t* qp = (const uint16_t*)a.q + b * a.qs[0] + h * a.qs[1];
  const uint16_t* kp = (const uint16_t*)a.k + b * a.ks[0] + h * a.ks[1];
  const uint16_t* vp = (const uint16_t*)a.v + b * a.vs[0] + h * a.vs[1];
  uint16_t* op = (uint16_t*)a.o + b * a.os[0] + h * a.os[1];
  float* lsep = a.lse ? a.lse + ((int64_t)b * a.heads + h) * N : nullptr;

  // ---- workgroup entirely in the padding: zero-fill and leave -----------------
  if (q0 >= n) {
    const int r = tid >> 3, c16 = tid & 7;
    for (int row = q0 + r; row < q0 + BM && row < N; row += 32) {
      *(uint4*)(op + row * a.os[2] + c16 * 8) = make_uint4(0, 0, 0, 0);
    }
    if (lsep) {
      for (int row = q0 + tid; row < q0 + BM && row < N; row += kThreads) lsep[row] = -INFINITY;
    }
    return;
  }

  // ---- key range of this workgroup ---------------------------------------------
  const int q_last = (q0 + BM < n ? q0 + BM : n) - 1;
  int lo = 0, hi = n;
  if (a.wl >= 0) lo = q0 - a.wl > 0 ? q0 - a.wl : 0;
  if (a.wr >= 0) hi = q_last + a.wr + 1 < n ? q_last + a.wr + 1 : n;
  const int t_lo = lo / kBN;
  const int t_hi = (hi + kBN - 1) / kBN;
  const bool windowed = (a.wl >= 0) || (a.wr >= 0);

  // ---- this wavefront's queries --------------------------------------------------
  const int qw0 = q0 + wave * 32 * NQB;
  const int qw_last = (qw0 + 32 * NQB < n ? qw0 + 32 * NQB : n) - 1;  // < qw0: all padding
  const bool wave_has_rows = qw_last >= qw0;

  typename T::v8 qreg[NQB][4];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    int row = qw0 + qb * 32 + l32;
    row = row < N ? row : N - 1;
    const uint16_t* src = qp + row * a.qs[2] + hh * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint4 u = *(const uint4*)(src + ks * 16);
      if (a.negate_q) {
        u.x ^= 0x80008000u; u.y ^= 0x80008000u; u.z ^= 0x80008000u; u.w ^= 0x80008000u;
      }
      qreg[qb][ks] = as_v8<T>(u);
    }
  }

  floatx16 oacc[NQB][2];
  float m_ref[NQB], mc[NQB], lsum[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    m_ref[qb] = -INFINITY;
    mc[qb] = 0.f;
    lsum[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[qb][db][r] = 0.f;
  }

  // ---- staging: thread t moves 16 bytes of rows t/8 and t/8 + 32 -------------------
  const int st_r = tid >> 3, st_c = (tid & 7) * 8;
  uint4 kst[2], vst[2];
  auto fetch = [&](int t) {
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const int jg = t * kBN + p * 32 + st_r;
      const int jc = jg < N ? jg : N - 1;
      kst[p] = *(const uint4*)(kp + jc * a.ks[2] + st_c);
      uint4 vv = *(const uint4*)(vp + jc * a.vs[2] + st_c);
      // padded V rows are replaced by zeros: 0 * (whatever is stored there) must be 0
      if (jg >= n) vv = make_uint4(0, 0, 0, 0);
      vst[p] = vv;
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      *(uint4*)&lds_k[buf][(p * 32 + st_r) * kSK + st_c] = kst[p];
      *(uint4*)&lds_v[buf][(p * 32 + st_r) * kSV + st_c] = vst[p];
    }
  };

  fetch(t_lo);
  stash(0);
  __syncthreads();

  int buf = 0;
  for (int t = t_lo; t < t_hi; ++t) {
    if (t + 1 < t_hi) fetch(t + 1);

    const int tile_j0 = t * kBN;
    // interior tiles (every key visible to every query of the workgroup) take the
    // instantiation without any per-element mask work
    auto tile_compute = [&](auto masked_tag) {
      constexpr bool masked = decltype(masked_tag)::value;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const int kb0 = tile_j0 + kb * 32;
        if (masked) {  // wavefront-uniform: skip key blocks no query of this wavefront sees
          if (kb0 >= n) continue;
          if (a.wl >= 0 && kb0 + 31 < qw0 - a.wl) continue;
          if (a.wr >= 0 && kb0 > qw_last + a.wr) continue;
        }

        // S^T block: 32 keys x 32 queries per qb
        floatx16 sacc[NQB];
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[qb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const uint4 ku = *(const uint4*)&lds_k[buf][(kb * 32 + l32) * kSK + ks * 16 + hh * 8];
          const typename T::v8 ka = as_v8<T>(ku);
#pragma unroll
          for (int qb = 0; qb < NQB; ++qb) sacc[qb] = T::mfma(ka, qreg[qb][ks], sacc[qb]);
        }

        // online softmax; lane holds query (qb, l32) and keys kb0 + 8*(r/4) + 4*hh + r%4
        uint32_t pk[NQB][8];
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
          const int ig = qw0 + qb * 32 + l32;
          uint32_t vis = 0xFFFFu;
          if (masked) {
            vis = 0;
            int jlo = 0, jhi = n - 1;
            if (a.wl >= 0 && ig - a.wl > jlo) jlo = ig - a.wl;
            if (a.wr >= 0 && ig + a.wr < jhi) jhi = ig + a.wr;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int jg = kb0 + 8 * (r >> 2) + 4 * hh + (r & 3);
              vis |= (jg >= jlo && jg <= jhi) ? (1u << r) : 0u;
            }
          }
          float tmax = -INFINITY;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float sv = (!masked || (vis >> r & 1)) ? sacc[qb][r] : -INFINITY;
            tmax = fmaxf(tmax, sv);
          }
          tmax = fmaxf(tmax, xor32(tmax));
          // A lane refreshes its reference only on its own row's evidence, so what a
          // row computes never depends on which other rows share its wavefront.
          const bool refresh = (tmax - m_ref[qb]) > a.tau_raw;
          if (__any(refresh)) {
            const float m_new = refresh ? tmax : m_ref[qb];
            const float mc_new = (m_new == -INFINITY) ? 0.f : m_new * a.c;
            const float alpha = __builtin_amdgcn_exp2f(mc[qb] - mc_new);
            m_ref[qb] = m_new;
            mc[qb] = mc_new;
            lsum[qb] *= alpha;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
              for (int r = 0; r < 16; ++r) oacc[qb][db][r] *= alpha;
          }
          const float nmc = -mc[qb];
          float p[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float e = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[qb][r], a.c, nmc));
            if (masked) e = (vis >> r & 1) ? e : 0.f;
            p[r] = e;
            lsum[qb] += e;
          }
#pragma unroll
          for (int r = 0; r < 8; ++r) pk[qb][r] = T::pack2(p[2 * r], p[2 * r + 1]);
        }

        // O^T += V^T * P^T ; summation slot (hh, e) of k-step ks2 is key
        // kb*32 + 16*ks2 + (e < 4 ? 4*hh + e : 8 + 4*hh + e - 4)
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
#pragma unroll
          for (int db = 0; db < 2; ++db) {
            typename T::v8 va;
            if (V_TR) {
              // within 16 lanes, lane p fetches 4 consecutive d of key row p/4; the
              // transpose hands lane i the 4 keys of column i.
              const int p16 = lane & 15;
              const int row = kb * 32 + ks2 * 16 + 4 * hh + (p16 >> 2);
              const int col = db * 32 + 16 * ((lane >> 4) & 1) + 4 * (p16 & 3);
              typedef __attribute__((address_space(3))) shortx4 lds_s4;
              const shortx4 x0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                  (lds_s4*)&lds_v[buf][row * kSV + col]);
              const shortx4 x1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                  (lds_s4*)&lds_v[buf][(row + 8) * kSV + col]);
              shortx8 x;
              x[0] = x0[0]; x[1] = x0[1]; x[2] = x0[2]; x[3] = x0[3];
              x[4] = x1[0]; x[5] = x1[1]; x[6] = x1[2]; x[7] = x1[3];
              va = __builtin_bit_cast(typename T::v8, x);
            } else {
              shortx8 x;
#pragma unroll
              for (int e = 0; e < 8; ++e) {
                const int row = kb * 32 + ks2 * 16 + (e < 4 ? 4 * hh + e : 8 + 4 * hh + e - 4);
                x[e] = (short)lds_v[buf][row * kSV + db * 32 + l32];
              }
              va = __builtin_bit_cast(typename T::v8, x);
            }
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) {
              uint4 pu = make_uint4(pk[qb][ks2 * 4 + 0], pk[qb][ks2 * 4 + 1], pk[qb][ks2 * 4 + 2],
                                    pk[qb][ks2 * 4 + 3]);
              oacc[qb][db] = T::mfma(va, as_v8<T>(pu), oacc[qb][db]);
            }
          }
        }
      }
    };
    if (wave_has_rows) {
      if (windowed || (tile_j0 + kBN > n)) tile_compute(std::true_type{});
      else tile_compute(std::false_type{});
    }

    if (t + 1 < t_hi) stash(buf ^ 1);
    __syncthreads();
    buf ^= 1;
  }

  // ---- epilogue -----------------------------------------------------------------------
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const int ig = qw0 + qb * 32 + l32;
    const float ltot = lsum[qb] + xor32(lsum[qb]);
    if (ig >= N) continue;
    const bool live = (ig < n) && (ltot > 0.f);
    const float inv = live ? 1.0f / ltot : 0.f;
    uint16_t* orow = op + ig * a.os[2];
#pragma unroll
    for (int db = 0; db < 2; ++db) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 w;
        w.x = T::pack2(oacc[qb][db][4 * g + 0] * inv, oacc[qb][db][4 * g + 1] * inv);
        w.y = T::pack2(oacc[qb][db][4 * g + 2] * inv, oacc[qb][db][4 * g + 3] * inv);
        if (!live) w = make_uint2(0, 0);
        *(uint2*)(orow + db * 32 + 8 * g + 4 * hh) = w;
      }
    }
    if (lsep && hh == 0) {
      lsep[ig] = live ? (mc[qb] + __builtin_amdgcn_logf(ltot)) * kLn2 : -INFINITY;
    }
  }
}

template <class T>
int launch(const FaKernelArgs& a, int bm, int v_path, void* stream) {
  dim3 block(kThreads);
  unsigned grid = (unsigned)a.total_tiles;
  if (a.map_xcd) grid = (unsigned)(((a.total_tiles + 7) / 8) * 8);
  hipStream_t s = (hipStream_t)stream;
  if (bm == 256) {
    if (v_path == 0) hipLaunchKernelGGL((fa_fwd_kernel<T, 2, true>), dim3(grid), block, 0, s, a);
    else hipLaunchKernelGGL((fa_fwd_kernel<T, 2, false>), dim3(grid), block, 0, s, a);
  } else {
    if (v_path == 0) hipLaunchKernelGGL((fa_fwd_kernel<T, 1, true>), dim3(grid), block, 0, s, a);
    else hipLaunchKernelGGL((fa_fwd_kernel<T, 1, false>), dim3(grid), block, 0, s, a);
  }
  return (int)hipGetLastError();
}

}  // namespace

int fa_launch_f16(const FaKernelArgs& a, int bm, int v_path, void* stream) {
  return launch<F16>(a, bm, v_path, stream);
}
int fa_launch_bf16(const FaKernelArgs& a, int bm, int v_path, void* stream) {
  return launch<BF16>(a, bm, v_path, stream);
}
