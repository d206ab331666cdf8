// Achievable ceilings of the machine this library runs on, measured rather than quoted:
//   * dense 32x32x16 matrix-core rate (fp16 and bf16) with nothing else going on, once with
//     all-zero operands and once with random operands.  The two differ a great deal on
//     MI355X: with random bits in the operands the chip lowers its clock to stay inside its
//     power limit, so the rate an attention kernel can hope for on real data is the second
//     number, not the data-sheet peak;
//   * streaming copy bandwidth (1 GiB read + 1 GiB written per pass).
// Prints one JSON line.  Standalone program: no part of the attention path uses it.
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define CK(x)                                                                          \
  do {                                                                                 \
    hipError_t e_ = (x);                                                               \
    if (e_ != hipSuccess) {                                                            \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
      return 1;                                                                        \
    }                                                                                  \
  } while (0)

// 8 wavefronts per compute unit, 16 independent-enough products per iteration: four
// accumulators, operands rotating over four A and four B fragments.
template <bool BF16>
__global__ __launch_bounds__(512) void mfma_loop(const uint4* in, float* out, int iters) {
  uint4 a[4], b[4];
  for (int i = 0; i < 4; ++i) {
    a[i] = in[threadIdx.x * 8 + i];
    b[i] = in[threadIdx.x * 8 + 4 + i];
  }
  floatx16 c[4];
  for (int j = 0; j < 4; ++j)
    for (int r = 0; r < 16; ++r) c[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (BF16)
          c[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf8, a[(i + j) & 3]),
                                                          __builtin_bit_cast(bf8, b[i]), c[j], 0, 0, 0);
        else
          c[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a[(i + j) & 3]),
                                                         __builtin_bit_cast(half8, b[i]), c[j], 0, 0, 0);
      }
  }
  float s = 0.f;
  for (int j = 0; j < 4; ++j)
    for (int r = 0; r < 16; ++r) s += c[j][r];
  if (s == 12345.678f) out[0] = s;  // keeps the loop alive
}

// each workgroup streams contiguous 16 KB pieces, four 16-byte accesses in flight per lane
__global__ __launch_bounds__(256) void copy16(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  const size_t piece = 1024;  // uint4 per workgroup step
  for (size_t base = (size_t)blockIdx.x * piece; base + piece <= n; base += (size_t)gridDim.x * piece) {
    uint4 r[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = src[base + j * 256 + threadIdx.x];
#pragma unroll
    for (int j = 0; j < 4; ++j) dst[base + j * 256 + threadIdx.x] = r[j];
  }
}

int main() {
  int cus = 0;
  CK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0));
  const int n16 = 512 * 8;  // uint4 per workgroup's worth of operands
  uint4* din;
  float* dout;
  CK(hipMalloc(&din, n16 * sizeof(uint4)));
  CK(hipMalloc(&dout, 4));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  const int iters = 4000, reps = 5;
  double tf[2][2];
  for (int bf = 0; bf < 2; ++bf)
    for (int rnd = 0; rnd < 2; ++rnd) {
      // values in (-1, 1) with random mantissas, from a fixed linear congruential sequence
      std::vector<uint16_t> h(n16 * 8, 0);
      if (rnd) {
        uint32_t x = 12345u;
        for (auto& v : h) {
          x = x * 1664525u + 1013904223u;
          const float f = ((int)(x >> 8) % 2001 - 1000) * 0.001f;
          if (bf) {
            uint32_t u;
            __builtin_memcpy(&u, &f, 4);
            v = (uint16_t)(u >> 16);
          } else {
            const _Float16 hf = (_Float16)f;
            __builtin_memcpy(&v, &hf, 2);
          }
        }
      }
      CK(hipMemcpy(din, h.data(), h.size() * 2, hipMemcpyHostToDevice));
      auto launch = [&] {
        if (bf) mfma_loop<true><<<cus, 512>>>(din, dout, iters);
        else mfma_loop<false><<<cus, 512>>>(din, dout, iters);
      };
      launch();
      CK(hipDeviceSynchronize());
      CK(hipEventRecord(e0));
      for (int r = 0; r < reps; ++r) launch();
      CK(hipEventRecord(e1));
      CK(hipEventSynchronize(e1));
      float ms;
      CK(hipEventElapsedTime(&ms, e0, e1));
      const double flops = 2.0 * 32 * 32 * 16 * 16.0 * iters * (double)cus * 8 * reps;
      tf[bf][rnd] = flops / (ms * 1e-3) / 1e12;
    }
  // copy
  const size_t bytes = (size_t)1 << 30, n = bytes / 16;
  uint4 *src, *dst;
  CK(hipMalloc(&src, bytes));
  CK(hipMalloc(&dst, bytes));
  CK(hipMemset(src, 1, bytes));
  copy16<<<cus * 32, 256>>>(src, dst, n);
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0));
  for (int r = 0; r < reps; ++r) copy16<<<cus * 32, 256>>>(src, dst, n);
  CK(hipEventRecord(e1));
  CK(hipEventSynchronize(e1));
  float ms;
  CK(hipEventElapsedTime(&ms, e0, e1));
  const double copy_gbs = 2.0 * bytes * reps / (ms * 1e-3) / 1e9;
  printf("{\"compute_units\": %d, \"mfma_f16_zero_tflops\": %.1f, \"mfma_f16_random_tflops\": %.1f, "
         "\"mfma_bf16_zero_tflops\": %.1f, \"mfma_bf16_random_tflops\": %.1f, \"copy_gbs\": %.1f}\n",
         cus, tf[0][0], tf[0][1], tf[1][0], tf[1][1], copy_gbs);
  CK(hipFree(src));
  CK(hipFree(dst));
  CK(hipFree(din));
  CK(hipFree(dout));
  return 0;
}
