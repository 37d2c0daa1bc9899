// Measures what the bf16 matrix cores of this GPU sustain on their own, next to which the
// Fisher-Gram kernel's rate is reported: a loop of independent v_mfma_f32_32x32x16_bf16 with
// no memory traffic at all, (a) on constant operands and (b) on operands with random sign and
// mantissa bits, as real activations have.  Under (b) the chip runs into its power limit and
// clocks down, so (b), not the data-sheet number, is the ceiling a dense bf16 kernel fed with
// real data can approach.  Prints one JSON line.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                                    \
  do {                                                                           \
    hipError_t e_ = (x);                                                         \
    if (e_ != hipSuccess) {                                                      \
      fprintf(stderr, "HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      return 1;                                                                  \
    }                                                                            \
  } while (0)

__device__ inline unsigned mix(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

template <int RANDOM>
__global__ __launch_bounds__(256) void mfma_only(float* out, int iters) {
  u32x4 aw[2], bw[8];
  for (int i = 0; i < 2; ++i)
    for (int q = 0; q < 4; ++q) {
      const unsigned h = mix(threadIdx.x * 131 + i * 17 + q);
      aw[i][q] = RANDOM ? ((h & 0x807f807fu) | 0x3f003f00u) : 0x3f803f80u;   // +-[0.5, 1) or 1.0
    }
  for (int i = 0; i < 8; ++i)
    for (int q = 0; q < 4; ++q) {
      const unsigned h = mix(threadIdx.x * 977 + i * 31 + q + 7);
      bw[i][q] = RANDOM ? ((h & 0x807f807fu) | 0x3f003f00u) : 0x3f803f80u;
    }
  f32x16 acc[16];
  for (int i = 0; i < 16; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aw[i & 1]),
                                                       __builtin_bit_cast(bf16x8, bw[i >> 1]), acc[i], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < 16; ++i)
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

template <int RANDOM>
static int run(float* d, int cus, double* tflops) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  const int iters = 40000;
  mfma_only<RANDOM><<<cus, 256>>>(d, 4000);   // warm up: clocks settle under load
  double best = 0;
  for (int rep = 0; rep < 3; ++rep) {
    CK(hipEventRecord(e0));
    mfma_only<RANDOM><<<cus, 256>>>(d, iters);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double tf = (double)cus * 4 * 16 * (double)iters * 32768.0 / ms / 1e9;
    if (rep > 0 && tf > best) best = tf;     // the first repetition still sees the ramp
  }
  *tflops = best;
  return 0;
}

int main() {
  hipDeviceProp_t p;
  CK(hipGetDeviceProperties(&p, 0));
  const int cus = p.multiProcessorCount;
  float* d;
  CK(hipMalloc(&d, (size_t)cus * 256 * sizeof(float)));
  double tc = 0, tr = 0;
  if (run<0>(d, cus, &tc)) return 1;
  if (run<1>(d, cus, &tr)) return 1;
  printf("{\"kernel\": \"v_mfma_f32_32x32x16_bf16 only, 1 wave per SIMD, %d CUs\", \"constant_operands_tflops\": %.1f, "
         "\"random_operands_tflops\": %.1f}\n", cus, tc, tr);
  return 0;
}
