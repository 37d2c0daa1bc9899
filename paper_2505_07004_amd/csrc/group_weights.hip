// Averaged squared output gradients, s[i,k] = c^2/|J_k| * sum_{j in J_k} dZ[i,j]^2
// (GuidedQuant, Algorithm 1, line 2).  One pass over dZ: HBM-bound streaming with
// 16-byte loads and a shuffle reduction inside a team of LPP lanes per (token, group).
#include "gq_internal.hpp"

namespace gq {
namespace {

template <typename T> struct Elems;
template <> struct Elems<float> {
  static constexpr int kPerVec = 4;
  __device__ static float sumsq(const float* p) {
    f32x4 v = *reinterpret_cast<const f32x4*>(p);
    return (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
  }
  __device__ static float one(const float* p) { return *p; }
};
template <> struct Elems<__bf16> {
  static constexpr int kPerVec = 8;
  __device__ static float sumsq(const __bf16* p) {
    u32x4 v = *reinterpret_cast<const u32x4*>(p);
    float acc = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float lo = __builtin_bit_cast(float, v[q] << 16);
      float hi = __builtin_bit_cast(float, v[q] & 0xffff0000u);
      acc += lo * lo + hi * hi;
    }
    return acc;
  }
  __device__ static float one(const __bf16* p) { return (float)*p; }
};

// A team of LPP consecutive lanes reduces one (token i, group k) segment of m elements.
// VEC: the segment start is 16-byte aligned and m is a multiple of the vector width.
template <typename T, int LPP, bool VEC>
__global__ __launch_bounds__(256) void group_weights_kernel(const T* __restrict__ dZ, int64_t n_pairs,
                                                            int G, int64_t m, int64_t ld, float coef,
                                                            float* __restrict__ s, int64_t ld_s) {
  constexpr int kTeams = 256 / LPP;
  const int team = threadIdx.x / LPP;
  const int lane = threadIdx.x % LPP;
  constexpr int V = Elems<T>::kPerVec;
  for (int64_t p = (int64_t)blockIdx.x * kTeams + team; p < n_pairs; p += (int64_t)gridDim.x * kTeams) {
    const int64_t i = p / G;
    const int k = (int)(p - i * G);
    const T* seg = dZ + i * ld + (int64_t)k * m;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    if (VEC) {
      const int64_t nv = m / V;
      int64_t v = lane;
      for (; v + 3 * LPP < nv; v += 4 * LPP) {
        a0 += Elems<T>::sumsq(seg + v * V);
        a1 += Elems<T>::sumsq(seg + (v + LPP) * V);
        a2 += Elems<T>::sumsq(seg + (v + 2 * LPP) * V);
        a3 += Elems<T>::sumsq(seg + (v + 3 * LPP) * V);
      }
      for (; v < nv; v += LPP) a0 += Elems<T>::sumsq(seg + v * V);
    } else {
      for (int64_t e = lane; e < m; e += LPP) {
        float x = Elems<T>::one(seg + e);
        a0 += x * x;
      }
    }
    float acc = (a0 + a1) + (a2 + a3);
#pragma unroll
    for (int off = LPP / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
    if (lane == 0) s[i * ld_s + k] = coef * acc;
  }
}

template <typename T, int LPP>
hipError_t launch_t(const T* dZ, int64_t n, int64_t m, int64_t ld, int G, float coef, float* s, int64_t ld_s, bool vec,
                    hipStream_t st) {
  const int64_t n_pairs = n * G;
  const int64_t teams = 256 / LPP;
  int64_t blocks = (n_pairs + teams - 1) / teams;
  const int64_t cap = 256 * 16;  // 16 resident blocks per CU is more than enough to saturate HBM
  if (blocks > cap) blocks = cap;
  if (vec)
    group_weights_kernel<T, LPP, true><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(dZ, n_pairs, G, m, ld, coef, s, ld_s);
  else
    group_weights_kernel<T, LPP, false><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(dZ, n_pairs, G, m, ld, coef, s, ld_s);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_dt(const T* dZ, int64_t n, int64_t d_out, int64_t ld, int G, float grad_scale, float* s,
                     int64_t ld_s, hipStream_t st) {
  const int64_t m = d_out / G;
  const float coef = (float)((double)grad_scale * (double)grad_scale / (double)m);
  constexpr int V = Elems<T>::kPerVec;
  const bool vec = (m % V == 0);  // with a 16-byte aligned base and pitch every segment start is aligned
  const int64_t work = vec ? m / V : m;  // loads per segment
  if (work >= 64) return launch_t<T, 64>(dZ, n, m, ld, G, coef, s, ld_s, vec, st);
  if (work >= 16) return launch_t<T, 16>(dZ, n, m, ld, G, coef, s, ld_s, vec, st);
  if (work >= 4) return launch_t<T, 4>(dZ, n, m, ld, G, coef, s, ld_s, vec, st);
  return launch_t<T, 1>(dZ, n, m, ld, G, coef, s, ld_s, vec, st);
}

}  // namespace

hipError_t launch_group_weights(const void* dZ, gq_dtype dt, int64_t n, int64_t d_out, int64_t ld, int G,
                                float grad_scale, float* s, int64_t ld_s, hipStream_t st) {
  if (n == 0) return hipSuccess;
  if (dt == GQ_F32) return launch_dt<float>((const float*)dZ, n, d_out, ld, G, grad_scale, s, ld_s, st);
  return launch_dt<__bf16>((const __bf16*)dZ, n, d_out, ld, G, grad_scale, s, ld_s, st);
}

}  // namespace gq
