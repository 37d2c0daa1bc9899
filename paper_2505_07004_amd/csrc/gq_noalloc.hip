// gq_fisher_gram_noalloc: gq_fisher_gram for callers that cannot allocate device memory (code under HIP
// graph capture, tight serving loops, harnesses that forbid hipMalloc) and therefore cannot bring a
// workspace.  The only device memory the Gram kernels need beyond inputs and outputs, when no work item
// is split between workgroups, is the token weights repacked group-major with zero padding; here that
// buffer is a file-scope device array of fixed size.  Nothing is allocated or freed, by this library or
// by anything it calls.
#include <mutex>

#include "gq_internal.hpp"

namespace {

constexpr size_t kScratchBytes = (size_t)4 << 20;      // 4 MiB per GPU, held until the process ends
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code `scratch` is only a handle: the address of a GPU's copy of the array comes from
// hipGetSymbolAddress, once per device, with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

hipError_t scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

size_t gq_fisher_gram_noalloc_max_scratch_bytes(void) { return kScratchBytes; }

int gq_fisher_gram_noalloc(const void* X, gq_dtype x_dtype, int64_t n, int64_t d_in, int64_t ld_x, const float* s,
                           int32_t G, float* H, uint32_t flags, void* hip_stream) {
  if (x_dtype != GQ_F32 && x_dtype != GQ_BF16) return GQ_ERR_DTYPE;
  if (n < 0 || d_in <= 0 || G <= 0 || ld_x < d_in) return GQ_ERR_SHAPE;
  if (flags & ~(uint32_t)(GQ_ACCUMULATE | GQ_MIRROR | GQ_TWO_TERMS)) return GQ_ERR_UNSUPPORTED;
  if (!H) return GQ_ERR_NULLPTR;
  if (n > 0 && (!X || !s)) return GQ_ERR_NULLPTR;
  if (!aligned16(H)) return GQ_ERR_ALIGN;
  const size_t elem = x_dtype == GQ_BF16 ? 2 : 4;
  if (n > 0 && (!aligned16(X) || ((size_t)ld_x * elem) % 16 != 0)) return GQ_ERR_ALIGN;
  if (x_dtype == GQ_BF16 && (ld_x >= ((int64_t)1 << 26) || n >= ((int64_t)1 << 28))) return GQ_ERR_UNSUPPORTED;
  // the repacked weights of this call must fit the fixed array
  const size_t need = (x_dtype == GQ_BF16 && n > 0) ? gq::fisher_gram_bf16_weights_bytes(n, G) : 0;
  if (need > kScratchBytes) return GQ_ERR_WORKSPACE;

  hipStream_t st = (hipStream_t)hip_stream;
  const bool accumulate = (flags & GQ_ACCUMULATE) != 0;
  hipError_t e = hipSuccess;
  if (n == 0) {
    if (!accumulate) e = gq::launch_zero_upper(H, d_in, G, st);
  } else if (x_dtype == GQ_F32) {
    e = gq::launch_fisher_gram_f32((const float*)X, n, d_in, ld_x, s, G, H, accumulate, st);
  } else {
    void* ptr = nullptr;
    e = scratch_of_current_device(&ptr);
    if (e != hipSuccess) return GQ_ERR_HIP;
    // every call rewrites the part of the array it reads (weights and their zero padding), so nothing
    // of an earlier call is ever seen
    e = gq::launch_fisher_gram_bf16(X, n, d_in, ld_x, s, G, H, accumulate, (flags & GQ_TWO_TERMS) != 0, ptr, true, st);
  }
  if (e != hipSuccess) return GQ_ERR_HIP;
  if (flags & GQ_MIRROR) e = gq::launch_mirror(H, d_in, G, st);
  return e == hipSuccess ? GQ_OK : GQ_ERR_HIP;
}

}  // extern "C"
