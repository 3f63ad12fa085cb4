// vf_gemm_noalloc: the sliced contraction of vf_gemm (nsplit > 1) for callers that cannot
// allocate device memory -- code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc.  vf_gemm hands the caller nsplit slabs of partial products to add up; here
// the slabs live in a file-scope device array of fixed size and the library's own fold kernel
// adds them in slab order into C.  The call allocates nothing: no hipMalloc, no hipFree, no
// library routine that allocates.
#include <mutex>

#include "vf_internal.h"

namespace vf {
namespace {

// The slabs of partial products.  Every GPU the library runs on holds its own copy of this
// array, at its own address, until the process ends.
constexpr int64_t kScratchFloats = VF_NOALLOC_SCRATCH_BYTES / 4;
static __device__ __align__(256) float scratch[kScratchFloats];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
float* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch`, per device

// In host code the array's name is a host-side stand-in, not a device address: the address on
// the device that is current comes from hipGetSymbolAddress, once per device.
int scratch_on_current_device(float** out) {
  int dev = -1;
  VF_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return VF_EINVAL;
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    VF_HIP(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
    if (!p) return VF_EDEVICE;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return VF_OK;
}

}  // namespace
}  // namespace vf

using namespace vf;

extern "C" int vf_gemm_noalloc(const void* A, int64_t lda, const void* B, int64_t ldb, float* C,
                               int32_t M, int32_t N, int32_t K, float alpha, int32_t accumulate,
                               int32_t nsplit, void* stream) {
  if (!A || !B || !C || M < 1 || N < 1 || K < 1 || lda < K || ldb < K || nsplit < 1) return VF_EINVAL;
  const int64_t slab = (int64_t)M * N;
  if (slab * nsplit > kScratchFloats) {
    set_last_error_text("vf_gemm_noalloc: nsplit * M * N floats exceed VF_NOALLOC_SCRATCH_BYTES");
    return VF_EINVAL;
  }
  float* slabs = nullptr;
  VF_TRY(scratch_on_current_device(&slabs));
  hipStream_t s = static_cast<hipStream_t>(stream);
  // every slice writes the whole of its slab (an empty slice writes zeros), so nothing has to be
  // cleared between calls
  Epilogue ep;
  ep.C = slabs; ep.ldc = N;
  VF_TRY(launch_gemm_bf16(static_cast<const bf16_t*>(A), lda, static_cast<const bf16_t*>(B), ldb, M, N, K,
                          nsplit, slab, ep, s));
  return launch_fold_slabs(slabs, nsplit, slab, slab, GradOut{C, alpha, accumulate ? 1 : 0}, s);
}
