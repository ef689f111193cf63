// The one entry point of the library that allocates nothing: fp_op_gemm_noalloc, for callers that
// cannot call hipMalloc (code under HIP graph capture, tight serving loops, harnesses that forbid
// allocation).  It is fp_op_gemm_ws with the split-K workspace taken from a file-scope device
// array instead of a caller buffer.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/flowprefill.h"
#include "kernels.h"

namespace {

constexpr size_t kScratchBytes = (size_t)FP_NOALLOC_SCRATCH_BYTES;

// Split-K partial sums [split][M][N] fp32.  One copy per GPU the library runs on, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};    // device address of `scratch` on each GPU, once known

// Device address of this GPU's copy of the array (looked up once per device, with that device
// current).  Returns null and sets *err on failure.
void* scratch_on_current_device(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

fp_status fail(fp_status code, const char* fmt, long long a = 0, long long b = 0) {
  char buf[256];
  snprintf(buf, sizeof(buf), fmt, a, b);
  fp::set_last_error(buf);
  return code;
}

}  // namespace

extern "C" fp_status fp_op_gemm_noalloc(int32_t dtype, const void* a, const void* w, void* c, int64_t m,
                                        int64_t n, int64_t k, int32_t residual, void* hip_stream) {
  if (!a || !w || !c || m <= 0 || n <= 0 || k <= 0 || (k % 8) || (n % 8) || m > INT32_MAX ||
      n > INT32_MAX || k > INT32_MAX || (dtype != 0 && dtype != 1))
    return fail(FP_ERR_INVALID, "fp_op_gemm_noalloc: bad size, alignment or dtype");
  const size_t need = fp::gemm_workspace_bytes(dtype, m, n, k);
  if (need > kScratchBytes)
    return fail(FP_ERR_INVALID,
                "fp_op_gemm_noalloc: the problem wants %lld bytes of split-K scratch, the static scratch holds %lld; "
                "use fp_op_gemm_ws with a caller workspace", (long long)need, (long long)kScratchBytes);
  hipError_t e = hipSuccess;
  void* ptr = scratch_on_current_device(&e);
  if (!ptr) {
    fp::set_last_error(hipGetErrorString(e));
    return FP_ERR_DEVICE;
  }
  // Nothing in the scratch has to start at zero: every launched K range stores its whole [M][N]
  // slab before the reduction kernel (next on the same stream) reads exactly those slabs.
  fp::launch_gemm(dtype, a, w, c, m, n, k, residual, ptr, kScratchBytes, reinterpret_cast<hipStream_t>(hip_stream));
  e = hipGetLastError();
  if (e != hipSuccess) {
    fp::set_last_error(hipGetErrorString(e));
    return FP_ERR_DEVICE;
  }
  return FP_OK;
}
