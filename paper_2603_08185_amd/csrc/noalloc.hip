// serq_linear_noalloc: serq_linear for callers that cannot allocate or bring a workspace (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The only scratch memory
// serq_linear's kernels use -- the words in which the K slices of a channel block meet -- lives here in
// a file-scope device array; each GPU the library runs on holds its own copy until the process ends.
#include <mutex>

#include "serq_device.h"

namespace {

// One 64-bit word per output of a 32-token block, for at most kMaxN output channels: 8 MiB.
constexpr int64_t kMaxN = 32768;
constexpr size_t kScratchWords = (size_t)(kMaxN / 32) * 1024;
static __device__ __align__(256) unsigned long long scratch[kScratchWords];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};          // per device: the address of ITS copy of `scratch`

// Device address of the current device's copy of the array (set up on the first call on that device).
// In host code the array's name is only a handle for the runtime: the address kernels and fills may use
// is the one hipGetSymbolAddress returns, and it differs from device to device.
int scratch_for_current_device(void** out, hipStream_t st) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return SERQ_EHIP;
  if (dev < 0 || dev >= kMaxDevices) return SERQ_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return SERQ_EHIP;
    // The array is zero when the code object is loaded; it is cleared once more here, with a plain fill
    // kernel (safe under stream capture), so that the first call does not depend on that.
    const int rc = serq_workspace_init(ptr, sizeof(unsigned long long) * kScratchWords, (void*)st);
    if (rc != SERQ_OK) return rc;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SERQ_OK;
}

}  // namespace

extern "C" int serq_linear_noalloc(const void* Xq, const float* scale, int abits,
                                   const void* Wq, const float* wscale,
                                   int s_begin, int r, const void* Rp, int r_dtype,
                                   int64_t M, int64_t N, int64_t K,
                                   void* Y, int y_dtype, int64_t ldy, int flags, void* stream) {
  if (N > kMaxN) return SERQ_ELIMIT;
  void* ws = nullptr;
  const int rc = scratch_for_current_device(&ws, (hipStream_t)stream);
  if (rc != SERQ_OK) return rc;
  // The kernels receive the device address as an argument, exactly as they receive a caller's workspace;
  // they return every word they used to zero before they finish, so nothing has to be cleared per call.
  // (The array holds the decode path's meeting words only: the tiled path, which could park K slices in a
  // larger workspace, finds none here and runs unsliced.)
  return serq_linear(Xq, scale, abits, Wq, wscale, s_begin, r, Rp, r_dtype, M, N, K, Y, y_dtype, ldy,
                     ws, sizeof(unsigned long long) * kScratchWords, flags, stream);
}
