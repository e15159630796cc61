// tmac_mpgemm for callers that cannot allocate: the split-K partial sums of the batched kernel go
// to a fixed device array that lives in this library's code object, one copy per GPU, instead of
// a workspace the caller brings.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "tmac.h"
#include "tmac_internal.h"

namespace tmac {

// The array.  In host code its name is only a handle for hipGetSymbolAddress: kernels and copies
// get the device address that call returns (a different one on every GPU).
static __device__ __align__(256) unsigned char scratch[TMAC_NOALLOC_MAX_WORKSPACE];

constexpr int NOALLOC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[NOALLOC_MAX_DEVICES];  // device address of `scratch` per GPU, null until asked

// Device address of the current GPU's copy of the array; looked up once per GPU.
static hipError_t scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace tmac

using namespace tmac;

extern "C" tmac_status tmac_mpgemm_noalloc(const tmac_wdesc* desc, const void* packed_dev, const void* lut_dev,
                                           tmac_lut_t lut, int32_t N, const float* act_scale_dev,
                                           float weight_scale, void* out_dev, tmac_out_t out, int64_t ldo,
                                           void* stream) {
  if (!desc || N <= 0) return TMAC_EINVAL;
  const size_t need_all = tmac_workspace_bytes(desc, N);  // (0: the descriptor is not valid)
  if (need_all == 0) return TMAC_EINVAL;
  // what the call would ask of a caller's workspace (the size query adds 256 bytes of slack)
  const size_t need = need_all > 256 ? need_all - 256 : 0;
  if (need > (size_t)TMAC_NOALLOC_MAX_WORKSPACE) {
    note_detail("tmac_mpgemm_noalloc: the split-K partial sums of this call exceed TMAC_NOALLOC_MAX_WORKSPACE bytes; "
                "use tmac_mpgemm with a workspace of tmac_workspace_bytes(desc, N) bytes");
    return TMAC_ESIZE;
  }
  void* ws = nullptr;
  const hipError_t e = scratch_of_current_device(&ws);
  if (e != hipSuccess) {
    note_hip_error((int)e);
    return TMAC_EHIP;
  }
  return tmac_mpgemm_ex(desc, packed_dev, lut_dev, lut, N, act_scale_dev, weight_scale, out_dev, out, ldo, ws,
                        (size_t)TMAC_NOALLOC_MAX_WORKSPACE, stream, nullptr);
}
