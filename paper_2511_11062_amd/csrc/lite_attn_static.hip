// The allocation-free entry point of the C ABI (include/lite_attn.h: lite_attn_fwd_static) and the static device array
// that stands in for everything the other entry points keep in allocated device memory besides the Skip-Mask: the
// Skip-List, the row schedule, V^T and the statistics counters of the call.
#include <hip/hip_runtime.h>

#include <mutex>

#include "lite_attn.h"
#include "lite_attn_kernels.h"

namespace {

// One copy per GPU, held from the moment the library's code object is loaded on that GPU until the process ends.
static __device__ __align__(256) unsigned char scratch[LITE_ATTN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
char* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, looked up on the first call there

// In host code the name `scratch` is only a handle for the symbol, not a device address: every use of the array's
// memory goes through the pointer that hipGetSymbolAddress returns for the current device.
int scratch_of_current_device(char** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return la::hip_fail(e);
  if (dev < 0 || dev >= kMaxDevices) return LITE_ATTN_EUNSUPPORTED;
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e == hipSuccess && !p) e = hipErrorInvalidSymbol;
    if (e == hipSuccess) e = la::prepare_fwd();  // function attributes of the fused kernel on this device
    if (e != hipSuccess) return la::hip_fail(e);
    g_scratch_ptr[dev] = static_cast<char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return LITE_ATTN_OK;
}

}  // namespace

extern "C" int lite_attn_fwd_static(const void* q, const void* k, const void* v, void* out,
                                    const lite_attn_desc_t* desc, uint64_t* dev_skip_mask, float threshold,
                                    void* hip_stream) {
  int rc = la::check_desc(desc);
  if (rc != LITE_ATTN_OK) return rc;
  rc = la::check_call(q, k, v, out, threshold);
  if (rc != LITE_ATTN_OK) return rc;
  if (!dev_skip_mask || ((uintptr_t)dev_skip_mask & 7)) return LITE_ATTN_EINVAL;
  const la::Geometry geo = la::geometry(*desc);
  const la::ListLayout ll = la::list_layout(geo);  // the lists first, V^T behind them
  if (ll.total + la::vt_bytes(geo) > (size_t)LITE_ATTN_STATIC_SCRATCH_BYTES) return LITE_ATTN_ESCRATCH;
  char* ptr = nullptr;
  rc = scratch_of_current_device(&ptr);
  if (rc != LITE_ATTN_OK) return rc;
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  // the array keeps the previous call's contents: the counters the kernels add to start at zero (fill kernel, not a
  // memset node); Skip-List, row schedule and V^T are written in full, for this call's shape, before they are read
  unsigned long long* stats = reinterpret_cast<unsigned long long*>(ptr + ll.stats);
  hipError_t e = la::launch_clear(nullptr, 0, stats, 3, stream);
  if (e == hipSuccess)  // lists rebuilt from the caller's mask on every call, none left behind for a next one
    e = la::launch_call(*desc, geo, ll, ptr, reinterpret_cast<uint16_t*>(ptr + ll.total), q, k, v, out, dev_skip_mask,
                        stats, threshold, /*lists_ready=*/false, /*build_next=*/false, stream, nullptr);
  return e == hipSuccess ? LITE_ATTN_OK : la::hip_fail(e);
}
