// spt_spmv_static: spt_spmv for callers that cannot hand over (or allocate) a workspace --
// code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. The
// scratch memory the SpMV kernels need (the per-chunk carries of the entry-balanced CSR /
// ordered-COO kernel, the bins of the unordered-COO scatter, ...) lives in a fixed array in
// device memory that is part of the library's code object; the kernels receive its address
// exactly as they receive the caller's workspace in spt_spmv.
#include <atomic>
#include <mutex>

#include "common.hpp"

namespace spt {

constexpr size_t kStaticScratchBytes = SPT_STATIC_SCRATCH_BYTES;  // held by every GPU the library runs on

// Every GPU holds its own copy of this array at its own address. In host code the name is
// only a handle for hipGetSymbolAddress: it is never passed to a kernel or a memset.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, looked up once per device.
static spt_status scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(SPT_ERR_DEVICE, "spmv_static: hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices)
    return fail(SPT_ERR_UNSUPPORTED, "spmv_static: device ordinal %d beyond %d", dev, kMaxDevices);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (!p) {
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p)
        return fail(SPT_ERR_DEVICE, "spmv_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
      g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return SPT_OK;
}

}  // namespace spt

using namespace spt;

extern "C" {

spt_status spt_spmv_static(const spt_tensor* A, const void* x, void* y, void* stream) {
  clear_error();
  const size_t need = spt_workspace_bytes(SPT_OP_SPMV, A, 0);  // 0: invalid descriptor, error set
  if (need == 0) return spt_spmv(A, x, y, nullptr, 0, stream);  // reports what is wrong with A
  if (need > kStaticScratchBytes)
    return fail(SPT_ERR_WORKSPACE,
                "spmv_static: this operand needs %zu bytes of scratch memory, the static array holds %zu; "
                "use spt_spmv with a workspace",
                need, kStaticScratchBytes);
  void* ws = nullptr;
  spt_status st = scratch_of_current_device(&ws);
  if (st != SPT_OK) return st;
  return spt_spmv(A, x, y, ws, kStaticScratchBytes, stream);
}

}  // extern "C"
