#include "common.hpp"
namespace spt {
size_t coo_to_csr_workspace(const spt_tensor*) { return 256; }
spt_status coo_to_csr_dispatch(const spt_tensor*, int32_t, int32_t*, int32_t*, void*, void*, size_t,
                               hipStream_t) {
  return fail(SPT_ERR_UNSUPPORTED, "coo_to_csr: not built yet");
}
}  // namespace spt
