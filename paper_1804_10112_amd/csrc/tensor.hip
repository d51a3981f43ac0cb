#include "common.hpp"
namespace spt {
size_t ttv_workspace(Format, const spt_tensor*) { return 256; }
size_t mttkrp_workspace(Format, const spt_tensor*, int32_t) { return 256; }
spt_status ttv_dispatch(Format, const spt_tensor*, const void*, int32_t*, int32_t*, void*, int64_t*,
                        void*, size_t, hipStream_t) {
  return fail(SPT_ERR_UNSUPPORTED, "ttv: not built yet");
}
spt_status mttkrp_dispatch(Format, const spt_tensor*, const void*, const void*, int32_t, void*,
                           void*, size_t, hipStream_t) {
  return fail(SPT_ERR_UNSUPPORTED, "mttkrp: not built yet");
}
}  // namespace spt
