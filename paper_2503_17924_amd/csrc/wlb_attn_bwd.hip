#include <hip/hip_runtime.h>
#include "wlb_device.h"
#include "wlb_internal.h"
namespace wlb {
wlb_status launch_bwd(const wlb_attn_desc& d, const wlb_plan_layout& L, const void* q, const void* k,
                      const void* v, const void* o, const float* lse, const void* d_o, void* dq,
                      void* dk, void* dv, char* ws, size_t off_delta, void* stream) {
    return fail(WLB_ERR_UNSUPPORTED, "backward not built yet");
}
}
