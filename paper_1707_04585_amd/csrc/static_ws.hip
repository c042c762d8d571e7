// revnet_stack_fwd_static: the forward pass of a stack for callers that cannot
// allocate device memory and have no workspace of their own to hand over (code
// under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  Same kernels and the same driver as revnet_stack_fwd; the only
// difference is where the workspace lives: in a fixed-size array of this
// library's device image instead of caller memory.
#include <mutex>

#include "api_common.h"

namespace {

constexpr size_t kStaticWsBytes = RVN_STATIC_WS_BYTES;  // what revnet_stack_fwd_static can plan into
constexpr int kMaxDevices = 64;

// The workspace itself.  One copy per GPU that loads the library, held until
// the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; it is not a device address.
static __device__ __align__(256) unsigned char scratch[kStaticWsBytes];

std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, once looked up

// Device address of `scratch` on the current device (looked up once per device,
// with that device current); null with *err set if HIP refuses.
void *scratch_on_current_device(hipError_t *err) {
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

using namespace rvn;
using namespace rvn::api;

extern "C" {

int revnet_stack_fwd_static(const rvn_block_desc *desc, int32_t depth, const rvn_tensor *x1, const rvn_tensor *x2,
                            const rvn_block_params *params, const rvn_tensor *y1, const rvn_tensor *y2,
                            void *hip_stream) {
    if (depth <= 0) return fail(RVN_ERR_SHAPE, "depth = %d must be positive", depth);
    // Everything that can be checked without the device first; the plan tells how much workspace the
    // shape needs.  (A placeholder base that is aligned and overlaps nothing stands in for the workspace.)
    Plan pl;
    Geo g;
    void *const nowhere = reinterpret_cast<void *>(uintptr_t{256});
    if (int rc = check_fwd_args(desc, x1, x2, y1, y2, nowhere, ~size_t{0}, &pl, &g, false)) return rc;
    if (!params) return fail(RVN_ERR_NULL, "params is NULL");
    for (int k = 0; k < depth; ++k)
        if (int rc = check_params(*desc, &params[k], "params")) return rc;
    if (pl.total > kStaticWsBytes)
        return fail(RVN_ERR_WORKSPACE,
                    "this shape needs a workspace of %zu bytes; the built-in workspace of revnet_stack_fwd_static holds "
                    "%zu (use revnet_stack_fwd with a workspace of the caller's)",
                    pl.total, kStaticWsBytes);
    hipError_t herr = hipSuccess;
    void *const ws = scratch_on_current_device(&herr);
    if (!ws) return fail(RVN_ERR_HIP, "cannot locate the built-in workspace: %s", hipGetErrorString(herr));
    const rvn_tensor *t[4] = {x1, x2, y1, y2};
    const char *nm[4] = {"x1", "x2", "y1", "y2"};
    for (int i = 0; i < 4; ++i)
        if (overlaps_range(t[i], ws, kStaticWsBytes)) return fail(RVN_ERR_ALIAS, "%s overlaps the built-in workspace", nm[i]);
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    // (stack_forward starts by clearing the ticket counters with a fill kernel: the array keeps
    // whatever the previous call left in it, and nothing else in the plan is read before it is written)
    stack_forward(cx, *desc, depth, pl, bind(pl, ws), g, view_of(x1), view_of(x2), params, view_of(y1), view_of(y2));
    return finish(cx);
}

}  // extern "C"
