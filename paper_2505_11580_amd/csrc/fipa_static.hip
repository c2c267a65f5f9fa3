// fipa_forward_static: fipa_forward for callers that cannot allocate device memory (code under HIP
// graph capture, serving loops, harnesses that forbid hipMalloc).  The workspace of fipa_forward
// is replaced by a scratch array that lives in the library's own device image: each GPU the
// library runs on holds one copy until the process ends.  The kernels are those of fipa_forward;
// they receive the array's device address as their workspace argument.
#include <mutex>

#include "fipa_internal.h"

namespace {

// File-scope device array.  In host code this name is only a handle for hipGetSymbolAddress: the
// device address differs per GPU and is looked up once per device below.
static __device__ __align__(256) unsigned char scratch[FIPA_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, once known

// Device address of this GPU's copy of the scratch array (looked up on the first call on a device,
// with that device current).  Returns nullptr and sets *err on failure.
void *scratch_address(hipError_t *err)
{
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (*err != hipSuccess || !ptr) {
            if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" int fipa_forward_static(const fipa_desc *desc, const void *q, const void *k, const void *v,
                                   const void *q_pts, const void *k_pts, const void *v_pts, const float *rot,
                                   const float *trans, const void *z1, const void *z2, const float *w_b,
                                   const float *gamma, const uint8_t *mask, float *o, float *o_pts, float *o_pair,
                                   float *lse, void *hip_stream)
{
    // host-side checks first: argument errors are reported without touching a device
    const fipa::FwdArgs a{q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask, o, o_pts, o_pair, lse};
    const int rc = fipa::check_forward_args(desc, a);
    if (rc != FIPA_OK) return rc;
    if (desc->flags & FIPA_FLAG_KEEP_FORWARD) return FIPA_ERR_UNSUPPORTED;  // (nothing is kept in the shared scratch)
    size_t need = 0;
    fipa_workspace_bytes(desc, &need, nullptr);
    if (need > (size_t)FIPA_STATIC_SCRATCH_BYTES) return FIPA_ERR_WORKSPACE;  // problem too large for the static scratch
    hipError_t e = hipSuccess;
    void *ws = scratch_address(&e);
    if (!ws) return FIPA_ERR_LAUNCH;
    // Everything the kernels expect to start at zero (the arrival counters of the key-range split)
    // is cleared by the first kernel of every call, so the previous call's contents do not matter.
    e = fipa::enqueue_forward(*desc, a, ws, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
}
