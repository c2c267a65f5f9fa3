// Internal declarations shared by the HIP sources of libfipa (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <atomic>
#include <stddef.h>
#include <stdint.h>

#include "fipa.h"

namespace fipa {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Dynamic-LDS limit of a kernel, raised once per device instead of on every launch: `state` is a
// function-local static of the launching function (one per kernel instantiation) that remembers
// the largest limit already set on each device.
struct LdsLimit {
    std::atomic<int> set[32] = {};
};
inline hipError_t raise_lds_limit(LdsLimit &state, const void *kernel, int bytes)
{
    int dev = 0;
    const bool known = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 32;
    if (known && state.set[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && known) {
        int cur = state.set[dev].load(std::memory_order_relaxed);
        while (cur < bytes && !state.set[dev].compare_exchange_weak(cur, bytes, std::memory_order_release)) {}
    }
    return e;
}

// All tensor arguments of fipa_forward, as passed by the caller.
struct FwdArgs {
    const void *q, *k, *v, *q_pts, *k_pts, *v_pts;
    const float *rot, *trans;
    const void *z1, *z2;
    const float *w_b, *gamma;
    const uint8_t *mask;
    float *o, *o_pts, *o_pair, *lse;
    // Packed batch (fipa_forward_packed / fipa_backward_packed): DEVICE pointer to B + 1 row offsets;
    // the tensors above then have [total] leading rows instead of [B, L], chain b at rows
    // cu[b] .. cu[b+1] - 1, and desc.L is an upper bound of the chain lengths.  Null: padded batch.
    const int *cu = nullptr;
    int total_rows = 0;  // with cu: the host's copy of cu[B]
};

struct BwdArgs {
    FwdArgs f;  // inputs and saved forward results (o, o_pts, o_pair, lse are read here)
    const float *d_o, *d_o_pts, *d_o_pair;
    void *d_q, *d_k, *d_v, *d_q_pts, *d_k_pts, *d_v_pts, *d_z1, *d_z2;
    float *d_gamma;
    float *d_w_b;            // may be null
    float *d_rot, *d_trans;  // both or neither
};

// Arguments of fipa_module_forward beyond the description.
struct ModuleArgs {
    const void *s, *w_in;
    const float *b_in;
    const float *rot, *trans;
    const void *z1, *z2;
    const float *w_b, *gamma;
    const uint8_t *mask;
    const void *w_out;
    const float *b_out;
    float *s_out;
};

// Arguments of fipa_module_backward beyond those of the forward.
struct ModuleBwdArgs {
    const float *d_s_out;
    float *d_s_in, *d_w_in, *d_b_in, *d_w_out, *d_b_out;  // the two bias gradients may be null
    void *d_z1, *d_z2;
    float *d_gamma, *d_w_b, *d_rot, *d_trans;             // d_w_b and the frame pair may be null
};

// Host-side checks of a description (sizes, dtype, flags, shapes the kernels are built for;
// backward: the shapes fipa_backward supports) and of a pointer's 16-byte alignment.
int check_desc(const fipa_desc *d, bool backward);
bool aligned16(const void *p);

// Host-side checks of fipa_forward's description and tensor pointers (null, alignment; the
// workspace is the caller's business), and the dispatch to the fp32 or bf16 chain.
int check_forward_args(const fipa_desc *desc, const FwdArgs &a);
hipError_t enqueue_forward(const fipa_desc &desc, const FwdArgs &a, void *workspace, hipStream_t stream);

// Stage timing (fipa_profile_begin / fipa_profile_end).  A StageTimer is created per API call;
// when profiling is inactive every method is a no-op.
class StageTimer {
   public:
    explicit StageTimer(hipStream_t stream);
    StageTimer() : stream_(nullptr), slot_(-1) {}  // never records
    void begin(int stage);  // record the start event of `stage`
    void end(int stage);    // record its stop event

   private:
    hipStream_t stream_;
    int slot_;
};

// Per-batch centroid of the valid translations (any common shift of all frames leaves the
// result unchanged, Section 2; subtracting it keeps global coordinates small) and the number
// of leading key slots that must be visited (1 + index of the last valid residue).
//   cen   [B,4] floats (x, y, z, unused),  kvlen [B] ints
// Also sets counters[0 .. n_counters) to zero (n_counters may be 0).
// cu: row offsets of a packed batch (see FwdArgs), or null.
hipError_t launch_prep(const fipa_desc &d, const float *trans, const uint8_t *mask, const int *cu, float *cen,
                       int *kvlen, int *counters, int n_counters, hipStream_t stream);

// fp32 direct path (fipa_f32.hip)
size_t f32_forward_workspace(const fipa_desc &d);
hipError_t f32_forward(const fipa_desc &d, const FwdArgs &a, void *ws, hipStream_t stream);

// bf16 MFMA path (fipa_bf16_*.hip)
size_t bf16_forward_workspace(const fipa_desc &d);
hipError_t bf16_forward(const fipa_desc &d, const FwdArgs &a, void *ws, hipStream_t stream);
size_t bf16_backward_workspace(const fipa_desc &d);

// IPA module around the core (fipa_module.hip)
bool module_shape_supported(const fipa_desc &d, int d_s);
bool module_backward_shape_supported(const fipa_desc &d, int d_s);
size_t module_forward_workspace(const fipa_desc &d, int d_s);
hipError_t module_forward(const fipa_desc &d, int d_s, const ModuleArgs &a, void *ws, hipStream_t stream);
size_t module_backward_workspace(const fipa_desc &d, int d_s);
hipError_t module_backward(const fipa_desc &d, int d_s, const ModuleArgs &a, const ModuleBwdArgs &g, void *ws,
                           hipStream_t stream);
hipError_t bf16_backward(const fipa_desc &d, const BwdArgs &a, void *ws, hipStream_t stream);
// bf16_backward in two calls on one workspace: `begin` runs the forward part and also writes the
// core's outputs f.o, f.o_pts, f.o_pair; `finish` takes the upstream gradients.
hipError_t bf16_backward_begin(const fipa_desc &d, const FwdArgs &f, void *ws, hipStream_t stream);
hipError_t bf16_backward_finish(const fipa_desc &d, const BwdArgs &a, void *ws, hipStream_t stream);

}  // namespace fipa
