// Optional per-stage timing with HIP events recorded on the caller's stream.
#include <vector>

#include "fipa_internal.h"

namespace fipa {

namespace {
struct ProfileState {
    bool active = false;
    int capacity = 0;
    int used = 0;
    int every = 1;   // time one call in `every`
    long calls = 0;  // calls seen since begin
    std::vector<hipEvent_t> ev;  // [capacity][FIPA_PROFILE_STAGES][2]
    std::vector<unsigned char> recorded;  // [capacity][FIPA_PROFILE_STAGES]
};
ProfileState g_prof;
}  // namespace

StageTimer::StageTimer(hipStream_t stream) : stream_(stream), slot_(-1)
{
    if (g_prof.active && g_prof.calls++ % g_prof.every == 0 && g_prof.used < g_prof.capacity) slot_ = g_prof.used++;
}

void StageTimer::begin(int stage)
{
    if (slot_ < 0) return;
    (void)hipEventRecord(g_prof.ev[((size_t)slot_ * FIPA_PROFILE_STAGES + stage) * 2], stream_);
}

void StageTimer::end(int stage)
{
    if (slot_ < 0) return;
    (void)hipEventRecord(g_prof.ev[((size_t)slot_ * FIPA_PROFILE_STAGES + stage) * 2 + 1], stream_);
    g_prof.recorded[(size_t)slot_ * FIPA_PROFILE_STAGES + stage] = 1;
}

}  // namespace fipa

using namespace fipa;

extern "C" int fipa_profile_begin(int capacity) { return fipa_profile_begin_every(capacity, 1); }

extern "C" int fipa_profile_begin_every(int capacity, int every)
{
    if (capacity <= 0 || capacity > 4096 || every <= 0 || g_prof.active) return FIPA_ERR_INVALID_ARG;
    g_prof.ev.assign((size_t)capacity * FIPA_PROFILE_STAGES * 2, nullptr);
    g_prof.recorded.assign((size_t)capacity * FIPA_PROFILE_STAGES, 0);
    for (auto &e : g_prof.ev)
        if (hipEventCreate(&e) != hipSuccess) return FIPA_ERR_LAUNCH;
    g_prof.capacity = capacity;
    g_prof.used = 0;
    g_prof.every = every;
    g_prof.calls = 0;
    g_prof.active = true;
    return FIPA_OK;
}

extern "C" int fipa_profile_end(float *stage_ms, int *n_calls)
{
    if (!g_prof.active) return FIPA_ERR_INVALID_ARG;
    g_prof.active = false;
    double sum[FIPA_PROFILE_STAGES] = {0};
    int cnt[FIPA_PROFILE_STAGES] = {0};
    int rc = FIPA_OK;
    for (int s = 0; s < g_prof.used; ++s)
        for (int st = 0; st < FIPA_PROFILE_STAGES; ++st) {
            if (!g_prof.recorded[(size_t)s * FIPA_PROFILE_STAGES + st]) continue;
            hipEvent_t a = g_prof.ev[((size_t)s * FIPA_PROFILE_STAGES + st) * 2];
            hipEvent_t b = g_prof.ev[((size_t)s * FIPA_PROFILE_STAGES + st) * 2 + 1];
            float ms = 0.f;
            if (hipEventSynchronize(b) != hipSuccess || hipEventElapsedTime(&ms, a, b) != hipSuccess) {
                rc = FIPA_ERR_LAUNCH;
                continue;
            }
            sum[st] += ms;
            cnt[st] += 1;
        }
    for (int st = 0; st < FIPA_PROFILE_STAGES; ++st)
        if (stage_ms) stage_ms[st] = cnt[st] ? (float)(sum[st] / cnt[st]) : 0.f;
    if (n_calls) *n_calls = g_prof.used;
    for (auto &e : g_prof.ev)
        if (e) (void)hipEventDestroy(e);
    g_prof.ev.clear();
    g_prof.recorded.clear();
    g_prof.capacity = g_prof.used = 0;
    return rc;
}

// ---- measured denominators for the benchmark -------------------------------------------------------
// A loop of independent 32x32x16 bf16 MFMAs (four accumulators per wave, operands in registers, no
// memory traffic): what the matrix pipes of this chip sustain at the clock they hold under that
// load.  2 * 32*32*16 flop per MFMA per wave.
namespace {
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;
typedef __attribute__((ext_vector_type(16))) float probe_f32x16;

__global__ __launch_bounds__(256) void fipa_probe_mfma_kernel(float *out, int iters)
{
    probe_bf16x8 a, b;
    for (int x = 0; x < 8; ++x) {
        a[x] = (__bf16)(float)((threadIdx.x + x) & 3);
        b[x] = (__bf16)1.0f;
    }
    probe_f32x16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j & 3], 0, 0, 0);
    }
    float r = 0.f;
    for (int i = 0; i < 4; ++i) r += acc[i][0];
    if (out) out[(size_t)blockIdx.x * 256 + threadIdx.x] = r;
}
}  // namespace

extern "C" int fipa_probe_mfma(int iters, int workgroups, float *out, void *hip_stream, double *flop)
{
    if (iters <= 0 || workgroups <= 0 || !out) return FIPA_ERR_INVALID_ARG;
    hipLaunchKernelGGL(fipa_probe_mfma_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(hip_stream), out, iters);
    if (flop) *flop = (double)workgroups * 4.0 * (double)iters * 16.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return hipGetLastError() == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
}
