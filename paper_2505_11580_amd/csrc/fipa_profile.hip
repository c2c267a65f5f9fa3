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
