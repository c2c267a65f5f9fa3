// Host side of the bf16 forward: workspace carving and the pack -> attention -> epilogue chain.
#include "fipa_bf16_common.h"

namespace fipa {

size_t bf16_forward_workspace(const fipa_desc &d)
{
    return bf16_layout(d, !(bf16_fused_epilogue(d) || bf16_wide_fused_epilogue(d))).total;
}

hipError_t bf16_forward(const fipa_desc &d, const FwdArgs &a, void *ws, hipStream_t stream)
{
    const bool wide_fused = bf16_wide_fused_epilogue(d);
    const bool fused = bf16_fused_epilogue(d);
    const Bf16Layout w = bf16_layout(d, !(fused || wide_fused));
    char *base = static_cast<char *>(ws);
    float *cen = reinterpret_cast<float *>(base + w.cen);
    int *kvlen = reinterpret_cast<int *>(base + w.kvlen);

    StageTimer timer(stream);
    timer.begin(0);
    int *counters = reinterpret_cast<int *>(base + w.counters);
    const int n_counters = w.plan.S > 1 ? w.plan.rem * 4 : 0;
    // With the AlphaFold2 head shape the pack kernel does the per-batch preparation itself.
    const bool prep_in_pack = d.c == 16 && d.Pq == 4 && d.Pv == 8;
    hipError_t e = hipSuccess;
    if (!prep_in_pack) {
        e = launch_prep(d, a.trans, a.mask, a.cu, cen, kvlen, counters, n_counters, stream);
        if (e != hipSuccess) return e;
    }

    PackParams pk;
    pk.q = (const bf16_t *)a.q; pk.k = (const bf16_t *)a.k; pk.v = (const bf16_t *)a.v;
    pk.q_pts = (const bf16_t *)a.q_pts; pk.k_pts = (const bf16_t *)a.k_pts;
    pk.v_pts = (const bf16_t *)a.v_pts;
    pk.z1 = (const bf16_t *)a.z1; pk.z2 = (const bf16_t *)a.z2;
    pk.rot = a.rot; pk.trans = a.trans; pk.w_b = a.w_b; pk.gamma = a.gamma; pk.cen = cen;
    pk.mask = a.mask; pk.cu = a.cu;
    pk.Qh = (bf16_t *)(base + w.Qh); pk.Qz = (bf16_t *)(base + w.Qz);
    pk.Kh = (bf16_t *)(base + w.Kh); pk.Z2 = (bf16_t *)(base + w.Z2);
    pk.Vh = (bf16_t *)(base + w.Vh);
    pk.kbias = (float *)(base + w.kbias); pk.qbias = (float *)(base + w.qbias);
    pk.B = d.B; pk.L = d.L; pk.Lp = w.Lp; pk.NT = w.NT; pk.H = d.H; pk.c = d.c; pk.Pq = d.Pq;
    pk.Pv = d.Pv; pk.cz = d.cz; pk.r = d.r; pk.DZ = w.DZ;
    pk.w_L = d.w_L; pk.w_C = d.w_C; pk.qk_scale = d.qk_scale;
    pk.skip_qz = (fused && w.DZ <= 256) || w.DZ > 256;  // those attention kernels form the factor vectors themselves
    pk.cen_out = prep_in_pack ? cen : nullptr; pk.kvlen_out = kvlen; pk.counters = counters; pk.n_counters = n_counters;
    e = launch_pack_bf16(pk, stream);
    if (e != hipSuccess) return e;
    timer.end(0);

    AttnParams at;
    at.Qh = pk.Qh; at.Qz = pk.Qz; at.Kh = pk.Kh; at.Vh = pk.Vh; at.Z2 = pk.Z2;
    at.kbias = pk.kbias; at.qbias = pk.qbias; at.kvlen = kvlen;
    at.Ohat = fused || wide_fused ? nullptr : (float *)(base + w.Ohat);
    at.lse2 = (float *)(base + w.lse2);
    at.rot = a.rot; at.trans = a.trans; at.cen = cen; at.z1 = pk.z1; at.mask = a.mask; at.cu = a.cu;
    at.o = a.o; at.o_pts = a.o_pts; at.o_pair = a.o_pair; at.lse = a.lse;
    at.B = d.B; at.L = d.L; at.Lp = w.Lp; at.H = d.H; at.NT = w.NT;
    at.nQT = w.Lp / kTileQ; at.total_tiles = at.nQT * d.B * d.H; at.cz = d.cz; at.r = d.r; at.w_b = a.w_b; at.w_L = d.w_L;
    at.plan = w.plan; at.partial = (float *)(base + w.partial); at.counters = counters;
    at.deal = a.mask != nullptr || a.cu != nullptr;  // chains of different lengths
    at.ws_base = base;
    // (the wave-specialised kernel is an opt-in variant: it measured slower than the default on every shape tried)
    const bool ws_kernel = (d.flags & FIPA_FLAG_WAVE_SPECIALISED) && fused && attn_fwd_ws_supported(w.DZ, d.cz) &&
                           w.total < (1ull << 32) && !a.cu;
    timer.begin(1);
    e = w.DZ > 256 ? launch_attn_fwd_wide_bf16(at, w.DZ, wide_fused, stream)
        : ws_kernel ? launch_attn_fwd_ws_bf16(at, w.DZ, stream)
                    : launch_attn_fwd_bf16(at, w.DZ, fused, stream);
    if (e != hipSuccess) return e;
    timer.end(1);
    if (fused || wide_fused) return hipSuccess;  // steps 8-9 ran inside the attention kernel

    EpiParams ep;
    ep.Ohat = at.Ohat; ep.lse2 = at.lse2; ep.qbias = pk.qbias; ep.rot = a.rot; ep.trans = a.trans;
    ep.cen = cen; ep.z1 = pk.z1; ep.mask = a.mask; ep.cu = a.cu;
    ep.o = a.o; ep.o_pts = a.o_pts; ep.o_pair = a.o_pair; ep.lse = a.lse;
    ep.B = d.B; ep.L = d.L; ep.Lp = w.Lp; ep.H = d.H; ep.c = d.c; ep.Pv = d.Pv; ep.cz = d.cz;
    ep.r = d.r; ep.DZ = w.DZ;
    timer.begin(2);
    e = launch_epilogue_bf16(ep, stream);
    timer.end(2);
    return e;
}


}  // namespace fipa
