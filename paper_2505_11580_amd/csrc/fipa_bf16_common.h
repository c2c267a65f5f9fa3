// Layout of the packed (lifted) tensors used by the bf16 MFMA path, shared by the pack,
// attention and epilogue kernels.
//
// Lifted features (Algorithm 1 steps 4-6, rewritten without changing the result):
//   q^ = [ q | Qhi Qhi Qlo Qlo | log2e * w_L * w_b (.) z1 ]
//   k^ = [ log2e*w_L/sqrt(c) * k | Khi Klo Khi Klo | z2 ]      K = log2e*gamma*w_L*w_C * (T o k_pts)
//   v^ = [ v | Vhi | Vlo | z2 ]
// Global point coordinates are carried as the sum of two bf16 numbers (hi + lo), so that the
// four partial products Qhi.Khi + Qhi.Klo + Qlo.Khi + Qlo.Klo reproduce the fp32 dot product;
// the per-key term -|K|^2/2 of the expanded squared distance is added in fp32 (kbias), and the
// per-query term |Q|^2 is constant along the softmax axis and is dropped (it returns in lse).
// The first kDH columns are head specific; the pair-factor part is shared by all heads and,
// on the key side, by k^ and v^.
#pragma once

#include "fipa_internal.h"

namespace fipa {

constexpr int kDH = 64;     // head-specific lifted columns (scalars + split points), zero padded
constexpr int kTileQ = 128; // query rows per workgroup (4 waves x 32 rows)
constexpr int kTileK = 64;  // keys per LDS tile

typedef unsigned short bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ bf16_t f2bf(float f)
{
    unsigned u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((unsigned)h) << 16); }

// Position of key kk (0..63) inside a transposed value tile row.  Within each group of 16
// keys the order is the one in which a lane of the S^T accumulator holds its keys, so that the
// probabilities can be fed to the second MFMA straight from registers.
__host__ __device__ __forceinline__ int vt_pos(int kk)
{
    const int grp = kk & ~15, x = kk & 15;
    const int g = (x >> 2) & 1, s = ((x >> 3) << 2) | (x & 3);
    return grp + 8 * g + s;
}

// Column of the head-specific value block holding part `lo` (0 = hi, 1 = lo) of global value
// coordinate cc (= 3*point + axis).
__host__ __device__ __forceinline__ int v_pt_col(int c, int Pv, int cc, int lo)
{
    return c + lo * 3 * Pv + cc;
}

struct Bf16Layout {
    int Lp, NT, DZ;
    size_t cen, kvlen, Qh, Qz, Kh, Z2, kbias, qbias, VhT, Z2T, Ohat, lse2, total;
};

inline Bf16Layout bf16_layout(const fipa_desc &d)
{
    Bf16Layout w;
    w.Lp = (int)align_up((size_t)d.L, kTileQ);
    w.NT = w.Lp / kTileK;
    w.DZ = d.r * d.cz;
    const size_t BH = (size_t)d.B * d.H;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    w.cen = take((size_t)d.B * 4 * sizeof(float));
    w.kvlen = take((size_t)d.B * sizeof(int));
    w.Qh = take(BH * w.Lp * kDH * 2);
    w.Qz = take(BH * w.Lp * (size_t)w.DZ * 2);
    w.Kh = take(BH * w.Lp * kDH * 2);
    w.Z2 = take((size_t)d.B * w.Lp * w.DZ * 2);
    w.kbias = take(BH * w.Lp * sizeof(float));
    w.qbias = take(BH * w.Lp * sizeof(float));
    w.VhT = take(BH * w.Lp * kDH * 2);
    w.Z2T = take((size_t)d.B * w.Lp * w.DZ * 2);
    w.Ohat = take(BH * w.Lp * (size_t)(kDH + w.DZ) * sizeof(float));
    w.lse2 = take(BH * w.Lp * sizeof(float));
    w.total = off;
    return w;
}

struct PackParams {
    const bf16_t *q, *k, *v, *q_pts, *k_pts, *v_pts, *z1, *z2;
    const float *rot, *trans, *w_b, *gamma, *cen;
    const uint8_t *mask;
    bf16_t *Qh, *Qz, *Kh, *Z2, *VhT, *Z2T;
    float *kbias, *qbias;
    int B, L, Lp, NT, H, c, Pq, Pv, cz, r, DZ;
    float w_L, w_C, qk_scale;
};

struct AttnParams {
    const bf16_t *Qh, *Qz, *Kh, *Z2, *VhT, *Z2T;
    const float *kbias;
    const int *kvlen;
    float *Ohat, *lse2;
    int B, L, Lp, H, NT, nQT, total_tiles;
};

struct EpiParams {
    const float *Ohat, *lse2, *qbias, *rot, *trans, *cen;
    const bf16_t *z1;
    const uint8_t *mask;
    float *o, *o_pts, *o_pair, *lse;
    int B, L, Lp, H, c, Pv, cz, r, DZ;
};

hipError_t launch_pack_bf16(const PackParams &p, hipStream_t stream);
hipError_t launch_attn_fwd_bf16(const AttnParams &p, int DZ, hipStream_t stream);
hipError_t launch_epilogue_bf16(const EpiParams &p, hipStream_t stream);

}  // namespace fipa
