// Layout of the packed (lifted) tensors used by the bf16 MFMA path, shared by the pack,
// attention and epilogue kernels.
//
// Lifted features (Algorithm 1 steps 4-6, rewritten without changing the result):
//   q^ = [ q | Qhi Qhi Qlo Qlo | log2e * w_L * w_b (.) z1 ]
//   k^ = [ log2e*w_L/sqrt(c) * k | Khi Klo Khi Klo | z2 ]      K = log2e*gamma*w_L*w_C * (T o k_pts)
//   v^ = [ v | Vhi, Vlo (interleaved per lane half, see v_pt_col) | z2 ]
// Global point coordinates are carried as the sum of two bf16 numbers (hi + lo), so that the
// four partial products Qhi.Khi + Qhi.Klo + Qlo.Khi + Qlo.Klo reproduce the fp32 dot product;
// the per-key term -|K|^2/2 of the expanded squared distance is added in fp32 (kbias), and the
// per-query term |Q|^2 is constant along the softmax axis and is dropped (it returns in lse).
// The first kDH columns are head specific; the pair-factor part z2 is stored once per batch
// element and serves every head, both as key features and as value features.
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

// Column of the head-specific value block that holds part `lo` (0 = hi, 1 = lo) of the global
// value coordinate (point pt, axis ax).  The transposed output accumulator gives the lanes
// 0-31 of a wave the columns d with (d/4)%2 == 0 and the lanes 32-63 the others; this layout
// puts all six numbers of a point into one half, so the inverse frame needs no lane exchange:
// half g' = pt / PH owns points g'*PH .. g'*PH+PH-1 (PH = ceil(Pv/2)).
__host__ __device__ __forceinline__ int v_pt_col(int c, int Pv, int pt, int ax, int lo)
{
    const int PH = (Pv + 1) / 2;
    const int gh = pt / PH;
    const int u = 3 * (pt - gh * PH) + ax + 3 * PH * lo;
    return c + 8 * (u >> 2) + 4 * gh + (u & 3);
}
// Largest column index + 1 that v_pt_col can return.
__host__ __device__ __forceinline__ int v_cols_needed(int c, int Pv)
{
    const int PH = (Pv + 1) / 2;
    return c + 8 * ((6 * PH + 3) / 4);
}

// Rows of the caller's tensors.  A padded batch keeps residue i of batch element b at row b L + i and
// every element has L residues; a packed batch (p.cu set: B + 1 row offsets in device memory, the
// variable-length batches of Section 3 stored back to back) keeps chain b at rows cu[b] .. cu[b+1] - 1.
// The workspace is laid out [B, .., Lp, ..] either way, Lp covering the longest chain.
template <class P>
__device__ __forceinline__ size_t user_row(const P &p, int b, int i)
{
    return p.cu ? (size_t)(p.cu[b] + i) : (size_t)b * p.L + i;
}
template <class P>
__device__ __forceinline__ int user_len(const P &p, int b)
{
    return p.cu ? p.cu[b + 1] - p.cu[b] : p.L;
}
// Element (b, h, i) of the log-sum-exp output: [B, H, L], or chain b's [H, len_b] block at H cu[b].
template <class P>
__device__ __forceinline__ size_t user_lse_index(const P &p, int b, int h, int i)
{
    return p.cu ? (size_t)p.cu[b] * p.H + (size_t)h * (p.cu[b + 1] - p.cu[b]) + i : ((size_t)b * p.H + h) * p.L + i;
}

// Key-range split of the fused attention launch.  A launch of T query tiles runs in ceil(T/256)
// rounds on the 256 compute units of the chip; when the last round would be at most half full,
// its tiles are cut into S parts along the key axis (each part one workgroup), so that the last
// round lasts about 1/S as long.  Each part reduces its accumulator to the unnormalised output
// row (scalars, global points, z1-contracted pair part: 20 + c_z floats per lane pair instead of
// 64 + r c_z) and leaves it in memory with its softmax reference and weight sum; the part that
// arrives last merges them.
struct SplitPlan {
    int full;  // leading tiles that run whole (a multiple of 256)
    int rem;   // remaining tiles
    int S;     // parts per remaining tile (1 = not split)
    // When the parts fill exactly one round (rem * S = 256) the last 256 whole tiles and the parts
    // are launched interleaved: half of the compute units take a part first and a whole tile
    // second, the other half the other way round.  Work per unit stays the same, but the
    // start-up loads and the output stores of the two halves no longer fall on the same instant
    // (those phases are bandwidth-bound when all 256 workgroups reach them together).
    int mixed;
    int units() const { return full + rem * S; }
};

inline SplitPlan attn_split_plan(int total_tiles, int Lp, int DZ, int cz, bool fused)
{
    constexpr int kCU = 256;
    SplitPlan s;
    s.full = (total_tiles / kCU) * kCU;
    s.rem = total_tiles - s.full;
    s.S = 1;
    if (fused && DZ <= 256 && cz >= 32 && s.rem > 0 && s.rem <= kCU / 2) {
        const int by_blocks = (Lp / 32) / 4;  // at least four 32-key blocks per part
        s.S = kCU / s.rem;
        if (s.S > 4) s.S = 4;
        if (s.S > by_blocks) s.S = by_blocks;
        if (s.S < 1) s.S = 1;
    }
    s.mixed = s.S > 1 && s.rem * s.S == kCU && s.full >= kCU;
    return s;
}

// The MFMA kernels give each XCD a contiguous run of work units, so that the tiles of one
// (batch, head) pair share that XCD's L2.  In launch order the pairs of one batch element are
// neighbours, and with chains of different lengths (a masked batch) whole XCDs would get only
// long or only short chains (lengths 5.8k, 7.5k, 7.5k, 1.6k at H = 12: four XCDs with 1.5 times
// the mean work, two with almost none).  deal_pair() renumbers the pairs so that position
// `pos` of the contiguous order holds pair x, x + 8, x + 16, ... for the x-th run: every XCD
// gets pairs of every batch element.  A bijection on [0, P) for any P.
__device__ __forceinline__ int deal_pair(int pos, int P)
{
    int x = 0;
    for (; x < 7; ++x) {
        const int n = (P - x + 7) / 8;  // pairs with index = x (mod 8)
        if (pos < n) break;
        pos -= n;
    }
    return x + 8 * pos;
}

// The pair that a masked batch's position `pos` of the contiguous order works on: the batch
// elements are ranked by descending chain length (kvlen; ties by index), their pairs listed in
// that order and dealt to the XCDs with deal_pair(), so that every XCD starts with its longest
// chains and ends with its shortest (a workgroup's run time is proportional to the length of its
// chain; the other way round the last, long workgroups run while most compute units are idle).
// Every lane of the wave calls it and gets the same answer.  More than 64 batch elements: no ranking.
__device__ __forceinline__ int dealt_pair_by_length(int pos, const int *kvlen, int B, int H, int lane)
{
    const int pi = deal_pair(pos, B * H);
    const int rb = pi / H, h = pi - rb * H;
    if (B > 64) return pi;
    const int mine = lane < B ? kvlen[lane] : -1;
    int rank = 0;
    for (int j = 0; j < B; ++j) {
        const int other = __builtin_amdgcn_readlane(mine, j);
        rank += (other > mine || (other == mine && j < lane)) ? 1 : 0;
    }
    const unsigned long long hit = __ballot(lane < B && rank == rb);
    const int b = __builtin_amdgcn_readfirstlane(__ffsll((long long)hit) - 1);
    return b * H + h;
}

// 16-byte groups per lane that one wave of one part leaves for the merge: 2 of scalars, 3 of
// point coordinates, 1 of (reference maximum, weight sum), 4 per 32-column block of the
// z1-contracted pair part (c_z / 32 blocks).
__host__ __device__ inline int attn_partial_groups(int cz) { return 6 + 4 * (cz / 32); }
constexpr int kMaxSplitUnits = 256;  // a split launch has at most this many part workgroups

struct Bf16Layout {
    int Lp, NT, DZ;
    SplitPlan plan;
    size_t cen, kvlen, Qh, Qz, Kh, Vh, Z2, kbias, qbias, Ohat, lse2, partial, counters, total;
};

// with_ohat: the unfused epilogue needs the lifted output O^ in memory.  with_qz: the per-head
// query-side factor vectors are wanted whatever the width (the gradient kernels stream them).
inline Bf16Layout bf16_layout(const fipa_desc &d, bool with_ohat, bool with_qz = false)
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
    // (per-head query-side factor vectors: only where the attention kernel does not form them itself,
    // i.e. the unfused path up to width 256, which the backward uses too)
    w.Qz = (with_ohat && w.DZ <= 256) || with_qz ? take(BH * w.Lp * (size_t)w.DZ * 2) : 0;
    w.Kh = take(BH * w.Lp * kDH * 2);
    w.Vh = take(BH * w.Lp * kDH * 2);
    w.Z2 = take((size_t)d.B * w.Lp * w.DZ * 2);
    w.kbias = take(BH * w.Lp * sizeof(float));
    w.qbias = take(BH * w.Lp * sizeof(float));
    w.lse2 = take(BH * w.Lp * sizeof(float));
    w.Ohat = with_ohat ? take(BH * w.Lp * (size_t)(kDH + w.DZ) * sizeof(float)) : 0;
    w.plan = attn_split_plan((int)(BH * (w.Lp / kTileQ)), w.Lp, w.DZ, d.cz, !with_ohat);
    // (sized for the largest split any length can give, so that the total stays affine in L)
    const bool can_split = !with_ohat && w.DZ <= 256 && d.cz >= 32;
    w.partial = can_split ? take((size_t)kMaxSplitUnits * 4 * attn_partial_groups(d.cz) * 64 * 16) : 0;
    w.counters = can_split ? take((size_t)kMaxSplitUnits * 4 * sizeof(int)) : 0;
    w.total = off;
    return w;
}

// The fused epilogue is compiled for the AlphaFold2-style head shape only.
inline bool bf16_fused_epilogue(const fipa_desc &d) { return d.c == 16 && d.Pv == 8 && d.r * d.cz <= 256; }
// The same for the two-window kernel of width r*cz = 512 (c_z such that half a factor slice is whole 32-column blocks).
bool attn_fwd_wide_fused_supported(int DZ, int cz);
inline bool bf16_wide_fused_epilogue(const fipa_desc &d)
{
    return d.c == 16 && d.Pv == 8 && attn_fwd_wide_fused_supported(d.r * d.cz, d.cz);
}

struct PackParams {
    const bf16_t *q, *k, *v, *q_pts, *k_pts, *v_pts, *z1, *z2;
    const float *rot, *trans, *w_b, *gamma, *cen;
    const uint8_t *mask;
    const int *cu;  // packed batch: row offsets of the chains (see user_row), else null
    bf16_t *Qh, *Qz, *Kh, *Vh, *Z2;
    float *kbias, *qbias;
    int B, L, Lp, NT, H, c, Pq, Pv, cz, r, DZ;
    float w_L, w_C, qk_scale;
    bool skip_qz;  // the attention kernel forms the query-side factor vectors itself
    // When cen_out is set, the AlphaFold2-shape pack kernel finds the per-batch reference point
    // and key-loop bound itself (no separate preparation launch), uses them, and leaves them
    // here for the attention kernel; it also clears `counters`.  `cen` is ignored then.
    float *cen_out;
    int *kvlen_out;
    int *counters;
    int n_counters;
};

struct AttnParams {
    const bf16_t *Qh, *Qz, *Kh, *Vh, *Z2;
    const float *kbias, *qbias;
    const int *kvlen;
    float *Ohat, *lse2;  // unfused epilogue only
    // fused epilogue: final outputs and what they need
    const float *rot, *trans, *cen, *w_b;
    const bf16_t *z1;
    const uint8_t *mask;
    const int *cu;  // packed batch: row offsets of the chains (see user_row), else null
    float *o, *o_pts, *o_pair, *lse;
    int B, L, Lp, H, NT, nQT, total_tiles, cz, r;
    int deal;  // set for masked batches: chain lengths come from kvlen, and the (batch, head) pairs are renumbered (see dealt_pair_by_length)
    float w_L;
    // key-range split (see SplitPlan): exchange buffer and one arrival counter per (split tile, wave)
    SplitPlan plan;
    float *partial;
    int *counters;
    // wave-specialised kernel: an address at or below Kh, Vh, Z2 and kbias, all of which lie less
    // than 4 GiB above it (the start of the workspace that holds them)
    const char *ws_base;
};

struct EpiParams {
    const float *Ohat, *lse2, *qbias, *rot, *trans, *cen;
    const bf16_t *z1;
    const uint8_t *mask;
    const int *cu;  // packed batch: row offsets of the chains (see user_row), else null
    float *o, *o_pts, *o_pair, *lse;
    int B, L, Lp, H, c, Pv, cz, r, DZ;
};

// ---- backward -----------------------------------------------------------------------------------
enum { FIPA_BWD_DQ = 0, FIPA_BWD_DK = 1, FIPA_BWD_DV = 2 };

struct BwdParams {
    const bf16_t *Qh, *Qz, *Kh, *Vh, *Z2, *dOhat;  // lifted tensors (dOhat: [B,H,Lp,64+DZ])
    const float *kbias;   // [B,H,Lp] per-key logit term (log2 units; -inf = masked)
    const float *nlse;    // [B,H,Lp] minus the log2 log-sum-exp of the kernel's logits (-inf = invalid query)
    const float *Dvec;    // [B,H,Lp] D_i = dO^_i . O^_i
    const int *kvlen;
    float *out;           // [B,H,Lp,64+DZ] dQ^ / dK^ / dV^
    float *wsum;          // [B,H,Lp] sum of the rounded dS over the streamed side, or NULL
    int B, L, Lp, H, total_tiles;
    int deal;     // set for masked batches: chain lengths come from kvlen, and the (batch, head) pairs are renumbered (see dealt_pair_by_length)
};

struct BwdPackParams {
    const float *d_o, *d_o_pts, *d_o_pair, *rot, *Ohat, *lse2;
    const bf16_t *z1;
    const uint8_t *mask;
    const int *cu;  // packed batch: row offsets of the chains (see user_row), else null
    bf16_t *dOhat;
    float *Dvec, *nlse;
    int B, L, Lp, H, c, Pv, cz, r, DZ;
};

struct BwdUnpackParams {
    const bf16_t *q_pts, *k_pts, *v_pts, *z1, *dOhat;
    const float *rot, *trans, *cen, *gamma, *w_b, *d_o_pair, *d_o_pts;
    const uint8_t *mask;
    const int *cu;  // packed batch: row offsets of the chains (see user_row), else null
    const float *dQhat, *dKhat, *dVhat, *Ohat, *rowsum, *colsum;
    bf16_t *d_q, *d_k, *d_v, *d_q_pts, *d_k_pts, *d_v_pts, *d_z1, *d_z2;
    float *gpart;   // [B,H,Lp] per-(b,h,i) contribution to d gamma
    float *d_gamma; // [H]
    float *d_w_b;   // [H, cz] or null
    float *d_rot, *d_trans;  // [B, L, 3, 3], [B, L, 3] or null
    float *wpart;   // [H, ceil(B*L/32), DZ] partial sums of d w_b
    int B, L, Lp, H, c, Pq, Pv, cz, r, DZ;
    int total_rows;  // rows of the caller's tensors: B L, or the total of a packed batch
    float w_L, w_C, qk_scale;
};

hipError_t launch_bwd_bf16(const BwdParams &p, int DZ, int mode, hipStream_t stream);
hipError_t launch_bwd_pack_bf16(const BwdPackParams &p, hipStream_t stream);
hipError_t launch_bwd_unpack_bf16(const BwdUnpackParams &p, hipStream_t stream);

hipError_t launch_pack_bf16(const PackParams &p, hipStream_t stream);
hipError_t launch_attn_fwd_bf16(const AttnParams &p, int DZ, bool fused, hipStream_t stream);
bool attn_fwd_ws_supported(int DZ, int cz);  // shapes of the wave-specialised fused kernel
hipError_t launch_attn_fwd_ws_bf16(const AttnParams &p, int DZ, hipStream_t stream);
hipError_t launch_attn_fwd_wide_bf16(const AttnParams &p, int DZ, bool fused, hipStream_t stream);  // r*cz = 512
hipError_t launch_epilogue_bf16(const EpiParams &p, hipStream_t stream);

}  // namespace fipa
