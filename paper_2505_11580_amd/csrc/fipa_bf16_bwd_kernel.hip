// MFMA kernels of the backward pass on the lifted features.  The paper gives no backward; this
// is the chain rule through softmax(Q^ K^T) V^ (Algorithm 1 step 7) with the usual
// recomputation of the weights from the saved log-sum-exp (the scheme of Algorithm 2 run again):
//     P_ij  = exp2(S_ij - lse_i),        S = Q^ K^T + kbias   (log2 units)
//     dP_ij = dO^_i . V^_j,              dS_ij = P_ij (dP_ij - D_i),   D_i = dO^_i . O^_i
//     dQ^_i = sum_j dS_ij K^_j,   dK^_j = sum_i dS_ij Q^_i,   dV^_j = sum_i P_ij dO^_i.
//
// One kernel template serves the three accumulations.  A workgroup keeps 128 "stationary" rows
// (32 per wave, their lifted features as MFMA B fragments in registers) and streams blocks of
// 32 rows of the other side through LDS:
//     DQ: stationary = queries (Y1 = q^, Y2 = dO^), streamed = keys    (X1 = k^, X2 = v^),  acc += X1^T dS
//     DK: stationary = keys    (Y1 = k^, Y2 = v^),  streamed = queries (X1 = q^, X2 = dO^), acc += X1^T dS
//     DV: stationary = keys    (Y1 = k^),           streamed = queries (X1 = q^, X2 = dO^), acc += X2^T P
// Both small products are formed transposed (streamed row = MFMA row, stationary row = lane), so
// the per-stationary-row scalars are per-lane values and the weights are already laid out as the
// B operand of the accumulating MFMA, whose A operand is read from the row-major streamed tile
// with the transposing LDS read.
//
// The streamed blocks arrive in a ring of three LDS stages by direct global -> LDS loads issued
// one block ahead; one barrier per block publishes the new stage and releases the oldest.
//
// Lifted width 576 (r*c_z = 512): the two sets of stationary fragments take 288 registers per lane,
// so a workgroup accumulates one of three windows of 192 output columns (template parameters NWIN,
// WIN; DV, with one set of fragments, one of two windows of 288) and the small products are formed once
// per window; a streamed block of queries (q^ and dO^,
// 78 KB) fits LDS twice only, so DK and DV run without the pipeline across blocks (everything of
// block n while block n+1 loads).  Plain forms that make the shape trainable; not tuned.
#include "fipa_gfx950.h"

namespace fipa {

namespace {

constexpr int kSB = 32;              // streamed rows per block
constexpr int kHS = kDH * 2 + 16;    // LDS row stride (bytes) of a 64-column head-specific tile

template <int DZ, int MODE, int NWIN = 1, int WIN = 0>
struct BwdCfg {
    static constexpr int D = kDH + DZ;           // lifted width
    static constexpr int KS = D / 16;            // k-steps of the small products
    static constexpr int KSH = kDH / 16;
    static constexpr int NB = D / 32;            // 32-row blocks of the accumulator
    static constexpr int NBH = kDH / 32;
    static_assert(NB % NWIN == 0, "windows must tile the output columns");
    static constexpr int NBW = NB / NWIN;        // blocks this workgroup accumulates: WIN * NBW .. + NBW - 1
    static constexpr int ZS = DZ * 2 + 48;       // LDS row stride of a pair-part tile: conflict free for row reads and transposing reads
    static constexpr int Z_SPR = ZS / 16, H_SPR = kHS / 16;   // 16-byte slots per row
    static constexpr int NZ = (kSB * Z_SPR + 63) / 64;         // wave-wide 1 KiB loads per pair-part tile
    static constexpr int NH = (kSB * H_SPR + 63) / 64;         // per head-part tile
    // DQ streams k^ and v^, whose pair parts are the same z2 rows: one copy serves both
    static constexpr bool kSharedZ = MODE == FIPA_BWD_DQ;
    // flat list of the wave-wide loads of one block: X1 pair | X1 head | X2 pair (unless shared) | X2 head
    static constexpr int X1Z_OFF = 0;
    static constexpr int X1H_OFF = NZ * 1024;
    static constexpr int X2Z_OFF = kSharedZ ? X1Z_OFF : (NZ + NH) * 1024;
    static constexpr int X2H_OFF = kSharedZ ? (NZ + NH) * 1024 : (2 * NZ + NH) * 1024;
    static constexpr int NI = (kSharedZ ? NZ : 2 * NZ) + 2 * NH;
    static constexpr int NIW = (NI + 3) / 4;     // per wave
    static constexpr int NSC = MODE == FIPA_BWD_DK ? 2 : 1;   // per-streamed-row scalars: logit term (+ D for DK)
    // Three stages where they fit.  Otherwise two, without the spare KiB for the surplus entries of
    // the last round of loads (the waves that would issue them skip them; every wait in this kernel
    // is for all outstanding loads, so the waves need not issue the same number).
    static constexpr bool PIPELINED = 3 * (NIW * 4 * 1024 + 2 * 1024) <= 160 * 1024;
    static constexpr bool kSkipSurplus = !PIPELINED;
    static constexpr int SC_OFF = (PIPELINED ? NIW * 4 : NI) * 1024;   // each scalar load covers 1 KiB (its first 128 bytes are data)
    static constexpr int STAGE = SC_OFF + 2 * 1024;
    static constexpr int NSTAGE = PIPELINED ? 3 : 2;
    static constexpr int LDS_BYTES = NSTAGE * STAGE;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static constexpr int VM_PER_BLOCK = NIW + NSC;             // vector-memory ops one wave issues per block
};

// The direct loads of one wave (see dma16): wave w issues entries w, w+4, ... of the flat list;
// surplus entries repeat entry 0 into the spare KiB the stage keeps for them.  Lanes whose slot
// lies in the row padding or past the last row fetch element 0 of the tile again (harmless).
template <class C>
struct BwdDma {
    const char *src[C::NIW + C::NSC];  // wave-uniform
    int step[C::NIW + C::NSC];         // wave-uniform: bytes from one block to the next
    int voff[C::NIW + C::NSC];         // per lane: byte offset of the previously requested block
    unsigned wave_lds;
    int wave;                          // wave-uniform
};

// Entry K of the loads of a block.  (Entry wave + 4 K of the flat list; past its end: a surplus entry.)
template <class C, int K>
__device__ __forceinline__ void bwd_issue_one(BwdDma<C> &d, unsigned stage)
{
    if constexpr (K < C::NIW) {
        if (C::kSkipSurplus && d.wave + 4 * K >= C::NI) return;
        dma16<4096 * K>(d.src[K], d.voff[K], d.step[K], stage + d.wave_lds);
    } else {
        dma16<C::SC_OFF + 1024 * (K - C::NIW)>(d.src[K], d.voff[K], d.step[K], stage);
    }
}

template <class C, int K = 0>
__device__ __forceinline__ void bwd_issue_block(BwdDma<C> &d, unsigned stage)
{
    if constexpr (K < C::NIW + C::NSC) {
        bwd_issue_one<C, K>(d, stage);
        bwd_issue_block<C, K + 1>(d, stage);
    }
}

// Entry k of the loads of a block (k is a compile-time constant after unrolling).
template <class C, int K = 0>
__device__ __forceinline__ void bwd_issue_entry(BwdDma<C> &d, unsigned stage, int k)
{
    if constexpr (K < C::NIW + C::NSC) {
        if (k == K)
            bwd_issue_one<C, K>(d, stage);
        else
            bwd_issue_entry<C, K + 1>(d, stage, k);
    }
}

struct BwdLane {
    int ka_h, ka_z, va_h, va_z, g;  // per-lane LDS offsets inside a stage, lane half
    float slane, dlane;             // per-stationary-row logit term and D
};

// The MFMAs of a steady step in issue order: per k-step the small products S (and dP) of the
// current block followed by its share of the first KS - kTail accumulation MFMAs of the previous
// block; then the held-back kTail accumulation MFMAs, which are issued among the exponentials of
// the new weights.  kind: 0 = S, 1 = dP, 2 = accumulation; idx: k-step, or accumulation number.
template <class C, int MODE>
struct BwdOps {
    static constexpr bool kNeedDP = MODE != FIPA_BWD_DV;
    static constexpr int KS = C::KS;
    static constexpr int NACC = 2 * C::NBW;  // accumulation MFMAs of a block (= KS when there is one window)
    static constexpr int kTail = NACC >= 16 ? 8 : NACC / 2;  // (8, 12 and 16 measured: 1.96, 2.00, 2.00 ms of gradient kernels at L = 4096)
    static constexpr int kInLoop = NACC - kTail;
    static constexpr int NL = (kNeedDP ? 2 : 1) * KS + kInLoop;  // before the weights
    static constexpr int NT = NL + kTail;
    struct Op {
        int kind, idx;
    };
    static constexpr Op op(int j)
    {
        int n = 0;
        for (int ks = 0; ks < KS; ++ks) {
            if (n == j) return {0, ks};
            ++n;
            if (kNeedDP) {
                if (n == j) return {1, ks};
                ++n;
            }
            for (int a = ks * kInLoop / KS; a < (ks + 1) * kInLoop / KS; ++a) {
                if (n == j) return {2, a};
                ++n;
            }
        }
        return {2, kInLoop + (j - NL)};
    }
    // first tail operation of weight pair t (t = 0..7), relative to NL
    static constexpr int tail_begin(int t) { return t * kTail / 8; }
};

// Steady step (current and previous block both present) with a fixed instruction order: the LDS
// operand of every MFMA is requested kLA MFMAs ahead, in order of use, into a small ring; one
// load entry of the next block goes out per k-step; the weights of the current block are formed
// pair by pair between the held-back accumulation MFMAs.
template <class C, int MODE, int WIN>
__device__ __forceinline__ void bwd_step_steady(const char *__restrict__ st, const char *__restrict__ st_prev, const BwdLane &ln,
                                                const bf16x8 (&y1f)[C::KS],
                                                const bf16x8 (&y2f)[MODE != FIPA_BWD_DV ? C::KS : 1],
                                                f32x16 (&acc)[C::NBW], bf16x8 (&wf)[2], float &wsum,
                                                BwdDma<C> &dma, unsigned next_stage)
{
    using O = BwdOps<C, MODE>;
    constexpr bool kNeedDP = MODE != FIPA_BWD_DV;
    constexpr int AZ_OFF = MODE == FIPA_BWD_DV ? C::X2Z_OFF : C::X1Z_OFF;
    constexpr int AH_OFF = MODE == FIPA_BWD_DV ? C::X2H_OFF : C::X1H_OFF;
    constexpr int kEntries = C::NIW + C::NSC;
    constexpr int kLA = 3, kRing = 4;
    // The load entries of the next block go out with the first kDmaSteps k-steps.  The block has
    // to have landed when the next step begins (three stages: one block of lead), so entries
    // issued late in the step are waited for; spread over all k-steps the last ones were.  In the
    // first quarter: dV^ -6 %, dQ^ -2 %; dK^, whose step is the longest, is 4 % slower that way
    // and keeps the even spread.
    constexpr int kDmaSteps = MODE == FIPA_BWD_DK ? C::KS : (C::KS >= 4 ? C::KS / 4 : 1);
    auto fetch = [&](auto J) -> bf16x8 {
        constexpr auto o = O::op(decltype(J)::value);
        if constexpr (o.kind == 0) {
            const int ks = o.idx;
            const char *s1 = ks < C::KSH ? st + C::X1H_OFF + ln.ka_h + ks * 32 : st + C::X1Z_OFF + ln.ka_z + (ks - C::KSH) * 32;
            return *reinterpret_cast<const bf16x8 *>(s1);
        } else if constexpr (o.kind == 1) {
            const int ks = o.idx;
            const char *s2 = ks < C::KSH ? st + C::X2H_OFF + ln.ka_h + ks * 32 : st + C::X2Z_OFF + ln.ka_z + (ks - C::KSH) * 32;
            return *reinterpret_cast<const bf16x8 *>(s2);
        } else {
            const int nb = WIN * C::NBW + (o.idx >> 1), tt = o.idx & 1;  // block of the whole lifted row
            const char *src = nb < C::NBH ? st_prev + AH_OFF + ln.va_h + 16 * tt * kHS + nb * 64
                                          : st_prev + AZ_OFF + ln.va_z + 16 * tt * C::ZS + (nb - C::NBH) * 64;
            const int rs = nb < C::NBH ? kHS : C::ZS;
            const bf16x4 lo = lds_read_tr(src);
            const bf16x4 hi = lds_read_tr(src + 8 * rs);
            bf16x8 av;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                av[x] = lo[x];
                av[4 + x] = hi[x];
            }
            return av;
        }
    };
    f32x16 sacc, dpacc;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const f32x4 sb = *reinterpret_cast<const f32x4 *>(st + C::SC_OFF + (8 * a + 4 * ln.g) * 4);
#pragma unroll
        for (int x = 0; x < 4; ++x) sacc[4 * a + x] = sb[x] + ln.slane;
        if constexpr (C::NSC == 2) {
            const f32x4 db = *reinterpret_cast<const f32x4 *>(st + C::SC_OFF + 1024 + (8 * a + 4 * ln.g) * 4);
#pragma unroll
            for (int x = 0; x < 4; ++x) dpacc[4 * a + x] = -(db[x] + ln.dlane);
        } else {
#pragma unroll
            for (int x = 0; x < 4; ++x) dpacc[4 * a + x] = -ln.dlane;
        }
    }
    bf16x8 fr[kRing];
    static_for<kLA>([&](auto J) { fr[decltype(J)::value] = fetch(J); });
    unsigned wp[8];
    static_for<O::NT>([&](auto J) {
        constexpr int j = decltype(J)::value;
        if constexpr (j + kLA < O::NT) fr[(j + kLA) % kRing] = fetch(std::integral_constant<int, j + kLA>{});
        constexpr auto o = O::op(j);
        // the weights of pair t, just before the first held-back MFMA of its group
        if constexpr (j >= O::NL) {
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                if (O::NL + O::tail_begin(t) != j) continue;
                // (several pairs fall on one MFMA when there are fewer held-back MFMAs than pairs)
                float w0 = __builtin_amdgcn_exp2f(sacc[2 * t]), w1 = __builtin_amdgcn_exp2f(sacc[2 * t + 1]);
                if constexpr (kNeedDP) {
                    w0 *= dpacc[2 * t];
                    w1 *= dpacc[2 * t + 1];
                }
                wp[t] = pack_pair(w0, w1, wsum);
            }
        }
        if constexpr (o.kind == 0) {
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % kRing], y1f[o.idx], sacc, 0, 0, 0);
            if (next_stage != 0xFFFFFFFFu) {
#pragma unroll
                for (int e = o.idx * kEntries / kDmaSteps; e < (o.idx + 1) * kEntries / kDmaSteps; ++e)
                    if (e < kEntries) bwd_issue_entry<C>(dma, next_stage, e);
            }
        } else if constexpr (o.kind == 1) {
            dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % kRing], y2f[kNeedDP ? o.idx : 0], dpacc, 0, 0, 0);
        } else {
            acc[o.idx >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % kRing], wf[o.idx & 1], acc[o.idx >> 1], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    });
    wf[0] = __builtin_bit_cast(bf16x8, (u32x4){wp[0], wp[1], wp[2], wp[3]});
    wf[1] = __builtin_bit_cast(bf16x8, (u32x4){wp[4], wp[5], wp[6], wp[7]});
}

// First and last step of the pipeline: the small products and the weights of the block in stage
// `st` (CUR: the first block, nothing to accumulate yet) or the accumulation of the last block
// (PREV: stage `st_prev`, weights `wf`).  On exit of a CUR step `wf` holds the block's weights.
// The loads of the next block (stage `next_stage`) are issued spread over the k-steps.
template <class C, int MODE, int WIN, bool CUR, bool PREV>
__device__ __forceinline__ void bwd_step(const char *__restrict__ st, const char *__restrict__ st_prev, const BwdLane &ln,
                                         const bf16x8 (&y1f)[C::KS],
                                         const bf16x8 (&y2f)[MODE != FIPA_BWD_DV ? C::KS : 1],
                                         f32x16 (&acc)[C::NBW], bf16x8 (&wf)[2], float &wsum,
                                         BwdDma<C> &dma, unsigned next_stage)
{
    static_assert(CUR != PREV, "the steady step is bwd_step_steady");
    constexpr bool kNeedDP = MODE != FIPA_BWD_DV;
    constexpr int AZ_OFF = MODE == FIPA_BWD_DV ? C::X2Z_OFF : C::X1Z_OFF;  // tile the accumulation reads
    constexpr int AH_OFF = MODE == FIPA_BWD_DV ? C::X2H_OFF : C::X1H_OFF;
    constexpr int kEntries = C::NIW + C::NSC;  // load entries of a block
    if constexpr (CUR) {
        f32x16 sacc, dpacc;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const f32x4 sb = *reinterpret_cast<const f32x4 *>(st + C::SC_OFF + (8 * a + 4 * ln.g) * 4);
#pragma unroll
            for (int x = 0; x < 4; ++x) sacc[4 * a + x] = sb[x] + ln.slane;
            if constexpr (C::NSC == 2) {
                const f32x4 db = *reinterpret_cast<const f32x4 *>(st + C::SC_OFF + 1024 + (8 * a + 4 * ln.g) * 4);
#pragma unroll
                for (int x = 0; x < 4; ++x) dpacc[4 * a + x] = -(db[x] + ln.dlane);
            } else {
#pragma unroll
                for (int x = 0; x < 4; ++x) dpacc[4 * a + x] = -ln.dlane;
            }
        }
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            // S (and dP) of the current block: [32 streamed rows] x [32 stationary rows (lanes)]
            const char *s1 = ks < C::KSH ? st + C::X1H_OFF + ln.ka_h + ks * 32 : st + C::X1Z_OFF + ln.ka_z + (ks - C::KSH) * 32;
            const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(s1);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, y1f[ks], sacc, 0, 0, 0);
            if constexpr (kNeedDP) {
                const char *s2 = ks < C::KSH ? st + C::X2H_OFF + ln.ka_h + ks * 32 : st + C::X2Z_OFF + ln.ka_z + (ks - C::KSH) * 32;
                const bf16x8 a2 = *reinterpret_cast<const bf16x8 *>(s2);
                dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, y2f[ks], dpacc, 0, 0, 0);
            }
            if (next_stage != 0xFFFFFFFFu) {
#pragma unroll
                for (int e = ks * kEntries / C::KS; e < (ks + 1) * kEntries / C::KS; ++e)
                    bwd_issue_entry<C>(dma, next_stage, e);
            }
        }
        // weights of the accumulating product: P (DV) or dS = P (dP - D) (DQ, DK)
        unsigned wp[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            float w0 = __builtin_amdgcn_exp2f(sacc[r]), w1 = __builtin_amdgcn_exp2f(sacc[r + 1]);
            if constexpr (kNeedDP) {
                w0 *= dpacc[r];
                w1 *= dpacc[r + 1];
            }
            wp[r >> 1] = pack_pair(w0, w1, wsum);
        }
        wf[0] = __builtin_bit_cast(bf16x8, (u32x4){wp[0], wp[1], wp[2], wp[3]});
        wf[1] = __builtin_bit_cast(bf16x8, (u32x4){wp[4], wp[5], wp[6], wp[7]});
    }
    if constexpr (PREV) {
#pragma unroll
        for (int i = 0; i < 2 * C::NBW; ++i) {
            // acc^T[feature, stationary row] += X^T[feature, streamed row] W[streamed row, stationary row]
            const int nb = WIN * C::NBW + (i >> 1), tt = i & 1;  // block of the whole lifted row
            const char *src = nb < C::NBH ? st_prev + AH_OFF + ln.va_h + 16 * tt * kHS + nb * 64
                                          : st_prev + AZ_OFF + ln.va_z + 16 * tt * C::ZS + (nb - C::NBH) * 64;
            const int rs = nb < C::NBH ? kHS : C::ZS;
            const bf16x4 lo = lds_read_tr(src);
            const bf16x4 hi = lds_read_tr(src + 8 * rs);
            bf16x8 a;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                a[x] = lo[x];
                a[4 + x] = hi[x];
            }
            acc[i >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, wf[tt], acc[i >> 1], 0, 0, 0);
        }
    }
}

// One window (of NWIN) of the output columns of one tile of stationary rows.
template <int DZ, int MODE, int NWIN, int WIN>
__device__ __forceinline__ void bwd_window(const BwdParams &p, char *smem, int logical)
{
    using C = BwdCfg<DZ, MODE, NWIN, WIN>;
    constexpr bool kNeedDP = MODE != FIPA_BWD_DV;
    const int nT = p.Lp / kTileQ;
    const int bh_pos = logical / nT, tile = logical - bh_pos * nT;
    const int bh = p.deal ? dealt_pair_by_length(bh_pos, p.kvlen, p.B, p.H, threadIdx.x & 63) : bh_pos;
    const int b = bh / p.H;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, g = lane >> 5;
    const int kvlen = p.deal ? p.kvlen[b] : p.L;  // (no mask: every chain has L residues)
    const int nblk = (kvlen + kSB - 1) / kSB;       // streamed blocks: residues past the last valid one contribute nothing
    const int srow = tile * kTileQ + wave * 32 + li;  // stationary row of this lane, < Lp

    // Stationary rows past the last valid residue of the chain (padding of a ragged batch) take
    // part in nothing: zero gradient.
    if (tile * kTileQ >= kvlen) {
        float *orow = p.out + ((size_t)bh * p.Lp + srow) * C::D + 32 * WIN * C::NBW;
#pragma unroll
        for (int nb = 0; nb < C::NBW; ++nb)
#pragma unroll
            for (int a = 0; a < 4; ++a)
                *reinterpret_cast<f32x4 *>(orow + 32 * nb + 8 * a + 4 * g) = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (WIN == 0 && p.wsum && g == 0) p.wsum[(size_t)bh * p.Lp + srow] = 0.f;
        return;
    }

    // streamed tiles (row 0 of block 0, row pitch in bytes) and stationary sources, by mode
    const bf16_t *Qh = p.Qh + (size_t)bh * p.Lp * kDH, *Qz = p.Qz + (size_t)bh * p.Lp * DZ;
    const bf16_t *Kh = p.Kh + (size_t)bh * p.Lp * kDH, *Vh = p.Vh + (size_t)bh * p.Lp * kDH;
    const bf16_t *Z2 = p.Z2 + (size_t)b * p.Lp * DZ;
    const bf16_t *dO = p.dOhat + (size_t)bh * p.Lp * C::D;
    const bf16_t *x1z, *x1h, *x2z, *x2h, *y1h, *y1z, *y2h, *y2z;
    int x1zp, x1hp, x2zp, x2hp, y1hp, y1zp, y2hp, y2zp;  // row pitches in elements
    const float *srow_src, *slane_src, *drow_src = nullptr, *dlane_src = nullptr;
    if (MODE == FIPA_BWD_DQ) {
        x1h = Kh; x1hp = kDH; x1z = Z2; x1zp = DZ; x2h = Vh; x2hp = kDH; x2z = Z2; x2zp = DZ;
        y1h = Qh; y1hp = kDH; y1z = Qz; y1zp = DZ; y2h = dO; y2hp = C::D; y2z = dO + kDH; y2zp = C::D;
        srow_src = p.kbias + (size_t)bh * p.Lp;
        slane_src = p.nlse + (size_t)bh * p.Lp;
        dlane_src = p.Dvec + (size_t)bh * p.Lp;
    } else {
        x1h = Qh; x1hp = kDH; x1z = Qz; x1zp = DZ; x2h = dO; x2hp = C::D; x2z = dO + kDH; x2zp = C::D;
        y1h = Kh; y1hp = kDH; y1z = Z2; y1zp = DZ; y2h = Vh; y2hp = kDH; y2z = Z2; y2zp = DZ;
        srow_src = p.nlse + (size_t)bh * p.Lp;
        slane_src = p.kbias + (size_t)bh * p.Lp;
        drow_src = p.Dvec + (size_t)bh * p.Lp;
    }

    // ---- direct global -> LDS loads of the streamed blocks -------------------------------------
    BwdDma<C> dma;
    dma.wave_lds = 1024u * wave;
    dma.wave = wave;
#pragma unroll
    for (int k = 0; k < C::NIW; ++k) {
        int i = wave + 4 * k;
        if (i >= C::NI) i = 0;
        // region of flat entry i
        const int r1 = C::NZ, r2 = C::NZ + C::NH, r3 = C::kSharedZ ? r2 : r2 + C::NZ;
        const bool is_z = i < r1 || (!C::kSharedZ && i >= r2 && i < r3);
        const bool is_x1 = i < r2;
        const int first = i < r1 ? 0 : (i < r2 ? r1 : (i < r3 ? r2 : r3));
        const bf16_t *base = is_x1 ? (is_z ? x1z : x1h) : (is_z ? x2z : x2h);
        const int pitch = 2 * (is_x1 ? (is_z ? x1zp : x1hp) : (is_z ? x2zp : x2hp));  // bytes
        const int spr = is_z ? C::Z_SPR : C::H_SPR;
        const int cols = is_z ? DZ / 8 : kDH / 8;  // 16-byte columns of a tile row
        const int s = 64 * (i - first) + lane;
        const int row = s / spr, col = s - row * spr;
        dma.src[k] = reinterpret_cast<const char *>(base);
        dma.step[k] = kSB * pitch;
        dma.voff[k] = ((row < kSB && col < cols) ? row * pitch + col * 16 : 0) - dma.step[k];
    }
    dma.src[C::NIW] = reinterpret_cast<const char *>(srow_src);
    dma.step[C::NIW] = kSB * 4;
    dma.voff[C::NIW] = min(lane, 7) * 16 - dma.step[C::NIW];
    if constexpr (C::NSC == 2) {
        dma.src[C::NIW + 1] = reinterpret_cast<const char *>(drow_src);
        dma.step[C::NIW + 1] = kSB * 4;
        dma.voff[C::NIW + 1] = min(lane, 7) * 16 - dma.step[C::NIW + 1];
    }
    const unsigned smem_lds = lds_address(smem);
    if (nblk > 0) bwd_issue_block<C>(dma, smem_lds);

    // stationary fragments: features 16*ks + 8*g .. +7 of row srow
    bf16x8 y1f[C::KS], y2f[kNeedDP ? C::KS : 1];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        const bf16_t *s1 = ks < C::KSH ? y1h + (size_t)srow * y1hp + ks * 16 + 8 * g
                                       : y1z + (size_t)srow * y1zp + (ks - C::KSH) * 16 + 8 * g;
        y1f[ks] = *reinterpret_cast<const bf16x8 *>(s1);
        if (kNeedDP) {
            const bf16_t *s2 = ks < C::KSH ? y2h + (size_t)srow * y2hp + ks * 16 + 8 * g
                                           : y2z + (size_t)srow * y2zp + (ks - C::KSH) * 16 + 8 * g;
            y2f[ks] = *reinterpret_cast<const bf16x8 *>(s2);
        }
    }
    // The stationary fragments go to accumulation registers, from where the MFMAs read their B
    // operand directly; the accumulators and the small products, which the vector ALU works on,
    // are left to the register allocator (this file is compiled with the MFMA results in the
    // general vector-register class: see build.py).
    // (At width 576 the two sets are 288 registers: 64 fragments fill the accumulation registers.)
    constexpr int kPin2 = !kNeedDP ? 0 : (2 * C::KS <= 64 ? C::KS : 64 - C::KS);
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        asm volatile("" : "+a"(y1f[ks]));
        if (ks < kPin2) asm volatile("" : "+a"(y2f[ks]));
    }
    const float slane = slane_src[srow];
    const float dlane = dlane_src ? dlane_src[srow] : 0.f;

    f32x16 acc[C::NBW];
#pragma unroll
    for (int nb = 0; nb < C::NBW; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[nb][r] = 0.f;
    float wsum = 0.f;  // sum over streamed rows of the rounded dS (DQ: row sums, DK: column sums)

    // per-lane LDS offsets inside a stage
    const int l16 = lane & 15, grp2 = (lane >> 4) & 1, e4 = l16 >> 2, j4 = l16 & 3;
    const int ka_h = li * kHS + g * 16, ka_z = li * C::ZS + g * 16;                    // row reads (small products)
    const int va_h = (4 * g + e4) * kHS + (16 * grp2 + 4 * j4) * 2;                     // transposing reads
    const int va_z = (4 * g + e4) * C::ZS + (16 * grp2 + 4 * j4) * 2;

    // Software pipeline over the streamed blocks: iteration n forms the small products S and dP
    // of block n and, interleaved with them, accumulates block n-1 with the weights computed
    // one iteration earlier -- two independent streams of MFMAs, so the matrix pipe does not
    // wait on either's operands; the last accumulation MFMAs are held back and run while the
    // weights of block n are formed.  Blocks n-1 and n are resident, block n+1 is on its way
    // into the third stage.
    bf16x8 wf[2] = {};         // weights of the previous block (B operands of the accumulation)
    BwdLane ln;
    ln.ka_h = ka_h; ln.ka_z = ka_z; ln.va_h = va_h; ln.va_z = va_z; ln.g = g; ln.slane = slane; ln.dlane = dlane;
    int sidx = 0;              // stage of block n
    const char *st_prev = smem;
    for (int n = 0; n < nblk; ++n) {
        const char *st = smem + sidx * C::STAGE;
        // block n must have landed; the barrier also tells everyone that the stage of block n-2
        // is free again
        wait_vmem<0>();
        wg_barrier();
        sidx = sidx + 1 < C::NSTAGE ? sidx + 1 : 0;
        // (0xFFFFFFFF: no next block)
        const unsigned next_stage = n + 1 < nblk ? smem_lds + sidx * C::STAGE : 0xFFFFFFFFu;
        if constexpr (C::PIPELINED) {
            if (n == 0)
                bwd_step<C, MODE, WIN, true, false>(st, st_prev, ln, y1f, y2f, acc, wf, wsum, dma, next_stage);
            else
                bwd_step_steady<C, MODE, WIN>(st, st_prev, ln, y1f, y2f, acc, wf, wsum, dma, next_stage);
        } else {
            // two stages: everything of block n now, while block n+1 loads into the other stage
            bwd_step<C, MODE, WIN, true, false>(st, st, ln, y1f, y2f, acc, wf, wsum, dma, next_stage);
            bwd_step<C, MODE, WIN, false, true>(st, st, ln, y1f, y2f, acc, wf, wsum, dma, 0xFFFFFFFFu);
        }
        st_prev = st;
    }
    if (C::PIPELINED && nblk > 0)
        bwd_step<C, MODE, WIN, false, true>(st_prev, st_prev, ln, y1f, y2f, acc, wf, wsum, dma, 0xFFFFFFFFu);

    // ---- write acc^T: row srow, columns 32*nb + 8*(r/4) + 4*g + r%4 -------------------------------
    float *orow = p.out + ((size_t)bh * p.Lp + srow) * C::D + 32 * WIN * C::NBW;
#pragma unroll
    for (int nb = 0; nb < C::NBW; ++nb)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            f32x4 out;
#pragma unroll
            for (int x = 0; x < 4; ++x) out[x] = acc[nb][4 * a + x];
            *reinterpret_cast<f32x4 *>(orow + 32 * nb + 8 * a + 4 * g) = out;
        }
    if (WIN == 0 && p.wsum) {  // (every window forms the same sums)
        const float tot = wsum + __shfl_xor(wsum, 32);
        if (g == 0) p.wsum[(size_t)bh * p.Lp + srow] = tot;
    }
}

template <int DZ, int MODE, int NWIN>
__global__ __launch_bounds__(256, 1) void fipa_bwd_kernel(BwdParams p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // each XCD gets a contiguous run of tiles; the windows of a tile are neighbours in its launch order
    const int chunk = (p.total_tiles + 7) / 8;
    const int slot = blockIdx.x / 8;
    const int logical = (blockIdx.x % 8) * chunk + slot / NWIN;
    if (logical >= p.total_tiles) return;
    if constexpr (NWIN == 1) {
        bwd_window<DZ, MODE, 1, 0>(p, smem, logical);
    } else {
        static_assert(NWIN == 2 || NWIN == 3, "window dispatch");
        const int win = slot % NWIN;
        if (win == 0)
            bwd_window<DZ, MODE, NWIN, 0>(p, smem, logical);
        else if (NWIN == 2 || win == 1)
            bwd_window<DZ, MODE, NWIN, 1>(p, smem, logical);
        else if constexpr (NWIN == 3)
            bwd_window<DZ, MODE, NWIN, 2>(p, smem, logical);
    }
}

template <int DZ, int MODE>
hipError_t launch(const BwdParams &p, hipStream_t stream)
{
    // (DV keeps one set of stationary fragments: half of the output columns fit beside it)
    constexpr int NWIN = DZ > 256 ? (MODE == FIPA_BWD_DV ? 2 : 3) : 1;
    using C = BwdCfg<DZ, MODE, NWIN, 0>;
    static LdsLimit lds_limit;
    hipError_t e = raise_lds_limit(lds_limit, (const void *)fipa_bwd_kernel<DZ, MODE, NWIN>, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int chunk = (p.total_tiles + 7) / 8;
    hipLaunchKernelGGL((fipa_bwd_kernel<DZ, MODE, NWIN>), dim3(chunk * 8 * NWIN), dim3(256), C::LDS_BYTES, stream, p);
    return hipGetLastError();
}

template <int DZ>
hipError_t launch_mode(const BwdParams &p, int mode, hipStream_t stream)
{
    switch (mode) {
        case FIPA_BWD_DQ: return launch<DZ, FIPA_BWD_DQ>(p, stream);
        case FIPA_BWD_DK: return launch<DZ, FIPA_BWD_DK>(p, stream);
        case FIPA_BWD_DV: return launch<DZ, FIPA_BWD_DV>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_bwd_bf16(const BwdParams &p, int DZ, int mode, hipStream_t stream)
{
    switch (DZ) {
        case 32: return launch_mode<32>(p, mode, stream);
        case 64: return launch_mode<64>(p, mode, stream);
        case 128: return launch_mode<128>(p, mode, stream);
        case 256: return launch_mode<256>(p, mode, stream);
        case 512: return launch_mode<512>(p, mode, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fipa
