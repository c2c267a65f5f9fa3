// Fused attention on the lifted features (Algorithm 1 step 7) for wide pair factors (r*c_z = 512,
// lifted width 576; and r*c_z = 1024, width 1088, see the end of this comment): same mathematics and
// register layout as the main kernel, but the output
// accumulator of 32 x 576 fp32 per wave does not fit the register file, so the value columns are
// cut into windows and each workgroup computes one window (recomputing S^T and the softmax).
// Key blocks of 32 residues arrive in a ring of three LDS stages by direct global -> LDS loads
// issued one block ahead (the z2 block is stored once and read in both roles, as in the main
// kernel).  The loop is software pipelined over two blocks: iteration n forms S^T of block n and,
// interleaved with it, accumulates P V of block n-1; the softmax of block n (running maximum of
// Algorithm 2, raised lazily) follows.
// Two ways of cutting the columns into the two windows (template parameter CZ of WideCfg):
//   CZ = 0   the lifted columns in their natural order, 288 each; the windows write the lifted
//            output O^ and a separate kernel runs steps 8-9 (any head shape, any c_z);
//   CZ = c_z window 0 takes the head-specific columns and, of every factor slice rho, the pair columns
//            d < c_z/2; window 1 the pair columns d >= c_z/2.  Every output of steps 8-9 then
//            depends on one window only -- o, o_pts and o_pair[d < c_z/2] on window 0,
//            o_pair[d >= c_z/2] on window 1 (the contraction over rho of step 9 stays inside a
//            window) -- and the epilogue runs on the accumulator registers as in the main kernel:
//            no O^ in memory, no epilogue kernel.  AlphaFold2 head shape, c_z a multiple of 64.
// Width 1088 (rank 8 at c_z = 128; the larger head widths that Section 4.1 names as the way to higher
// rank): the query fragments alone take 272 registers per lane, which leaves room for a quarter of the
// output columns, so there are four natural-order windows (the 34 column blocks padded to 36, nine per
// window; S^T is formed four times), a key block is 77 KB and only two stages fit LDS, so the loop is
// not pipelined across blocks (S^T, softmax and P V of a block one after the other while the next block
// loads), and the epilogue is the separate kernel.  It makes the shape usable; it is not tuned.
#include "fipa_gfx950.h"

namespace fipa {

namespace {

constexpr int kKB = 32;              // keys per block
constexpr int kHS = kDH * 2 + 16;    // LDS row stride (bytes) of the head-specific k^ / v^ blocks
constexpr float kTauW = 8.f;

template <int DZ, int CZ, int NWIN, int WIN>
struct WideCfg {
    static constexpr bool FUSED = CZ > 0;
    static constexpr int D = kDH + DZ;
    static constexpr int KS = D / 16, KSH = kDH / 16;
    static constexpr int NB = D / 32, NBH = kDH / 32, NZB = DZ / 32;
    static_assert(!FUSED || (CZ % 64 == 0 && DZ % CZ == 0), "half a factor slice must be whole 32-column blocks");
    static_assert(!FUSED || NWIN == 2, "the slice-halving windows come in pairs");
    // 32-column blocks of this window (natural order: the last window may end in padding blocks,
    // col_block() >= NB, which are neither multiplied nor stored)
    static constexpr int NBW = FUSED ? (WIN == 0 ? NBH + NZB / 2 : NZB / 2) : (NB + NWIN - 1) / NWIN;
    static constexpr int HB = FUSED ? CZ / 64 : 1;   // blocks per half factor slice
    // Column block (0 .. NB-1 in the natural order; the first NBH are head-specific) that block nbw
    // of this window accumulates.
    static constexpr int col_block(int nbw)
    {
        if (!FUSED) return WIN * NBW + nbw;
        if (WIN == 0 && nbw < NBH) return nbw;
        const int t = WIN == 0 ? nbw - NBH : nbw;
        return NBH + (t / HB) * (CZ / 32) + WIN * HB + t % HB;
    }
    static constexpr int ZS = DZ * 2 + 48;       // LDS row stride of the z2 block (conflict free for both read patterns)
    static constexpr int Z_SPR = ZS / 16, H_SPR = kHS / 16;
    static constexpr int NZ = (kKB * Z_SPR + 63) / 64;   // wave-wide 1 KiB loads for the z2 block
    static constexpr int NH = (kKB * H_SPR + 63) / 64;   // for one head block
    static constexpr int NI = NZ + 2 * NH;               // flat list: z2 | k^ head | v^ head
    static constexpr int NIW = (NI + 3) / 4;             // per wave
    static constexpr int Z_OFF = 0, KH_OFF = NZ * 1024, VH_OFF = (NZ + NH) * 1024;
    static constexpr int KB_OFF = NIW * 4 * 1024;        // 32 per-key fp32 biases (a full 1 KiB load lands here)
    static constexpr int STAGE = KB_OFF + 1024;
    static constexpr int NSTAGE = STAGE * 3 + DZ * 4 <= 160 * 1024 ? 3 : 2;
    static constexpr bool PIPELINED = NSTAGE == 3;       // S^T of block n together with P V of block n-1
    static constexpr int CW_OFF = NSTAGE * STAGE;        // per-head scale vector of the query-side factors (DZ floats)
    static constexpr int LDS_BYTES = CW_OFF + DZ * 4;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

// The direct loads of one wave (see dma16): wave w issues entries w, w+4, ... of the flat list,
// then the bias entry; surplus entries repeat entry 0 into the spare KiB of the stage.
template <class C>
struct WideDma {
    const char *src[C::NIW + 1];
    int step[C::NIW + 1];
    int voff[C::NIW + 1];
    unsigned wave_lds;
};

template <class C, int K = 0>
__device__ __forceinline__ void wide_issue_block(WideDma<C> &d, unsigned stage)
{
    if constexpr (K < C::NIW) {
        dma16<4096 * K>(d.src[K], d.voff[K], d.step[K], stage + d.wave_lds);
        wide_issue_block<C, K + 1>(d, stage);
    } else if constexpr (K == C::NIW) {
        dma16<C::KB_OFF>(d.src[K], d.voff[K], d.step[K], stage);
    }
}

// Entry k of the loads of the next block (k is a compile-time constant after unrolling).
template <class C, int K = 0>
__device__ __forceinline__ void wide_issue_entry(WideDma<C> &d, unsigned stage, int k)
{
    if constexpr (K <= C::NIW) {
        if (k == K) {
            if constexpr (K < C::NIW)
                dma16<4096 * K>(d.src[K], d.voff[K], d.step[K], stage + d.wave_lds);
            else
                dma16<C::KB_OFF>(d.src[K], d.voff[K], d.step[K], stage);
        } else {
            wide_issue_entry<C, K + 1>(d, stage, k);
        }
    }
}

struct WideLane {
    int kaddr_h, kaddr_z, vaddr_h, vaddr_z, g;
};

// LDS operand of P V operation i (= 2 * window block + key half) from the stage at `st`: 32 v^ columns x 16 keys.
template <class C, int I>
__device__ __forceinline__ bf16x8 wide_load_pv(const char *__restrict__ st, const WideLane &ln)
{
    constexpr int nbw = I >> 1, tt = I & 1;
    constexpr int nb = C::col_block(nbw);
    constexpr bool head = nb < C::NBH;
    const char *src = head ? st + C::VH_OFF + ln.vaddr_h + 16 * tt * kHS + nb * 64
                           : st + C::Z_OFF + ln.vaddr_z + 16 * tt * C::ZS + (nb - C::NBH) * 64;
    constexpr int rs = head ? kHS : C::ZS;
    const bf16x4 lo = lds_read_tr(src);
    const bf16x4 hi = lds_read_tr(src + 8 * rs);
    bf16x8 a;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        a[x] = lo[x];
        a[4 + x] = hi[x];
    }
    return a;
}

// One step of the pipeline: S^T and the softmax of the block in stage `st` (CUR), interleaved
// with P V of the previous block (stage `st_prev`, probabilities `pf` on entry) (PREV).  On exit
// `pf` holds the probabilities of the current block.  When `load_next` is set the loads of the
// next block are issued between the MFMAs, one entry every few of them (issued back to back they
// cost about 60 cycles each).
template <class C, bool CUR, bool PREV>
__device__ __forceinline__ void wide_step(const char *__restrict__ st, const char *__restrict__ st_prev, const WideLane &ln,
                                          const bf16x8 (&qf)[C::KS], f32x16 (&acc)[C::NBW],
                                          bf16x8 (&pf)[2], float &m_run, float &l_run,
                                          WideDma<C> &dma, unsigned next_stage, bool load_next)
{
    constexpr int kDmaEvery = C::KS / (C::NIW + 1);
    static_assert(kDmaEvery >= 1, "more load entries than S^T MFMAs");
    f32x16 sacc;
    if constexpr (CUR) {
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const f32x4 bias = *reinterpret_cast<const f32x4 *>(st + C::KB_OFF + (8 * a + 4 * ln.g) * 4);
#pragma unroll
            for (int x = 0; x < 4; ++x) sacc[4 * a + x] = bias[x];
        }
        // (unrolled by recursion: at width 1088 the 68 steps are more than an unroll pragma will take, and
        // a loop that stays a loop indexes the fragments at run time, which moves them to scratch memory)
        static_for<C::KS>([&](auto I) {
            constexpr int ks = decltype(I)::value;
            const char *src = ks < C::KSH ? st + C::KH_OFF + ln.kaddr_h + ks * 32 : st + C::Z_OFF + ln.kaddr_z + (ks - C::KSH) * 32;
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(src);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sacc, 0, 0, 0);
            if (load_next && ks % kDmaEvery == 0) wide_issue_entry<C>(dma, next_stage, ks / kDmaEvery);
        });
    }
    if constexpr (PREV) {
        static_for<2 * C::NBW>([&](auto I) {
            constexpr int i = decltype(I)::value;
            if constexpr (C::col_block(i >> 1) < C::NB) {
                const bf16x8 a = wide_load_pv<C, i>(st_prev, ln);
                acc[i >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[i & 1], acc[i >> 1], 0, 0, 0);
            }
        });
    }
    if constexpr (CUR) {
        float mx = sacc[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        if (__any(mx > m_run + kTauW)) {
            const float m_new = fmaxf(m_run, mx);
            const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int nb = 0; nb < C::NBW; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[nb][r] *= alpha;
        }
        const float m_use = m_run == -INFINITY ? 0.f : m_run;
        unsigned pp[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2)
            pp[r >> 1] = pack_pair(__builtin_amdgcn_exp2f(sacc[r] - m_use), __builtin_amdgcn_exp2f(sacc[r + 1] - m_use), l_run);
        pf[0] = __builtin_bit_cast(bf16x8, (u32x4){pp[0], pp[1], pp[2], pp[3]});
        pf[1] = __builtin_bit_cast(bf16x8, (u32x4){pp[4], pp[5], pp[6], pp[7]});
    }
}

// The MFMAs of a steady step in issue order: the S^T MFMAs of the current block with the first
// NPV - kTail P V MFMAs of the previous block spread between them, then the held-back kTail P V
// MFMAs, which run while the row maximum and the exponentials of the current block are formed.
// kind: 0 = S^T (idx = k-step), 1 = P V (idx = 2 * output block + key half).
template <class C>
struct WideOps {
    static constexpr int KS = C::KS, NPV = 2 * C::NBW;
    static constexpr int kTail = 8;
    static constexpr int kInLoop = NPV - kTail;
    static constexpr int NL = KS + kInLoop, NT = KS + NPV;
    static_assert(kInLoop >= 0, "fewer P V MFMAs than held back");
    struct Op {
        int kind, idx;
    };
    static constexpr Op op(int j)
    {
        int n = 0;
        for (int ks = 0; ks < KS; ++ks) {
            if (n == j) return {0, ks};
            ++n;
            for (int a = ks * kInLoop / KS; a < (ks + 1) * kInLoop / KS; ++a) {
                if (n == j) return {1, a};
                ++n;
            }
        }
        return {1, kInLoop + (j - NL)};
    }
};

// Steady step (current and previous block both present) with a fixed instruction order: LDS
// operands requested kLA MFMAs ahead into a small ring, the loads of the next block spread over
// the S^T MFMAs, and the softmax of the current block -- row maximum, then the exponentials pair
// by pair -- between the held-back P V MFMAs of the previous block.  Those still use the old
// reference, so when the reference has to be raised the accumulator is rescaled only at the end
// of the step, after the last of them.
template <class C>
__device__ __forceinline__ void wide_step_steady(const char *__restrict__ st, const char *__restrict__ st_prev, const WideLane &ln,
                                                 const bf16x8 (&qf)[C::KS], f32x16 (&acc)[C::NBW],
                                                 bf16x8 (&pf)[2], float &m_run, float &l_run,
                                                 WideDma<C> &dma, unsigned next_stage, bool load_next)
{
    using O = WideOps<C>;
    constexpr int kDmaEvery = C::KS / (C::NIW + 1);
    constexpr int kLA = 3, kRing = 4;
    auto fetch = [&](auto J) -> bf16x8 {
        constexpr auto o = O::op(decltype(J)::value);
        if constexpr (o.kind == 0) {
            constexpr int ks = o.idx;
            const char *src = ks < C::KSH ? st + C::KH_OFF + ln.kaddr_h + ks * 32 : st + C::Z_OFF + ln.kaddr_z + (ks - C::KSH) * 32;
            return *reinterpret_cast<const bf16x8 *>(src);
        } else {
            return wide_load_pv<C, o.idx>(st_prev, ln);
        }
    };
    f32x16 sacc;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const f32x4 bias = *reinterpret_cast<const f32x4 *>(st + C::KB_OFF + (8 * a + 4 * ln.g) * 4);
#pragma unroll
        for (int x = 0; x < 4; ++x) sacc[4 * a + x] = bias[x];
    }
    bf16x8 fr[kRing];
    static_for<kLA>([&](auto J) { fr[decltype(J)::value] = fetch(J); });
    unsigned pp[8];
    float mx = 0.f, m_use = 0.f, alpha = 1.f, psum = 0.f;
    bool raise = false;
    static_for<O::NT>([&](auto J) {
        constexpr int j = decltype(J)::value;
        if constexpr (j + kLA < O::NT) fr[(j + kLA) % kRing] = fetch(std::integral_constant<int, j + kLA>{});
        constexpr auto o = O::op(j);
        constexpr int t = j - O::NL;  // position among the held-back MFMAs
        if constexpr (t == 0) {
            // row maximum of the current block (first half of the tree)
            mx = sacc[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[r]);
        } else if constexpr (t == 1) {
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            raise = __any(mx > m_run + kTauW);
            const float m_new = raise ? fmaxf(m_run, mx) : m_run;
            alpha = m_new == -INFINITY || !raise ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            m_use = m_new == -INFINITY ? 0.f : m_new;
        }
        if constexpr (t >= 2) {
            constexpr int first = (t - 2) * 8 / (O::kTail - 2), last = (t - 1) * 8 / (O::kTail - 2);
#pragma unroll
            for (int q = first; q < last; ++q)
                pp[q] = pack_pair(__builtin_amdgcn_exp2f(sacc[2 * q] - m_use), __builtin_amdgcn_exp2f(sacc[2 * q + 1] - m_use), psum);
        }
        if constexpr (o.kind == 0) {
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % kRing], qf[o.idx], sacc, 0, 0, 0);
            if (load_next && o.idx % kDmaEvery == 0) wide_issue_entry<C>(dma, next_stage, o.idx / kDmaEvery);
        } else {
            acc[o.idx >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % kRing], pf[o.idx & 1], acc[o.idx >> 1], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    });
    if (raise) {  // rare: every P V MFMA of the previous block has been issued; bring the accumulator to the new reference
        l_run *= alpha;
#pragma unroll
        for (int nb = 0; nb < C::NBW; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nb][r] *= alpha;
    }
    l_run += psum;
    pf[0] = __builtin_bit_cast(bf16x8, (u32x4){pp[0], pp[1], pp[2], pp[3]});
    pf[1] = __builtin_bit_cast(bf16x8, (u32x4){pp[4], pp[5], pp[6], pp[7]});
}

// One window of one query tile.
template <int DZ, int CZ, int NWIN, int WIN>
__device__ __forceinline__ void wide_window(const AttnParams &p, char *smem, int logical)
{
    using C = WideCfg<DZ, CZ, NWIN, WIN>;
    const int bh_pos = logical / p.nQT, qt = logical - bh_pos * p.nQT;
    const int bh = p.deal ? dealt_pair_by_length(bh_pos, p.kvlen, p.B, p.H, threadIdx.x & 63) : bh_pos;
    const int b = bh / p.H;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, g = lane >> 5;
    const int kvlen = p.deal ? p.kvlen[b] : p.L;  // (no mask: every chain has L residues)
    const int nblk = (kvlen + kKB - 1) / kKB;
    const int irow = qt * kTileQ + wave * 32 + li;

    // rows of this chain in the caller's tensors (a packed batch stores the chains back to back)
    [[maybe_unused]] const int ulen = user_len(p, b);
    [[maybe_unused]] const size_t urow0 = user_row(p, b, 0);
    [[maybe_unused]] const int h = bh - b * p.H;

    // A tile whose rows all lie past the last valid residue of its chain has nothing to attend
    // from: zero output.
    if (qt * kTileQ >= kvlen) {
        if constexpr (!C::FUSED) {
            float *orow = p.Ohat + ((size_t)bh * p.Lp + irow) * C::D;
#pragma unroll
            for (int nbw = 0; nbw < C::NBW; ++nbw)
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    if (C::col_block(nbw) < C::NB)
                        *reinterpret_cast<f32x4 *>(orow + 32 * C::col_block(nbw) + 8 * a + 4 * g) = (f32x4){0.f, 0.f, 0.f, 0.f};
            if (WIN == 0 && g == 0) p.lse2[(size_t)bh * p.Lp + irow] = -INFINITY;
        } else if (irow < ulen) {
            const size_t row = (urow0 + irow) * p.H + h;
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            if constexpr (WIN == 0) {
#pragma unroll
                for (int a = 0; a < 2; ++a) *reinterpret_cast<f32x4 *>(p.o + row * 16 + 8 * a + 4 * g) = zero;
#pragma unroll
                for (int a = 0; a < 3; ++a) *reinterpret_cast<f32x4 *>(p.o_pts + row * 24 + 12 * g + 4 * a) = zero;
                if (p.lse && g == 0) p.lse[user_lse_index(p, b, h, irow)] = 0.f;
            }
#pragma unroll
            for (int q = 0; q < C::HB; ++q)
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    *reinterpret_cast<f32x4 *>(p.o_pair + row * CZ + 32 * (WIN * C::HB + q) + 8 * a + 4 * g) = zero;
        }
        return;
    }

    // start at the block holding the tile's own residues (see the main kernel) and wrap around
    // (Rounded down to a multiple of kStartGroup blocks: the four tiles whose own residues lie in
    // one group start at the same block and, running side by side, fetch every block once from
    // beyond L2 instead of four times -- at this width a chain's keys and values do not fit L2.
    // The tiles that start up to 12 blocks before their own residues raise the reference a few
    // times more.  Workload 3: 4 % faster at 16; 8 and 32 to 64 measure within 1 % of it.)
    constexpr int kStartGroup = 16;
    const int first_blk = min(((qt * (kTileQ / kKB)) / kStartGroup) * kStartGroup, max(nblk - 1, 0));

    WideDma<C> dma;
    dma.wave_lds = 1024u * wave;
    {
        const char *Z2b = reinterpret_cast<const char *>(p.Z2 + (size_t)b * p.Lp * DZ);
        const char *Khb = reinterpret_cast<const char *>(p.Kh + (size_t)bh * p.Lp * kDH);
        const char *Vhb = reinterpret_cast<const char *>(p.Vh + (size_t)bh * p.Lp * kDH);
#pragma unroll
        for (int k = 0; k < C::NIW; ++k) {
            int i = wave + 4 * k;
            if (i >= C::NI) i = 0;
            const bool isz = i < C::NZ;
            const bool isk = !isz && i < C::NZ + C::NH;
            const int first = isz ? 0 : (isk ? C::NZ : C::NZ + C::NH);
            const int spr = isz ? C::Z_SPR : C::H_SPR;        // 16-byte slots per LDS row
            const int cols = isz ? DZ / 8 : kDH / 8;          // 16-byte columns of a global row
            const int s = 64 * (i - first) + lane;
            const int row = s / spr, col = s - row * spr;
            dma.step[k] = kKB * cols * 16;
            dma.src[k] = isz ? Z2b : (isk ? Khb : Vhb);
            // one block before the first block: every request advances the offset first
            dma.voff[k] = ((row < kKB && col < cols) ? row * (cols * 16) + col * 16 : 0) + (first_blk - 1) * dma.step[k];
        }
        dma.step[C::NIW] = kKB * 4;
        dma.src[C::NIW] = reinterpret_cast<const char *>(p.kbias + (size_t)bh * p.Lp);
        dma.voff[C::NIW] = min(lane, 7) * 16 + (first_blk - 1) * dma.step[C::NIW];
    }
    const unsigned smem_lds = lds_address(smem);
    int next_blk = first_blk;
    if (nblk > 0) {
        wide_issue_block<C>(dma, smem_lds);
        ++next_blk;
    }

    bf16x8 qf[C::KS];
    {
        const bf16_t *qh = p.Qh + ((size_t)bh * p.Lp + irow) * kDH;
#pragma unroll
        for (int ks = 0; ks < C::KSH; ++ks) qf[ks] = *reinterpret_cast<const bf16x8 *>(qh + ks * 16 + 8 * g);
        // The pair part of q^ -- the bias vector b^{h1} = log2e * w_L * w_b[h] (.) z1 of Algorithm 1
        // steps 2-3 -- is formed here from z1, which all heads of a residue share, instead of being
        // packed per head (24 KiB per residue at this width) and read back.  The per-head scale
        // vector goes through LDS; rows that do not exist or are masked get zeros.
        {
            float *cw = reinterpret_cast<float *>(smem + C::CW_OFF);
            for (int x = tid; x < DZ; x += 256) cw[x] = kLog2e * p.w_L * p.w_b[(size_t)h * p.cz + x % p.cz];
            __syncthreads();
            const bool ok = irow < ulen && (p.mask ? p.mask[urow0 + irow] != 0 : true);
            const unsigned keep = ok ? 0xFFFFFFFFu : 0u;
            const bf16_t *z1row = p.z1 + (urow0 + min(irow, ulen - 1)) * DZ + 8 * g;
#pragma unroll
            for (int ks = 0; ks < C::KS - C::KSH; ++ks) {
                const uint4 zr = *reinterpret_cast<const uint4 *>(z1row + 16 * ks);
                const f32x4 w0 = *reinterpret_cast<const f32x4 *>(cw + 16 * ks + 8 * g);
                const f32x4 w1 = *reinterpret_cast<const f32x4 *>(cw + 16 * ks + 8 * g + 4);
                const unsigned zw[4] = {zr.x, zr.y, zr.z, zr.w};  // two bf16 values each
                unsigned pk[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const float wl = x < 2 ? w0[2 * x] : w1[2 * x - 4], wh = x < 2 ? w0[2 * x + 1] : w1[2 * x - 3];
                    const float lo = wl * __uint_as_float(zw[x] << 16), hi = wh * __uint_as_float(zw[x] & 0xFFFF0000u);
                    // (round to nearest even, as the pack kernel's conversion; one v_cvt_pk_bf16_f32)
                    pk[x] = __builtin_bit_cast(unsigned, __builtin_convertvector((f32x2){lo, hi}, bf16x2)) & keep;
                }
                qf[C::KSH + ks] = __builtin_bit_cast(bf16x8, (u32x4){pk[0], pk[1], pk[2], pk[3]});
            }
        }
        // Most q^ fragments live in accumulation registers, from where the MFMA reads its B
        // operand directly (left to itself the compiler parks them there and copies each one to
        // an architectural register before its MFMA): 16 * NBW registers hold the output
        // accumulator, 16 the S^T accumulator, the rest of the 256 takes fragments.
        // (Width 1088: the fragments fill the accumulation registers and the accumulators live in the
        // architectural ones.)
        constexpr int kWant = C::KS * 4 > 256 ? 64 : (256 - 16 * C::NBW - 16) / 4;
        constexpr int kInAcc = kWant < C::KS ? kWant : C::KS;
#pragma unroll
        for (int ks = 0; ks < kInAcc; ++ks) asm volatile("" : "+a"(qf[ks]));
    }
    f32x16 acc[C::NBW];
#pragma unroll
    for (int nb = 0; nb < C::NBW; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[nb][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    WideLane ln;
    {
        const int l16 = lane & 15, grp2 = (lane >> 4) & 1, e4 = l16 >> 2, j4 = l16 & 3;
        ln.kaddr_h = li * kHS + g * 16;
        ln.kaddr_z = li * C::ZS + g * 16;
        ln.vaddr_h = (4 * g + e4) * kHS + (16 * grp2 + 4 * j4) * 2;
        ln.vaddr_z = (4 * g + e4) * C::ZS + (16 * grp2 + 4 * j4) * 2;
        ln.g = g;
    }

    bf16x8 pf[2] = {};
    int sidx = 0;  // stage of block n
    const char *st_prev = smem;
    for (int n = 0; n < nblk; ++n) {
        const char *st = smem + sidx * C::STAGE;
        // block n must have landed; the barrier also tells everyone that the stage of block n-2
        // is free again
        wait_vmem<0>();
        wg_barrier();
        sidx = sidx + 1 < C::NSTAGE ? sidx + 1 : 0;
        const bool load_next = n + 1 < nblk;
        unsigned next_stage = 0;
        if (load_next) {
            if (next_blk == nblk) {  // continue at block 0
#pragma unroll
                for (int k = 0; k <= C::NIW; ++k) dma.src[k] -= (size_t)nblk * dma.step[k];
                next_blk = 0;
            }
            next_stage = smem_lds + sidx * C::STAGE;
            ++next_blk;
        }
        if constexpr (C::PIPELINED) {
            if (n == 0)
                wide_step<C, true, false>(st, st_prev, ln, qf, acc, pf, m_run, l_run, dma, next_stage, load_next);
            else
                wide_step_steady<C>(st, st_prev, ln, qf, acc, pf, m_run, l_run, dma, next_stage, load_next);
        } else {
            // two stages: everything of block n now, while block n+1 loads into the other stage
            wide_step<C, true, false>(st, st, ln, qf, acc, pf, m_run, l_run, dma, next_stage, load_next);
            wide_step<C, false, true>(st, st, ln, qf, acc, pf, m_run, l_run, dma, 0u, false);
        }
        st_prev = st;
    }
    if (C::PIPELINED && nblk > 0) wide_step<C, false, true>(st_prev, st_prev, ln, qf, acc, pf, m_run, l_run, dma, 0u, false);

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    const float lse2 = l_tot > 0.f ? m_run + __log2f(l_tot) : -INFINITY;
    if constexpr (!C::FUSED) {
        float *orow = p.Ohat + ((size_t)bh * p.Lp + irow) * C::D;
#pragma unroll
        for (int nbw = 0; nbw < C::NBW; ++nbw)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 out;
#pragma unroll
                for (int x = 0; x < 4; ++x) out[x] = acc[nbw][4 * a + x] * inv;
                if (C::col_block(nbw) < C::NB) *reinterpret_cast<f32x4 *>(orow + 32 * C::col_block(nbw) + 8 * a + 4 * g) = out;
            }
        if (WIN == 0 && g == 0) p.lse2[(size_t)bh * p.Lp + irow] = lse2;
    } else {
        // ---- split, inverse frame, z1 contraction (Algorithm 1 steps 8-9, Eq. 4) on the accumulator;
        // c = 16, N_value = 8.  This window holds, for its half of the pair columns d, all R = DZ / CZ
        // factor slices: block z0 + rho * HB + q is slice rho, columns 32 (WIN * HB + q) .. + 31.
        constexpr int R = DZ / CZ, HB = C::HB, z0 = WIN == 0 ? C::NBH : 0;
        const bool in_range = irow < ulen;
        const int irow_c = min(irow, ulen - 1);  // rows past the end compute on a valid address and store nothing
        const bool valid = (p.mask ? p.mask[urow0 + irow_c] != 0 : true) && l_tot > 0.f;
        const float sc = valid ? inv : 0.f;
        const size_t row = (urow0 + irow_c) * p.H + h;
        {
            // (read per lane from memory: 8 bytes of each of the wave's 32 rows per load.  Staging the rows
            // through the free LDS stages during the last block, as the main kernel does, measured 2 %
            // slower here -- the epilogue is 1 % of a unit at this width, the extra barrier is not free)
            const bf16_t *z1row = p.z1 + (urow0 + irow_c) * DZ + 32 * WIN * HB + 4 * g;
#pragma unroll
            for (int rho = 0; rho < R; ++rho)
#pragma unroll
                for (int q = 0; q < HB; ++q)
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const uint2 zraw = *reinterpret_cast<const uint2 *>(z1row + rho * CZ + 32 * q + 8 * a);
                        const bf16_t *zb16 = reinterpret_cast<const bf16_t *>(&zraw);
#pragma unroll
                        for (int x = 0; x < 4; ++x) acc[z0 + rho * HB + q][4 * a + x] *= bf2f(zb16[x]);
                    }
#pragma unroll
            for (int q = 0; q < HB; ++q)
#pragma unroll
                for (int rho = 1; rho < R; ++rho)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[z0 + q][r] += acc[z0 + rho * HB + q][r];
        }
        if (in_range) {
            float *dst = p.o_pair + row * CZ + 32 * WIN * HB;
#pragma unroll
            for (int q = 0; q < HB; ++q)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    f32x4 out;
#pragma unroll
                    for (int x = 0; x < 4; ++x) out[x] = acc[z0 + q][4 * a + x] * sc;
                    *reinterpret_cast<f32x4 *>(dst + 32 * q + 8 * a + 4 * g) = out;
                }
        }
        if constexpr (WIN == 0) {
            constexpr int c = 16, Pv = 8;
            // point part: this half owns points 4g .. 4g+3, hi parts in slots u = 0..11, lo parts in
            // slots 12..23; slot u sits in column 16 + 8*(u/4) + 4g + u%4 (see v_pt_col)
            float Gv[12];
#pragma unroll
            for (int u = 0; u < 12; ++u) {
                const int dh = 16 + 8 * (u >> 2) + (u & 3);  // column for g = 0; g = 1 adds 4
                const int dl = 16 + 8 * ((u + 12) >> 2) + ((u + 12) & 3);
                Gv[u] = acc[dh >> 5][4 * ((dh & 31) >> 3) + (dh & 3)] + acc[dl >> 5][4 * ((dl & 31) >> 3) + (dl & 3)];
            }
            if (in_range) {
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    f32x4 out;
#pragma unroll
                    for (int x = 0; x < 4; ++x) out[x] = acc[0][4 * a + x] * sc;
                    *reinterpret_cast<f32x4 *>(p.o + row * c + 8 * a + 4 * g) = out;
                }
            }
            const float *Rp = p.rot + (urow0 + irow_c) * 9;
            const float *tr = p.trans + (urow0 + irow_c) * 3;
            float Rm[9], tc[3];
#pragma unroll
            for (int a = 0; a < 9; ++a) Rm[a] = Rp[a];
#pragma unroll
            for (int a = 0; a < 3; ++a) tc[a] = tr[a] - p.cen[4 * b + a];
            float outp[12];
#pragma unroll
            for (int pp = 0; pp < 4; ++pp) {
                const float rx = Gv[3 * pp] * inv - tc[0], ry = Gv[3 * pp + 1] * inv - tc[1],
                            rz = Gv[3 * pp + 2] * inv - tc[2];
#pragma unroll
                for (int x = 0; x < 3; ++x) {
                    const float val = Rm[x] * rx + Rm[3 + x] * ry + Rm[6 + x] * rz;  // R^T
                    outp[3 * pp + x] = valid ? val : 0.f;
                }
            }
            if (in_range) {
                float *dst = p.o_pts + row * (Pv * 3) + 12 * g;
#pragma unroll
                for (int a = 0; a < 3; ++a)
                    *reinterpret_cast<f32x4 *>(dst + 4 * a) =
                        (f32x4){outp[4 * a], outp[4 * a + 1], outp[4 * a + 2], outp[4 * a + 3]};
                if (p.lse && g == 0)
                    p.lse[user_lse_index(p, b, h, irow)] = valid ? lse2 * kLn2 - p.qbias[(size_t)bh * p.Lp + irow] : 0.f;
            }
        }
    }
}

template <int DZ, int CZ, int NWIN>
__global__ __launch_bounds__(256, 1) void fipa_attn_fwd_wide_kernel(AttnParams p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    // Workgroups are dealt round-robin to the 8 XCDs; each XCD gets a contiguous run of tiles, and the
    // windows of a tile are neighbours in that XCD's launch order, so that they run side by side and
    // the key blocks one of them brings in are found in the XCD's L2 by the other (launched as a
    // second grid dimension the windows of a tile ran far apart in time: 6.49 -> 5.92 ms at the
    // ragged rank-4 workload).  Going further -- all heads of a group of four query tiles side by side,
    // so that 32 workgroups share one z2 stream -- measured 7 % slower: the same lines are then
    // wanted by every compute unit of the XCD at the same moment.
    const int chunk = (p.total_tiles + 7) / 8;
    const int slot = blockIdx.x / 8;
    const int logical = (blockIdx.x % 8) * chunk + slot / NWIN;
    if (logical >= p.total_tiles) return;
    const int win = slot % NWIN;
    if (win == 0)
        wide_window<DZ, CZ, NWIN, 0>(p, smem, logical);
    else if (NWIN == 2 || win == 1)
        wide_window<DZ, CZ, NWIN, 1>(p, smem, logical);
    else if constexpr (NWIN > 2) {
        if (win == 2)
            wide_window<DZ, CZ, NWIN, 2>(p, smem, logical);
        else
            wide_window<DZ, CZ, NWIN, 3>(p, smem, logical);
    }
}

}  // namespace

bool attn_fwd_wide_fused_supported(int DZ, int cz) { return DZ == 512 && (cz == 64 || cz == 128 || cz == 256); }

namespace {

template <int DZ, int CZ, int NWIN>
hipError_t launch_wide(const AttnParams &p, hipStream_t stream)
{
    static_assert(NWIN == 2 || NWIN == 4, "window dispatch of the kernel");
    constexpr int lds = WideCfg<DZ, CZ, NWIN, 0>::LDS_BYTES;
    static LdsLimit lds_limit;
    hipError_t e = raise_lds_limit(lds_limit, (const void *)fipa_attn_fwd_wide_kernel<DZ, CZ, NWIN>, lds);
    if (e != hipSuccess) return e;
    const int chunk = (p.total_tiles + 7) / 8;
    hipLaunchKernelGGL((fipa_attn_fwd_wide_kernel<DZ, CZ, NWIN>), dim3(chunk * 8 * NWIN), dim3(256), lds, stream, p);
    return hipGetLastError();
}

}  // namespace

// fused: steps 8-9 of Algorithm 1 run inside the kernel (width 576, AlphaFold2 head shape, c_z of
// attn_fwd_wide_fused_supported); otherwise the kernel leaves O^ and the log-sum-exp in the workspace.
hipError_t launch_attn_fwd_wide_bf16(const AttnParams &p, int DZ, bool fused, hipStream_t stream)
{
    if (DZ == 1024) return fused ? hipErrorInvalidValue : launch_wide<1024, 0, 4>(p, stream);
    if (DZ != 512) return hipErrorInvalidValue;
    if (!fused) return launch_wide<512, 0, 2>(p, stream);
    switch (p.cz) {
        case 64: return launch_wide<512, 64, 2>(p, stream);
        case 128: return launch_wide<512, 128, 2>(p, stream);
        case 256: return launch_wide<512, 256, 2>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fipa
