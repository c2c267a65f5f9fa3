// Fused attention on the lifted features (Algorithm 1 step 7) for wide pair factors (r*c_z = 512,
// lifted width 576): same mathematics and register layout as the main kernel, but the output
// accumulator of 32 x 576 fp32 per wave does not fit the register file, so the value columns are
// cut into windows and each workgroup computes one window (recomputing S^T and the softmax).
// Key blocks of 32 residues arrive in a ring of three LDS stages by direct global -> LDS loads
// issued one block ahead (the z2 block is stored once and read in both roles, as in the main
// kernel).  The loop is software pipelined over two blocks: iteration n forms S^T of block n and,
// interleaved with it, accumulates P V of block n-1; the softmax of block n (running maximum of
// Algorithm 2, raised lazily) follows.  Unfused epilogue.
#include "fipa_gfx950.h"

namespace fipa {

namespace {

constexpr int kKB = 32;              // keys per block
constexpr int kHS = kDH * 2 + 16;    // LDS row stride (bytes) of the head-specific k^ / v^ blocks
constexpr float kTauW = 8.f;

template <int DZ, int NWIN>
struct WideCfg {
    static constexpr int D = kDH + DZ;
    static constexpr int KS = D / 16, KSH = kDH / 16;
    static constexpr int NB = D / 32, NBH = kDH / 32;
    static constexpr int NBW = NB / NWIN;
    static_assert(NB % NWIN == 0, "windows must tile the value columns");
    static_assert(KS == 4 * NBW, "one P V MFMA per two S^T MFMAs");
    static constexpr int ZS = DZ * 2 + 48;       // LDS row stride of the z2 block (conflict free for both read patterns)
    static constexpr int Z_SPR = ZS / 16, H_SPR = kHS / 16;
    static constexpr int NZ = (kKB * Z_SPR + 63) / 64;   // wave-wide 1 KiB loads for the z2 block
    static constexpr int NH = (kKB * H_SPR + 63) / 64;   // for one head block
    static constexpr int NI = NZ + 2 * NH;               // flat list: z2 | k^ head | v^ head
    static constexpr int NIW = (NI + 3) / 4;             // per wave
    static constexpr int Z_OFF = 0, KH_OFF = NZ * 1024, VH_OFF = (NZ + NH) * 1024;
    static constexpr int KB_OFF = NIW * 4 * 1024;        // 32 per-key fp32 biases (a full 1 KiB load lands here)
    static constexpr int STAGE = KB_OFF + 1024;
    static constexpr int NSTAGE = 3;
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
    int kaddr_h, kaddr_z, vaddr_h, vaddr_z, g, win;
};

// One step of the pipeline: S^T and the softmax of the block in stage `st` (CUR), interleaved
// with P V of the previous block (stage `st_prev`, probabilities `pf` on entry) (PREV).  On exit
// `pf` holds the probabilities of the current block.  When `load_next` is set the loads of the
// next block are issued between the MFMAs, one entry every few of them (issued back to back they
// cost about 60 cycles each).
template <int DZ, int NWIN, bool CUR, bool PREV>
__device__ __forceinline__ void wide_step(const char *__restrict__ st, const char *__restrict__ st_prev, const WideLane &ln,
                                          const bf16x8 (&qf)[WideCfg<DZ, NWIN>::KS], f32x16 (&acc)[WideCfg<DZ, NWIN>::NBW],
                                          bf16x8 (&pf)[2], float &m_run, float &l_run,
                                          WideDma<WideCfg<DZ, NWIN>> &dma, unsigned next_stage, bool load_next)
{
    using C = WideCfg<DZ, NWIN>;
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
    }
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        if constexpr (CUR) {
            const char *src = ks < C::KSH ? st + C::KH_OFF + ln.kaddr_h + ks * 32 : st + C::Z_OFF + ln.kaddr_z + (ks - C::KSH) * 32;
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(src);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sacc, 0, 0, 0);
            if (load_next && ks % kDmaEvery == 0) wide_issue_entry<C>(dma, next_stage, ks / kDmaEvery);
        }
        if constexpr (PREV) {
            if ((ks & 1) == 0) {
                const int i = ks >> 1, nbw = i >> 1, tt = i & 1;
                const int nb = ln.win * C::NBW + nbw;  // global 32-column block (win is uniform)
                const bool head = nb < C::NBH;
                const char *src = head ? st_prev + C::VH_OFF + ln.vaddr_h + 16 * tt * kHS + nb * 64
                                       : st_prev + C::Z_OFF + ln.vaddr_z + 16 * tt * C::ZS + (nb - C::NBH) * 64;
                const int rs = head ? kHS : C::ZS;
                const bf16x4 lo = lds_read_tr(src);
                const bf16x4 hi = lds_read_tr(src + 8 * rs);
                bf16x8 a;
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    a[x] = lo[x];
                    a[4 + x] = hi[x];
                }
                acc[nbw] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[tt], acc[nbw], 0, 0, 0);
            }
        }
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
template <int DZ, int NWIN>
struct WideOps {
    using C = WideCfg<DZ, NWIN>;
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
template <int DZ, int NWIN>
__device__ __forceinline__ void wide_step_steady(const char *__restrict__ st, const char *__restrict__ st_prev, const WideLane &ln,
                                                 const bf16x8 (&qf)[WideCfg<DZ, NWIN>::KS], f32x16 (&acc)[WideCfg<DZ, NWIN>::NBW],
                                                 bf16x8 (&pf)[2], float &m_run, float &l_run,
                                                 WideDma<WideCfg<DZ, NWIN>> &dma, unsigned next_stage, bool load_next)
{
    using C = WideCfg<DZ, NWIN>;
    using O = WideOps<DZ, NWIN>;
    constexpr int kDmaEvery = C::KS / (C::NIW + 1);
    constexpr int kLA = 3, kRing = 4;
    auto fetch = [&](auto J) -> bf16x8 {
        constexpr auto o = O::op(decltype(J)::value);
        if constexpr (o.kind == 0) {
            constexpr int ks = o.idx;
            const char *src = ks < C::KSH ? st + C::KH_OFF + ln.kaddr_h + ks * 32 : st + C::Z_OFF + ln.kaddr_z + (ks - C::KSH) * 32;
            return *reinterpret_cast<const bf16x8 *>(src);
        } else {
            constexpr int nbw = o.idx >> 1, tt = o.idx & 1;
            const int nb = ln.win * C::NBW + nbw;  // global 32-column block (win is uniform)
            const bool head = nb < C::NBH;
            const char *src = head ? st_prev + C::VH_OFF + ln.vaddr_h + 16 * tt * kHS + nb * 64
                                   : st_prev + C::Z_OFF + ln.vaddr_z + 16 * tt * C::ZS + (nb - C::NBH) * 64;
            const int rs = head ? kHS : C::ZS;
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

template <int DZ, int NWIN>
__global__ __launch_bounds__(256, 1) void fipa_attn_fwd_wide_kernel(AttnParams p)
{
    using C = WideCfg<DZ, NWIN>;
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
    const int bh_pos = logical / p.nQT, qt = logical - bh_pos * p.nQT;
    const int bh = p.deal ? dealt_pair_by_length(bh_pos, p.kvlen, p.B, p.H, threadIdx.x & 63) : bh_pos;
    const int b = bh / p.H;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, g = lane >> 5;
    const int kvlen = p.deal ? p.kvlen[b] : p.L;  // (no mask: every chain has L residues)
    const int nblk = (kvlen + kKB - 1) / kKB;
    const int irow = qt * kTileQ + wave * 32 + li;

    // A tile whose rows all lie past the last valid residue of its chain has nothing to attend
    // from: zero output.
    if (qt * kTileQ >= kvlen) {
        float *orow = p.Ohat + ((size_t)bh * p.Lp + irow) * C::D + win * C::NBW * 32;
#pragma unroll
        for (int nbw = 0; nbw < C::NBW; ++nbw)
#pragma unroll
            for (int a = 0; a < 4; ++a)
                *reinterpret_cast<f32x4 *>(orow + 32 * nbw + 8 * a + 4 * g) = (f32x4){0.f, 0.f, 0.f, 0.f};
        if (win == 0 && g == 0) p.lse2[(size_t)bh * p.Lp + irow] = -INFINITY;
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
            for (int x = tid; x < DZ; x += 256) cw[x] = kLog2e * p.w_L * p.w_b[(size_t)(bh - b * p.H) * p.cz + x % p.cz];
            __syncthreads();
            const int ulen = user_len(p, b);
            const size_t urow0 = user_row(p, b, 0);  // (a packed batch stores the chains back to back)
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
        constexpr int kInAcc = (256 - 16 * C::NBW - 16) / 4 < C::KS ? (256 - 16 * C::NBW - 16) / 4 : C::KS;
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
        ln.win = win;
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
        if (n == 0)
            wide_step<DZ, NWIN, true, false>(st, st_prev, ln, qf, acc, pf, m_run, l_run, dma, next_stage, load_next);
        else
            wide_step_steady<DZ, NWIN>(st, st_prev, ln, qf, acc, pf, m_run, l_run, dma, next_stage, load_next);
        st_prev = st;
    }
    if (nblk > 0) wide_step<DZ, NWIN, false, true>(st_prev, st_prev, ln, qf, acc, pf, m_run, l_run, dma, 0u, false);

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    float *orow = p.Ohat + ((size_t)bh * p.Lp + irow) * C::D + win * C::NBW * 32;
#pragma unroll
    for (int nbw = 0; nbw < C::NBW; ++nbw)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            f32x4 out;
#pragma unroll
            for (int x = 0; x < 4; ++x) out[x] = acc[nbw][4 * a + x] * inv;
            *reinterpret_cast<f32x4 *>(orow + 32 * nbw + 8 * a + 4 * g) = out;
        }
    if (win == 0 && g == 0) p.lse2[(size_t)bh * p.Lp + irow] = l_tot > 0.f ? m_run + __log2f(l_tot) : -INFINITY;
}

}  // namespace

hipError_t launch_attn_fwd_wide_bf16(const AttnParams &p, int DZ, hipStream_t stream)
{
    if (DZ != 512) return hipErrorInvalidValue;
    using C = WideCfg<512, 2>;
    static LdsLimit lds_limit;
    hipError_t e = raise_lds_limit(lds_limit, (const void *)fipa_attn_fwd_wide_kernel<512, 2>, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int chunk = (p.total_tiles + 7) / 8;
    hipLaunchKernelGGL((fipa_attn_fwd_wide_kernel<512, 2>), dim3(chunk * 8 * 2), dim3(256), C::LDS_BYTES, stream, p);
    return hipGetLastError();
}

}  // namespace fipa
