// Fused attention on the lifted features (Algorithm 1 step 7, with steps 2-3 on the query side and
// steps 8-9 / Eq. 4 on the accumulator) for gfx950, with the work of a query tile divided between
// two kinds of waves, so that every SIMD holds two waves whose waits overlap.
//
// One workgroup = one (batch, head, 128-query tile) = 8 waves.  Row group g (32 query rows) is served
// by a pair of waves:
//   * the S wave (waves 0-3) keeps q^ as MFMA B fragments in registers, forms S^T = K^ Q^T of a key
//     block (bf16 MFMA 32x32x16, the per-key fp32 bias as initial accumulator), evaluates the online
//     softmax of Algorithm 2 (reference maximum raised lazily, running sum) and leaves the block's
//     weights P^T -- already in B-operand layout, rounded to bf16 -- in LDS together with the factor
//     by which earlier contributions have to be rescaled;
//   * the PV wave (waves 4-7) keeps the 32 x (64 + DZ) fp32 output accumulator, reads P^T from LDS
//     and accumulates O^T += V^T P^T (the v^ operand comes from the row-major key block through the
//     transposing LDS read), issues the direct global -> LDS loads of the key blocks, and runs the
//     epilogue (z1 contraction, inverse frame, stores; or the key-range-split exchange).
// An S wave needs about 180 registers and a PV wave about 220, so two waves fit a SIMD (one wave
// holding both q^ and the accumulator needs 240 + working registers: one wave per SIMD, nothing to
// cover its waits).  The MFMA work of the two kinds is equal (KS = 2 NB MFMAs per key block each).
//
// Pipeline, one workgroup barrier per key block: in iteration t the S waves form S^T of block t and
// (between those MFMAs) the softmax of block t-1, whose weights they publish before the next
// barrier; the PV waves accumulate block t-2 and request block t+2.  A key block lives in one of
// five LDS stages from its request to its accumulation.
#include "fipa_gfx950.h"

namespace fipa {

namespace {

constexpr float kTau = 32.0f;
constexpr float kTauPow = 4294967296.0f;  // 2^kTau
constexpr int kBlk = 32;           // keys per LDS stage
constexpr int kHS = kDH * 2 + 16;  // LDS row stride (bytes) of the head-specific k^ / v^ blocks

template <int DZ>
struct WsCfg {
    static constexpr int DV = kDH + DZ;
    static constexpr int KSZ = DZ / 16;      // k-steps of S^T over the pair part
    static constexpr int KSH = kDH / 16;     // k-steps over the head-specific part
    static constexpr int KS = KSZ + KSH;
    static constexpr int NB = DV / 32;       // 32-row blocks of O^T
    static constexpr int NBH = kDH / 32;     // of which head specific
    static constexpr int NPV = 2 * NB;       // P V MFMAs per key block
    static_assert(KS == NPV, "S^T and P V use the same number of MFMAs per block");
    static constexpr int ZS = DZ * 2 + 48;   // LDS row stride of the z2 block: conflict free for the row reads
    static constexpr int Z_SPR = ZS / 16;    // 16-byte slots per row
    static constexpr int H_SPR = kHS / 16;
    // A stage is a flat list of 16-byte slots: z2 block | k^ head block | v^ head block | 32 biases,
    // filled by NE wave-wide loads of 64 slots each.
    static constexpr int Z_SLOTS = kBlk * Z_SPR, H_SLOTS = kBlk * H_SPR, B_SLOTS = kBlk * 4 / 16;
    static constexpr int Z_OFF = 0;
    static constexpr int KH_OFF = Z_SLOTS * 16;
    static constexpr int VH_OFF = KH_OFF + H_SLOTS * 16;
    static constexpr int KB_OFF = VH_OFF + H_SLOTS * 16;
    static constexpr int SLOTS = Z_SLOTS + 2 * H_SLOTS + B_SLOTS;
    static constexpr int NE = (SLOTS + 63) / 64;   // load entries per block
    static constexpr int NEW = (NE + 3) / 4;       // per PV wave (a surplus entry repeats entry 0)
    static constexpr int STAGE = NE * 1024;
    static constexpr int NSTAGE = 5;
    // Weights of a block: per row group 2 KiB of P^T (two B operands) and 32 rescale factors; two
    // buffers (one is written while the other is read).
    static constexpr int PB_OFF = NSTAGE * STAGE;
    static constexpr int PB_RG = 2048 + 256;
    static constexpr int PB_BUF = 4 * PB_RG;
    static constexpr int CW_OFF = PB_OFF + 2 * PB_BUF;  // per-head scale vector of the query-side factors (DZ floats)
    static constexpr int ST_OFF = CW_OFF + DZ * 4;      // final (reference, weight sum) of every row: 4 x 32 x 2 floats
    static constexpr int LDS_BYTES = ST_OFF + 1024;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    // Start-up: the z1 rows of the tile (4 x 32 rows x 2 DZ bytes) pass through LDS on their way into
    // the query-side factor fragments; they sit behind the first three stages and may cover the
    // weight buffers, which are not in use yet, but not the scale vector.
    static constexpr int Z1P_OFF = 3 * STAGE;
    static_assert(Z1P_OFF + 4 * 32 * DZ * 2 <= CW_OFF, "z1 staging overlaps the scale vector");
    static_assert(32 * DZ * 2 <= STAGE, "epilogue z1 staging: a wave's rows fit one stage");
    static constexpr int LA_S = 3 < KS ? 3 : KS - 1;   // LDS operands are fetched this many MFMAs ahead of their use
    static constexpr int LA_PV = 3 < KS ? 3 : KS - 1;  // (3, 5, 8 and 12 measured the same)
    static constexpr int RING_S = LA_S + 1;  // operand buffers
    static constexpr int RING_PV = LA_PV + 1;
    static constexpr int DMA_EVERY = NPV / NEW;  // one load entry every DMA_EVERY P V MFMAs
    static_assert(DMA_EVERY >= 1, "more load entries than MFMAs");
};

__device__ __forceinline__ void wait_lgkm0() { __builtin_amdgcn_s_waitcnt(0xC07F); }  // s_waitcnt lgkmcnt(0) only

// ---- direct global -> LDS loads of the key blocks (issued by the PV waves) ---------------------
// Entry k of PV wave w is entry e = w + 4k of the flat list (e >= NE: entry 0 again, same data to
// the same place, so that every wave issues the same number of loads per block).  Lane l of entry
// e fills slot 64 e + l of the stage; the slot decides which tensor, row and 16-byte column the
// lane fetches.  All four tensors live in one workspace: addresses are a common base plus a 32-bit
// per-lane offset, which advances by the tensor's block stride with every request (signed: a
// key-range part may walk downwards).
template <int DZ>
struct Dma {
    using C = WsCfg<DZ>;
    const char *base;       // wave-uniform
    int voff[C::NEW];       // per lane: offset of the PREVIOUSLY requested block
    int vstep[C::NEW];      // per lane: bytes from one key block to the next in walking direction
    unsigned lds_off[C::NEW];  // wave-uniform: 1024 * entry
};

__device__ __forceinline__ void dma16v(const char *base, int &voff, int vstep, int adv, unsigned lds_addr)
{
    // adv = 1: advance to the next block first; adv = 0: fetch the previously requested block again
    asm volatile(
        "s_mov_b32 m0, %1\n\t"
        "v_mad_i32_i24 %0, %2, %4, %0\n\t"
        "global_load_lds_dwordx4 %0, %3"
        : "+v"(voff)
        : "s"(lds_addr), "v"(vstep), "s"(base), "s"(adv)
        : "memory", "m0");
}

template <int DZ, int K>
__device__ __forceinline__ void dma_entry(Dma<DZ> &d, unsigned stage, int adv)
{
    dma16v(d.base, d.voff[K], d.vstep[K], adv, stage + d.lds_off[K]);
}

template <int DZ, int K = 0>
__device__ __forceinline__ void issue_block(Dma<DZ> &d, unsigned stage)
{
    if constexpr (K < WsCfg<DZ>::NEW) {
        dma_entry<DZ, K>(d, stage, 1);
        issue_block<DZ, K + 1>(d, stage);
    }
}

// Load entry (j / DMA_EVERY) is issued right before MFMA j when j is a multiple of DMA_EVERY.
template <int DZ, int K = 0>
__device__ __forceinline__ void dma_slot(Dma<DZ> &d, unsigned stage, int adv, int j)
{
    using C = WsCfg<DZ>;
    if constexpr (K < C::NEW) {
        if (j == K * C::DMA_EVERY)
            dma_entry<DZ, K>(d, stage, adv);
        else
            dma_slot<DZ, K + 1>(d, stage, adv, j);
    }
}

// After the last block in walking direction the sequence continues at the other end.
template <int DZ>
__device__ __forceinline__ void dma_wrap(Dma<DZ> &d, int nblk_chain)
{
#pragma unroll
    for (int k = 0; k < WsCfg<DZ>::NEW; ++k) d.voff[k] -= nblk_chain * d.vstep[k];
}

// ---- per-lane LDS addressing ---------------------------------------------------------------------
struct LaneAddr {
    int kaddr_h, kaddr_z, vaddr_h, vaddr_z, baddr;  // per-lane offsets inside a stage
};

template <int DZ>
__device__ __forceinline__ LaneAddr lane_addresses(int lane)
{
    using C = WsCfg<DZ>;
    const int li = lane & 31, g = lane >> 5;
    const int l16 = lane & 15, grp2 = (lane >> 4) & 1, e4 = l16 >> 2, j4 = l16 & 3;
    LaneAddr a;
    a.kaddr_h = C::KH_OFF + li * kHS + g * 16;
    a.kaddr_z = C::Z_OFF + li * C::ZS + g * 16;
    a.vaddr_h = C::VH_OFF + (4 * g + e4) * kHS + (16 * grp2 + 4 * j4) * 2;
    a.vaddr_z = C::Z_OFF + (4 * g + e4) * C::ZS + (16 * grp2 + 4 * j4) * 2;
    a.baddr = C::KB_OFF + 16 * g;
    return a;
}

// P V operation i of a key block works on the 32-column block pv_nb(i) of O^T and on the keys
// 16 pv_tt(i) .. + 15.  The two operations of a column block depend on each other through the
// accumulator; column blocks are taken in pairs so that consecutive MFMAs are independent.
template <int DZ>
__host__ __device__ constexpr int pv_nb(int i)
{
    constexpr int NB = WsCfg<DZ>::NB;
    return i < 4 * (NB / 2) ? 2 * (i / 4) + (i & 1) : NB - 1;
}
template <int DZ>
__host__ __device__ constexpr int pv_tt(int i)
{
    constexpr int NB = WsCfg<DZ>::NB;
    return i < 4 * (NB / 2) ? (i >> 1) & 1 : i & 1;
}

// LDS operand of P V operation `i` from the stage at `st`: 32 v^ columns x 16 keys.
template <int DZ>
__device__ __forceinline__ bf16x8 load_pv(const LaneAddr &w, const char *st, int i)
{
    using C = WsCfg<DZ>;
    const int nb = pv_nb<DZ>(i), tt = pv_tt<DZ>(i);
    const char *src = nb < C::NBH ? st + w.vaddr_h + 16 * tt * kHS + nb * 64
                                  : st + w.vaddr_z + 16 * tt * C::ZS + (nb - C::NBH) * 64;
    const int rs = nb < C::NBH ? kHS : C::ZS;
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

// LDS operand of S^T operation `ks` from the stage at `st`: 32 keys x 16 k^ features.
template <int DZ>
__device__ __forceinline__ bf16x8 load_s(const LaneAddr &w, const char *st, int ks)
{
    using C = WsCfg<DZ>;
    const char *src = ks < C::KSH ? st + w.kaddr_h + ks * 32 : st + w.kaddr_z + (ks - C::KSH) * 32;
    return *reinterpret_cast<const bf16x8 *>(src);
}

// Per-key bias (norm term, mask) of the stage at `st` in the layout of the S^T accumulator.
__device__ __forceinline__ f32x16 load_bias(const LaneAddr &w, const char *st)
{
    f32x16 sacc;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const f32x4 bias = *reinterpret_cast<const f32x4 *>(st + w.baddr + a * 32);
#pragma unroll
        for (int x = 0; x < 4; ++x) sacc[4 * a + x] = bias[x];
    }
    return sacc;
}

__device__ __forceinline__ float row_max16(const f32x16 &s)
{
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
    return fmaxf(mx, __shfl_xor(mx, 32));
}

// All 16 exponentials of an S^T block against the reference maximum -> MFMA B operands.
__device__ __forceinline__ void exp_block(const f32x16 &sacc, float m_use, bf16x8 (&pf)[2], float &psum)
{
    unsigned pp[8];
#pragma unroll
    for (int r = 0; r < 16; r += 2)
        pp[r >> 1] = pack_pair(__builtin_amdgcn_exp2f(sacc[r] - m_use), __builtin_amdgcn_exp2f(sacc[r + 1] - m_use), psum);
    pf[0] = __builtin_bit_cast(bf16x8, (u32x4){pp[0], pp[1], pp[2], pp[3]});
    pf[1] = __builtin_bit_cast(bf16x8, (u32x4){pp[4], pp[5], pp[6], pp[7]});
}

// ---- S wave ----------------------------------------------------------------------------------------
template <int DZ>
struct SWave {
    using C = WsCfg<DZ>;
    bf16x8 qf[C::KS];
    float m_ref, l_run;
    LaneAddr ad;
    int lane;
};

// S^T block (32 keys x 32 queries) of the stage at `st`, accumulator preset with the per-key bias.
template <int DZ>
__device__ __forceinline__ f32x16 s_block(const SWave<DZ> &w, const char *__restrict__ st)
{
    using C = WsCfg<DZ>;
    f32x16 sacc = load_bias(w.ad, st);
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks)
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_s<DZ>(w.ad, st, ks), w.qf[ks], sacc, 0, 0, 0);
    return sacc;
}

// Leave a block's weights and the rescale factor of the earlier contributions for the PV wave.
__device__ __forceinline__ void publish(char *pb, int lane, const bf16x8 (&pf)[2], float alpha)
{
    *reinterpret_cast<bf16x8 *>(pb + lane * 16) = pf[0];
    *reinterpret_cast<bf16x8 *>(pb + 1024 + lane * 16) = pf[1];
    if (lane < 32) *reinterpret_cast<float *>(pb + 2048 + lane * 4) = alpha;
}

// Raise the reference maximum to cover mx; returns the factor for everything accumulated so far.
template <int DZ>
__device__ __forceinline__ float raise_reference(SWave<DZ> &w, float mx)
{
    const float m_new = fmaxf(w.m_ref, mx);
    const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(w.m_ref - m_new);  // (no reference yet: nothing accumulated, factor 0)
    w.m_ref = m_new;
    w.l_run *= alpha;
    return alpha;
}

// The MFMAs of a key block are not all issued in the iteration that forms the block: the last HB of
// them are held back, with their LDS operands already in registers, and issued right after the
// next workgroup barrier, where they cover the time the first LDS reads of the new block take.
constexpr int kHoldS = 2;   // held-back S^T MFMAs per block
constexpr int kHoldPV = 2;  // held-back P V MFMAs per block

// First part of S^T of the block in stage `st` (no softmax work interleaved): the accumulation chain
// up to the held-back MFMAs, whose operands go to `hold`.
template <int DZ>
__device__ __forceinline__ void s_start(const SWave<DZ> &w, f32x16 &sacc, bf16x8 (&hold)[kHoldS], const char *st)
{
    using C = WsCfg<DZ>;
    constexpr int N = C::KS, NM = N - kHoldS;
    sacc = load_bias(w.ad, st);
#pragma unroll
    for (int ks = 0; ks < NM; ++ks)
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_s<DZ>(w.ad, st, ks), w.qf[ks], sacc, 0, 0, 0);
#pragma unroll
    for (int h = 0; h < kHoldS; ++h) hold[h] = load_s<DZ>(w.ad, st, NM + h);
}

// The held-back MFMAs of the pending block: completes its S^T in `sacc`.
template <int DZ>
__device__ __forceinline__ void s_held(const SWave<DZ> &w, f32x16 &sacc, const bf16x8 (&hold)[kHoldS])
{
    using C = WsCfg<DZ>;
#pragma unroll
    for (int h = 0; h < kHoldS; ++h)
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hold[h], w.qf[C::KS - kHoldS + h], sacc, 0, 0, 0);
}

// Softmax of the pending block without new MFMAs (the last block of a sequence).
template <int DZ>
__device__ __forceinline__ void s_finish(SWave<DZ> &w, f32x16 &sacc, const bf16x8 (&hold)[kHoldS], char *pb)
{
    s_held<DZ>(w, sacc, hold);
    const float mx = row_max16(sacc);
    float alpha = 1.f;
    if (__any(mx > w.m_ref + kTau)) alpha = raise_reference<DZ>(w, mx);
    bf16x8 pf[2];
    float psum = 0.f;
    exp_block(sacc, w.m_ref == -INFINITY ? 0.f : w.m_ref, pf, psum);
    w.l_run += psum;
    publish(pb, w.lane, pf, alpha);
}

// Steady step of an S wave.  On entry `sacc` / `hold` describe the pending block (its chain without
// the held-back MFMAs).  The step requests the first operands of the block in stage `st`, issues
// the held-back MFMAs, then forms the new block's chain (up to its own held-back MFMAs) with the
// exponentials of the pending block between the MFMAs, and publishes those weights to `pb` a few
// MFMAs before the end, so that the LDS writes have completed when the wave reaches the barrier.
// LDS operands are requested LA_S MFMAs ahead in order of use: each MFMA waits for exactly its own.
template <int DZ>
__device__ __forceinline__ void s_step(SWave<DZ> &w, f32x16 &sacc, bf16x8 (&hold)[kHoldS], const char *st, char *pb)
{
    using C = WsCfg<DZ>;
    constexpr int N = C::KS, NM = N - kHoldS;
    constexpr int kFirstExp = 2;                         // the held-back MFMAs need a moment to finish
    constexpr int kPublish = NM >= 8 ? NM - 4 : NM - 1;  // MFMA slot in which the weights are published
    static_assert(NM > kFirstExp && kPublish >= kFirstExp, "not enough MFMAs to spread the softmax over");
    const float m_use = w.m_ref == -INFINITY ? 0.f : w.m_ref;
    bf16x8 fr[C::RING_S];
    f32x16 snew = load_bias(w.ad, st);
#pragma unroll
    for (int j = 0; j < C::LA_S; ++j) fr[j] = load_s<DZ>(w.ad, st, j);
    __builtin_amdgcn_sched_barrier(0);
    s_held<DZ>(w, sacc, hold);
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 pn[2];
    unsigned pp[8];
    float ex[16];
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < NM; ++j) {
        {
            const int jn = j + C::LA_S;
            if (jn < NM)
                fr[jn % C::RING_S] = load_s<DZ>(w.ad, st, jn);
            else if (jn < N)
                hold[jn - NM] = load_s<DZ>(w.ad, st, jn);
        }
        snew = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % C::RING_S], w.qf[j], snew, 0, 0, 0);
        // softmax slices of the pending block, spread over the MFMA slots kFirstExp .. kPublish:
        // the 16 exponentials (pairs are rounded to bf16 together)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (kFirstExp + (r * (kPublish - kFirstExp + 1)) / 16 != j) continue;
            ex[r] = __builtin_amdgcn_exp2f(sacc[r] - m_use);
            // (the empty asm keeps the value here: the rare path below recomputes it, and the
            // optimiser would otherwise move this work behind the MFMAs)
            asm volatile("" : "+v"(ex[r]));
            if (r & 1) {
                pp[r >> 1] = pack_pair(ex[r - 1], ex[r], psum);
                asm volatile("" : "+v"(pp[r >> 1]), "+v"(psum));
            }
        }
        if (j == kPublish) {
            pn[0] = __builtin_bit_cast(bf16x8, (u32x4){pp[0], pp[1], pp[2], pp[3]});
            pn[1] = __builtin_bit_cast(bf16x8, (u32x4){pp[4], pp[5], pp[6], pp[7]});
            float alpha = 1.f;
            // psum <= 2^kTau bounds every weight of the block; a larger (or infinite) sum means the
            // reference is too small for this block
            if (__any(!(psum <= kTauPow) || w.m_ref == -INFINITY)) {  // (no reference yet: take the block's maximum)
                alpha = raise_reference<DZ>(w, row_max16(sacc));
                psum = 0.f;
                exp_block(sacc, w.m_ref == -INFINITY ? 0.f : w.m_ref, pn, psum);
            }
            w.l_run += psum;
            publish(pb, w.lane, pn, alpha);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    sacc = snew;
}

// ---- PV wave ---------------------------------------------------------------------------------------
template <int DZ>
struct PvWave {
    using C = WsCfg<DZ>;
    f32x16 oacc[C::NB];
    LaneAddr ad;
    int lane;
};

// O^T += V^T P^T for the block in stage `st` with the weights published at `pb`.  The step first
// requests those weights and the first operands, then issues the held-back MFMAs of the previous
// block (operands `hold`, weights `pf_old`, both in registers), applies the rescale factor that
// came with the new weights (rare), and forms the new block's products -- all of them when LAST,
// else all but the last kHoldPV, whose operands it leaves in `hold` (and the weights in `pf_old`).
// When DMA is set the load entries of a block go out between the MFMAs, into the stage at LDS
// address `st_dma`: the next block of the sequence (adv = 1) or, when the sequence has no further
// block, the previously requested one again (adv = 0: same bytes to the same place, which keeps
// the number of loads per iteration, and with it the wait counts, the same for every iteration).
template <int DZ, bool DMA, bool LAST>
__device__ __forceinline__ void pv_step(PvWave<DZ> &w, bf16x8 (&hold)[kHoldPV], bf16x8 (&pf_old)[2], const char *st,
                                        const char *pb, Dma<DZ> &dma, unsigned st_dma, int adv)
{
    using C = WsCfg<DZ>;
    constexpr int N = C::NPV, NM = LAST ? N : N - kHoldPV;
    bf16x8 pf[2];
    pf[0] = *reinterpret_cast<const bf16x8 *>(pb + w.lane * 16);
    pf[1] = *reinterpret_cast<const bf16x8 *>(pb + 1024 + w.lane * 16);
    const float alpha = *reinterpret_cast<const float *>(pb + 2048 + (w.lane & 31) * 4);
    bf16x8 fr[C::RING_PV];
#pragma unroll
    for (int j = 0; j < C::LA_PV; ++j) fr[j] = load_pv<DZ>(w.ad, st, j);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int h = 0; h < kHoldPV; ++h) {
        constexpr int i0 = N - kHoldPV;
        w.oacc[pv_nb<DZ>(i0 + h)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hold[h], pf_old[pv_tt<DZ>(i0 + h)],
                                                                              w.oacc[pv_nb<DZ>(i0 + h)], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (__any(alpha != 1.f)) {
        // rare: the S wave raised its reference for this block
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) w.oacc[nb][r] *= alpha;
            __builtin_amdgcn_sched_barrier(0);  // one block at a time: keeps the register demand of this rare path small
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NM; ++i) {
        {
            const int in = i + C::LA_PV;
            if (in < NM)
                fr[in % C::RING_PV] = load_pv<DZ>(w.ad, st, in);
            else if (in < N)
                hold[in - NM] = load_pv<DZ>(w.ad, st, in);
        }
        if constexpr (DMA) dma_slot<DZ>(dma, st_dma, adv, i);
        w.oacc[pv_nb<DZ>(i)] =
            __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % C::RING_PV], pf[pv_tt<DZ>(i)], w.oacc[pv_nb<DZ>(i)], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (!LAST) {
        pf_old[0] = pf[0];
        pf_old[1] = pf[1];
    }
}

// Accesses to the exchange buffer of the key-range split: 16-byte buffer accesses with the sc1
// cache-policy bit, which makes a store write through to, and a load read from, the device's
// coherence point instead of the non-coherent caches, so that a part sees what a part on
// another compute unit (or XCD) wrote once that part's stores have completed.
constexpr int kXchgPolicy = 16;  // sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t xchg_resource(float *base)
{
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, 0x7fffffff, 0x00020000);  // raw dword buffer
}
__device__ __forceinline__ void xchg_store(__amdgpu_buffer_rsrc_t rs, int off, f32x4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), rs, off, 0, kXchgPolicy);
}
__device__ __forceinline__ f32x4 xchg_load(__amdgpu_buffer_rsrc_t rs, int off)
{
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, kXchgPolicy));
}

// What the epilogue needs to know about the unit of work.
struct Unit {
    int b, bh, qt, irow, part, nparts, tile_local;
};

// Split, inverse frame, z1 contraction (Algorithm 1 steps 8-9, Eq. 4) on the accumulator of a PV
// wave, for c = 16, N_value = 8 and BPS = c_z / 32 column blocks per factor slice; the key-range-split
// exchange when the unit is a part.  z1l: this lane's staged z1 row in LDS.
template <int DZ, int BPS>
__device__ __forceinline__ void epilogue(const AttnParams &p, const Unit &u, PvWave<DZ> &w, float m_ref, float l_tot,
                                         const char *z1_rows)
{
    using C = WsCfg<DZ>;
    constexpr int c = 16, Pv = 8;
    constexpr int NZB = C::NB - C::NBH;  // 32-column blocks of the pair part
    static_assert(NZB % BPS == 0, "factor slices tile the pair part");
    constexpr int cz = 32 * BPS;
    const int lane = w.lane, li = lane & 31, g = lane >> 5;
    const int wave = (threadIdx.x >> 6) & 3;
    f32x16(&oacc)[C::NB] = w.oacc;
    const bool in_range = u.irow < p.L;
    const int irow_c = min(u.irow, p.L - 1);  // rows past the end compute on a valid address and store nothing
    // point part: this half owns points 4g .. 4g+3, hi parts in slots u = 0..11, lo parts in
    // slots 12..23; slot u sits in column 16 + 8*(u/4) + 4g + u%4 (see v_pt_col)
    float Gv[12];
#pragma unroll
    for (int s = 0; s < 12; ++s) {
        const int dh = 16 + 8 * (s >> 2) + (s & 3);  // column for g = 0; g = 1 adds 4
        const int dl = 16 + 8 * ((s + 12) >> 2) + ((s + 12) & 3);
        const float hi = oacc[dh >> 5][4 * ((dh & 31) >> 3) + (dh & 3)];
        const float lo = oacc[dl >> 5][4 * ((dl & 31) >> 3) + (dl & 3)];
        Gv[s] = hi + lo;
    }
    float sc8[8];  // scalar columns 8a + 4g + x, a = 0, 1
#pragma unroll
    for (int r = 0; r < 8; ++r) sc8[r] = oacc[0][r];
    // pair part: o~[d'] = sum_rho z1[rho, d'] * U[rho, d']; the lane holds columns 8a + 4g + x
    f32x16 pr[BPS];
    {
        constexpr int kCpr = DZ / 8;
        const char *z1l = z1_rows + li * (DZ * 2) + 8 * g;
#pragma unroll
        for (int zb = 0; zb < NZB; ++zb)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                // columns 32 zb + 8 a + 4 g .. + 3 of row li: half g of chunk 4 zb + a
                const uint2 zraw = *reinterpret_cast<const uint2 *>(z1l + 16 * ((4 * zb + a) ^ (li % kCpr)));
                const bf16_t *zb16 = reinterpret_cast<const bf16_t *>(&zraw);
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const float t = oacc[C::NBH + zb][4 * a + x] * bf2f(zb16[x]);
                    // sum over rho: column dz of U belongs to output d' = dz % cz
                    if (zb < BPS)
                        pr[zb][4 * a + x] = t;
                    else
                        pr[zb % BPS][4 * a + x] += t;
                }
            }
    }

    // ---- key-range split: leave this part's unnormalised row in memory; the part that arrives
    // last merges all parts of the tile.  A part's words are complete (vmcnt = 0) before it takes
    // its ticket.
    if (u.nparts > 1) {
        // per lane: 2 groups of scalars, 3 of point coordinates, 1 of (m, l), 4 per pair block
        constexpr int groups = 6 + 4 * BPS;
        // wave-uniform base: this row group's rows in part 0 of the tile; byte offsets within 32 bits
        const __amdgpu_buffer_rsrc_t xr =
            xchg_resource(p.partial + ((size_t)u.tile_local * u.nparts * 4 + wave) * (groups * 64 * 4));
        constexpr int kPartBytes = 4 * groups * 64 * 16;
        const int mine = u.part * kPartBytes + lane * 16;
        xchg_store(xr, mine + 0 * 1024, (f32x4){sc8[0], sc8[1], sc8[2], sc8[3]});
        xchg_store(xr, mine + 1 * 1024, (f32x4){sc8[4], sc8[5], sc8[6], sc8[7]});
#pragma unroll
        for (int a = 0; a < 3; ++a)
            xchg_store(xr, mine + (2 + a) * 1024, (f32x4){Gv[4 * a], Gv[4 * a + 1], Gv[4 * a + 2], Gv[4 * a + 3]});
        xchg_store(xr, mine + 5 * 1024, (f32x4){m_ref, l_tot, 0.f, 0.f});
#pragma unroll
        for (int zb = 0; zb < BPS; ++zb)
#pragma unroll
            for (int a = 0; a < 4; ++a)
                xchg_store(xr, mine + (6 + 4 * zb + a) * 1024,
                           (f32x4){pr[zb][4 * a], pr[zb][4 * a + 1], pr[zb][4 * a + 2], pr[zb][4 * a + 3]});
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        int ticket = 0;
        if (lane == 0)
            ticket = __hip_atomic_fetch_add(p.counters + u.tile_local * 4 + wave, 1, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);
        ticket = __builtin_amdgcn_readfirstlane(ticket);
        if (ticket != u.nparts - 1) return;
        asm volatile("" ::: "memory");
        // Merge all parts in the order of their key ranges, this wave's own included (read
        // back), so that the result does not depend on which part happened to come last.
        float m_acc = -INFINITY;
        l_tot = 0.f;
#pragma unroll
        for (int r = 0; r < 8; ++r) sc8[r] = 0.f;
#pragma unroll
        for (int s = 0; s < 12; ++s) Gv[s] = 0.f;
#pragma unroll
        for (int zb = 0; zb < BPS; ++zb)
#pragma unroll
            for (int r = 0; r < 16; ++r) pr[zb][r] = 0.f;
        for (int q = 0; q < u.nparts; ++q) {
            const int other = q * kPartBytes + lane * 16;
            f32x4 head[6], pair[BPS][4];
#pragma unroll
            for (int k = 0; k < 6; ++k) head[k] = xchg_load(xr, other + k * 1024);
#pragma unroll
            for (int zb = 0; zb < BPS; ++zb)
#pragma unroll
                for (int a = 0; a < 4; ++a) pair[zb][a] = xchg_load(xr, other + (6 + 4 * zb + a) * 1024);
            const float m_o = head[5][0], l_o = head[5][1];
            const float m_new = fmaxf(m_acc, m_o);
            const float a_own = m_acc == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_acc - m_new);
            const float a_oth = m_o == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_o - m_new);
            m_acc = m_new;
            l_tot = l_tot * a_own + l_o * a_oth;
#pragma unroll
            for (int r = 0; r < 8; ++r) sc8[r] = sc8[r] * a_own + head[r >> 2][r & 3] * a_oth;
#pragma unroll
            for (int s = 0; s < 12; ++s) Gv[s] = Gv[s] * a_own + head[2 + (s >> 2)][s & 3] * a_oth;
#pragma unroll
            for (int zb = 0; zb < BPS; ++zb)
#pragma unroll
                for (int r = 0; r < 16; ++r) pr[zb][r] = pr[zb][r] * a_own + pair[zb][r >> 2][r & 3] * a_oth;
        }
        m_ref = m_acc;
    }

    // ---- normalise, apply the inverse frame, store ---------------------------------------------
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    const float lse2 = l_tot > 0.f ? m_ref + __log2f(l_tot) : -INFINITY;
    const int h = u.bh - u.b * p.H;
    const bool valid = (p.mask ? p.mask[(size_t)u.b * p.L + irow_c] != 0 : true) && l_tot > 0.f;
    const float sc = valid ? inv : 0.f;
    const size_t row = ((size_t)u.b * p.L + irow_c) * p.H + h;
    if (in_range) {
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            f32x4 out;
#pragma unroll
            for (int x = 0; x < 4; ++x) out[x] = sc8[4 * a + x] * sc;
            *reinterpret_cast<f32x4 *>(p.o + row * c + 8 * a + 4 * g) = out;
        }
    }
    {
        const float *R = p.rot + ((size_t)u.b * p.L + irow_c) * 9;
        const float *tr = p.trans + ((size_t)u.b * p.L + irow_c) * 3;
        float Rm[9], tc[3];
#pragma unroll
        for (int a = 0; a < 9; ++a) Rm[a] = R[a];
#pragma unroll
        for (int a = 0; a < 3; ++a) tc[a] = tr[a] - p.cen[4 * u.b + a];
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
        }
    }
    if (in_range) {
        float *dst = p.o_pair + row * cz;
#pragma unroll
        for (int zb = 0; zb < BPS; ++zb)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 out;
#pragma unroll
                for (int x = 0; x < 4; ++x) out[x] = pr[zb][4 * a + x] * sc;
                *reinterpret_cast<f32x4 *>(dst + 32 * zb + 8 * a + 4 * g) = out;
            }
        if (p.lse && g == 0)
            p.lse[(size_t)u.bh * p.L + u.irow] = valid ? lse2 * kLn2 - p.qbias[(size_t)u.bh * p.Lp + u.irow] : 0.f;
    }
}

template <int DZ>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void fipa_attn_fwd_ws_kernel(AttnParams p)
{
    using C = WsCfg<DZ>;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of work
    // units so that the query tiles of one (batch, head) share that XCD's L2 copy of k^ and v^.
    // The first plan.full workgroups take whole tiles; the others take one of the plan.S key-range
    // parts of a remaining tile (the parts of a tile are neighbours in the launch order).
    // In a mixed launch (see SplitPlan) the last 512 workgroups alternate, per XCD, between runs of
    // 16 whole tiles and 16 parts.
    Unit u;
    u.part = 0;
    u.tile_local = 0;
    u.nparts = 1;
    int logical;
    int wg = blockIdx.x;        // position in the plain order: whole tiles, then parts
    if (p.plan.mixed && wg >= p.plan.full - 256) {
        const int i = wg - (p.plan.full - 256), x = i % 8, j = i / 8;  // XCD, slot 0..63
        const int run = j / 16, k = j % 16 + 16 * (run / 2);            // k-th whole tile / part of this XCD's 32
        wg = (run % 2 == 0 ? p.plan.full - 256 : p.plan.full) + 8 * k + x;
    }
    if (wg < p.plan.full) {
        logical = (wg % 8) * (p.plan.full / 8) + wg / 8;
    } else {
        u.nparts = p.plan.S;
        const int uu = wg - p.plan.full, n_units = p.plan.rem * u.nparts;
        if (uu >= n_units) return;
        const int lin = n_units % 8 == 0 ? (uu % 8) * (n_units / 8) + uu / 8 : uu;
        u.tile_local = lin / u.nparts;
        u.part = lin - u.tile_local * u.nparts;
        logical = p.plan.full + u.tile_local;
    }
    const int bh_pos = logical / p.nQT;
    u.qt = logical - bh_pos * p.nQT;
    u.bh = p.deal ? dealt_pair_by_length(bh_pos, p.kvlen, p.B, p.H, threadIdx.x & 63) : bh_pos;
    u.b = u.bh / p.H;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool s_role = wave8 < 4;   // waves 0-3: S waves, waves 4-7: PV waves
    const int rg = wave8 & 3;        // row group
    const int li = lane & 31, g = lane >> 5;
    const int b = u.b, bh = u.bh, qt = u.qt, part = u.part, nparts = u.nparts;
    // (without a mask every chain has L residues: no dependent load in front of everything else)
    const int kvlen = p.deal ? p.kvlen[b] : p.L;
    const int nkb = (kvlen + kBlk - 1) / kBlk;      // key blocks of this chain
    const int irow = qt * kTileQ + rg * 32 + li;    // < Lp always
    u.irow = irow;

    // A tile whose rows all lie past the last valid residue of its chain (padding of a ragged
    // batch) has nothing to attend from: its outputs are zero by definition.
    if (qt * kTileQ >= kvlen) {
        if (!s_role && irow < p.L && part == 0) {
            const size_t row = ((size_t)b * p.L + irow) * p.H + (bh - b * p.H);
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int a = 0; a < 2; ++a) *reinterpret_cast<f32x4 *>(p.o + row * 16 + 8 * a + 4 * g) = zero;
#pragma unroll
            for (int a = 0; a < 3; ++a) *reinterpret_cast<f32x4 *>(p.o_pts + row * 24 + 12 * g + 4 * a) = zero;
            for (int d = 4 * g; d < p.cz; d += 8) *reinterpret_cast<f32x4 *>(p.o_pair + row * p.cz + d) = zero;
            if (p.lse && g == 0) p.lse[(size_t)bh * p.L + irow] = 0.f;
        }
        return;
    }

    // Key blocks are visited starting at the block that holds the tile's own residues and
    // wrapping around.  With distance-dominated logits the row maximum sits near the diagonal,
    // so the reference maximum is found in the first blocks and is rarely raised afterwards.
    // A key-range part takes its share of that rotated sequence: positions pos0 .. pos0 + nblk - 1.
    // The first part gets a quarter of a share more than the others: it holds the diagonal blocks
    // and never has to raise its softmax reference, while the others may.
    const int pos0 = part == 0 ? 0 : (4 * part + 1) * nkb / (4 * nparts + 1);
    const int pos1 = part + 1 == nparts ? nkb : (4 * part + 5) * nkb / (4 * nparts + 1);
    const int nblk = pos1 - pos0;  // key blocks this workgroup processes
    // A part walks its range away from the diagonal too: upwards from its first position when
    // that end is the nearer one (always so for a whole tile), downwards from its last otherwise.
    const bool downwards = pos0 > nkb - (pos0 + nblk);
    const int dir = downwards ? -1 : 1;
    int first_blk = min(qt * (kTileQ / kBlk), max(nkb - 1, 0)) + (downwards ? pos0 + nblk - 1 : pos0);
    if (first_blk >= nkb) first_blk -= nkb;  // (nkb = 0: stays 0 and is never used)
    const int wrap_at = downwards ? -1 : nkb, wrap_to = downwards ? nkb - 1 : 0;
    // waves 1-3 of a whole tile (or of its first part) take their first reference from their own diagonal block
    const bool diag = pos0 == 0 && !downwards && nblk >= 4;

    const unsigned smem_lds = lds_address(smem);
    char *pbuf = smem + C::PB_OFF + rg * C::PB_RG;  // + (block & 1) * PB_BUF
    float *stats = reinterpret_cast<float *>(smem + C::ST_OFF) + rg * 64;

    if (s_role) {
        // =========================== S wave ===========================================================
        SWave<DZ> w;
        w.lane = lane;
        w.ad = lane_addresses<DZ>(lane);
        w.m_ref = -INFINITY;
        w.l_run = 0.f;
        // q^ row fragments: features 16*ks + 8*g .. +7 of row irow, loaded straight into accumulation
        // registers (the MFMA reads its B operand from there).  The loads are invisible to the
        // compiler's wait-count bookkeeping; the wait_vmem<0>() below covers them, and the empty asm
        // after it orders every use behind that wait.
        {
            const bf16_t *qh = p.Qh + ((size_t)bh * p.Lp + irow) * kDH;
#pragma unroll
            for (int ks = 0; ks < C::KSH; ++ks)
                asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(w.qf[ks]) : "v"(qh + ks * 16 + 8 * g) : "memory");
        }
        // The pair part of q^ -- the bias vector b^{h1} = log2e * w_L * w_b[h] (.) z1 of Algorithm 1
        // steps 2-3 -- is formed here from z1, which all heads of a residue share.  This wave's 32 z1
        // rows go to LDS as whole rows (coalesced), the 16-byte chunks of row r stored at position
        // chunk ^ (r mod chunks-per-row) so that the reads below -- one chunk index across 32 rows --
        // spread over the banks.  The per-head scale vector goes to LDS as well.
        constexpr int kRowBytes = DZ * 2, kWaveBytes = 32 * kRowBytes, kCpr = DZ / 8;
        {
            const char *zbase = reinterpret_cast<const char *>(p.z1 + (size_t)b * p.L * DZ);
            const int row0 = qt * kTileQ + rg * 32;
#pragma unroll
            for (int k = 0; k < kWaveBytes / 1024; ++k) {
                const int slot = 64 * k + lane, r = slot / kCpr, c = (slot % kCpr) ^ (r % kCpr);
                int voff = min(row0 + r, p.L - 1) * kRowBytes + 16 * c;
                dma16<0>(zbase, voff, 0, smem_lds + C::Z1P_OFF + rg * kWaveBytes + 1024 * k);
            }
            if (tid < DZ)
                reinterpret_cast<float *>(smem + C::CW_OFF)[tid] =
                    kLog2e * p.w_L * p.w_b[(size_t)(bh - b * p.H) * p.cz + tid % p.cz];
        }
        wait_vmem<0>();
        wait_lgkm0();
        wg_barrier();  // B1: z1 rows, scale vector and the first two key blocks are in LDS
        {
            // q^ pair part: bf16(scale[col] * z1[row, col]); rows that do not exist or are masked get 0
            const bool ok = irow < p.L && (p.mask ? p.mask[(size_t)b * p.L + irow] != 0 : true);
            const unsigned keep = ok ? 0xFFFFFFFFu : 0u;
            const float *cw = reinterpret_cast<const float *>(smem + C::CW_OFF) + 8 * g;
            const char *z1l = smem + C::Z1P_OFF + rg * kWaveBytes + li * kRowBytes;
#pragma unroll
            for (int ks = 0; ks < C::KSZ; ++ks) {
                const f32x4 w0 = *reinterpret_cast<const f32x4 *>(cw + 16 * ks);
                const f32x4 w1 = *reinterpret_cast<const f32x4 *>(cw + 16 * ks + 4);
                // features 16 ks + 8 g .. + 7 of row li: chunk 2 ks + g
                const uint4 zr = *reinterpret_cast<const uint4 *>(z1l + 16 * ((2 * ks + g) ^ (li % kCpr)));
                const unsigned zw[4] = {zr.x, zr.y, zr.z, zr.w};  // two bf16 values each
                unsigned pk[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const float wl = x < 2 ? w0[2 * x] : w1[2 * x - 4], wh = x < 2 ? w0[2 * x + 1] : w1[2 * x - 3];
                    const float lo = wl * __uint_as_float(zw[x] << 16), hi = wh * __uint_as_float(zw[x] & 0xFFFF0000u);
                    // (round to nearest even, as the pack kernel's conversion; one v_cvt_pk_bf16_f32)
                    pk[x] = __builtin_bit_cast(unsigned, __builtin_convertvector((f32x2){lo, hi}, bf16x2)) & keep;
                }
                w.qf[C::KSH + ks] = __builtin_bit_cast(bf16x8, (u32x4){pk[0], pk[1], pk[2], pk[3]});
            }
        }
        wait_lgkm0();
        wg_barrier();  // B2: the z1 rows have been consumed (key block 3 goes where they sat)
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) asm volatile("" : "+v"(w.qf[ks]));
        f32x16 sacc;
        bf16x8 hold[kHoldS];
        if (nblk > 0) {
            sacc = s_block<DZ>(w, smem);
            float mx = row_max16(sacc);
            if (diag) {
                wg_barrier();  // B3: blocks 2 and 3 have landed
                if (rg > 0) mx = fmaxf(mx, row_max16(s_block<DZ>(w, smem + rg * C::STAGE)));
            }
            w.m_ref = mx;
            bf16x8 pf[2];
            float psum = 0.f;
            exp_block(sacc, mx == -INFINITY ? 0.f : mx, pf, psum);
            w.l_run = psum;
            publish(pbuf, lane, pf, 1.f);
            if (nblk > 1) s_start<DZ>(w, sacc, hold, smem + C::STAGE);  // block 1 becomes the pending block
        }
        int st = 2;  // stage of block t
        for (int t = 2; t < nblk + 2; ++t) {
            wait_lgkm0();
            wg_barrier();  // block t has landed; the weights of block t-2 are published
            char *pb = pbuf + ((t - 1) & 1) * C::PB_BUF;
            if (t < nblk)
                s_step<DZ>(w, sacc, hold, smem + st * C::STAGE, pb);
            else if (t == nblk)
                s_finish<DZ>(w, sacc, hold, pb);
            st = st + 1 < C::NSTAGE ? st + 1 : 0;
        }
        const float l_tot = w.l_run + __shfl_xor(w.l_run, 32);
        if (lane < 32) {
            stats[2 * lane] = w.m_ref;
            stats[2 * lane + 1] = l_tot;
        }
        wait_lgkm0();
        wg_barrier();  // BF: the rows' final reference and weight sum are in LDS
        return;
    }

    // =============================== PV wave ==========================================================
    PvWave<DZ> w;
    w.lane = lane;
    w.ad = lane_addresses<DZ>(lane);
    Dma<DZ> dma;
    dma.base = p.ws_base;
    {
        const unsigned z2_off = (unsigned)(reinterpret_cast<const char *>(p.Z2 + (size_t)b * p.Lp * DZ) - p.ws_base);
        const unsigned kh_off = (unsigned)(reinterpret_cast<const char *>(p.Kh + (size_t)bh * p.Lp * kDH) - p.ws_base);
        const unsigned vh_off = (unsigned)(reinterpret_cast<const char *>(p.Vh + (size_t)bh * p.Lp * kDH) - p.ws_base);
        const unsigned kb_off = (unsigned)(reinterpret_cast<const char *>(p.kbias + (size_t)bh * p.Lp) - p.ws_base);
#pragma unroll
        for (int k = 0; k < C::NEW; ++k) {
            int e = rg + 4 * k;
            if (e >= C::NE) e = 0;
            dma.lds_off[k] = 1024u * e;
            const int s = 64 * e + lane;
            unsigned off = z2_off;   // slots in the row padding or past the last slot fetch the first 16 bytes of the z2 block
            int step = kBlk * DZ * 2;
            if (s < C::Z_SLOTS) {
                const int row = s / C::Z_SPR, col = s - row * C::Z_SPR;
                if (col < DZ / 8) off = z2_off + row * (DZ * 2) + col * 16;
            } else if (s < C::Z_SLOTS + 2 * C::H_SLOTS) {
                const bool isk = s < C::Z_SLOTS + C::H_SLOTS;
                const int s2 = s - C::Z_SLOTS - (isk ? 0 : C::H_SLOTS);
                const int row = s2 / C::H_SPR, col = s2 - row * C::H_SPR;
                if (col < kDH / 8) {
                    off = (isk ? kh_off : vh_off) + row * (kDH * 2) + col * 16;
                    step = kBlk * kDH * 2;
                }
            } else if (s < C::SLOTS) {
                off = kb_off + (s - C::Z_SLOTS - 2 * C::H_SLOTS) * 16;
                step = kBlk * 4;
            }
            dma.vstep[k] = dir * step;
            // one block before the first block: every request advances the offset first
            dma.voff[k] = (int)off + (first_blk * dir - 1) * dma.vstep[k];
        }
    }
    int next_blk = first_blk;  // next key block to request
    int requested = 0;         // blocks requested so far
    auto request = [&](int stage) {
        if (next_blk == wrap_at) {
            dma_wrap<DZ>(dma, nkb);
            next_blk = wrap_to;
        }
        issue_block<DZ>(dma, smem_lds + stage * C::STAGE);
        next_blk += dir;
        requested += 1;
    };
    if (nblk > 0) request(0);
    if (nblk > 1) request(1);
#pragma unroll
    for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) w.oacc[nb][r] = 0.f;
    wait_vmem<0>();
    wg_barrier();  // B1
    wg_barrier();  // B2
    if (nblk > 2) request(2);
    if (nblk > 3) request(3);
    if (nblk > 0 && diag) {
        wait_vmem<0>();
        wg_barrier();  // B3
    }
    int st = 2;       // stage of block t
    int z1_off = 0;   // where this wave's z1 rows are staged for the epilogue
    bf16x8 hold[kHoldPV], pf_old[2];  // held-back operands and weights of the previous block: none yet
#pragma unroll
    for (int h = 0; h < kHoldPV; ++h)
#pragma unroll
        for (int x = 0; x < 8; ++x) hold[h][x] = (__bf16)0.f;
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int x = 0; x < 8; ++x) pf_old[h][x] = (__bf16)0.f;
    int st_req = requested > 0 ? requested - 1 : 0;  // stage of the block requested last
    int t = 2;
    // Block t must have landed before the barrier of iteration t; the loads requested after it (one
    // block's worth: block 3 here, later what the previous iteration requested) may still be on their way.
    if (nblk > 3)
        wait_vmem<C::NEW>();
    else
        wait_vmem<0>();
    for (; t < nblk; ++t) {
        wg_barrier();
        const int s_pv = st >= 2 ? st - 2 : st + C::NSTAGE - 2;             // stage of block t-2
        const char *pb = pbuf + (t & 1) * C::PB_BUF;
        const int adv = t + 2 < nblk ? 1 : 0;
        if (adv) {
            if (next_blk == wrap_at) {
                dma_wrap<DZ>(dma, nkb);
                next_blk = wrap_to;
            }
            next_blk += dir;
            st_req = st_req + 1 < C::NSTAGE ? st_req + 1 : 0;  // (= the stage of block t-3, free since the barrier)
        }
        pv_step<DZ, true, false>(w, hold, pf_old, smem + s_pv * C::STAGE, pb, dma, smem_lds + st_req * C::STAGE, adv);
        st = st + 1 < C::NSTAGE ? st + 1 : 0;
        wait_vmem<C::NEW>();  // block t+1 (requested an iteration ago or earlier)
        wait_lgkm0();         // the held-back operands are in registers before their stage is given up
    }
    if (nblk > 0) {
        // iteration t = max(nblk, 2): every key block has landed and the three stages after the last
        // block are free: this wave's 32 z1 rows (for the contraction of step 9) go there while the last
        // blocks are being multiplied.  Row-major with the 16-byte chunks of row r stored at position
        // chunk ^ (r mod chunks-per-row).
        wait_vmem<0>();
        wg_barrier();
        {
            constexpr int kRowBytes = DZ * 2, kWaveBytes = 32 * kRowBytes, kCpr = DZ / 8;
            const int f0 = nblk % C::NSTAGE;                                   // first free stage (cyclically)
            const int room = min(C::NSTAGE - f0, 3) * C::STAGE;                // free bytes before the ring wraps
            const int n_head = min(4, room / kWaveBytes);                     // waves that fit there; the rest start at 0
            z1_off = rg < n_head ? f0 * C::STAGE + rg * kWaveBytes : (rg - n_head) * kWaveBytes;
            const char *zbase = reinterpret_cast<const char *>(p.z1 + (size_t)b * p.L * DZ);
            const int row0 = qt * kTileQ + rg * 32;
#pragma unroll
            for (int k = 0; k < kWaveBytes / 1024; ++k) {
                const int slot = 64 * k + lane, r = slot / kCpr, c = (slot % kCpr) ^ (r % kCpr);
                int voff = min(row0 + r, p.L - 1) * kRowBytes + 16 * c;
                dma16<0>(zbase, voff, 0, smem_lds + z1_off + 1024 * k);
            }
        }
        if (nblk > 1) {
            // the last block but one, then (iteration nblk + 1) the last block
            const int s_pv = st >= 2 ? st - 2 : st + C::NSTAGE - 2;
            pv_step<DZ, false, false>(w, hold, pf_old, smem + s_pv * C::STAGE, pbuf + (t & 1) * C::PB_BUF, dma, 0u, 0);
            st = st + 1 < C::NSTAGE ? st + 1 : 0;
            ++t;
            wait_lgkm0();
            wg_barrier();
        }
        {
            const int s_pv = st >= 2 ? st - 2 : st + C::NSTAGE - 2;
            pv_step<DZ, false, true>(w, hold, pf_old, smem + s_pv * C::STAGE, pbuf + (t & 1) * C::PB_BUF, dma, 0u, 0);
        }
    }
    float m_ref = -INFINITY, l_tot = 0.f;
    wg_barrier();  // BF
    if (nblk > 0) {
        m_ref = stats[2 * li];
        l_tot = stats[2 * li + 1];
    } else {
        // (an empty part: nothing was staged; stage this wave's z1 rows now, the contraction reads them)
        constexpr int kRowBytes = DZ * 2, kWaveBytes = 32 * kRowBytes, kCpr = DZ / 8;
        z1_off = rg * kWaveBytes;
        const char *zbase = reinterpret_cast<const char *>(p.z1 + (size_t)b * p.L * DZ);
        const int row0 = qt * kTileQ + rg * 32;
#pragma unroll
        for (int k = 0; k < kWaveBytes / 1024; ++k) {
            const int slot = 64 * k + lane, r = slot / kCpr, c = (slot % kCpr) ^ (r % kCpr);
            int voff = min(row0 + r, p.L - 1) * kRowBytes + 16 * c;
            dma16<0>(zbase, voff, 0, smem_lds + z1_off + 1024 * k);
        }
    }
    wait_vmem<0>();  // the z1 rows staged above (this wave's own loads, no barrier needed)
    asm volatile("" ::: "memory");
    switch (p.cz) {
        case 32:
            if constexpr (DZ >= 32) epilogue<DZ, 1>(p, u, w, m_ref, l_tot, smem + z1_off);
            break;
        case 64:
            if constexpr (DZ >= 64) epilogue<DZ, 2>(p, u, w, m_ref, l_tot, smem + z1_off);
            break;
        case 128:
            if constexpr (DZ >= 128) epilogue<DZ, 4>(p, u, w, m_ref, l_tot, smem + z1_off);
            break;
        case 256:
            if constexpr (DZ >= 256) epilogue<DZ, 8>(p, u, w, m_ref, l_tot, smem + z1_off);
            break;
        default: break;
    }
}

template <int DZ>
hipError_t launch(const AttnParams &p, hipStream_t stream)
{
    using C = WsCfg<DZ>;
    static LdsLimit lds_limit;
    hipError_t e = raise_lds_limit(lds_limit, (const void *)fipa_attn_fwd_ws_kernel<DZ>, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    if (p.plan.full % 8 != 0 || p.plan.full + p.plan.rem != p.total_tiles || p.plan.S < 1 || p.cz < 32 ||
        p.cz % 32 != 0 || DZ % p.cz != 0 || !p.ws_base)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL((fipa_attn_fwd_ws_kernel<DZ>), dim3(p.plan.units()), dim3(512), C::LDS_BYTES, stream, p);
    return hipGetLastError();
}

}  // namespace

// Shapes this kernel is built for: the AlphaFold2 head shape (fused epilogue), c_z a power of two >= 32.
bool attn_fwd_ws_supported(int DZ, int cz)
{
    return (DZ == 32 || DZ == 64 || DZ == 128 || DZ == 256) && (cz == 32 || cz == 64 || cz == 128 || cz == 256) &&
           DZ % cz == 0;
}

hipError_t launch_attn_fwd_ws_bf16(const AttnParams &p, int DZ, hipStream_t stream)
{
    switch (DZ) {
        case 32: return launch<32>(p, stream);
        case 64: return launch<64>(p, stream);
        case 128: return launch<128>(p, stream);
        case 256: return launch<256>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fipa
