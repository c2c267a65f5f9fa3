// Fused attention on the lifted features (Algorithm 1 step 7) for gfx950: online softmax over
// key blocks (the recurrences of Algorithm 2: running maximum m, running sum l, rescaled
// accumulator), bf16 MFMA 32x32x16 for both contractions, fp32 accumulation, and -- for the
// AlphaFold2-style head shape -- the split / inverse frame / z1 contraction of steps 8-9 on the
// accumulator registers, so the lifted output never goes to memory.
//
// Work split: one workgroup = one (batch, head, 128-query tile); each of its 4 waves owns 32
// query rows and keeps q^ (as MFMA B fragments) and the 32 x (64+DZ) output accumulator in
// registers for the whole key loop.  Key blocks of 32 residues are brought into a ring of LDS
// stages by direct global->LDS loads, two iterations ahead of their first use, and are shared
// by the four waves.  Both products are computed transposed,
//     S^T = K^ Q^T        (A = k^ rows from LDS, B = q^ registers)
//     O^T += V^T P^T      (A = v^ columns, read from the row-major block with the transposing
//                          LDS read, B = P^T registers)
// so that a lane owns one query row: the softmax statistics are per-lane scalars and the
// exponentiated S^T accumulator already has the layout of the B operand of the second
// product.  The pair-factor block z2 is stored once and read in both roles.
//
// The loop is software pipelined over three blocks: iteration n accumulates P V of block n,
// evaluates the exponentials of block n+1 (whose S^T was formed one iteration earlier) and
// forms S^T of block n+2.  The 2*KS MFMAs of an iteration are issued in a fixed order with
// their LDS operands fetched a few MFMAs ahead and the VALU work of the softmax cut into
// slices placed between them, so that it runs in the shadow of the matrix pipe.
//
// The softmax reference ("running maximum" m of Algorithm 2) is only raised when the weights of
// a block, taken against the current reference, sum to more than 2^kTau; until then nothing is
// rescaled.  The result is the same softmax: numerator and denominator carry the same factor
// 2^(m_true - m_ref), and fp32 / bf16 keep their relative precision over that range.
#include "fipa_gfx950.h"

namespace fipa {

namespace {

constexpr float kTau = 32.0f;
constexpr float kTauPow = 4294967296.0f;  // 2^kTau
constexpr int kBlk = 32;           // keys per LDS stage
constexpr int kHS = kDH * 2 + 16;  // LDS row stride (bytes) of the head-specific k^ / v^ blocks

template <int DZ>
struct AttnCfg {
    static constexpr int DV = kDH + DZ;
    static constexpr int KSZ = DZ / 16;      // k-steps of S^T over the pair part
    static constexpr int KSH = kDH / 16;     // k-steps over the head-specific part
    static constexpr int KS = KSZ + KSH;
    static constexpr int NB = DV / 32;       // 32-row blocks of O^T
    static constexpr int NBH = kDH / 32;     // of which head specific
    static constexpr int ZS = DZ * 2 + 48;   // LDS row stride of the z2 block: this pad keeps both
                                             // the row reads and the transposing reads conflict free
    static constexpr int Z_SPR = ZS / 16;    // 16-byte slots per row
    static constexpr int H_SPR = kHS / 16;
    static constexpr int NZ = (kBlk * Z_SPR + 63) / 64;  // wave-wide 1 KiB loads for the z2 block
    static constexpr int NH = (kBlk * H_SPR + 63) / 64;  // for one head block
    static constexpr int NI = NZ + 2 * NH;   // flat list of wave-wide loads: z2 | k^ head | v^ head
    static constexpr int NIW = (NI + 3) / 4; // per wave
    static constexpr int Z_OFF = 0;
    static constexpr int KH_OFF = NZ * 1024;
    static constexpr int VH_OFF = (NZ + NH) * 1024;
    static constexpr int KB_OFF = NIW * 4 * 1024;        // 32 per-key fp32 biases (a full 1 KiB load lands here)
    static constexpr int STAGE = KB_OFF + 1024;
    static constexpr int NSTAGE = 5 * STAGE <= 160 * 1024 ? 5 : 4;
    // Start-up of the fused kernel: the z1 rows of the tile (4 waves x 32 rows x 2 DZ bytes) pass
    // through LDS on their way into the query-side factor fragments.  They sit behind the first
    // three stages (which the first three key blocks fill meanwhile) and may reach past the ring.
    static constexpr int Z1P_OFF = 3 * STAGE;
    static constexpr int Z1P_END = Z1P_OFF + 4 * 32 * DZ * 2;
    static constexpr int CW_OFF = Z1P_END > NSTAGE * STAGE ? Z1P_END : NSTAGE * STAGE;  // per-head scale vector of the query-side factors (DZ floats)
    static constexpr int LDS_BYTES = CW_OFF + DZ * 4;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static constexpr int NOPS = 2 * KS;      // MFMAs per pipelined iteration (KS == 2*NB)
    static_assert(KS == 2 * NB, "S^T and P V use the same number of MFMAs per block");
    static constexpr int LA = 3;             // LDS operands are fetched LA MFMAs ahead of their use
    static constexpr int RING = LA + 1;      // operand buffers
    static_assert(KS > LA && NOPS % RING == 0, "pipeline depth");
    static constexpr int VM_PER_BLOCK = NIW + 1;          // vector-memory ops one wave issues per block
    static constexpr int DMA_EVERY = NOPS / (NIW + 1);   // one load entry every DMA_EVERY MFMAs
};

template <int DZ>
struct Wave {
    using C = AttnCfg<DZ>;
    bf16x8 qf[C::KS];
    f32x16 oacc[C::NB];
    float m_ref, l_run;
    int kaddr_h, kaddr_z, vaddr_h, vaddr_z, baddr;  // per-lane LDS offsets inside a stage
};

// S^T block (32 keys x 32 queries) of the stage at `st`, accumulator preset with the per-key bias.
template <int DZ>
__device__ __forceinline__ f32x16 s_block(const Wave<DZ> &w, const char *__restrict__ st)
{
    using C = AttnCfg<DZ>;
    f32x16 sacc;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const f32x4 bias = *reinterpret_cast<const f32x4 *>(st + w.baddr + a * 32);
#pragma unroll
        for (int x = 0; x < 4; ++x) sacc[4 * a + x] = bias[x];
    }
#pragma unroll
    for (int ks = 0; ks < C::KSH; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(st + w.kaddr_h + ks * 32);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, w.qf[ks], sacc, 0, 0, 0);
    }
#pragma unroll
    for (int ks = 0; ks < C::KSZ; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(st + w.kaddr_z + ks * 32);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, w.qf[C::KSH + ks], sacc, 0, 0, 0);
    }
    return sacc;
}

// One 32-row block of O^T += V^T P^T for the 32 keys of the stage at `st`.
template <int DZ>
__device__ __forceinline__ void pv_block(Wave<DZ> &w, const char *__restrict__ st, const bf16x8 (&pf)[2], int nb)
{
    using C = AttnCfg<DZ>;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
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
        w.oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[tt], w.oacc[nb], 0, 0, 0);
    }
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

// The direct global->LDS loads of one wave.  A wave-wide load writes 64 consecutive 16-byte
// slots of a stage; the slot decides which (row, 16-byte column) of the global block the lane
// fetches.  Slots in the row padding or past the last row fetch element 0 of the block again
// (harmless).  Wave w issues entries w, w+4, ... of the flat list z2 | k^ head | v^ head; surplus
// entries repeat entry 0 so that every wave issues the same number of loads per block.  The
// per-lane offsets run ahead by one block per call, so the blocks must be requested in the
// order in which they are stored (wrap-arounds are handled by moving the bases).
template <int DZ>
struct Dma {
    using C = AttnCfg<DZ>;
    const char *src[C::NIW + 1];  // wave-uniform: tensor the entry reads (the last entry is the bias)
    int step[C::NIW + 1];         // wave-uniform: bytes from one key block to the next
    int voff[C::NIW + 1];         // per lane: byte offset of the PREVIOUSLY requested block
    unsigned wave_lds;            // wave-uniform: 1024 * wave
};

// Entry k of the loads of the next key block, into the stage whose LDS address is `stage`.
template <int DZ, int K>
__device__ __forceinline__ void dma_entry(Dma<DZ> &d, unsigned stage)
{
    using C = AttnCfg<DZ>;
    if constexpr (K < C::NIW)
        dma16<4096 * K>(d.src[K], d.voff[K], d.step[K], stage + d.wave_lds);
    else
        dma16<C::KB_OFF>(d.src[K], d.voff[K], d.step[K], stage);
}

template <int DZ, int K = 0>
__device__ __forceinline__ void issue_block(Dma<DZ> &d, unsigned stage)
{
    using C = AttnCfg<DZ>;
    if constexpr (K <= C::NIW) {
        dma_entry<DZ, K>(d, stage);
        issue_block<DZ, K + 1>(d, stage);
    }
}

// After the last block in walking direction has been requested the sequence continues at the
// other end (the steps are signed).
template <int DZ>
__device__ __forceinline__ void dma_wrap(Dma<DZ> &d, int nblk)
{
    using C = AttnCfg<DZ>;
#pragma unroll
    for (int k = 0; k <= C::NIW; ++k) d.src[k] -= (size_t)nblk * d.step[k];
}

// ---- the hand-ordered MFMA sequence of one pipelined iteration -------------------------------
// Operations 0 .. NOPS-1: the first LA are P V MFMAs (their operands come from a stage
// that has been visible for a whole iteration, so they can be fetched across the barrier), then
// S^T and P V MFMAs alternate (the S^T MFMAs form one dependent chain; alternating hides its
// latency), and the last LA are S^T MFMAs.
template <int DZ>
struct Ops {
    using C = AttnCfg<DZ>;
    static constexpr int F = C::LA;
    __host__ __device__ static constexpr bool is_pv(int j)
    {
        return j < F ? true : (j >= C::NOPS - F ? false : ((j - F) & 1) == 1);
    }
    // index of the operation within its kind: P V -> 2*nb + tt, S^T -> ks
    __host__ __device__ static constexpr int idx(int j)
    {
        return j < F ? j : (j >= C::NOPS - F ? C::KS - (C::NOPS - j) : (((j - F) & 1) ? F + (j - F) / 2 : (j - F) / 2));
    }
};

// LDS operand of P V operation `i` (= 2*nb + tt) from the stage at `st`: 32 v^ columns x 16 keys.
template <int DZ>
__device__ __forceinline__ bf16x8 load_pv(const Wave<DZ> &w, const char *st, int i)
{
    using C = AttnCfg<DZ>;
    const int nb = i >> 1, tt = i & 1;
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
__device__ __forceinline__ bf16x8 load_s(const Wave<DZ> &w, const char *st, int ks)
{
    using C = AttnCfg<DZ>;
    const char *src = ks < C::KSH ? st + w.kaddr_h + ks * 32 : st + w.kaddr_z + (ks - C::KSH) * 32;
    return *reinterpret_cast<const bf16x8 *>(src);
}

// Per-key bias (norm term, mask) of the stage at `st` in the layout of the S^T accumulator.
template <int DZ>
__device__ __forceinline__ f32x16 load_bias(const Wave<DZ> &w, const char *st)
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

// Raise the reference maximum to cover mx: rescale everything accumulated so far.
template <int DZ>
__device__ __forceinline__ void raise_reference(Wave<DZ> &w, float mx)
{
    using C = AttnCfg<DZ>;
    const float m_new = fmaxf(w.m_ref, mx);
    const float alpha = m_new == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(w.m_ref - m_new);
    w.m_ref = m_new;
    w.l_run *= alpha;
#pragma unroll
    for (int nb = 0; nb < C::NB; ++nb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) w.oacc[nb][r] *= alpha;
        __builtin_amdgcn_sched_barrier(0);  // one block at a time: keeps the register demand of this rare path small
    }
}

// Load entry (j / DMA_EVERY) is issued right after MFMA j when j is a multiple of DMA_EVERY.
template <int DZ, int K = 0>
__device__ __forceinline__ void dma_slot(Dma<DZ> &d, unsigned stage, int j)
{
    using C = AttnCfg<DZ>;
    if constexpr (K <= C::NIW) {
        if (j == K * C::DMA_EVERY)
            dma_entry<DZ, K>(d, stage);
        else
            dma_slot<DZ, K + 1>(d, stage, j);
    }
}

// Steady-state iteration n (blocks n, n+1, n+2 exist):
//   O^T += V^T P^T of block n (stage st_pv, probabilities pf),
//   exponentials of block n+1 from its S^T accumulator `sacc` -> pf (for the next iteration),
//   S^T of block n+2 (stage st_s) -> sacc,
//   and the operand prefetch for the first P V MFMAs of the next iteration (stage st_pv_next).
// `fr` is the operand ring; on entry it holds the operands of operations 0 .. LA-1.
// Operation 0 needs nothing but registers, so it is issued first and `head` -- the wait for block
// n+2, the workgroup barrier and the ring bookkeeping, which yields the stages st_s, st_pv_next
// and the load target st_dma -- runs behind it instead of in front of an idle matrix pipe.
template <int DZ, class Head>
__device__ __forceinline__ void steady_iteration(Wave<DZ> &w, bf16x8 (&pf)[2], f32x16 &sacc, bf16x8 (&fr)[AttnCfg<DZ>::RING],
                                                 const char *st_pv, Dma<DZ> &dma, Head &&head)
{
    const char *st_s = nullptr, *st_pv_next = nullptr;
    unsigned st_dma = 0;
    using C = AttnCfg<DZ>;
    using O = Ops<DZ>;
    constexpr int N = C::NOPS;
    constexpr int kRing = C::RING;
    constexpr int kLookahead = C::LA;
    const float m_use = w.m_ref == -INFINITY ? 0.f : w.m_ref;
    f32x16 snew;
    bf16x8 pn[2];
    unsigned pp[8];
    float ex[16];
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        if (j == 0) {
            static_assert(O::is_pv(0) && O::idx(0) == 0, "operation 0 is the first P V MFMA");
            w.oacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[0], pf[0], w.oacc[0], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            head(st_s, st_pv_next, st_dma);
        }
        // operand fetch, LA operations ahead (wrapping into the next iteration), in order of use:
        // LDS returns data in order, so each MFMA waits for exactly its own operand.  (Fetching
        // groups of four operations with one wait per group measured 3 % slower; depths 3 to 6
        // measure the same.)
        {
            const int jn = j + kLookahead;
            if (jn < N) {
                if (O::is_pv(jn))
                    fr[jn % kRing] = load_pv<DZ>(w, st_pv, O::idx(jn));
                else
                    fr[jn % kRing] = load_s<DZ>(w, st_s, O::idx(jn));
            } else {
                fr[jn % kRing] = load_pv<DZ>(w, st_pv_next, O::idx(jn - N));
            }
        }
        if (j == kLookahead - 1) snew = load_bias<DZ>(w, st_s);  // before the first S^T MFMA
        // one entry of the loads of the block four ahead, every few MFMAs
        dma_slot<DZ>(dma, st_dma, j);
        // the MFMA
        if (j == 0) {
            // (issued above)
        } else if (O::is_pv(j)) {
            const int i = O::idx(j);
            w.oacc[i >> 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % kRing], pf[i & 1], w.oacc[i >> 1], 0, 0, 0);
        } else {
            snew = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % kRing], w.qf[O::idx(j)], snew, 0, 0, 0);
        }
        // softmax slices of block n+1, spread evenly over the operations: the 16 exponentials
        // (pairs are rounded to bf16 together)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if ((r * N) / 16 != j) continue;
            ex[r] = __builtin_amdgcn_exp2f(sacc[r] - m_use);
            // (the empty asm keeps the value here: the rare path below recomputes it, and the
            // optimiser would otherwise move this work out of the MFMA shadow)
            asm volatile("" : "+v"(ex[r]));
            if (r & 1) {
                pp[r >> 1] = pack_pair(ex[r - 1], ex[r], psum);
                asm volatile("" : "+v"(pp[r >> 1]), "+v"(psum));
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    pn[0] = __builtin_bit_cast(bf16x8, (u32x4){pp[0], pp[1], pp[2], pp[3]});
    pn[1] = __builtin_bit_cast(bf16x8, (u32x4){pp[4], pp[5], pp[6], pp[7]});
    // psum <= 2^kTau bounds every weight of the block; a larger (or infinite) sum means the
    // reference is too small for this block
    if (__any(!(psum <= kTauPow) || w.m_ref == -INFINITY)) {  // (no reference yet: take the block's maximum)
        // rare: redo the exponentials after raising the reference to the block's true maximum
        raise_reference<DZ>(w, row_max16(sacc));
        const float m_new = w.m_ref == -INFINITY ? 0.f : w.m_ref;
        psum = 0.f;
        exp_block(sacc, m_new, pn, psum);
    }
    w.l_run += psum;
    pf[0] = pn[0];
    pf[1] = pn[1];
    sacc = snew;
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

template <int DZ, bool FUSED>
__global__ __launch_bounds__(256, 1) void fipa_attn_fwd_bf16_kernel(AttnParams p)
{
    using C = AttnCfg<DZ>;
    extern __shared__ __attribute__((aligned(16))) char smem[];

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of work
    // units so that the query tiles of one (batch, head) share that XCD's L2 copy of k^ and v^.
    // The first plan.full workgroups take whole tiles; the others take one of the plan.S key-range
    // parts of a remaining tile (the parts of a tile are neighbours in the launch order).
    // In a mixed launch (see SplitPlan) the last 512 workgroups alternate, per XCD, between runs of
    // 16 whole tiles and 16 parts.
    int logical, part = 0, tile_local = 0, nparts = 1;
    int wg = blockIdx.x;        // position in the plain order: whole tiles, then parts
    if (p.plan.mixed && wg >= p.plan.full - 256) {
        const int i = wg - (p.plan.full - 256), x = i % 8, j = i / 8;  // XCD, slot 0..63
        const int run = j / 16, k = j % 16 + 16 * (run / 2);            // k-th whole tile / part of this XCD's 32
        wg = (run % 2 == 0 ? p.plan.full - 256 : p.plan.full) + 8 * k + x;
    }
    if (wg < p.plan.full) {
        logical = (wg % 8) * (p.plan.full / 8) + wg / 8;
    } else {
        nparts = p.plan.S;
        const int u = wg - p.plan.full, n_units = p.plan.rem * nparts;
        if (u >= n_units) return;
        const int lin = n_units % 8 == 0 ? (u % 8) * (n_units / 8) + u / 8 : u;
        tile_local = lin / nparts;
        part = lin - tile_local * nparts;
        logical = p.plan.full + tile_local;
    }
    const int bh_pos = logical / p.nQT, qt = logical - bh_pos * p.nQT;
    const int bh = p.deal ? dealt_pair_by_length(bh_pos, p.kvlen, p.B, p.H, threadIdx.x & 63) : bh_pos;
    const int b = bh / p.H;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, g = lane >> 5;
    // (without a mask every chain has L residues: no dependent load in front of everything else)
    const int kvlen = p.deal ? p.kvlen[b] : p.L;
    // rows of this chain in the caller's tensors (a packed batch stores the chains back to back)
    const int ulen = user_len(p, b);
    const size_t urow0 = user_row(p, b, 0);
    const int nkb = (kvlen + kBlk - 1) / kBlk;      // key blocks of this chain
    const int irow = qt * kTileQ + wave * 32 + li;  // < Lp always

    // A tile whose rows all lie past the last valid residue of its chain (padding of a ragged
    // batch) has nothing to attend from: its outputs are zero by definition.
    if (qt * kTileQ >= kvlen) {
        if constexpr (!FUSED) {
            float *orow = p.Ohat + ((size_t)bh * p.Lp + irow) * C::DV;
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    *reinterpret_cast<f32x4 *>(orow + 32 * nb + 8 * a + 4 * g) = (f32x4){0.f, 0.f, 0.f, 0.f};
            if (g == 0) p.lse2[(size_t)bh * p.Lp + irow] = -INFINITY;
        } else if (irow < ulen && part == 0) {
            const size_t row = (urow0 + irow) * p.H + (bh - b * p.H);
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int a = 0; a < 2; ++a) *reinterpret_cast<f32x4 *>(p.o + row * 16 + 8 * a + 4 * g) = zero;
#pragma unroll
            for (int a = 0; a < 3; ++a) *reinterpret_cast<f32x4 *>(p.o_pts + row * 24 + 12 * g + 4 * a) = zero;
            for (int d = 4 * g; d < p.cz; d += 8) *reinterpret_cast<f32x4 *>(p.o_pair + row * p.cz + d) = zero;
            if (p.lse && g == 0) p.lse[user_lse_index(p, b, bh - b * p.H, irow)] = 0.f;
        }
        return;
    }

    // ---- direct global->LDS loads ------------------------------------------------------------
    // A wave-wide load writes 64 consecutive 16-byte slots of a stage; the slot decides which
    // (row, 16-byte column) of the global block the lane fetches.  Slots in the row padding or
    // past the last row fetch element 0 of the block again (harmless).  Wave w issues entries
    // w, w+4, ... of the flat list z2 | k^ head | v^ head; surplus entries repeat entry 0 so that
    // every wave issues the same number of loads per block.
    // Key blocks are visited starting at the block that holds the tile's own residues and
    // wrapping around.  With distance-dominated logits the row maximum sits near the diagonal,
    // so the reference maximum is found in the first blocks and is rarely raised afterwards.
    // (The staggered starts also spread the tiles of a head over different blocks at any one
    // time; visiting the blocks in the same order everywhere measured slower.)
    // A key-range part takes its share of that rotated sequence: positions pos0 .. pos0 + nblk - 1.
    // The first part gets a quarter of a share more than the others: it holds the diagonal blocks
    // and never has to raise its softmax reference, while the others may (in a compact chain a
    // later block can lie closer in space than all earlier ones), so equal shares would leave it
    // waiting.
    const int pos0 = part == 0 ? 0 : (4 * part + 1) * nkb / (4 * nparts + 1);
    const int pos1 = part + 1 == nparts ? nkb : (4 * part + 5) * nkb / (4 * nparts + 1);
    const int nblk = pos1 - pos0;  // key blocks this workgroup processes
    // A part walks its range away from the diagonal too: upwards from its first position when
    // that end is the nearer one (always so for a whole tile), downwards from its last otherwise;
    // a range that approached the diagonal would raise the reference at every block.
    const bool downwards = pos0 > nkb - (pos0 + nblk);
    const int dir = downwards ? -1 : 1;
    int first_blk = min(qt * (kTileQ / kBlk), max(nkb - 1, 0)) + (downwards ? pos0 + nblk - 1 : pos0);
    if (first_blk >= nkb) first_blk -= nkb;  // (nkb = 0: stays 0 and is never used)
    const int wrap_at = downwards ? -1 : nkb, wrap_to = downwards ? nkb - 1 : 0;

    Dma<DZ> dma;
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
            dma.step[k] = dir * kBlk * cols * 16;
            dma.src[k] = isz ? Z2b : (isk ? Khb : Vhb);
            // one block before the first block: every request advances the offset first
            dma.voff[k] = ((row < kBlk && col < cols) ? row * (cols * 16) + col * 16 : 0) + (first_blk * dir - 1) * dma.step[k];
            // (entry wave + 4k lands (wave + 4k) KiB into the stage; a surplus entry refetches
            // entry 0 into the unused KiB that the stage keeps for it)
        }
        dma.step[C::NIW] = dir * kBlk * 4;
        dma.src[C::NIW] = reinterpret_cast<const char *>(p.kbias + (size_t)bh * p.Lp);
        dma.voff[C::NIW] = min(lane, 7) * 16 + (first_blk * dir - 1) * dma.step[C::NIW];
        if (downwards) {
            // the hardware adds the per-lane offset as an unsigned number: when walking downwards
            // keep it positive over the whole walk (at most nkb + 4 requests) by moving a bias
            // from the offset into the base
#pragma unroll
            for (int k = 0; k <= C::NIW; ++k) {
                const int bias = -(nkb + 8) * dma.step[k];
                dma.voff[k] += bias;
                dma.src[k] -= bias;
            }
        }
    }

    const unsigned smem_lds = lds_address(smem);
    int next_blk = first_blk;  // next key block to request

    if (nblk > 0) {
        // the first two blocks of the sequence; the next two follow once the query fragments
        // have been requested, so that what the first products need arrives first.  (Beyond the
        // end of a short sequence the requests simply go round again: every stage they touch is free.)
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (next_blk == wrap_at) {
                dma_wrap<DZ>(dma, nkb);
                next_blk = wrap_to;
            }
            issue_block<DZ>(dma, smem_lds + i * C::STAGE);
            next_blk += dir;
        }
    }

    // ---- q^ row fragments: features 16*ks + 8*g .. +7 of row irow ---------------------------
    // They are loaded straight into accumulation registers (the MFMA reads its B operand from
    // there), which leaves the architectural registers to the operand ring and the softmax.
    // The loads are invisible to the compiler's wait-count bookkeeping; the wait_vmem<0>()
    // below covers them, and the empty asm after it orders every use behind that wait.
    // With the fused epilogue (AlphaFold2 head shape) the pair part of q^ -- the bias vector
    // b^{h1} = log2e * w_L * w_b[h] (.) z1 of Algorithm 1 steps 2-3 -- is formed here from z1,
    // which all heads of a residue share, instead of being read per head from memory.
    Wave<DZ> w;
    {
        const bf16_t *qh = p.Qh + ((size_t)bh * p.Lp + irow) * kDH;
#pragma unroll
        for (int ks = 0; ks < C::KSH; ++ks)
            asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(w.qf[ks]) : "v"(qh + ks * 16 + 8 * g) : "memory");
        if constexpr (!FUSED) {
            const bf16_t *qz = p.Qz + ((size_t)bh * p.Lp + irow) * DZ;
#pragma unroll
            for (int ks = 0; ks < C::KSZ; ++ks)
                asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(w.qf[C::KSH + ks]) : "v"(qz + ks * 16 + 8 * g) : "memory");
            if (nblk > 0) {
#pragma unroll
                for (int i = 2; i < 4; ++i) {
                    if (next_blk == wrap_at) {
                        dma_wrap<DZ>(dma, nkb);
                        next_blk = wrap_to;
                    }
                    issue_block<DZ>(dma, smem_lds + i * C::STAGE);
                    next_blk += dir;
                }
            }
        } else {
            // This wave's 32 z1 rows go to LDS as whole rows (coalesced; read per lane from memory,
            // 16 bytes of each of 32 rows per load, they take several times as long), the 16-byte
            // chunks of row r stored at position chunk ^ (r mod chunks-per-row) so that the reads
            // below -- one chunk index across 32 rows -- spread over the banks.  The per-head
            // scale vector goes to LDS as well.
            constexpr int kRowBytes = DZ * 2, kWaveBytes = 32 * kRowBytes, kCpr = DZ / 8;
            const char *zbase = reinterpret_cast<const char *>(p.z1 + urow0 * DZ);
            const int row0 = qt * kTileQ + wave * 32;
#pragma unroll
            for (int k = 0; k < kWaveBytes / 1024; ++k) {
                const int slot = 64 * k + lane, r = slot / kCpr, c = (slot % kCpr) ^ (r % kCpr);
                int voff = min(row0 + r, ulen - 1) * kRowBytes + 16 * c;
                dma16<0>(zbase, voff, 0, smem_lds + C::Z1P_OFF + wave * kWaveBytes + 1024 * k);
            }
            if (tid < DZ)
                reinterpret_cast<float *>(smem + C::CW_OFF)[tid] =
                    kLog2e * p.w_L * p.w_b[(size_t)(bh - b * p.H) * p.cz + tid % p.cz];
        }
    }
#pragma unroll
    for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) w.oacc[nb][r] = 0.f;
    w.m_ref = -INFINITY;
    w.l_run = 0.f;
    {
        const int l16 = lane & 15, grp2 = (lane >> 4) & 1, e4 = l16 >> 2, j4 = l16 & 3;
        w.kaddr_h = C::KH_OFF + li * kHS + g * 16;
        w.kaddr_z = C::Z_OFF + li * C::ZS + g * 16;
        w.vaddr_h = C::VH_OFF + (4 * g + e4) * kHS + (16 * grp2 + 4 * j4) * 2;
        w.vaddr_z = C::Z_OFF + (4 * g + e4) * C::ZS + (16 * grp2 + 4 * j4) * 2;
        w.baddr = C::KB_OFF + 16 * g;
    }

    // ---- prologue: blocks 0 and 1 ----------------------------------------------------------------
    bf16x8 pf[2];
    f32x16 sacc;
    bf16x8 fr[C::RING];
    // q^ fragments and the first two stages.  (Unfused: blocks 2 and 3 may still be on their way;
    // the steady loop waits for them.)  Nothing the compiler tracks stays pending.
    if (!FUSED && nblk > 0)
        wait_vmem<2 * C::VM_PER_BLOCK>();
    else
        wait_vmem<0>();
    if (nblk > 0) {
        if constexpr (FUSED)
            __syncthreads();  // (with its fence: the scale vector written above is read by every wave)
        else
            wg_barrier();
        if constexpr (FUSED) {
            // q^ pair part: bf16(scale[col] * z1[row, col]); rows that do not exist or are masked get 0
            const bool ok = irow < ulen && (p.mask ? p.mask[urow0 + irow] != 0 : true);
            const unsigned keep = ok ? 0xFFFFFFFFu : 0u;
            const float *cw = reinterpret_cast<const float *>(smem + C::CW_OFF) + 8 * g;
            constexpr int kCpr = DZ / 8;
            const char *z1l = smem + C::Z1P_OFF + wave * (32 * DZ * 2) + li * (DZ * 2);
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
            // blocks 2 and 3 of the sequence (the steady loop waits for them); block 3 goes where
            // z1 rows sit until every wave has its fragments
            wg_barrier();
#pragma unroll
            for (int i = 2; i < 4; ++i) {
                if (next_blk == wrap_at) {
                    dma_wrap<DZ>(dma, nkb);
                    next_blk = wrap_to;
                }
                issue_block<DZ>(dma, smem_lds + i * C::STAGE);
                next_blk += dir;
            }
        }
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) asm volatile("" : "+a"(w.qf[ks]));
        sacc = s_block<DZ>(w, smem);
        float mx = row_max16(sacc);
        // The sequence of a whole tile (or of its first part) starts with the four blocks that
        // hold the tile's own residues, wave v's in block v.  With distance-dominated logits a
        // row's largest logits sit there, far above those of the neighbouring blocks, so waves
        // 1-3 would raise the reference (and every wave would wait for them) when they get to
        // their own block.  They look at it now instead and start from its maximum.
        if (pos0 == 0 && !downwards && nblk >= 4) {
            wait_vmem<0>();  // blocks 2 and 3
            wg_barrier();
            if (wave > 0) mx = fmaxf(mx, row_max16(s_block<DZ>(w, smem + wave * C::STAGE)));
        }
        w.m_ref = mx;
        float psum = 0.f;
        exp_block(sacc, mx == -INFINITY ? 0.f : mx, pf, psum);
        w.l_run = psum;
        if (nblk > 1) sacc = s_block<DZ>(w, smem + C::STAGE);
#pragma unroll
        for (int j = 0; j < C::LA; ++j) fr[j] = load_pv<DZ>(w, smem, j);
    }

    // ---- steady state: iteration n works on blocks n (P V), n+1 (exp), n+2 (S^T) ---------------
    int s0 = 0;  // stage of block n
    for (int n = 0; n + 2 < nblk; ++n) {
        steady_iteration<DZ>(w, pf, sacc, fr, smem + s0 * C::STAGE, dma,
                             [&](const char *&st_s, const char *&st_pv_next, unsigned &st_dma) {
            // Block n+2 must have landed (the requests of the previous iteration may still be in
            // flight); the barrier also tells everyone that the stage of block n-1 is free again.
            wait_vmem<C::VM_PER_BLOCK>();
            wg_barrier();
            const int s1 = s0 + 1 < C::NSTAGE ? s0 + 1 : s0 + 1 - C::NSTAGE;
            const int s2 = s0 + 2 < C::NSTAGE ? s0 + 2 : s0 + 2 - C::NSTAGE;
            const int s4 = s0 + 4 < C::NSTAGE ? s0 + 4 : s0 + 4 - C::NSTAGE;
            if (next_blk == wrap_at) {
                dma_wrap<DZ>(dma, nkb);
                next_blk = wrap_to;
            }
            next_blk += dir;
            st_s = smem + s2 * C::STAGE;
            st_pv_next = smem + s1 * C::STAGE;
            st_dma = smem_lds + s4 * C::STAGE;
            s0 = s1;
        });
    }
    wait_vmem<0>();  // requests past the end of the sequence went to free stages; let them finish

    // ---- fused epilogue, first step: this wave's 32 z1 rows go to LDS while the last blocks are
    // being multiplied.  After the barrier every wave has left the loop and every block load has
    // landed, so the three stages that do not hold the last two blocks are free; each wave takes
    // 32 * 2 DZ bytes of them.  Row-major with the 16-byte chunks of row r stored at position
    // chunk ^ (r mod chunks-per-row): the loads are whole rows (coalesced) and the reads below,
    // one chunk index across 32 rows, spread over the banks.
    [[maybe_unused]] int z1_off = 0;
    if constexpr (FUSED) {
        static_assert(C::NSTAGE == 5 && 32 * DZ * 2 <= C::STAGE, "z1 staging needs three free stages");
        constexpr int kRowBytes = DZ * 2, kWaveBytes = 32 * kRowBytes, kCpr = DZ / 8;  // 16-byte chunks per row
        wg_barrier();
        const int f0 = s0 + 2 < C::NSTAGE ? s0 + 2 : s0 + 2 - C::NSTAGE;  // first free stage (cyclically)
        const int room = min(C::NSTAGE - f0, 3) * C::STAGE;                // free bytes before the ring wraps
        const int n_head = min(4, room / kWaveBytes);                     // waves that fit there; the rest start at 0
        z1_off = wave < n_head ? f0 * C::STAGE + wave * kWaveBytes : (wave - n_head) * kWaveBytes;
        const char *zbase = reinterpret_cast<const char *>(p.z1 + urow0 * DZ);
        const int row0 = qt * kTileQ + wave * 32;
#pragma unroll
        for (int k = 0; k < kWaveBytes / 1024; ++k) {
            const int slot = 64 * k + lane, r = slot / kCpr, c = (slot % kCpr) ^ (r % kCpr);
            int voff = min(row0 + r, ulen - 1) * kRowBytes + 16 * c;
            dma16<0>(zbase, voff, 0, smem_lds + z1_off + 1024 * k);
        }
    }

    // ---- drain: the last two blocks -----------------------------------------------------------------
    if (nblk > 1) {
        // P V of the last block but one, exponentials of the last block
        const char *st = smem + s0 * C::STAGE;
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) pv_block<DZ>(w, st, pf, nb);
        const float mx = row_max16(sacc);
        if (__any(mx > w.m_ref + kTau)) raise_reference<DZ>(w, mx);
        float psum = 0.f;
        exp_block(sacc, w.m_ref == -INFINITY ? 0.f : w.m_ref, pf, psum);
        w.l_run += psum;
        s0 = s0 + 1 < C::NSTAGE ? s0 + 1 : s0 + 1 - C::NSTAGE;
    }
    if (nblk > 0) {
        const char *st = smem + s0 * C::STAGE;
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) pv_block<DZ>(w, st, pf, nb);
    }

    float l_tot = w.l_run + __shfl_xor(w.l_run, 32);
    f32x16(&oacc)[C::NB] = w.oacc;

    if constexpr (!FUSED) {
        // write O^ (row irow, columns 32*nb + 8*(r/4) + 4*g + r%4) and the log2 LSE
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        const float lse2 = l_tot > 0.f ? w.m_ref + __log2f(l_tot) : -INFINITY;
        float *orow = p.Ohat + ((size_t)bh * p.Lp + irow) * C::DV;
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                f32x4 out;
#pragma unroll
                for (int x = 0; x < 4; ++x) out[x] = oacc[nb][4 * a + x] * inv;
                *reinterpret_cast<f32x4 *>(orow + 32 * nb + 8 * a + 4 * g) = out;
            }
        if (g == 0) p.lse2[(size_t)bh * p.Lp + irow] = lse2;
    } else {
        // ---- split, inverse frame, z1 contraction (Algorithm 1 steps 8-9, Eq. 4); c = 16, Pv = 8
        // First everything that is linear in the accumulator, still unnormalised:
        //   the scalar columns, the global points (hi + lo parts), and the contraction with z1.
        constexpr int c = 16, Pv = 8;
        constexpr int NZB = C::NB - C::NBH;  // 32-column blocks of the pair part
        const bool in_range = irow < ulen;
        const int irow_c = min(irow, ulen - 1);  // rows past the end compute on a valid address and store nothing
        const int cz = p.cz;
        const int bps = cz / 32;                // 32-column blocks per factor slice (cz >= 32)
        // point part: this half owns points 4g .. 4g+3, hi parts in slots u = 0..11, lo parts in
        // slots 12..23; slot u sits in column 16 + 8*(u/4) + 4g + u%4 (see v_pt_col)
        float Gv[12];
#pragma unroll
        for (int u = 0; u < 12; ++u) {
            const int dh = 16 + 8 * (u >> 2) + (u & 3);  // column for g = 0; g = 1 adds 4
            const int dl = 16 + 8 * ((u + 12) >> 2) + ((u + 12) & 3);
            const float hi = oacc[dh >> 5][4 * ((dh & 31) >> 3) + (dh & 3)];
            const float lo = oacc[dl >> 5][4 * ((dl & 31) >> 3) + (dl & 3)];
            Gv[u] = hi + lo;
        }
        // pair part: o~[d'] = sum_rho z1[rho, d'] * U[rho, d']; the lane holds columns 8a + 4g + x
        {
            wait_vmem<0>();  // the z1 rows staged before the drain (this wave's own loads, no barrier needed)
            asm volatile("" ::: "memory");
            constexpr int kCpr = DZ / 8;
            const char *z1l = smem + z1_off + li * (DZ * 2) + 8 * g;
#pragma unroll
            for (int zb = 0; zb < NZB; ++zb)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    // columns 32 zb + 8 a + 4 g .. + 3 of row li: half g of chunk 4 zb + a
                    const uint2 zraw = *reinterpret_cast<const uint2 *>(z1l + 16 * ((4 * zb + a) ^ (li % kCpr)));
                    const bf16_t *zb16 = reinterpret_cast<const bf16_t *>(&zraw);
#pragma unroll
                    for (int x = 0; x < 4; ++x) oacc[C::NBH + zb][4 * a + x] *= bf2f(zb16[x]);
                }
            // sum over rho: column dz of U belongs to output d' = dz % cz.  For cz >= 32 the sums
            // end up in blocks 0 .. bps-1 of the pair part.
            if (cz >= 32) {
#pragma unroll
                for (int zb = 0; zb < NZB; ++zb) {
                    if (zb >= bps) break;
#pragma unroll
                    for (int z2_ = zb + 1; z2_ < NZB; ++z2_)
                        if ((z2_ - zb) % bps == 0)
#pragma unroll
                            for (int r = 0; r < 16; ++r) oacc[C::NBH + zb][r] += oacc[C::NBH + z2_][r];
                }
            }
        }

        // ---- key-range split: leave this part's unnormalised row in memory; the part that
        // arrives last merges all parts of the tile.  Every exchanged word is written and read
        // with device-scope atomic accesses (which go to the coherence point, not through the
        // non-coherent caches); a part's words are complete (vmcnt = 0) before it takes its ticket.
        if (nparts > 1) {
            // per lane: 2 groups of scalars, 3 of point coordinates, 1 of (m, l), 4 per pair block
            const int groups = attn_partial_groups(cz);
            // wave-uniform base: this wave's rows in part 0 of the tile; byte offsets within 32 bits
            const __amdgpu_buffer_rsrc_t xr =
                xchg_resource(p.partial + ((size_t)tile_local * nparts * 4 + wave) * (groups * 64 * 4));
            const int kPartBytes = 4 * groups * 64 * 16;
            const int mine = part * kPartBytes + lane * 16;
            xchg_store(xr, mine + 0 * 1024, (f32x4){oacc[0][0], oacc[0][1], oacc[0][2], oacc[0][3]});
            xchg_store(xr, mine + 1 * 1024, (f32x4){oacc[0][4], oacc[0][5], oacc[0][6], oacc[0][7]});
#pragma unroll
            for (int a = 0; a < 3; ++a)
                xchg_store(xr, mine + (2 + a) * 1024, (f32x4){Gv[4 * a], Gv[4 * a + 1], Gv[4 * a + 2], Gv[4 * a + 3]});
            xchg_store(xr, mine + 5 * 1024, (f32x4){w.m_ref, l_tot, 0.f, 0.f});
#pragma unroll
            for (int zb = 0; zb < NZB; ++zb) {
                if (zb >= bps) break;
#pragma unroll
                for (int a = 0; a < 4; ++a)
                    xchg_store(xr, mine + (6 + 4 * zb + a) * 1024,
                               (f32x4){oacc[C::NBH + zb][4 * a], oacc[C::NBH + zb][4 * a + 1],
                                       oacc[C::NBH + zb][4 * a + 2], oacc[C::NBH + zb][4 * a + 3]});
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            int ticket = 0;
            if (lane == 0)
                ticket = __hip_atomic_fetch_add(p.counters + tile_local * 4 + wave, 1, __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
            ticket = __builtin_amdgcn_readfirstlane(ticket);
            if (ticket != nparts - 1) return;
            asm volatile("" ::: "memory");
            // Merge all parts in the order of their key ranges, this wave's own included (read
            // back), so that the result does not depend on which part happened to come last.
            float m_acc = -INFINITY;
            l_tot = 0.f;
#pragma unroll
            for (int r = 0; r < 8; ++r) oacc[0][r] = 0.f;
#pragma unroll
            for (int u = 0; u < 12; ++u) Gv[u] = 0.f;
#pragma unroll
            for (int zb = 0; zb < NZB; ++zb)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[C::NBH + zb][r] = 0.f;
            for (int q = 0; q < nparts; ++q) {
                const int other = q * kPartBytes + lane * 16;
                f32x4 head[6], pair[NZB][4];
#pragma unroll
                for (int k = 0; k < 6; ++k) head[k] = xchg_load(xr, other + k * 1024);
#pragma unroll
                for (int zb = 0; zb < NZB; ++zb) {
                    if (zb >= bps) break;
#pragma unroll
                    for (int a = 0; a < 4; ++a) pair[zb][a] = xchg_load(xr, other + (6 + 4 * zb + a) * 1024);
                }
                const float m_o = head[5][0], l_o = head[5][1];
                const float m_new = fmaxf(m_acc, m_o);
                const float a_own = m_acc == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_acc - m_new);
                const float a_oth = m_o == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_o - m_new);
                m_acc = m_new;
                l_tot = l_tot * a_own + l_o * a_oth;
#pragma unroll
                for (int r = 0; r < 8; ++r) oacc[0][r] = oacc[0][r] * a_own + head[r >> 2][r & 3] * a_oth;
#pragma unroll
                for (int u = 0; u < 12; ++u) Gv[u] = Gv[u] * a_own + head[2 + (u >> 2)][u & 3] * a_oth;
#pragma unroll
                for (int zb = 0; zb < NZB; ++zb) {
                    if (zb >= bps) break;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        oacc[C::NBH + zb][r] = oacc[C::NBH + zb][r] * a_own + pair[zb][r >> 2][r & 3] * a_oth;
                }
            }
            w.m_ref = m_acc;
        }

        // ---- normalise, apply the inverse frame, store ---------------------------------------------
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        const float lse2 = l_tot > 0.f ? w.m_ref + __log2f(l_tot) : -INFINITY;
        const int h = bh - b * p.H;
        const bool valid = (p.mask ? p.mask[urow0 + irow_c] != 0 : true) && l_tot > 0.f;
        const float sc = valid ? inv : 0.f;
        const size_t row = (urow0 + irow_c) * p.H + h;
        if (in_range) {
            // scalar part: columns 8a + 4g + x, a = 0, 1
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                f32x4 out;
#pragma unroll
                for (int x = 0; x < 4; ++x) out[x] = oacc[0][4 * a + x] * sc;
                *reinterpret_cast<f32x4 *>(p.o + row * c + 8 * a + 4 * g) = out;
            }
        }
        {
            const float *R = p.rot + (urow0 + irow_c) * 9;
            const float *tr = p.trans + (urow0 + irow_c) * 3;
            float Rm[9], tc[3];
#pragma unroll
            for (int a = 0; a < 9; ++a) Rm[a] = R[a];
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
            }
        }
        if (in_range) {
            float *dst = p.o_pair + row * cz;
            if (cz >= 32) {
#pragma unroll
                for (int zb = 0; zb < NZB; ++zb) {
                    if (zb >= bps) break;
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        f32x4 out;
#pragma unroll
                        for (int x = 0; x < 4; ++x) out[x] = oacc[C::NBH + zb][4 * a + x] * sc;
                        *reinterpret_cast<f32x4 *>(dst + 32 * zb + 8 * a + 4 * g) = out;
                    }
                }
            } else {
                // cz in {8, 16}: slices are narrower than a block (such launches are never split)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    if (8 * a >= cz) break;
                    f32x4 out = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int zb = 0; zb < NZB; ++zb)
#pragma unroll
                        for (int a2 = 0; a2 < 4; ++a2) {
                            const int dz = 32 * zb + 8 * a2;
                            if (dz % cz == 8 * a)
#pragma unroll
                                for (int x = 0; x < 4; ++x) out[x] += oacc[C::NBH + zb][4 * a2 + x] * sc;
                        }
                    *reinterpret_cast<f32x4 *>(dst + 8 * a + 4 * g) = out;
                }
            }
            if (p.lse && g == 0)
                p.lse[user_lse_index(p, b, h, irow)] = valid ? lse2 * kLn2 - p.qbias[(size_t)bh * p.Lp + irow] : 0.f;
        }
    }
}

template <int DZ, bool FUSED>
hipError_t launch(const AttnParams &p, hipStream_t stream)
{
    using C = AttnCfg<DZ>;
    static LdsLimit lds_limit;
    hipError_t e = raise_lds_limit(lds_limit, (const void *)fipa_attn_fwd_bf16_kernel<DZ, FUSED>, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    if (p.plan.full % 8 != 0 || p.plan.full + p.plan.rem != p.total_tiles || p.plan.S < 1 ||
        (p.plan.S > 1 && (!FUSED || p.cz < 32)))
        return hipErrorInvalidValue;
    hipLaunchKernelGGL((fipa_attn_fwd_bf16_kernel<DZ, FUSED>), dim3(p.plan.units()), dim3(256),
                       C::LDS_BYTES, stream, p);
    return hipGetLastError();
}

template <int DZ>
hipError_t launch_dz(const AttnParams &p, bool fused, hipStream_t stream)
{
    return fused ? launch<DZ, true>(p, stream) : launch<DZ, false>(p, stream);
}

}  // namespace

hipError_t launch_attn_fwd_bf16(const AttnParams &p, int DZ, bool fused, hipStream_t stream)
{
    switch (DZ) {
        case 32: return launch_dz<32>(p, fused, stream);
        case 64: return launch_dz<64>(p, fused, stream);
        case 128: return launch_dz<128>(p, fused, stream);
        case 256: return launch_dz<256>(p, fused, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fipa
