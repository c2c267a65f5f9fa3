// Fused attention on the lifted features (Algorithm 1 step 7) for gfx950: online softmax over
// key tiles (the recurrences of Algorithm 2: running maximum m, running sum l, rescaled
// accumulator), bf16 MFMA 32x32x16 for both contractions, fp32 accumulation.
//
// Work split: one workgroup = one (batch, head, 128-query tile); each of its 4 waves owns 32
// query rows and keeps q^ (as MFMA B fragments) and the 32 x (64+DZ) output accumulator in
// registers for the whole key loop; K^ and V^ tiles of 64 keys are staged in LDS and shared by
// the four waves.  Both products are computed transposed,
//     S^T = K^ Q^T        (A = K^ tile from LDS, B = q^ registers)
//     O^T += V^T P^T      (A = transposed V^ tile from LDS, B = P^T registers)
// so that a lane owns one query row: the softmax statistics are per-lane scalars and the
// exponentiated S^T accumulator is already laid out as the B operand of the second product.
#include "fipa_bf16_common.h"

namespace fipa {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int DZ>
struct AttnCfg {
    static constexpr int DQK = kDH + DZ;
    static constexpr int DV = kDH + DZ;
    static constexpr int KS = DQK / 16;         // k-steps of S^T
    static constexpr int NB = DV / 32;          // 32-row blocks of O^T
    static constexpr int KSTR = DQK * 2 + 16;   // bytes per key row of the K^ tile (padded)
    static constexpr int VSTR = kTileK * 2 + 16;  // bytes per feature row of the V^T tile (padded)
    static constexpr int K_BYTES = kTileK * KSTR;
    static constexpr int V_BYTES = DV * VSTR;
    static constexpr int LDS_BYTES = K_BYTES + V_BYTES + kTileK * 4;
    static constexpr int K_CHUNKS = kTileK * DQK / 8 / 256;  // 16-byte chunks per thread
    static constexpr int V_CHUNKS = DV * kTileK / 8 / 256;
};

template <int DZ>
__global__ __launch_bounds__(256, 1) void fipa_attn_fwd_bf16_kernel(AttnParams p)
{
    using C = AttnCfg<DZ>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char *ldsK = smem;
    char *ldsV = smem + C::K_BYTES;
    float *ldsB = reinterpret_cast<float *>(smem + C::K_BYTES + C::V_BYTES);

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles
    // so that the query tiles of one (batch, head) share that XCD's L2 copy of K^ and V^.
    const int chunk = (p.total_tiles + 7) / 8;
    const int logical = (blockIdx.x % 8) * chunk + blockIdx.x / 8;
    if (logical >= p.total_tiles) return;
    const int bh = logical / p.nQT, qt = logical - bh * p.nQT;
    const int b = bh / p.H;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int li = lane & 31, g = lane >> 5;
    const int kvlen = p.kvlen[b];
    const int ntiles = (kvlen + kTileK - 1) / kTileK;
    const int irow = qt * kTileQ + wave * 32 + li;  // < Lp always

    // q^ row fragments: features 16*ks + 8*g .. +7 of row irow
    bf16x8 qf[C::KS];
    {
        const bf16_t *qh = p.Qh + ((size_t)bh * p.Lp + irow) * kDH;
        const bf16_t *qz = p.Qz + ((size_t)bh * p.Lp + irow) * DZ;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const bf16_t *src = ks < kDH / 16 ? qh + ks * 16 + 8 * g : qz + (ks - kDH / 16) * 16 + 8 * g;
            qf[ks] = *reinterpret_cast<const bf16x8 *>(src);
        }
    }

    f32x16 oacc[C::NB];
#pragma unroll
    for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[nb][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const bf16_t *Kh = p.Kh + (size_t)bh * p.Lp * kDH;
    const bf16_t *Z2 = p.Z2 + (size_t)b * p.Lp * DZ;
    const bf16_t *VhT = p.VhT + (size_t)bh * p.Lp * kDH;
    const bf16_t *Z2T = p.Z2T + (size_t)b * p.Lp * DZ;
    const float *kbias = p.kbias + (size_t)bh * p.Lp;

    uint4 kreg[C::K_CHUNKS], vreg[C::V_CHUNKS];
    float kbreg = 0.f;

#define FIPA_LOAD_K(T)                                                                             \
    do {                                                                                           \
        const int j0_ = (T) * kTileK;                                                              \
        _Pragma("unroll") for (int it = 0; it < C::K_CHUNKS; ++it) {                               \
            const int q_ = it * 256 + tid;                                                         \
            const int row_ = q_ / (C::DQK / 8), cc_ = q_ - row_ * (C::DQK / 8);                    \
            const bf16_t *src_ = cc_ < kDH / 8 ? Kh + (size_t)(j0_ + row_) * kDH + cc_ * 8         \
                                               : Z2 + (size_t)(j0_ + row_) * DZ + (cc_ - kDH / 8) * 8; \
            kreg[it] = *reinterpret_cast<const uint4 *>(src_);                                     \
        }                                                                                          \
        if (tid < kTileK) kbreg = kbias[j0_ + tid];                                                \
    } while (0)
#define FIPA_STORE_K()                                                                             \
    do {                                                                                           \
        _Pragma("unroll") for (int it = 0; it < C::K_CHUNKS; ++it) {                               \
            const int q_ = it * 256 + tid;                                                         \
            const int row_ = q_ / (C::DQK / 8), cc_ = q_ - row_ * (C::DQK / 8);                    \
            *reinterpret_cast<uint4 *>(ldsK + row_ * C::KSTR + cc_ * 16) = kreg[it];               \
        }                                                                                          \
        if (tid < kTileK) ldsB[tid] = kbreg;                                                       \
    } while (0)
#define FIPA_LOAD_V(T)                                                                             \
    do {                                                                                           \
        const bf16_t *vh_ = VhT + (size_t)(T) * kDH * kTileK;                                      \
        const bf16_t *zt_ = Z2T + (size_t)(T) * DZ * kTileK;                                       \
        _Pragma("unroll") for (int it = 0; it < C::V_CHUNKS; ++it) {                               \
            const int q_ = it * 256 + tid;                                                         \
            const int row_ = q_ >> 3, cc_ = q_ & 7;                                                \
            const bf16_t *src_ = row_ < kDH ? vh_ + row_ * kTileK + cc_ * 8                        \
                                            : zt_ + (row_ - kDH) * kTileK + cc_ * 8;               \
            vreg[it] = *reinterpret_cast<const uint4 *>(src_);                                     \
        }                                                                                          \
    } while (0)
#define FIPA_STORE_V()                                                                             \
    do {                                                                                           \
        _Pragma("unroll") for (int it = 0; it < C::V_CHUNKS; ++it) {                               \
            const int q_ = it * 256 + tid;                                                         \
            const int row_ = q_ >> 3, cc_ = q_ & 7;                                                \
            *reinterpret_cast<uint4 *>(ldsV + row_ * C::VSTR + cc_ * 16) = vreg[it];               \
        }                                                                                          \
    } while (0)

    if (ntiles > 0) {
        FIPA_LOAD_K(0);
        FIPA_STORE_K();
    }
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        FIPA_LOAD_V(t);

        // S^T = K^ Q^T, accumulator preset with the per-key bias (norm term, mask)
        f32x16 sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const f32x4 bias = *reinterpret_cast<const f32x4 *>(&ldsB[32 * kb + 8 * a + 4 * g]);
#pragma unroll
                for (int x = 0; x < 4; ++x) sacc[kb][4 * a + x] = bias[x];
            }
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(ldsK + (32 * kb + li) * C::KSTR + ks * 32 + g * 16);
                sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sacc[kb], 0, 0, 0);
            }

        // online softmax for this lane's query row (its keys: 16 per block here, the other 16
        // in the lane 32 away)
        float mx = sacc[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
        m_run = m_new;
        bf16x8 pf[2][2];
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float e = __builtin_amdgcn_exp2f(sacc[kb][r] - m_use);
                const __bf16 eb = (__bf16)e;
                pf[kb][r >> 3][r & 7] = eb;
                psum += (float)eb;  // the denominator sums the rounded weights the MFMA will use
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[nb][r] *= alpha;

        FIPA_STORE_V();
        __syncthreads();
        if (t + 1 < ntiles) FIPA_LOAD_K(t + 1);

        // O^T += V^T P^T
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(
                        ldsV + (32 * nb + li) * C::VSTR + (kb * 32 + tt * 16 + 8 * g) * 2);
                    oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[kb][tt], oacc[nb], 0, 0, 0);
                }

        if (t + 1 < ntiles) FIPA_STORE_K();
        __syncthreads();
    }

    // normalise and write O^ (row irow, columns 32*nb + 8*(r/4) + 4*g + r%4) and the log2 LSE
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
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
    if (g == 0) p.lse2[(size_t)bh * p.Lp + irow] = l_tot > 0.f ? m_run + __log2f(l_tot) : -INFINITY;
}

template <int DZ>
hipError_t launch(const AttnParams &p, hipStream_t stream)
{
    using C = AttnCfg<DZ>;
    hipError_t e = hipFuncSetAttribute((const void *)fipa_attn_fwd_bf16_kernel<DZ>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int chunk = (p.total_tiles + 7) / 8;
    hipLaunchKernelGGL(fipa_attn_fwd_bf16_kernel<DZ>, dim3(chunk * 8), dim3(256), C::LDS_BYTES,
                       stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_fwd_bf16(const AttnParams &p, int DZ, hipStream_t stream)
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
