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
// with the transposing LDS read.  Plain structure (one LDS stage, loads through registers): this
// is the first correct version, not yet pipelined like the forward kernel.
#include "fipa_bf16_common.h"

namespace fipa {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int kSB = 32;  // streamed rows per block

template <int DZ>
struct BwdCfg {
    static constexpr int D = kDH + DZ;           // lifted width
    static constexpr int KS = D / 16;            // k-steps of the small products
    static constexpr int KSH = kDH / 16;
    static constexpr int NB = D / 32;            // 32-row blocks of the accumulator
    static constexpr int RS = D * 2 + 48;        // LDS row stride (bytes): conflict free for row reads and transposing reads
    static constexpr int X_BYTES = kSB * RS;
    static constexpr int X1_OFF = 0;
    static constexpr int X2_OFF = X_BYTES;
    static constexpr int SROW_OFF = 2 * X_BYTES;        // 32 floats: per-streamed-row logit term
    static constexpr int DROW_OFF = SROW_OFF + 128;     // 32 floats: per-streamed-row D (DK only)
    static constexpr int LDS_BYTES = DROW_OFF + 128;
    static constexpr int NCHUNK = kSB * D / 8;          // 16-byte chunks per tile
    static constexpr int CHUNKS = (NCHUNK + 255) / 256; // per thread
};

__device__ __forceinline__ bf16x4 lds_read_tr(const char *ptr)
{
    return __builtin_bit_cast(
        bf16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(ptr)));
}

__device__ __forceinline__ unsigned pack_pair(float e0, float e1, float &sum)
{
    const bf16x2 b = __builtin_convertvector((f32x2){e0, e1}, bf16x2);
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    sum = __builtin_amdgcn_fdot2_f32_bf16(b, ones, sum, false);
    return __builtin_bit_cast(unsigned, b);
}

template <int DZ, int MODE>
__global__ __launch_bounds__(256, 1) void fipa_bwd_kernel(BwdParams p)
{
    using C = BwdCfg<DZ>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr bool kNeedDP = MODE != FIPA_BWD_DV;

    const int chunk = (p.total_tiles + 7) / 8;
    const int logical = (blockIdx.x % 8) * chunk + blockIdx.x / 8;
    if (logical >= p.total_tiles) return;
    const int nT = p.Lp / kTileQ;
    const int bh = logical / nT, tile = logical - bh * nT;
    const int b = bh / p.H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, g = lane >> 5;
    const int kvlen = p.kvlen[b];
    const int nblk = (kvlen + kSB - 1) / kSB;       // streamed blocks: residues past the last valid one contribute nothing
    const int srow = tile * kTileQ + wave * 32 + li;  // stationary row of this lane, < Lp

    // streamed sources (row pointers of block 0) and stationary sources, by mode
    const bf16_t *x1h, *x1z, *x2h, *x2z, *y1h, *y1z, *y2h, *y2z;
    int x1hp, x1zp, x2hp, x2zp, y1hp, y1zp, y2hp, y2zp;  // row pitches in elements
    const float *srow_src, *slane_src, *drow_src = nullptr, *dlane_src = nullptr;
    const bf16_t *Qh = p.Qh + (size_t)bh * p.Lp * kDH, *Qz = p.Qz + (size_t)bh * p.Lp * DZ;
    const bf16_t *Kh = p.Kh + (size_t)bh * p.Lp * kDH, *Vh = p.Vh + (size_t)bh * p.Lp * kDH;
    const bf16_t *Z2 = p.Z2 + (size_t)b * p.Lp * DZ;
    const bf16_t *dO = p.dOhat + (size_t)bh * p.Lp * C::D;
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
    const float slane = slane_src[srow];
    const float dlane = dlane_src ? dlane_src[srow] : 0.f;

    f32x16 acc[C::NB];
#pragma unroll
    for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[nb][r] = 0.f;
    float wsum = 0.f;  // sum over streamed rows of the rounded dS (DQ: row sums, DK: column sums)

    const int kaddr = li * C::RS + g * 16;
    const int l16 = lane & 15, grp2 = (lane >> 4) & 1, e4 = l16 >> 2, j4 = l16 & 3;
    const int vaddr = (4 * g + e4) * C::RS + (16 * grp2 + 4 * j4) * 2;

    for (int blk = 0; blk < nblk; ++blk) {
        const int r0 = blk * kSB;
        // ---- stage the streamed block: two row-major tiles [32][D] and the per-row scalars ----
        uint4 st1[C::CHUNKS], st2[C::CHUNKS];
#pragma unroll
        for (int it = 0; it < C::CHUNKS; ++it) {
            const int q = min(it * 256 + tid, C::NCHUNK - 1);
            const int row = q / (C::D / 8), cc = q - row * (C::D / 8);
            const bf16_t *s1 = cc < kDH / 8 ? x1h + (size_t)(r0 + row) * x1hp + cc * 8
                                            : x1z + (size_t)(r0 + row) * x1zp + (cc - kDH / 8) * 8;
            const bf16_t *s2 = cc < kDH / 8 ? x2h + (size_t)(r0 + row) * x2hp + cc * 8
                                            : x2z + (size_t)(r0 + row) * x2zp + (cc - kDH / 8) * 8;
            st1[it] = *reinterpret_cast<const uint4 *>(s1);
            st2[it] = *reinterpret_cast<const uint4 *>(s2);
        }
        float sr = 0.f, dr = 0.f;
        if (tid < kSB) {
            sr = srow_src[r0 + tid];
            dr = drow_src ? drow_src[r0 + tid] : 0.f;
        }
        __syncthreads();  // everyone is done with the previous block
#pragma unroll
        for (int it = 0; it < C::CHUNKS; ++it) {
            const int q = min(it * 256 + tid, C::NCHUNK - 1);  // (surplus threads rewrite the last chunk)
            const int row = q / (C::D / 8), cc = q - row * (C::D / 8);
            *reinterpret_cast<uint4 *>(smem + C::X1_OFF + row * C::RS + cc * 16) = st1[it];
            *reinterpret_cast<uint4 *>(smem + C::X2_OFF + row * C::RS + cc * 16) = st2[it];
        }
        if (tid < kSB) {
            *reinterpret_cast<float *>(smem + C::SROW_OFF + tid * 4) = sr;
            *reinterpret_cast<float *>(smem + C::DROW_OFF + tid * 4) = dr;
        }
        __syncthreads();

        // ---- S and dP blocks: [32 streamed rows] x [32 stationary rows (lanes)] ----------------
        f32x16 sacc, dpacc;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const f32x4 sb = *reinterpret_cast<const f32x4 *>(smem + C::SROW_OFF + (8 * a + 4 * g) * 4);
            const f32x4 db = *reinterpret_cast<const f32x4 *>(smem + C::DROW_OFF + (8 * a + 4 * g) * 4);
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                sacc[4 * a + x] = sb[x] + slane;
                dpacc[4 * a + x] = -(db[x] + dlane);
            }
        }
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(smem + C::X1_OFF + kaddr + ks * 32);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, y1f[ks], sacc, 0, 0, 0);
            if (kNeedDP) {
                const bf16x8 a2 = *reinterpret_cast<const bf16x8 *>(smem + C::X2_OFF + kaddr + ks * 32);
                dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, y2f[ks], dpacc, 0, 0, 0);
            }
        }
        // ---- weights of the accumulating product: P (DV) or dS = P (dP - D) (DQ, DK) -----------
        unsigned wp[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            float w0 = __builtin_amdgcn_exp2f(sacc[r]), w1 = __builtin_amdgcn_exp2f(sacc[r + 1]);
            if (kNeedDP) {
                w0 *= dpacc[r];
                w1 *= dpacc[r + 1];
            }
            wp[r >> 1] = pack_pair(w0, w1, wsum);
        }
        const bf16x8 wf[2] = {__builtin_bit_cast(bf16x8, (u32x4){wp[0], wp[1], wp[2], wp[3]}),
                              __builtin_bit_cast(bf16x8, (u32x4){wp[4], wp[5], wp[6], wp[7]})};
        // ---- acc^T[feature, stationary row] += X^T[feature, streamed row] W[streamed row, stationary row]
        constexpr int XOFF = MODE == FIPA_BWD_DV ? C::X2_OFF : C::X1_OFF;
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const char *src = smem + XOFF + vaddr + 16 * tt * C::RS + nb * 64;
                const bf16x4 lo = lds_read_tr(src);
                const bf16x4 hi = lds_read_tr(src + 8 * C::RS);
                bf16x8 a;
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    a[x] = lo[x];
                    a[4 + x] = hi[x];
                }
                acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, wf[tt], acc[nb], 0, 0, 0);
            }
    }

    // ---- write acc^T: row srow, columns 32*nb + 8*(r/4) + 4*g + r%4 -------------------------------
    float *orow = p.out + ((size_t)bh * p.Lp + srow) * C::D;
#pragma unroll
    for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            f32x4 out;
#pragma unroll
            for (int x = 0; x < 4; ++x) out[x] = acc[nb][4 * a + x];
            *reinterpret_cast<f32x4 *>(orow + 32 * nb + 8 * a + 4 * g) = out;
        }
    if (p.wsum) {
        const float tot = wsum + __shfl_xor(wsum, 32);
        if (g == 0) p.wsum[(size_t)bh * p.Lp + srow] = tot;
    }
}

template <int DZ, int MODE>
hipError_t launch(const BwdParams &p, hipStream_t stream)
{
    using C = BwdCfg<DZ>;
    hipError_t e = hipFuncSetAttribute((const void *)fipa_bwd_kernel<DZ, MODE>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int chunk = (p.total_tiles + 7) / 8;
    hipLaunchKernelGGL((fipa_bwd_kernel<DZ, MODE>), dim3(chunk * 8), dim3(256), C::LDS_BYTES, stream, p);
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
        default: return hipErrorInvalidValue;
    }
}

}  // namespace fipa
