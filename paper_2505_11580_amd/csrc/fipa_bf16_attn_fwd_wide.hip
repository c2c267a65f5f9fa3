// Fused attention on the lifted features (Algorithm 1 step 7) for wide pair factors (r*c_z = 512,
// lifted width 576): same mathematics and register layout as the main kernel, but the output
// accumulator of 32 x 576 fp32 per wave does not fit the register file, so the value columns are
// cut into windows and each workgroup computes one window (recomputing S^T and the softmax).
// Plain structure: one LDS stage filled through registers, online softmax with the running
// maximum of Algorithm 2 (raised lazily), unfused epilogue.  First correct version for this
// width, not pipelined.
#include "fipa_gfx950.h"

namespace fipa {

namespace {

constexpr int kKB = 32;      // keys per block
constexpr float kTauW = 8.f;

template <int DZ, int NWIN>
struct WideCfg {
    static constexpr int D = kDH + DZ;
    static constexpr int KS = D / 16, KSH = kDH / 16;
    static constexpr int NB = D / 32, NBH = kDH / 32;
    static constexpr int NBW = NB / NWIN;
    static_assert(NB % NWIN == 0, "windows must tile the value columns");
    static constexpr int RS = D * 2 + 48;     // k^ tile row stride (bytes)
    static constexpr int VS = kDH * 2 + 48;   // v^ head tile row stride
    static constexpr int K_OFF = 0;
    static constexpr int V_OFF = kKB * RS;
    static constexpr int B_OFF = V_OFF + kKB * VS;
    static constexpr int LDS_BYTES = B_OFF + kKB * 4;
    static constexpr int KCH = kKB * D / 8;      // 16-byte chunks of the k^ tile
    static constexpr int VCH = kKB * kDH / 8;    // of the v^ head tile
    static constexpr int KCT = (KCH + 255) / 256, VCT = (VCH + 255) / 256;
};

template <int DZ, int NWIN>
__global__ __launch_bounds__(256, 1) void fipa_attn_fwd_wide_kernel(AttnParams p)
{
    using C = WideCfg<DZ, NWIN>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int chunk = (p.total_tiles + 7) / 8;
    const int logical = (blockIdx.x % 8) * chunk + blockIdx.x / 8;
    if (logical >= p.total_tiles) return;
    const int win = blockIdx.y;
    const int bh = logical / p.nQT, qt = logical - bh * p.nQT;
    const int b = bh / p.H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, g = lane >> 5;
    const int kvlen = p.kvlen[b];
    const int nblk = (kvlen + kKB - 1) / kKB;
    const int irow = qt * kTileQ + wave * 32 + li;

    const bf16_t *Kh = p.Kh + (size_t)bh * p.Lp * kDH, *Vh = p.Vh + (size_t)bh * p.Lp * kDH;
    const bf16_t *Z2 = p.Z2 + (size_t)b * p.Lp * DZ;
    const float *kbias = p.kbias + (size_t)bh * p.Lp;

    bf16x8 qf[C::KS];
    {
        const bf16_t *qh = p.Qh + ((size_t)bh * p.Lp + irow) * kDH;
        const bf16_t *qz = p.Qz + ((size_t)bh * p.Lp + irow) * DZ;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const bf16_t *src = ks < C::KSH ? qh + ks * 16 + 8 * g : qz + (ks - C::KSH) * 16 + 8 * g;
            qf[ks] = *reinterpret_cast<const bf16x8 *>(src);
        }
    }
    f32x16 acc[C::NBW];
#pragma unroll
    for (int nb = 0; nb < C::NBW; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[nb][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const int kaddr = C::K_OFF + li * C::RS + g * 16;
    const int l16 = lane & 15, grp2 = (lane >> 4) & 1, e4 = l16 >> 2, j4 = l16 & 3;
    const int vaddr_z = C::K_OFF + (4 * g + e4) * C::RS + (16 * grp2 + 4 * j4) * 2 + kDH * 2;  // pair part of the k^ tile
    const int vaddr_h = C::V_OFF + (4 * g + e4) * C::VS + (16 * grp2 + 4 * j4) * 2;

    // start at the block holding the tile's own residues (see the main kernel) and wrap around
    const int first_blk = min(qt * (kTileQ / kKB), max(nblk - 1, 0));
    for (int n = 0; n < nblk; ++n) {
        const int blk = first_blk + n < nblk ? first_blk + n : first_blk + n - nblk;
        const int r0 = blk * kKB;
        uint4 kst[C::KCT], vst[C::VCT];
#pragma unroll
        for (int it = 0; it < C::KCT; ++it) {
            const int q = min(it * 256 + tid, C::KCH - 1);
            const int row = q / (C::D / 8), cc = q - row * (C::D / 8);
            const bf16_t *src = cc < kDH / 8 ? Kh + (size_t)(r0 + row) * kDH + cc * 8
                                             : Z2 + (size_t)(r0 + row) * DZ + (cc - kDH / 8) * 8;
            kst[it] = *reinterpret_cast<const uint4 *>(src);
        }
#pragma unroll
        for (int it = 0; it < C::VCT; ++it) {
            const int q = min(it * 256 + tid, C::VCH - 1);
            vst[it] = *reinterpret_cast<const uint4 *>(Vh + (size_t)r0 * kDH + q * 8);
        }
        float kb = 0.f;
        if (tid < kKB) kb = kbias[r0 + tid];
        __syncthreads();
#pragma unroll
        for (int it = 0; it < C::KCT; ++it) {
            const int q = min(it * 256 + tid, C::KCH - 1);
            const int row = q / (C::D / 8), cc = q - row * (C::D / 8);
            *reinterpret_cast<uint4 *>(smem + C::K_OFF + row * C::RS + cc * 16) = kst[it];
        }
#pragma unroll
        for (int it = 0; it < C::VCT; ++it) {
            const int q = min(it * 256 + tid, C::VCH - 1);
            const int row = q / (kDH / 8), cc = q - row * (kDH / 8);
            *reinterpret_cast<uint4 *>(smem + C::V_OFF + row * C::VS + cc * 16) = vst[it];
        }
        if (tid < kKB) *reinterpret_cast<float *>(smem + C::B_OFF + tid * 4) = kb;
        __syncthreads();

        f32x16 sacc;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const f32x4 bias = *reinterpret_cast<const f32x4 *>(smem + C::B_OFF + (8 * a + 4 * g) * 4);
#pragma unroll
            for (int x = 0; x < 4; ++x) sacc[4 * a + x] = bias[x];
        }
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(smem + kaddr + ks * 32);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], sacc, 0, 0, 0);
        }
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
        const bf16x8 pf[2] = {__builtin_bit_cast(bf16x8, (u32x4){pp[0], pp[1], pp[2], pp[3]}),
                              __builtin_bit_cast(bf16x8, (u32x4){pp[4], pp[5], pp[6], pp[7]})};
#pragma unroll
        for (int nbw = 0; nbw < C::NBW; ++nbw) {
            const int nb = win * C::NBW + nbw;  // global 32-column block (win is uniform)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const bool head = nb < C::NBH;
                const char *src = head ? smem + vaddr_h + 16 * tt * C::VS + nb * 64
                                       : smem + vaddr_z + 16 * tt * C::RS + (nb - C::NBH) * 64;
                const int rs = head ? C::VS : C::RS;
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
    hipError_t e = hipFuncSetAttribute((const void *)fipa_attn_fwd_wide_kernel<512, 2>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    const int chunk = (p.total_tiles + 7) / 8;
    hipLaunchKernelGGL((fipa_attn_fwd_wide_kernel<512, 2>), dim3(chunk * 8, 2), dim3(256), C::LDS_BYTES, stream, p);
    return hipGetLastError();
}

}  // namespace fipa
