// The IPA module around the attention core (Eq. 1 and Eq. 5 of the paper; Algorithm 1 steps 1
// and 10): input projection of the single representation, core, output projection of the
// concatenated results.  Both projections are small next to the attention (2.4 and 4.4 GFLOP
// against 117 GFLOP at B=2, L=2048, d_s=256), so one plain MFMA GEMM kernel serves them:
//     C[M, N] = A[M, K] W[N, K]^T + bias[N]        (weights stored [out, in])
// Two variations:
//   - the input projection scatters its bf16 results into the six tensors the core takes;
//   - the output projection reads its A operand directly from the core's fp32 outputs, forming
//     the concatenation (o_pair | o | o_pts | norms of o_pts) and the norms on the fly.
#include "fipa_gfx950.h"

namespace fipa {

namespace {

struct GemmParams {
    int M, N, K;
    const bf16_t *W;     // [N, K]
    const float *bias;   // [N] or null
    const bf16_t *A;     // [M, K]                              (input projection)
    const float *o_pair, *o, *o_pts;  // [M, k_pair], [M, k_o], [M, k_pts]   (output projection)
    int k_pair, k_o, k_pts;           // K = k_pair + k_o + k_pts + k_pts / 3
    float *C;            // [M, N] float32                      (output projection)
    bf16_t *seg_ptr[6];  // six row-major bf16 tensors [M, width] (input projection)
    int seg_start[7];    // first column of each, and N
};

__device__ __forceinline__ bf16x8 to_bf16x8(const float (&v)[8])
{
    unsigned pk[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const bf16x2 b = __builtin_convertvector((f32x2){v[2 * x], v[2 * x + 1]}, bf16x2);
        pk[x] = __builtin_bit_cast(unsigned, b);
    }
    return __builtin_bit_cast(bf16x8, (u32x4){pk[0], pk[1], pk[2], pk[3]});
}

// Eight consecutive entries k .. k+7 of row `row` of the concatenation of Eq. 5 (segment widths
// are multiples of 8, so a chunk never straddles two segments).  direct_chunk serves the three
// copied segments without branching; concat_chunk serves any k.
__device__ __forceinline__ void direct_chunk(const GemmParams &p, int row, int k, f32x4 &lo, f32x4 &hi)
{
    const int e1 = p.k_pair, e2 = e1 + p.k_o;
    const float *src = k < e1 ? p.o_pair + (size_t)row * p.k_pair + k
                              : (k < e2 ? p.o + (size_t)row * p.k_o + (k - e1) : p.o_pts + (size_t)row * p.k_pts + (k - e2));
    lo = *reinterpret_cast<const f32x4 *>(src);
    hi = *reinterpret_cast<const f32x4 *>(src + 4);
}

__device__ __forceinline__ bf16x8 chunk_to_bf16(const f32x4 &lo, const f32x4 &hi)
{
    const float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return to_bf16x8(v);
}

__device__ __forceinline__ bf16x8 concat_chunk(const GemmParams &p, int row, int k)
{
    const int e3 = p.k_pair + p.k_o + p.k_pts;
    if (k < e3) {
        f32x4 lo, hi;
        direct_chunk(p, row, k, lo, hi);
        return chunk_to_bf16(lo, hi);
    }
    float v[8];
    const float *src = p.o_pts + (size_t)row * p.k_pts + 3 * (k - e3);  // points k-e3 .. +7
#pragma unroll
    for (int x = 0; x < 8; ++x) {
        const float px = src[3 * x], py = src[3 * x + 1], pz = src[3 * x + 2];
        v[x] = sqrtf(px * px + py * py + pz * pz);
    }
    return to_bf16x8(v);
}

// Four waves arranged WM x WN, each computing (32 MTW) x (32 NTW) outputs; K in chunks of 64
// staged through LDS in two buffers (the next chunk is fetched into registers while the current
// one is multiplied; one barrier per chunk).  The products are computed transposed,
// C^T = W A^T (MFMA rows = output features, lanes = rows of A), so that a lane ends up with
// runs of four consecutive output features of one row: 16-byte stores.
// At the sizes of this module (a few GFLOP, K = 256 or about 2000) the products are bound by the
// chain of dependent memory round trips of each workgroup, not by the matrix pipe: 64 x 64
// tiles, which give one workgroup per compute unit at B*L = 4096 rows, measured fastest (14 and
// 28 microseconds); 128 x 128 or 32 x 256 tiles read less through L2 but leave fewer, longer
// chains (18 and 35), 32 x 64 tiles with 256-wide K chunks become bound by L2 re-reads (19 and 35).
constexpr int kGK = 64;               // K chunk
constexpr int kGRS = kGK * 2 + 16;    // LDS row stride in bytes (conflict free for 16-byte row reads)

template <int WM, int WN, int MTW, int NTW>
struct GemmTile {
    static_assert(WM * WN == 4, "four waves");
    static constexpr int WM_ = WM, MTW_ = MTW, NTW_ = NTW;
    static constexpr int TM = 32 * MTW * WM, TN = 32 * NTW * WN;   // workgroup tile
    static constexpr int CA = TM * (kGK / 8) / 256, CW = TN * (kGK / 8) / 256;  // 16-byte chunks per thread and K chunk
    static_assert(CA >= 1 && CW >= 1, "tile too small for 256 threads");
    static constexpr int LDS_BYTES = 2 * (TM + TN) * kGRS;
};

template <class T, bool CONCAT_A, bool SCATTER>
__global__ __launch_bounds__(256) void fipa_gemm_kernel(GemmParams p)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];  // [buffer][A tile | W tile]
    constexpr int kBuf = (T::TM + T::TN) * kGRS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, kg = lane >> 5;
    const int m0 = blockIdx.x * T::TM, n0 = blockIdx.y * T::TN;

    // staging: thread t moves chunks (row t/8 + 32 j, 8 k-values t%8): j < CA of A, j < CW of W
    // (fetch only requests; whatever needs the loaded values -- the float -> bfloat16 conversion
    // of the concatenation -- happens in stash, after the MFMAs of the current chunk)
    const int srow = tid >> 3, sch = tid & 7;
    struct Staged {
        uint4 a[CONCAT_A ? 1 : T::CA], w[T::CW];                    // bf16 chunks (a: input projection only)
        f32x4 lo[CONCAT_A ? T::CA : 1], hi[CONCAT_A ? T::CA : 1];    // float32 chunks of the concatenation
    };
    const int e3 = CONCAT_A ? p.k_pair + p.k_o + p.k_pts : 0;  // first norm column
    auto fetch = [&](int kc, Staged &st) {
        const int k = kc * kGK + 8 * sch;
        const int kk = min(k, p.K - 8);  // K is a multiple of 8, not necessarily of the chunk
#pragma unroll
        for (int j = 0; j < T::CA; ++j) {
            const int mg = min(m0 + srow + 32 * j, p.M - 1);  // past the end: recompute the last one
            if constexpr (CONCAT_A)
                direct_chunk(p, mg, min(kk, e3 - 8), st.lo[j], st.hi[j]);
            else
                st.a[j] = *reinterpret_cast<const uint4 *>(p.A + (size_t)mg * p.K + kk);
        }
#pragma unroll
        for (int j = 0; j < T::CW; ++j)
            st.w[j] = *reinterpret_cast<const uint4 *>(p.W + (size_t)min(n0 + srow + 32 * j, p.N - 1) * p.K + kk);
    };
    auto stash = [&](int buf, int kc, const Staged &st) {
        const int k = kc * kGK + 8 * sch;
        const bool in_k = k < p.K;
        char *ab = lds + buf * kBuf, *wb = ab + T::TM * kGRS;
#pragma unroll
        for (int j = 0; j < T::CA; ++j) {
            uint4 av = make_uint4(0, 0, 0, 0);
            if constexpr (CONCAT_A) {
                if (k < e3)
                    av = __builtin_bit_cast(uint4, chunk_to_bf16(st.lo[j], st.hi[j]));
                else if (in_k)  // the norms: few columns at the end of K
                    av = __builtin_bit_cast(uint4, concat_chunk(p, min(m0 + srow + 32 * j, p.M - 1), k));
            } else {
                av = st.a[j];
            }
            *reinterpret_cast<uint4 *>(ab + (srow + 32 * j) * kGRS + sch * 16) = in_k ? av : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < T::CW; ++j)
            *reinterpret_cast<uint4 *>(wb + (srow + 32 * j) * kGRS + sch * 16) = in_k ? st.w[j] : make_uint4(0, 0, 0, 0);
    };

    constexpr int MTW = T::MTW_, NTW = T::NTW_;
    const int wm = wave % T::WM_, wn = wave / T::WM_;
    f32x16 acc[MTW][NTW];
#pragma unroll
    for (int a = 0; a < MTW; ++a)
#pragma unroll
        for (int b = 0; b < NTW; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    const int nkc = (p.K + kGK - 1) / kGK;
    Staged st;
    fetch(0, st);
    stash(0, 0, st);
    __syncthreads();
    for (int kc = 0; kc < nkc; ++kc) {
        const int buf = kc & 1;
        if (kc + 1 < nkc) fetch(kc + 1, st);
        const char *at = lds + buf * kBuf + (32 * MTW * wm + li) * kGRS + kg * 16;
        const char *wt = lds + buf * kBuf + T::TM * kGRS + (32 * NTW * wn + li) * kGRS + kg * 16;
#pragma unroll
        for (int ks = 0; ks < kGK / 16; ++ks) {
            bf16x8 af[MTW], wf[NTW];
#pragma unroll
            for (int a = 0; a < MTW; ++a) af[a] = *reinterpret_cast<const bf16x8 *>(at + a * 32 * kGRS + ks * 32);
#pragma unroll
            for (int b = 0; b < NTW; ++b) wf[b] = *reinterpret_cast<const bf16x8 *>(wt + b * 32 * kGRS + ks * 32);
#pragma unroll
            for (int a = 0; a < MTW; ++a)
#pragma unroll
                for (int b = 0; b < NTW; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[b], af[a], acc[a][b], 0, 0, 0);
        }
        if (kc + 1 < nkc) stash(buf ^ 1, kc + 1, st);
        __syncthreads();
    }

    // the lane holds rows m0 + 32 (MTW wm + a) + li and output features
    // n0 + 32 (NTW wn + b) + 8 q + 4 kg + x, x = 0..3
#pragma unroll
    for (int a = 0; a < MTW; ++a) {
        const int row = m0 + 32 * (MTW * wm + a) + li;
        if (row >= p.M) continue;
#pragma unroll
        for (int b = 0; b < NTW; ++b)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = n0 + 32 * (NTW * wn + b) + 8 * q + 4 * kg;
                if (col >= p.N) continue;
                float val[4];
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    val[x] = acc[a][b][4 * q + x] + ((p.bias && col + x < p.N) ? p.bias[col + x] : 0.f);
                if constexpr (SCATTER) {
                    int seg = 0;
#pragma unroll
                    for (int s = 1; s < 6; ++s)
                        if (col >= p.seg_start[s]) seg = s;
                    const int start = p.seg_start[seg], width = p.seg_start[seg + 1] - start;
                    if (col + 3 < p.seg_start[seg + 1] && ((width | (col - start)) & 3) == 0) {
                        const unsigned lo = (unsigned)f2bf(val[0]) | ((unsigned)f2bf(val[1]) << 16);
                        const unsigned hi = (unsigned)f2bf(val[2]) | ((unsigned)f2bf(val[3]) << 16);
                        *reinterpret_cast<uint2 *>(p.seg_ptr[seg] + (size_t)row * width + (col - start)) = make_uint2(lo, hi);
                    } else {
                        for (int x = 0; x < 4 && col + x < p.N; ++x) {  // a run that crosses into the next tensor
                            int sx = seg;
                            while (col + x >= p.seg_start[sx + 1]) ++sx;
                            const int wx = p.seg_start[sx + 1] - p.seg_start[sx];
                            p.seg_ptr[sx][(size_t)row * wx + (col + x - p.seg_start[sx])] = f2bf(val[x]);
                        }
                    }
                } else {
                    if (col + 3 < p.N && (p.N & 3) == 0) {
                        *reinterpret_cast<f32x4 *>(p.C + (size_t)row * p.N + col) = (f32x4){val[0], val[1], val[2], val[3]};
                    } else {
                        for (int x = 0; x < 4 && col + x < p.N; ++x) p.C[(size_t)row * p.N + col + x] = val[x];
                    }
                }
            }
    }
}

template <class T, bool CONCAT_A, bool SCATTER>
hipError_t launch_gemm(const GemmParams &g, hipStream_t stream)
{
    hipError_t e = hipFuncSetAttribute((const void *)fipa_gemm_kernel<T, CONCAT_A, SCATTER>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((fipa_gemm_kernel<T, CONCAT_A, SCATTER>), dim3((g.M + T::TM - 1) / T::TM, (g.N + T::TN - 1) / T::TN),
                       dim3(256), T::LDS_BYTES, stream, g);
    return hipGetLastError();
}

struct ModuleLayout {
    size_t core, q, k, v, q_pts, k_pts, v_pts, o, o_pts, o_pair, total;
};

ModuleLayout module_layout(const fipa_desc &d)
{
    ModuleLayout w;
    const size_t M = (size_t)d.B * d.L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    w.core = take(bf16_forward_workspace(d));
    w.q = take(M * d.H * d.c * 2);
    w.k = take(M * d.H * d.c * 2);
    w.v = take(M * d.H * d.c * 2);
    w.q_pts = take(M * d.H * d.Pq * 3 * 2);
    w.k_pts = take(M * d.H * d.Pq * 3 * 2);
    w.v_pts = take(M * d.H * d.Pv * 3 * 2);
    w.o = take(M * d.H * d.c * 4);
    w.o_pts = take(M * d.H * d.Pv * 3 * 4);
    w.o_pair = take(M * d.H * d.cz * 4);
    w.total = off;
    return w;
}

}  // namespace

bool module_shape_supported(const fipa_desc &d, int d_s)
{
    const int n_cat = d.H * (d.cz + d.c + 4 * d.Pv);
    return d_s > 0 && d_s % 16 == 0 && (d.H * d.cz) % 8 == 0 && (d.H * d.c) % 8 == 0 && (d.H * d.Pv) % 8 == 0 &&
           n_cat % 16 == 0;
}

size_t module_forward_workspace(const fipa_desc &d) { return module_layout(d).total; }

hipError_t module_forward(const fipa_desc &d, int d_s, const ModuleArgs &a, void *ws, hipStream_t stream)
{
    const ModuleLayout w = module_layout(d);
    char *base = static_cast<char *>(ws);
    const int M = d.B * d.L;

    // ---- Eq. 1: q | k | v | q_pts | k_pts | v_pts = s W_in^T + b_in, as bf16 -------------------------
    GemmParams g1 = {};
    g1.M = M; g1.K = d_s;
    g1.W = (const bf16_t *)a.w_in; g1.bias = a.b_in; g1.A = (const bf16_t *)a.s;
    const int widths[6] = {d.H * d.c, d.H * d.c, d.H * d.c, d.H * d.Pq * 3, d.H * d.Pq * 3, d.H * d.Pv * 3};
    const size_t offs[6] = {w.q, w.k, w.v, w.q_pts, w.k_pts, w.v_pts};
    g1.seg_start[0] = 0;
    for (int s = 0; s < 6; ++s) {
        g1.seg_ptr[s] = (bf16_t *)(base + offs[s]);
        g1.seg_start[s + 1] = g1.seg_start[s] + widths[s];
    }
    g1.N = g1.seg_start[6];
    hipError_t e = launch_gemm<GemmTile<2, 2, 1, 1>, false, true>(g1, stream);
    if (e != hipSuccess) return e;

    // ---- the core (Algorithm 1 steps 2-9) ------------------------------------------------------------
    FwdArgs f{base + w.q, base + w.k, base + w.v, base + w.q_pts, base + w.k_pts, base + w.v_pts,
              a.rot, a.trans, a.z1, a.z2, a.w_b, a.gamma, a.mask,
              (float *)(base + w.o), (float *)(base + w.o_pts), (float *)(base + w.o_pair), nullptr};
    e = bf16_forward(d, f, base + w.core, stream);
    if (e != hipSuccess) return e;

    // ---- Eq. 5: s_out = concat(o_pair, o, o_pts, |o_pts|) W_out^T + b_out --------------------------
    GemmParams g2 = {};
    g2.M = M; g2.N = d_s;
    g2.W = (const bf16_t *)a.w_out; g2.bias = a.b_out;
    g2.o_pair = f.o_pair; g2.o = f.o; g2.o_pts = f.o_pts;
    g2.k_pair = d.H * d.cz; g2.k_o = d.H * d.c; g2.k_pts = d.H * d.Pv * 3;
    g2.K = g2.k_pair + g2.k_o + g2.k_pts + d.H * d.Pv;
    g2.C = a.s_out;
    return launch_gemm<GemmTile<2, 2, 1, 1>, true, false>(g2, stream);
}

}  // namespace fipa
