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

#include <type_traits>

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
    int chunks_per_split;  // 0: one workgroup sums all of K; else blockIdx.z takes this many K chunks
                           // and writes its partial product to C + blockIdx.z * M * N
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
// C^T = W A^T (MFMA rows = output features, lanes = rows of A); the finished tile leaves through
// LDS (see the end of the kernel).
// At the sizes of this module (a few GFLOP, K = 256 or about 2000) the matrix pipe is idle most
// of the time.  Measured at B*L = 4096 rows, d_s = 256 (input / output projection, microseconds):
// 64 x 64 tiles 10.8 / 28; 128 x 128 or 32 x 256 tiles read less through L2 but leave fewer,
// longer chains of round trips (18 / 35 with the earlier store path); 64 x 64 tiles with 256-wide
// K chunks, a quarter of the round trips, are 15 % slower; with loads, MFMAs and stores all taken
// out the input projection still takes 5.  The output projection uses 64 x 128 tiles with K split
// (see OutTile).
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
    static constexpr int LDS_TOTAL = LDS_BYTES + TN * 4;   // + the tile's slice of the bias vector
};

template <class T, bool CONCAT_A, bool SCATTER>
__global__ __launch_bounds__(256) void fipa_gemm_kernel(GemmParams p)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];  // [buffer][A tile | W tile]
    constexpr int kBuf = (T::TM + T::TN) * kGRS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, kg = lane >> 5;
    const int m0 = blockIdx.x * T::TM, n0 = blockIdx.y * T::TN;
    // the tile's slice of the bias (zero where there is none; a split-K product adds it in its first part only);
    // the first barrier below publishes it
    float *bias_l = reinterpret_cast<float *>(lds + T::LDS_BYTES);
    if (tid < T::TN) bias_l[tid] = (p.bias && n0 + tid < p.N && blockIdx.z == 0) ? p.bias[n0 + tid] : 0.f;

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
    int kc0 = 0, nkc = (p.K + kGK - 1) / kGK;
    if (p.chunks_per_split > 0) {
        kc0 = blockIdx.z * p.chunks_per_split;
        nkc = min(nkc, kc0 + p.chunks_per_split);
    }
    Staged st;
    fetch(kc0, st);
    stash(0, kc0, st);
    __syncthreads();
    for (int kc = kc0; kc < nkc; ++kc) {
        const int buf = (kc - kc0) & 1;
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

    // The lane holds rows 32 (MTW wm + a) + li of the tile and output features
    // 32 (NTW wn + b) + 8 q + 4 kg + x, x = 0..3.  Stored from here, every lane of a store would
    // touch a different row, 8 or 16 bytes of a 64-byte line each, and the number of partial-line
    // writes, not their bytes, is what the memory system then counts (at B*L = 4096 the input
    // projection spent 6 of its 14 microseconds on them).  The tile goes through LDS instead, in
    // its final type, and leaves as 16-byte pieces that are neighbours along a row.
    // (The loop above ended with a barrier: both operand buffers are free.)
    using OutT = std::conditional_t<SCATTER, bf16_t, float>;
    constexpr int kPer = 16 / (int)sizeof(OutT);               // outputs per 16-byte piece
    constexpr int kORS = T::TN * (int)sizeof(OutT) + 16;       // LDS row stride of the staged tile
    static_assert(T::TM * kORS <= T::LDS_BYTES, "the staged output tile must fit the operand buffers");
#pragma unroll
    for (int a = 0; a < MTW; ++a)
#pragma unroll
        for (int b = 0; b < NTW; ++b)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int rl = 32 * (MTW * wm + a) + li, cl = 32 * (NTW * wn + b) + 8 * q + 4 * kg;
                const f32x4 bv = *reinterpret_cast<const f32x4 *>(bias_l + cl);
                float val[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) val[x] = acc[a][b][4 * q + x] + bv[x];
                char *dst = lds + rl * kORS + cl * (int)sizeof(OutT);
                if constexpr (SCATTER) {
                    const unsigned lo = (unsigned)f2bf(val[0]) | ((unsigned)f2bf(val[1]) << 16);
                    const unsigned hi = (unsigned)f2bf(val[2]) | ((unsigned)f2bf(val[3]) << 16);
                    *reinterpret_cast<uint2 *>(dst) = make_uint2(lo, hi);
                } else {
                    *reinterpret_cast<f32x4 *>(dst) = (f32x4){val[0], val[1], val[2], val[3]};
                }
            }
    __syncthreads();
    constexpr int kPieces = T::TN / kPer;  // per row
    for (int idx = tid; idx < T::TM * kPieces; idx += 256) {
        const int rl = idx / kPieces, pc = idx - rl * kPieces;
        const int row = m0 + rl, col = n0 + pc * kPer;
        if (row >= p.M || col >= p.N) continue;
        const uint4 piece = *reinterpret_cast<const uint4 *>(lds + rl * kORS + pc * 16);
        const OutT *vals = reinterpret_cast<const OutT *>(&piece);
        if constexpr (SCATTER) {
            int seg = 0;
#pragma unroll
            for (int sg = 1; sg < 6; ++sg)
                if (col >= p.seg_start[sg]) seg = sg;
            const int start = p.seg_start[seg], width = p.seg_start[seg + 1] - start;
            if (col + kPer <= p.seg_start[seg + 1] && ((width | (col - start)) & (kPer - 1)) == 0) {
                *reinterpret_cast<uint4 *>(p.seg_ptr[seg] + (size_t)row * width + (col - start)) = piece;
            } else {
                for (int x = 0; x < kPer && col + x < p.N; ++x) {  // a piece that crosses into the next tensor, or is not aligned
                    int sx = seg;
                    while (col + x >= p.seg_start[sx + 1]) ++sx;
                    const int wx = p.seg_start[sx + 1] - p.seg_start[sx];
                    p.seg_ptr[sx][(size_t)row * wx + (col + x - p.seg_start[sx])] = vals[x];
                }
            }
        } else {
            float *C = p.C + (p.chunks_per_split > 0 ? (size_t)blockIdx.z * p.M * p.N : 0);
            if (col + kPer <= p.N && (p.N & (kPer - 1)) == 0) {
                *reinterpret_cast<uint4 *>(C + (size_t)row * p.N + col) = piece;
            } else {
                for (int x = 0; x < kPer && col + x < p.N; ++x) C[(size_t)row * p.N + col + x] = vals[x];
            }
        }
    }
}

template <class T, bool CONCAT_A, bool SCATTER>
hipError_t launch_gemm(const GemmParams &g, hipStream_t stream)
{
    static LdsLimit lds_limit;
    hipError_t e = raise_lds_limit(lds_limit, (const void *)fipa_gemm_kernel<T, CONCAT_A, SCATTER>, T::LDS_TOTAL);
    if (e != hipSuccess) return e;
    const int nkc = (g.K + kGK - 1) / kGK;
    const int nsplit = g.chunks_per_split > 0 ? (nkc + g.chunks_per_split - 1) / g.chunks_per_split : 1;
    hipLaunchKernelGGL((fipa_gemm_kernel<T, CONCAT_A, SCATTER>),
                       dim3((g.M + T::TM - 1) / T::TM, (g.N + T::TN - 1) / T::TN, nsplit), dim3(256), T::LDS_TOTAL,
                       stream, g);
    return hipGetLastError();
}

struct ModuleLayout {
    size_t core, q, k, v, q_pts, k_pts, v_pts, o, o_pts, o_pair, part, total;
};

// The output projection (Eq. 5) at B*L rows has few output tiles for 256 compute units (N = d_s
// is small, K = H (c_z + c + 4 P_v) long): 64 x 128 tiles -- the float32 concatenation is then read
// through L2 twice at d_s = 256 instead of four times -- with K split into up to four parts that
// leave partial products, summed in a fixed order afterwards.  (Measured at B*L = 4096, d_s = 256:
// 64 x 64 tiles unsplit 28 us; this form 16 + 5 us; 128 x 128 tiles split in eight 23 + 7 us.)
using OutTile = GemmTile<2, 2, 1, 2>;
struct OutSplit {
    int chunks_per_split, nsplit;  // nsplit = 1: no partial products
};
OutSplit out_projection_split(int M, int d_s, int n_cat)
{
    const int tiles = ((M + OutTile::TM - 1) / OutTile::TM) * ((d_s + OutTile::TN - 1) / OutTile::TN);
    const int nkc = (n_cat + kGK - 1) / kGK;
    int want = 512 / (tiles > 0 ? tiles : 1);
    want = want > 4 ? 4 : (want < 1 ? 1 : want);
    OutSplit o;
    o.chunks_per_split = (nkc + want - 1) / want;
    o.nsplit = (nkc + o.chunks_per_split - 1) / o.chunks_per_split;
    return o;
}

ModuleLayout module_layout(const fipa_desc &d, int d_s)
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
    const OutSplit os = out_projection_split((int)M, d_s, d.H * (d.cz + d.c + 4 * d.Pv));
    w.part = os.nsplit > 1 ? take((size_t)os.nsplit * M * d_s * 4) : 0;
    w.total = off;
    return w;
}

// ---- small memory-bound kernels of the module's backward ----------------------------------------

// dst[c][r] = bf16(src[r][c]) for a row-major [R, C] matrix of float or bf16 (32 x 32 tiles through
// LDS); dst has rows of length ld >= R, the tail of each row is set to zero.
template <class SrcT>
__global__ __launch_bounds__(256) void fipa_transpose_bf16_kernel(const SrcT *__restrict__ src, bf16_t *__restrict__ dst,
                                                                  int R, int C, int ld)
{
    __shared__ bf16_t tile[32][33];
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    for (int j = ty; j < 32; j += 8) {
        const int r = r0 + j, c = c0 + tx;
        bf16_t v = 0;
        if (r < R && c < C) {
            if constexpr (sizeof(SrcT) == 4)
                v = f2bf(((const float *)src)[(size_t)r * C + c]);
            else
                v = ((const bf16_t *)src)[(size_t)r * C + c];
        }
        tile[j][tx] = v;
    }
    __syncthreads();
    for (int j = ty; j < 32; j += 8) {
        const int c = c0 + j, r = r0 + tx;
        if (r < ld && c < C) dst[(size_t)c * ld + r] = tile[tx][j];  // (tile entries with r >= R hold zero)
    }
}

template <class SrcT>
hipError_t launch_transpose(const SrcT *src, bf16_t *dst, int R, int C, int ld, hipStream_t stream)
{
    hipLaunchKernelGGL((fipa_transpose_bf16_kernel<SrcT>), dim3((C + 31) / 32, (ld + 31) / 32), dim3(256), 0, stream, src, dst,
                       R, C, ld);
    return hipGetLastError();
}

// float32 -> bf16 copy.
__global__ __launch_bounds__(256) void fipa_to_bf16_kernel(const float *__restrict__ src, bf16_t *__restrict__ dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = f2bf(src[i]);
}

// Row r of the concatenation of Eq. 5 as bf16: [o_pair | o | o_pts | norms].
__global__ __launch_bounds__(256) void fipa_concat_bf16_kernel(GemmParams p, bf16_t *__restrict__ cat)
{
    const int row = blockIdx.x;
    for (int k = 8 * threadIdx.x; k < p.K; k += 8 * 256)
        *reinterpret_cast<bf16x8 *>(cat + (size_t)row * p.K + k) = concat_chunk(p, row, k);
}

// Gradient of the concatenation back to the core's upstream gradients:
//   d_o_pair, d_o copied; d_o_pts = its own columns + d_norm * o_pts / |o_pts| (zero at a zero vector).
__global__ __launch_bounds__(256) void fipa_split_dcat_kernel(const float *__restrict__ dcat, const float *__restrict__ o_pts,
                                                               float *__restrict__ d_o_pair, float *__restrict__ d_o,
                                                               float *__restrict__ d_o_pts, int k_pair, int k_o, int k_pts)
{
    const int row = blockIdx.x;
    const int K = k_pair + k_o + k_pts + k_pts / 3;
    const float *src = dcat + (size_t)row * K;
    for (int k = threadIdx.x; k < k_pair; k += 256) d_o_pair[(size_t)row * k_pair + k] = src[k];
    for (int k = threadIdx.x; k < k_o; k += 256) d_o[(size_t)row * k_o + k] = src[k_pair + k];
    for (int pt = threadIdx.x; pt < k_pts / 3; pt += 256) {
        const float *op = o_pts + (size_t)row * k_pts + 3 * pt;
        const float nrm = sqrtf(op[0] * op[0] + op[1] * op[1] + op[2] * op[2]);
        const float gn = nrm > 0.f ? src[k_pair + k_o + k_pts + pt] / nrm : 0.f;
        for (int x = 0; x < 3; ++x)
            d_o_pts[(size_t)row * k_pts + 3 * pt + x] = src[k_pair + k_o + 3 * pt + x] + gn * op[x];
    }
}

// The six bf16 gradient tensors of the core, side by side: dX [M, N_in].
__global__ __launch_bounds__(256) void fipa_gather6_kernel(GemmParams p, bf16_t *__restrict__ dst)
{
    const int row = blockIdx.x;
    for (int col = threadIdx.x; col < p.N; col += 256) {
        int seg = 0;
#pragma unroll
        for (int s = 1; s < 6; ++s)
            if (col >= p.seg_start[s]) seg = s;
        const int width = p.seg_start[seg + 1] - p.seg_start[seg];
        dst[(size_t)row * p.N + col] = p.seg_ptr[seg][(size_t)row * width + (col - p.seg_start[seg])];
    }
}

// out[i] = sum over the nsplit partial matrices (fixed order), n entries each; n is a multiple of 4
// (every matrix summed here has d_s, a multiple of 16, as one of its dimensions).
__global__ __launch_bounds__(256) void fipa_sum_partials_kernel(const float *__restrict__ part, float *__restrict__ out,
                                                                 size_t n, int nsplit)
{
    const size_t i = 4 * ((size_t)blockIdx.x * 256 + threadIdx.x);
    if (i >= n) return;
    f32x4 s = *reinterpret_cast<const f32x4 *>(part + i);
    for (int z = 1; z < nsplit; ++z) {
        const f32x4 t = *reinterpret_cast<const f32x4 *>(part + (size_t)z * n + i);
#pragma unroll
        for (int x = 0; x < 4; ++x) s[x] += t[x];
    }
    *reinterpret_cast<f32x4 *>(out + i) = s;
}

// out[r] = sum over the C entries of row r of a bf16 matrix [R, C] (one workgroup per row, fixed order).
__global__ __launch_bounds__(256) void fipa_rowsum_bf16_kernel(const bf16_t *__restrict__ src, float *__restrict__ out, int C)
{   // (rows may carry a zero tail: C is the stored row length)
    __shared__ float red[256];
    const int r = blockIdx.x;
    float s = 0.f;
    for (int c = threadIdx.x; c < C; c += 256) s += bf2f(src[(size_t)r * C + c]);
    red[threadIdx.x] = s;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if (threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[r] = red[0];
}

constexpr int kWgradChunks = 8;  // K chunks (of 64 rows of the batch) per workgroup of a weight-gradient product

struct ModuleBwdLayout {
    ModuleLayout f;   // forward part: core workspace slot (sized for the backward), core inputs and outputs
    size_t g16, gT, w_outT, w_inT, sT, dcat, d_o, d_o_pts, d_o_pair, dq, dk, dv, dq_pts, dk_pts, dv_pts, dX, dXT, cat,
        catT, part, total;
};

ModuleBwdLayout module_bwd_layout(const fipa_desc &d, int d_s)
{
    ModuleBwdLayout w;
    const size_t M = (size_t)d.B * d.L, Mp = align_up(M, kGK);  // transposed matrices carry rows of Mp entries
    const size_t n_in = (size_t)d.H * (3 * d.c + 3 * (2 * d.Pq + d.Pv)), n_cat = (size_t)d.H * (d.cz + d.c + 4 * d.Pv);

    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    // the forward layout with the core slot enlarged to what the core's backward needs
    w.f.core = take(bf16_backward_workspace(d) > bf16_forward_workspace(d) ? bf16_backward_workspace(d)
                                                                           : bf16_forward_workspace(d));
    w.f.q = take(M * d.H * d.c * 2);
    w.f.k = take(M * d.H * d.c * 2);
    w.f.v = take(M * d.H * d.c * 2);
    w.f.q_pts = take(M * d.H * d.Pq * 3 * 2);
    w.f.k_pts = take(M * d.H * d.Pq * 3 * 2);
    w.f.v_pts = take(M * d.H * d.Pv * 3 * 2);
    w.f.o = take(M * d.H * d.c * 4);
    w.f.o_pts = take(M * d.H * d.Pv * 3 * 4);
    w.f.o_pair = take(M * d.H * d.cz * 4);
    // (for a forward call that runs in this layout, FIPA_FLAG_KEEP_FORWARD: its partial products)
    const OutSplit os = out_projection_split((int)M, d_s, (int)n_cat);
    w.f.part = os.nsplit > 1 ? take((size_t)os.nsplit * M * d_s * 4) : 0;
    w.f.total = 0;
    w.g16 = take(M * d_s * 2);
    w.gT = take(Mp * d_s * 2);
    w.w_outT = take(n_cat * d_s * 2);
    w.w_inT = take(n_in * d_s * 2);
    w.sT = take(Mp * d_s * 2);
    w.dcat = take(M * n_cat * 4);
    w.d_o = take(M * d.H * d.c * 4);
    w.d_o_pts = take(M * d.H * d.Pv * 3 * 4);
    w.d_o_pair = take(M * d.H * d.cz * 4);
    w.dq = take(M * d.H * d.c * 2);
    w.dk = take(M * d.H * d.c * 2);
    w.dv = take(M * d.H * d.c * 2);
    w.dq_pts = take(M * d.H * d.Pq * 3 * 2);
    w.dk_pts = take(M * d.H * d.Pq * 3 * 2);
    w.dv_pts = take(M * d.H * d.Pv * 3 * 2);
    w.dX = take(M * n_in * 2);
    w.dXT = take(Mp * n_in * 2);
    w.cat = take(M * n_cat * 2);
    w.catT = take(Mp * n_cat * 2);
    const size_t nsplit = ((M + kGK - 1) / kGK + kWgradChunks - 1) / kWgradChunks;
    w.part = take(nsplit * (n_cat > n_in ? n_cat : n_in) * d_s * 4);
    w.total = off;
    return w;
}

}  // namespace

bool module_backward_shape_supported(const fipa_desc &d, int d_s)
{
    const int n_in = d.H * (3 * d.c + 3 * (2 * d.Pq + d.Pv));
    return module_shape_supported(d, d_s) && n_in % 8 == 0 && (long long)d.r * d.cz <= 512;
}

bool module_shape_supported(const fipa_desc &d, int d_s)
{
    const int n_cat = d.H * (d.cz + d.c + 4 * d.Pv);
    return d_s > 0 && d_s % 16 == 0 && (d.H * d.cz) % 8 == 0 && (d.H * d.c) % 8 == 0 && (d.H * d.Pv) % 8 == 0 &&
           n_cat % 16 == 0;
}

size_t module_forward_workspace(const fipa_desc &d, int d_s) { return module_layout(d, d_s).total; }

hipError_t module_forward(const fipa_desc &d, int d_s, const ModuleArgs &a, void *ws, hipStream_t stream)
{
    // With FIPA_FLAG_KEEP_FORWARD the call runs in the backward's layout and leaves there what the
    // backward call would otherwise compute again: the projected inputs, the core's outputs, and
    // inside the core's slot the lifted operands, O^ and the log-sum-exp.
    const bool keep = (d.flags & FIPA_FLAG_KEEP_FORWARD) != 0;
    const ModuleLayout w = keep ? module_bwd_layout(d, d_s).f : module_layout(d, d_s);
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
    e = keep ? bf16_backward_begin(d, f, base + w.core, stream) : bf16_forward(d, f, base + w.core, stream);
    if (e != hipSuccess) return e;

    // ---- Eq. 5: s_out = concat(o_pair, o, o_pts, |o_pts|) W_out^T + b_out --------------------------
    GemmParams g2 = {};
    g2.M = M; g2.N = d_s;
    g2.W = (const bf16_t *)a.w_out; g2.bias = a.b_out;
    g2.o_pair = f.o_pair; g2.o = f.o; g2.o_pts = f.o_pts;
    g2.k_pair = d.H * d.cz; g2.k_o = d.H * d.c; g2.k_pts = d.H * d.Pv * 3;
    g2.K = g2.k_pair + g2.k_o + g2.k_pts + d.H * d.Pv;
    const OutSplit os = out_projection_split(M, d_s, g2.K);
    if (os.nsplit == 1) {
        g2.C = a.s_out;
        return launch_gemm<OutTile, true, false>(g2, stream);
    }
    g2.C = (float *)(base + w.part);
    g2.chunks_per_split = os.chunks_per_split;
    e = launch_gemm<OutTile, true, false>(g2, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fipa_sum_partials_kernel, dim3((unsigned)(((size_t)M * d_s / 4 + 255) / 256)), dim3(256), 0, stream,
                       g2.C, a.s_out, (size_t)M * d_s, os.nsplit);
    return hipGetLastError();
}

size_t module_backward_workspace(const fipa_desc &d, int d_s) { return module_bwd_layout(d, d_s).total; }

hipError_t module_backward(const fipa_desc &d, int d_s, const ModuleArgs &a, const ModuleBwdArgs &g, void *ws,
                           hipStream_t stream)
{
    const ModuleBwdLayout w = module_bwd_layout(d, d_s);
    char *base = static_cast<char *>(ws);
    const int M = d.B * d.L, Mp = (int)align_up((size_t)M, kGK);
    const int widths[6] = {d.H * d.c, d.H * d.c, d.H * d.c, d.H * d.Pq * 3, d.H * d.Pq * 3, d.H * d.Pv * 3};
    const int n_cat = d.H * (d.cz + d.c + 4 * d.Pv);
    hipError_t e;
#define FIPA_TRY(call)        \
    do {                      \
        e = (call);           \
        if (e != hipSuccess)  \
            return e;         \
    } while (0)

    // ---- forward again: Eq. 1 and the core (its outputs feed the norm's derivative and d W_out) ----
    GemmParams g1 = {};
    g1.M = M; g1.K = d_s;
    g1.W = (const bf16_t *)a.w_in; g1.bias = a.b_in; g1.A = (const bf16_t *)a.s;
    const size_t in_offs[6] = {w.f.q, w.f.k, w.f.v, w.f.q_pts, w.f.k_pts, w.f.v_pts};
    g1.seg_start[0] = 0;
    for (int s = 0; s < 6; ++s) {
        g1.seg_ptr[s] = (bf16_t *)(base + in_offs[s]);
        g1.seg_start[s + 1] = g1.seg_start[s] + widths[s];
    }
    g1.N = g1.seg_start[6];
    const int n_in = g1.N;
    const bool kept = (d.flags & FIPA_FLAG_KEEP_FORWARD) != 0;  // the forward call left all of this in the workspace
    if (!kept) FIPA_TRY((launch_gemm<GemmTile<2, 2, 1, 1>, false, true>(g1, stream)));
    FwdArgs f{base + w.f.q, base + w.f.k, base + w.f.v, base + w.f.q_pts, base + w.f.k_pts, base + w.f.v_pts,
              a.rot, a.trans, a.z1, a.z2, a.w_b, a.gamma, a.mask,
              (float *)(base + w.f.o), (float *)(base + w.f.o_pts), (float *)(base + w.f.o_pair), nullptr};
    // (the forward part of the core's backward, which leaves O^ and the log-sum-exp for the gradient
    // kernels, also gives the core's outputs: no separate forward call)
    if (!kept) FIPA_TRY(bf16_backward_begin(d, f, base + w.f.core, stream));

    // ---- through Eq. 5: d cat = d s_out W_out; d W_out = d s_out^T cat; d b_out = column sums ----------
    bf16_t *g16 = (bf16_t *)(base + w.g16), *gT = (bf16_t *)(base + w.gT);
    hipLaunchKernelGGL(fipa_to_bf16_kernel, dim3((unsigned)(((size_t)M * d_s + 255) / 256)), dim3(256), 0, stream,
                       g.d_s_out, g16, (size_t)M * d_s);
    FIPA_TRY(launch_transpose<float>(g.d_s_out, gT, M, d_s, Mp, stream));                                // [d_s, Mp]
    FIPA_TRY(launch_transpose<bf16_t>((const bf16_t *)a.w_out, (bf16_t *)(base + w.w_outT), d_s, n_cat, d_s, stream));  // [N_cat, d_s]
    GemmParams gc = {};
    gc.M = M; gc.N = n_cat; gc.K = d_s;
    gc.A = g16; gc.W = (const bf16_t *)(base + w.w_outT); gc.C = (float *)(base + w.dcat);
    FIPA_TRY((launch_gemm<GemmTile<2, 2, 1, 1>, false, false>(gc, stream)));
    GemmParams cp = {};  // description of the concatenation (as for the forward's output projection)
    cp.M = M; cp.o_pair = f.o_pair; cp.o = f.o; cp.o_pts = f.o_pts;
    cp.k_pair = d.H * d.cz; cp.k_o = d.H * d.c; cp.k_pts = d.H * d.Pv * 3; cp.K = n_cat;
    hipLaunchKernelGGL(fipa_split_dcat_kernel, dim3(M), dim3(256), 0, stream, gc.C, f.o_pts, (float *)(base + w.d_o_pair),
                       (float *)(base + w.d_o), (float *)(base + w.d_o_pts), cp.k_pair, cp.k_o, cp.k_pts);
    hipLaunchKernelGGL(fipa_concat_bf16_kernel, dim3(M), dim3(256), 0, stream, cp, (bf16_t *)(base + w.cat));
    FIPA_TRY(launch_transpose<bf16_t>((const bf16_t *)(base + w.cat), (bf16_t *)(base + w.catT), M, n_cat, Mp, stream));  // [N_cat, Mp]
    const int nkc = Mp / kGK, nsplit = (nkc + kWgradChunks - 1) / kWgradChunks;
    GemmParams gw = {};
    gw.M = d_s; gw.N = n_cat; gw.K = Mp;
    gw.A = gT; gw.W = (const bf16_t *)(base + w.catT); gw.C = (float *)(base + w.part); gw.chunks_per_split = kWgradChunks;
    FIPA_TRY((launch_gemm<GemmTile<2, 2, 1, 1>, false, false>(gw, stream)));
    hipLaunchKernelGGL(fipa_sum_partials_kernel, dim3((unsigned)(((size_t)d_s * n_cat / 4 + 255) / 256)), dim3(256), 0, stream,
                       gw.C, g.d_w_out, (size_t)d_s * n_cat, nsplit);
    if (g.d_b_out) hipLaunchKernelGGL(fipa_rowsum_bf16_kernel, dim3(d_s), dim3(256), 0, stream, gT, g.d_b_out, Mp);
    FIPA_TRY(hipGetLastError());

    // ---- the core's backward -----------------------------------------------------------------------
    BwdArgs b;
    b.f = f;
    b.d_o = (const float *)(base + w.d_o); b.d_o_pts = (const float *)(base + w.d_o_pts);
    b.d_o_pair = (const float *)(base + w.d_o_pair);
    b.d_q = base + w.dq; b.d_k = base + w.dk; b.d_v = base + w.dv;
    b.d_q_pts = base + w.dq_pts; b.d_k_pts = base + w.dk_pts; b.d_v_pts = base + w.dv_pts;
    b.d_z1 = g.d_z1; b.d_z2 = g.d_z2; b.d_gamma = g.d_gamma; b.d_w_b = g.d_w_b; b.d_rot = g.d_rot; b.d_trans = g.d_trans;
    FIPA_TRY(bf16_backward_finish(d, b, base + w.f.core, stream));

    // ---- through Eq. 1: d s = dX W_in; d W_in = dX^T s; d b_in = column sums of dX ---------------------
    GemmParams gx = {};
    gx.M = M; gx.N = n_in;
    const size_t gr_offs[6] = {w.dq, w.dk, w.dv, w.dq_pts, w.dk_pts, w.dv_pts};
    gx.seg_start[0] = 0;
    for (int s = 0; s < 6; ++s) {
        gx.seg_ptr[s] = (bf16_t *)(base + gr_offs[s]);
        gx.seg_start[s + 1] = gx.seg_start[s] + widths[s];
    }
    bf16_t *dX = (bf16_t *)(base + w.dX), *dXT = (bf16_t *)(base + w.dXT);
    hipLaunchKernelGGL(fipa_gather6_kernel, dim3(M), dim3(256), 0, stream, gx, dX);
    FIPA_TRY(launch_transpose<bf16_t>(dX, dXT, M, n_in, Mp, stream));                                                  // [N_in, Mp]
    FIPA_TRY(launch_transpose<bf16_t>((const bf16_t *)a.w_in, (bf16_t *)(base + w.w_inT), n_in, d_s, n_in, stream));  // [d_s, N_in]
    FIPA_TRY(launch_transpose<bf16_t>((const bf16_t *)a.s, (bf16_t *)(base + w.sT), M, d_s, Mp, stream));              // [d_s, Mp]
    GemmParams gs = {};
    gs.M = M; gs.N = d_s; gs.K = n_in;
    gs.A = dX; gs.W = (const bf16_t *)(base + w.w_inT); gs.C = g.d_s_in;
    FIPA_TRY((launch_gemm<GemmTile<2, 2, 1, 1>, false, false>(gs, stream)));
    GemmParams gi = {};
    gi.M = n_in; gi.N = d_s; gi.K = Mp;
    gi.A = dXT; gi.W = (const bf16_t *)(base + w.sT); gi.C = (float *)(base + w.part); gi.chunks_per_split = kWgradChunks;
    FIPA_TRY((launch_gemm<GemmTile<2, 2, 1, 1>, false, false>(gi, stream)));
    hipLaunchKernelGGL(fipa_sum_partials_kernel, dim3((unsigned)(((size_t)n_in * d_s / 4 + 255) / 256)), dim3(256), 0, stream,
                       gi.C, g.d_w_in, (size_t)n_in * d_s, nsplit);
    if (g.d_b_in) hipLaunchKernelGGL(fipa_rowsum_bf16_kernel, dim3(n_in), dim3(256), 0, stream, dXT, g.d_b_in, Mp);
#undef FIPA_TRY
    return hipGetLastError();
}

}  // namespace fipa
