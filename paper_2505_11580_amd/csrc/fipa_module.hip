// The IPA module around the attention core (Eq. 1 and Eq. 5 of the paper; Algorithm 1 steps 1
// and 10): input projection of the single representation, core, output projection of the
// concatenated results.  Both projections are small next to the attention (2.4 and 4.4 GFLOP
// against 117 GFLOP at B=2, L=2048, d_s=256), so one plain MFMA GEMM kernel serves them:
//     C[M, N] = A[M, K] W[N, K]^T + bias[N]        (weights stored [out, in])
// Each wave owns 32 rows and 32*NT columns; A and W fragments are read straight from memory in
// the MFMA operand layout (a lane reads 8 consecutive k of its row), no LDS.  Two variations:
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
// are multiples of 8, so a chunk never straddles two segments).
__device__ __forceinline__ bf16x8 load_concat(const GemmParams &p, int row, int k)
{
    float v[8];
    const int e1 = p.k_pair, e2 = e1 + p.k_o, e3 = e2 + p.k_pts;
    if (k < e3) {
        const float *src = k < e1 ? p.o_pair + (size_t)row * p.k_pair + k
                                  : (k < e2 ? p.o + (size_t)row * p.k_o + (k - e1) : p.o_pts + (size_t)row * p.k_pts + (k - e2));
        const f32x4 a = *reinterpret_cast<const f32x4 *>(src), b = *reinterpret_cast<const f32x4 *>(src + 4);
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            v[x] = a[x];
            v[4 + x] = b[x];
        }
    } else {
        const float *src = p.o_pts + (size_t)row * p.k_pts + 3 * (k - e3);  // points k-e3 .. +7
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const float px = src[3 * x], py = src[3 * x + 1], pz = src[3 * x + 2];
            v[x] = sqrtf(px * px + py * py + pz * pz);
        }
    }
    return to_bf16x8(v);
}

template <int NT, bool CONCAT_A, bool SCATTER>
__global__ __launch_bounds__(256) void fipa_gemm_kernel(GemmParams p)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, kg = lane >> 5;
    const int m_base = blockIdx.x * 128 + wave * 32;
    const int n_base = blockIdx.y * 32 * NT;
    const int row_a = min(m_base + li, p.M - 1);  // rows / columns past the end are computed on the last one and not stored
    const bf16_t *wrow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) wrow[t] = p.W + (size_t)min(n_base + 32 * t + li, p.N - 1) * p.K + 8 * kg;
    const bf16_t *arow = CONCAT_A ? nullptr : p.A + (size_t)row_a * p.K + 8 * kg;

    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

#pragma unroll 4
    for (int k0 = 0; k0 < p.K; k0 += 16) {
        bf16x8 a;
        if constexpr (CONCAT_A)
            a = load_concat(p, row_a, k0 + 8 * kg);
        else
            a = *reinterpret_cast<const bf16x8 *>(arow + k0);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const bf16x8 b = *reinterpret_cast<const bf16x8 *>(wrow[t] + k0);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
        }
    }

    // the lane holds column n_base + 32 t + li and rows m_base + 8 (r / 4) + 4 kg + r % 4
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int col = n_base + 32 * t + li;
        if (col >= p.N) continue;
        const float bias = p.bias ? p.bias[col] : 0.f;
        int seg = 0;
        if constexpr (SCATTER) {
#pragma unroll
            for (int s = 1; s < 6; ++s)
                if (col >= p.seg_start[s]) seg = s;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = m_base + 8 * (r >> 2) + 4 * kg + (r & 3);
            if (row >= p.M) continue;
            const float val = acc[t][r] + bias;
            if constexpr (SCATTER) {
                const int width = p.seg_start[seg + 1] - p.seg_start[seg];
                p.seg_ptr[seg][(size_t)row * width + (col - p.seg_start[seg])] = f2bf(val);
            } else {
                p.C[(size_t)row * p.N + col] = val;
            }
        }
    }
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
    hipLaunchKernelGGL((fipa_gemm_kernel<4, false, true>), dim3((M + 127) / 128, (g1.N + 127) / 128), dim3(256), 0,
                       stream, g1);
    hipError_t e = hipGetLastError();
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
    hipLaunchKernelGGL((fipa_gemm_kernel<2, true, false>), dim3((M + 127) / 128, (g2.N + 63) / 64), dim3(256), 0,
                       stream, g2);
    return hipGetLastError();
}

}  // namespace fipa
