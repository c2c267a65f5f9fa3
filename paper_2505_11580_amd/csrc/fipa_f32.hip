// fp32 direct path: logits from explicit point differences (Eq. 3), online softmax over key
// tiles, fp32 accumulation of the lifted values (Algorithm 1 steps 6-7), and the split /
// inverse frame / z1 contraction (steps 8-9, Eq. 4) in the same kernel.  Plain VALU
// arithmetic; this is the accuracy path (1e-4), not the throughput path.
#include "fipa_internal.h"

namespace fipa {

namespace {

struct F32Params {
    const float *q, *k, *v, *z1, *z2, *rot, *trans, *gamma;
    const uint8_t *mask;
    const float *Qg, *Kg, *Vg, *Qz, *cen;
    const int *kvlen;
    float *o, *o_pts, *o_pair, *lse;
    int B, L, H, c, Pq, Pv, cz, r, DZ;
    int TK;    // keys per LDS tile
    int REC;   // floats per key record: k | Kg | z2 | v | Vg
    int SK;    // record stride in floats (odd, so that lanes hit distinct banks)
    int NCOL;  // lifted value width c + 3Pv + DZ
    float w_L, w_C, qk_scale;
};

constexpr int kRowsPerWave = 4;
constexpr int kRowsPerBlock = 16;

// Global-frame points relative to the batch centroid, T_i o x - centroid (Algorithm 1 steps 4-6).
__global__ __launch_bounds__(256) void fipa_pack_points_f32_kernel(
    const float *__restrict__ q_pts, const float *__restrict__ k_pts,
    const float *__restrict__ v_pts, const float *__restrict__ rot,
    const float *__restrict__ trans, const float *__restrict__ cen, float *__restrict__ Qg,
    float *__restrict__ Kg, float *__restrict__ Vg, int L, int H, int Pq, int Pv)
{
    const int b = blockIdx.y;
    const int idx = blockIdx.x * 256 + threadIdx.x;  // (i, h)
    if (idx >= L * H) return;
    const int i = idx / H, h = idx % H;
    const float *R = rot + ((size_t)b * L + i) * 9;
    const float *t = trans + ((size_t)b * L + i) * 3;
    float Rm[9], tc[3];
    for (int a = 0; a < 9; ++a) Rm[a] = R[a];
    for (int a = 0; a < 3; ++a) tc[a] = t[a] - cen[4 * b + a];
    auto apply = [&](const float *src, float *dst, int P) {
        for (int p = 0; p < P; ++p) {
            const float x = src[3 * p], y = src[3 * p + 1], z = src[3 * p + 2];
            for (int a = 0; a < 3; ++a)
                dst[3 * p + a] = Rm[3 * a] * x + Rm[3 * a + 1] * y + Rm[3 * a + 2] * z + tc[a];
        }
    };
    const size_t in_q = (((size_t)b * L + i) * H + h) * Pq * 3;
    const size_t in_v = (((size_t)b * L + i) * H + h) * Pv * 3;
    const size_t out_q = (((size_t)b * H + h) * L + i) * Pq * 3;
    const size_t out_v = (((size_t)b * H + h) * L + i) * Pv * 3;
    apply(q_pts + in_q, Qg + out_q, Pq);
    apply(k_pts + in_q, Kg + out_q, Pq);
    apply(v_pts + in_v, Vg + out_v, Pv);
}

// Query-side factor bias vector b^{h1}_i = w_L * w_b[h] (.) z1_i (Algorithm 1 step 2, with
// Eq. 3's w_L on the bias), laid out [B,H,L,DZ].
__global__ __launch_bounds__(256) void fipa_pack_qz_f32_kernel(const float *__restrict__ z1,
                                                               const float *__restrict__ w_b,
                                                               float *__restrict__ Qz, int L, int H,
                                                               int cz, int DZ, float w_L,
                                                               size_t total)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int x = (int)(idx % DZ);
    const size_t rest = idx / DZ;
    const int i = (int)(rest % L);
    const size_t bh = rest / L;
    const int h = (int)(bh % H);
    const size_t b = bh / H;
    Qz[idx] = w_L * w_b[(size_t)h * cz + x % cz] * z1[(b * L + i) * DZ + x];
}

__device__ __forceinline__ float wave_max(float x)
{
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
    return x;
}
__device__ __forceinline__ float wave_sum(float x)
{
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

template <int MC>
__global__ __launch_bounds__(256) void fipa_attn_f32_kernel(F32Params p)
{
    extern __shared__ float smem[];
    float *tile = smem;                                 // [TK][SK]
    float *mbias = smem + (size_t)p.TK * p.SK;          // [TK] 0 or -inf
    float *rowbuf = smem;                               // [16][NCOL], aliases the tile at the end

    const int b = blockIdx.z, h = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    const int i0 = blockIdx.x * kRowsPerBlock + wave * kRowsPerWave;
    const int L = p.L, H = p.H, c = p.c, DZ = p.DZ, TK = p.TK, SK = p.SK;
    const int nq = 3 * p.Pq, nv = 3 * p.Pv;
    const int kvlen = p.kvlen[b];

    const float *qrow[kRowsPerWave], *Qgrow[kRowsPerWave], *Qzrow[kRowsPerWave];
    for (int rr = 0; rr < kRowsPerWave; ++rr) {
        const int i = min(i0 + rr, L - 1);
        qrow[rr] = p.q + (((size_t)b * L + i) * H + h) * c;
        Qgrow[rr] = p.Qg + (((size_t)b * H + h) * L + i) * nq;
        Qzrow[rr] = p.Qz + (((size_t)b * H + h) * L + i) * DZ;
    }
    const float coef = 0.5f * p.gamma[h] * p.w_L * p.w_C;
    const float sc = p.w_L * p.qk_scale;

    // value column owned by this lane in slot mc, as an offset into a key record
    int coloff[MC];
    for (int mc = 0; mc < MC; ++mc) {
        const int col = lane + 64 * mc;
        int off = 0;
        if (col < c + nv)
            off = c + nq + DZ + col;
        else if (col < p.NCOL)
            off = c + nq + (col - c - nv);
        coloff[mc] = off;
    }

    float m[kRowsPerWave], l[kRowsPerWave], acc[kRowsPerWave][MC];
    for (int rr = 0; rr < kRowsPerWave; ++rr) {
        m[rr] = -INFINITY;
        l[rr] = 0.f;
        for (int mc = 0; mc < MC; ++mc) acc[rr][mc] = 0.f;
    }

    for (int j0 = 0; j0 < kvlen; j0 += TK) {
        __syncthreads();
        // stage the key records k | Kg | z2 | v | Vg
        for (int idx = threadIdx.x; idx < TK * p.REC; idx += 256) {
            const int jj = idx / p.REC, x = idx - jj * p.REC;
            const int j = j0 + jj;
            float val = 0.f;
            if (j < L) {
                if (x < c)
                    val = p.k[(((size_t)b * L + j) * H + h) * c + x];
                else if (x < c + nq)
                    val = p.Kg[(((size_t)b * H + h) * L + j) * nq + (x - c)];
                else if (x < c + nq + DZ)
                    val = p.z2[((size_t)b * L + j) * DZ + (x - c - nq)];
                else if (x < 2 * c + nq + DZ)
                    val = p.v[(((size_t)b * L + j) * H + h) * c + (x - c - nq - DZ)];
                else
                    val = p.Vg[(((size_t)b * H + h) * L + j) * nv + (x - 2 * c - nq - DZ)];
            }
            tile[(size_t)jj * SK + x] = val;
        }
        for (int jj = threadIdx.x; jj < TK; jj += 256) {
            const int j = j0 + jj;
            const bool ok = j < kvlen && (p.mask ? p.mask[(size_t)b * L + j] != 0 : true);
            mbias[jj] = ok ? 0.f : -INFINITY;
        }
        __syncthreads();

        // logits of this lane's key against the wave's four query rows (Eq. 3)
        const int lj = lane < TK ? lane : 0;
        const float *rec = tile + (size_t)lj * SK;
        float s[kRowsPerWave];
        {
            float dotk[kRowsPerWave] = {0.f, 0.f, 0.f, 0.f};
            for (int d = 0; d < c; ++d) {
                const float kd = rec[d];
                for (int rr = 0; rr < kRowsPerWave; ++rr) dotk[rr] += qrow[rr][d] * kd;
            }
            float dist[kRowsPerWave] = {0.f, 0.f, 0.f, 0.f};
            for (int d = 0; d < nq; ++d) {
                const float kd = rec[c + d];
                for (int rr = 0; rr < kRowsPerWave; ++rr) {
                    const float df = Qgrow[rr][d] - kd;
                    dist[rr] += df * df;
                }
            }
            float bias[kRowsPerWave] = {0.f, 0.f, 0.f, 0.f};
            for (int d = 0; d < DZ; ++d) {
                const float zd = rec[c + nq + d];
                for (int rr = 0; rr < kRowsPerWave; ++rr) bias[rr] += Qzrow[rr][d] * zd;
            }
            const float mb = lane < TK ? mbias[lj] : -INFINITY;
            for (int rr = 0; rr < kRowsPerWave; ++rr)
                s[rr] = sc * dotk[rr] + bias[rr] - coef * dist[rr] + mb;
        }
        // online softmax update (running maximum, running sum, rescaled accumulator)
        float pw[kRowsPerWave];
        for (int rr = 0; rr < kRowsPerWave; ++rr) {
            const float m_new = fmaxf(m[rr], wave_max(s[rr]));
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            pw[rr] = __expf(s[rr] - m_use);
            const float alpha = __expf(m[rr] - m_use);
            l[rr] = l[rr] * alpha + wave_sum(pw[rr]);
            m[rr] = m_new;
            for (int mc = 0; mc < MC; ++mc) acc[rr][mc] *= alpha;
        }
        // weighted sum of the lifted values: lanes own value columns
        for (int jj = 0; jj < TK; ++jj) {
            float pj[kRowsPerWave];
            for (int rr = 0; rr < kRowsPerWave; ++rr)
                pj[rr] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(pw[rr]), jj));
            const float *vrec = tile + (size_t)jj * SK;
            for (int mc = 0; mc < MC; ++mc) {
                const float val = vrec[coloff[mc]];
                for (int rr = 0; rr < kRowsPerWave; ++rr) acc[rr][mc] += pj[rr] * val;
            }
        }
    }

    // split, inverse frame, z1 contraction (Algorithm 1 steps 8-9, Eq. 4)
    __syncthreads();
    for (int rr = 0; rr < kRowsPerWave; ++rr) {
        const float inv = l[rr] > 0.f ? 1.f / l[rr] : 0.f;
        float *rb = rowbuf + (size_t)(wave * kRowsPerWave + rr) * p.NCOL;
        for (int mc = 0; mc < MC; ++mc) {
            const int col = lane + 64 * mc;
            if (col < p.NCOL) rb[col] = acc[rr][mc] * inv;
        }
    }
    __syncthreads();
    for (int rr = 0; rr < kRowsPerWave; ++rr) {
        const int i = i0 + rr;
        if (i >= L) break;
        const bool valid = (p.mask ? p.mask[(size_t)b * L + i] != 0 : true) && l[rr] > 0.f;
        const float *rb = rowbuf + (size_t)(wave * kRowsPerWave + rr) * p.NCOL;
        const size_t row = ((size_t)b * L + i) * H + h;
        for (int d = lane; d < c; d += 64) p.o[row * c + d] = valid ? rb[d] : 0.f;
        const float *R = p.rot + ((size_t)b * L + i) * 9;
        const float *t = p.trans + ((size_t)b * L + i) * 3;
        for (int idx = lane; idx < nv; idx += 64) {
            const int pp = idx / 3, x = idx - 3 * pp;
            float val = 0.f;
            for (int y = 0; y < 3; ++y)
                val += R[3 * y + x] * (rb[c + 3 * pp + y] - (t[y] - p.cen[4 * b + y]));
            p.o_pts[row * nv + idx] = valid ? val : 0.f;
        }
        for (int d = lane; d < p.cz; d += 64) {
            float val = 0.f;
            for (int rho = 0; rho < p.r; ++rho)
                val += p.z1[((size_t)b * L + i) * DZ + rho * p.cz + d] * rb[c + nv + rho * p.cz + d];
            p.o_pair[row * p.cz + d] = valid ? val : 0.f;
        }
        if (p.lse && lane == 0)
            p.lse[((size_t)b * H + h) * L + i] = valid ? m[rr] + __logf(l[rr]) : 0.f;
    }
}

struct F32Layout {
    size_t cen, kvlen, Qg, Kg, Vg, Qz, total;
};

F32Layout f32_layout(const fipa_desc &d)
{
    F32Layout w;
    const size_t BHL = (size_t)d.B * d.H * d.L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    w.cen = take((size_t)d.B * 4 * sizeof(float));
    w.kvlen = take((size_t)d.B * sizeof(int));
    w.Qg = take(BHL * 3 * d.Pq * sizeof(float));
    w.Kg = take(BHL * 3 * d.Pq * sizeof(float));
    w.Vg = take(BHL * 3 * d.Pv * sizeof(float));
    w.Qz = take(BHL * (size_t)d.r * d.cz * sizeof(float));
    w.total = off;
    return w;
}

constexpr size_t kF32LdsBudget = 150 * 1024;

}  // namespace

size_t f32_forward_workspace(const fipa_desc &d) { return f32_layout(d).total; }

hipError_t f32_forward(const fipa_desc &d, const FwdArgs &a, void *ws, hipStream_t stream)
{
    const F32Layout w = f32_layout(d);
    char *base = static_cast<char *>(ws);
    float *cen = reinterpret_cast<float *>(base + w.cen);
    int *kvlen = reinterpret_cast<int *>(base + w.kvlen);
    float *Qg = reinterpret_cast<float *>(base + w.Qg);
    float *Kg = reinterpret_cast<float *>(base + w.Kg);
    float *Vg = reinterpret_cast<float *>(base + w.Vg);
    float *Qz = reinterpret_cast<float *>(base + w.Qz);
    const int DZ = d.r * d.cz;

    StageTimer timer(stream);
    timer.begin(0);
    hipError_t e = launch_prep(d, a.trans, a.mask, nullptr, cen, kvlen, nullptr, 0, stream);
    if (e != hipSuccess) return e;

    hipLaunchKernelGGL(fipa_pack_points_f32_kernel, dim3((d.L * d.H + 255) / 256, d.B), dim3(256),
                       0, stream, (const float *)a.q_pts, (const float *)a.k_pts,
                       (const float *)a.v_pts, a.rot, a.trans, cen, Qg, Kg, Vg, d.L, d.H, d.Pq,
                       d.Pv);
    const size_t total = (size_t)d.B * d.H * d.L * DZ;
    hipLaunchKernelGGL(fipa_pack_qz_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       stream, (const float *)a.z1, a.w_b, Qz, d.L, d.H, d.cz, DZ, d.w_L, total);
    timer.end(0);

    F32Params p;
    p.q = (const float *)a.q; p.k = (const float *)a.k; p.v = (const float *)a.v;
    p.z1 = (const float *)a.z1; p.z2 = (const float *)a.z2;
    p.rot = a.rot; p.trans = a.trans; p.gamma = a.gamma; p.mask = a.mask;
    p.Qg = Qg; p.Kg = Kg; p.Vg = Vg; p.Qz = Qz; p.cen = cen; p.kvlen = kvlen;
    p.o = a.o; p.o_pts = a.o_pts; p.o_pair = a.o_pair; p.lse = a.lse;
    p.B = d.B; p.L = d.L; p.H = d.H; p.c = d.c; p.Pq = d.Pq; p.Pv = d.Pv; p.cz = d.cz; p.r = d.r;
    p.DZ = DZ;
    p.REC = 2 * d.c + 3 * d.Pq + 3 * d.Pv + DZ;
    p.SK = p.REC | 1;
    p.NCOL = d.c + 3 * d.Pv + DZ;
    p.w_L = d.w_L; p.w_C = d.w_C; p.qk_scale = d.qk_scale;
    int TK = 64;
    auto lds_bytes = [&](int tk) {
        const size_t tile = ((size_t)tk * p.SK + tk) * sizeof(float);
        const size_t rows = (size_t)kRowsPerBlock * p.NCOL * sizeof(float);
        return tile > rows ? tile : rows;
    };
    while (TK > 8 && lds_bytes(TK) > kF32LdsBudget) TK >>= 1;
    p.TK = TK;
    const size_t lds = lds_bytes(TK);
    const int MC = (p.NCOL + 63) / 64;
    const dim3 grid((d.L + kRowsPerBlock - 1) / kRowsPerBlock, d.H, d.B);
    timer.begin(1);  // the fp32 kernel contains the epilogue; stage 2 stays empty

#define FIPA_F32_CASE(N)                                                                        \
    case N: {                                                                                   \
        static LdsLimit lim;                                                                    \
        e = raise_lds_limit(lim, (const void *)fipa_attn_f32_kernel<N>, (int)lds);              \
        if (e != hipSuccess) return e;                                                          \
        hipLaunchKernelGGL(fipa_attn_f32_kernel<N>, grid, dim3(256), lds, stream, p);           \
        break;                                                                                  \
    }
    switch (MC) {
        FIPA_F32_CASE(1)
        FIPA_F32_CASE(2)
        FIPA_F32_CASE(3)
        FIPA_F32_CASE(4)
        FIPA_F32_CASE(5)
        FIPA_F32_CASE(6)
        FIPA_F32_CASE(7)
        FIPA_F32_CASE(8)
        FIPA_F32_CASE(9)
        default:
            return hipErrorInvalidValue;
    }
#undef FIPA_F32_CASE
    timer.end(1);
    return hipGetLastError();
}

}  // namespace fipa
