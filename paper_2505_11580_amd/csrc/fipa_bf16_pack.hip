// Frame application, hi/lo splitting, norm folding and feature packing for the bf16 MFMA path
// (Algorithm 1 steps 2-6).  Memory bound: one pass over the residues.
#include "fipa_bf16_common.h"

namespace fipa {

namespace {

constexpr int kRowStride = kDH + 8;  // bf16 per staged row; the 16-byte pad spreads LDS banks

// One wave per (batch, head, 64-residue tile); lane <-> residue.  Writes the head-specific
// columns of q^, k^ and v^ (row major), the fp32 per-key bias -|K|^2/2 (-inf for masked keys)
// and the per-query term |Q|^2/2 that the softmax drops.
__global__ __launch_bounds__(256) void fipa_pack_heads_bf16_kernel(PackParams p)
{
    extern __shared__ __attribute__((aligned(16))) bf16_t stage_raw[];
    bf16_t(*stage)[3][64][kRowStride] = reinterpret_cast<bf16_t(*)[3][64][kRowStride]>(stage_raw);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int tile = blockIdx.x, b = blockIdx.z;
    const bool head_ok = (int)(blockIdx.y * 4 + wave) < p.H;
    const int h = head_ok ? blockIdx.y * 4 + wave : p.H - 1;  // surplus waves redo the last head, store nothing
    const int i = tile * kTileK + lane;
    const int c = p.c, Pq = p.Pq, Pv = p.Pv, nq = 3 * Pq;
    bf16_t *rq = stage[wave][0][lane], *rk = stage[wave][1][lane], *rv = stage[wave][2][lane];
    for (int x = 0; x < kDH; ++x) {
        rq[x] = 0;
        rk[x] = 0;
        rv[x] = 0;
    }
    const size_t urow = user_row(p, b, i);  // (only used where i < the chain's length)
    const bool ok = i < user_len(p, b) && (p.mask ? p.mask[urow] != 0 : true);
    float kb = -INFINITY, qb = 0.f;
    if (ok) {
        const float *R = p.rot + urow * 9;
        const float *t = p.trans + urow * 3;
        float Rm[9], tc[3];
        for (int a = 0; a < 9; ++a) Rm[a] = R[a];
        for (int a = 0; a < 3; ++a) tc[a] = t[a] - p.cen[4 * b + a];
        const size_t row = urow * p.H + h;
        const float pscale = p.gamma[h] * p.w_L * p.w_C;  // weight of Q.K in the expanded distance
        const float kscale = kLog2e * pscale;
        const float sscale = kLog2e * p.w_L * p.qk_scale;
        for (int x = 0; x < c; ++x) {
            rq[x] = p.q[row * c + x];
            rk[x] = f2bf(sscale * bf2f(p.k[row * c + x]));
            rv[x] = p.v[row * c + x];
        }
        float ksq = 0.f, qsq = 0.f;
        for (int pp = 0; pp < Pq; ++pp) {
            float ql[3], kl[3];
            for (int a = 0; a < 3; ++a) {
                ql[a] = bf2f(p.q_pts[(row * Pq + pp) * 3 + a]);
                kl[a] = bf2f(p.k_pts[(row * Pq + pp) * 3 + a]);
            }
            for (int a = 0; a < 3; ++a) {
                const float Qg =
                    Rm[3 * a] * ql[0] + Rm[3 * a + 1] * ql[1] + Rm[3 * a + 2] * ql[2] + tc[a];
                const float Kg = kscale * (Rm[3 * a] * kl[0] + Rm[3 * a + 1] * kl[1] +
                                           Rm[3 * a + 2] * kl[2] + tc[a]);
                const bf16_t qh = f2bf(Qg), qlo = f2bf(Qg - bf2f(qh));
                const bf16_t kh = f2bf(Kg), klo = f2bf(Kg - bf2f(kh));
                const int cc = 3 * pp + a;
                rq[c + cc] = qh;
                rq[c + nq + cc] = qh;
                rq[c + 2 * nq + cc] = qlo;
                rq[c + 3 * nq + cc] = qlo;
                rk[c + cc] = kh;
                rk[c + nq + cc] = klo;
                rk[c + 2 * nq + cc] = kh;
                rk[c + 3 * nq + cc] = klo;
                const float qe = bf2f(qh) + bf2f(qlo), ke = bf2f(kh) + bf2f(klo);
                qsq += qe * qe;
                ksq += ke * ke;
            }
        }
        kb = kscale != 0.f ? -ksq / (2.f * kscale) : 0.f;
        qb = 0.5f * pscale * qsq;
        for (int pp = 0; pp < Pv; ++pp) {
            float vl[3];
            for (int a = 0; a < 3; ++a) vl[a] = bf2f(p.v_pts[(row * Pv + pp) * 3 + a]);
            for (int a = 0; a < 3; ++a) {
                const float Vg =
                    Rm[3 * a] * vl[0] + Rm[3 * a + 1] * vl[1] + Rm[3 * a + 2] * vl[2] + tc[a];
                const bf16_t vh = f2bf(Vg), vlo = f2bf(Vg - bf2f(vh));
                rv[v_pt_col(c, Pv, pp, a, 0)] = vh;
                rv[v_pt_col(c, Pv, pp, a, 1)] = vlo;
            }
        }
    }
    const size_t bh = (size_t)b * p.H + h;
    __syncthreads();
    if (!head_ok) return;
    p.kbias[bh * p.Lp + i] = kb;
    p.qbias[bh * p.Lp + i] = qb;
    // the wave's 64 rows x 128 bytes of each tensor are contiguous in memory
    const size_t tile_off = (bh * p.Lp + (size_t)tile * kTileK) * kDH;
    uint4 *dq = reinterpret_cast<uint4 *>(p.Qh + tile_off);
    uint4 *dk = reinterpret_cast<uint4 *>(p.Kh + tile_off);
    uint4 *dv = reinterpret_cast<uint4 *>(p.Vh + tile_off);
    for (int it = 0; it < 8; ++it) {
        const int chunk = it * 64 + lane, r_ = chunk >> 3, cc = chunk & 7;
        dq[chunk] = *reinterpret_cast<const uint4 *>(&stage[wave][0][r_][cc * 8]);
        dk[chunk] = *reinterpret_cast<const uint4 *>(&stage[wave][1][r_][cc * 8]);
        dv[chunk] = *reinterpret_cast<const uint4 *>(&stage[wave][2][r_][cc * 8]);
    }
}

// z2 copy (zeroing masked and padded residues): one thread per 8 consecutive features.
__device__ __forceinline__ void pack_z2_chunk(const PackParams &p, size_t idx)
{
    const int cpr = p.DZ / 8;  // 16-byte chunks per row
    if (idx >= (size_t)p.B * p.Lp * cpr) return;
    const int cc = (int)(idx % cpr);
    const size_t bi = idx / cpr;
    const int i = (int)(bi % p.Lp), b = (int)(bi / p.Lp);
    const size_t urow = user_row(p, b, i);
    const bool ok = i < user_len(p, b) && (p.mask ? p.mask[urow] != 0 : true);
    uint4 val = make_uint4(0, 0, 0, 0);
    if (ok) val = *reinterpret_cast<const uint4 *>(p.z2 + urow * p.DZ + cc * 8);
    *reinterpret_cast<uint4 *>(p.Z2 + ((size_t)b * p.Lp + i) * p.DZ + cc * 8) = val;
}

__global__ __launch_bounds__(256) void fipa_pack_z2_bf16_kernel(PackParams p)
{
    pack_z2_chunk(p, (size_t)blockIdx.x * 256 + threadIdx.x);
}

// Query-side factor bias vectors b^{h1} = log2e * w_L * w_b[h] (.) z1 for every head (Algorithm 1
// steps 2-3; Eq. 3 puts w_L on the bias, the log2e turns exp into exp2): one thread per
// (batch, head, residue, 8 consecutive features).
__global__ __launch_bounds__(256) void fipa_pack_qz_bf16_kernel(PackParams p)
{
    const int cpr = p.DZ / 8;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)p.B * p.H * p.Lp * cpr) return;
    const int cc = (int)(idx % cpr);
    size_t rest = idx / cpr;
    const int i = (int)(rest % p.Lp);
    rest /= p.Lp;
    const int h = (int)(rest % p.H), b = (int)(rest / p.H);
    const size_t urow = user_row(p, b, i);
    const bool ok = i < user_len(p, b) && (p.mask ? p.mask[urow] != 0 : true);
    __attribute__((aligned(16))) bf16_t out[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (ok) {
        const float bscale = kLog2e * p.w_L;
        const uint4 val = *reinterpret_cast<const uint4 *>(p.z1 + urow * p.DZ + cc * 8);
        const bf16_t *e = reinterpret_cast<const bf16_t *>(&val);
        const int col0 = (cc * 8) % p.cz;  // cz is a multiple of 8: the chunk stays inside one factor slice
        const float *wb = p.w_b + (size_t)h * p.cz + col0;
#pragma unroll
        for (int x = 0; x < 8; ++x) out[x] = f2bf(bscale * wb[x] * bf2f(e[x]));
    }
    *reinterpret_cast<uint4 *>(p.Qz + (((size_t)b * p.H + h) * p.Lp + i) * p.DZ + cc * 8) =
        *reinterpret_cast<const uint4 *>(out);
}

// Head-specific columns for the AlphaFold2-style head shape (c = 16, N_query = 4, N_value = 8):
// one thread per (batch, residue, head) and per role (blockIdx.y: 0 = q^, 1 = k^, 2 = v^),
// rows assembled in registers.  Consecutive threads read consecutive (residue, head) records.
// The finished row is not stored by its thread (a wave would then write 16 bytes into each of 64
// different rows per instruction): the wave's 64 rows go through `stage` (this wave's 64 x 128
// bytes of LDS, chunk c of row r at position (c + r) mod 8) and leave as whole 128-byte rows,
// eight per instruction.  `active` is false for the threads past the end of the launch.
template <int ROLE>
__device__ __forceinline__ void pack_head_row(const PackParams &p, int b, int i, int h, const float (&cen)[3],
                                              bool active, char *stage, unsigned long long *dst_of_row)
{
    constexpr int c = 16, Pq = 4, Pv = 8;
    const size_t bh = (size_t)b * p.H + h;
    const size_t urow = user_row(p, b, i);
    const bool ok = active && i < user_len(p, b) && (p.mask ? p.mask[urow] != 0 : true);
    __attribute__((aligned(16))) bf16_t row[kDH];
#pragma unroll
    for (int x = 0; x < kDH; ++x) row[x] = 0;
    float bias = ROLE == 1 ? -INFINITY : 0.f;
    if (ok) {
        const float *R = p.rot + urow * 9;
        const float *t = p.trans + urow * 3;
        float Rm[9], tc[3];
#pragma unroll
        for (int a = 0; a < 9; ++a) Rm[a] = R[a];
#pragma unroll
        for (int a = 0; a < 3; ++a) tc[a] = t[a] - cen[a];
        const size_t rec = urow * p.H + h;
        const float pscale = p.gamma[h] * p.w_L * p.w_C;  // weight of Q.K in the expanded distance
        const bf16_t *sc_src = ROLE == 0 ? p.q : (ROLE == 1 ? p.k : p.v);
        __attribute__((aligned(16))) bf16_t sc[c];
        *reinterpret_cast<uint4 *>(sc) = *reinterpret_cast<const uint4 *>(sc_src + rec * c);
        *reinterpret_cast<uint4 *>(sc + 8) = *reinterpret_cast<const uint4 *>(sc_src + rec * c + 8);
        if (ROLE == 1) {
            const float sscale = kLog2e * p.w_L * p.qk_scale;
#pragma unroll
            for (int x = 0; x < c; ++x) row[x] = f2bf(sscale * bf2f(sc[x]));
        } else {
#pragma unroll
            for (int x = 0; x < c; ++x) row[x] = sc[x];
        }
        constexpr int P = ROLE == 2 ? Pv : Pq;
        const bf16_t *pt_src = (ROLE == 0 ? p.q_pts : (ROLE == 1 ? p.k_pts : p.v_pts)) + rec * P * 3;
        __attribute__((aligned(8))) bf16_t pts[P * 3];
#pragma unroll
        for (int x = 0; x < P * 3 / 4; ++x)
            *reinterpret_cast<uint2 *>(pts + 4 * x) = *reinterpret_cast<const uint2 *>(pt_src + 4 * x);
        const float kscale = kLog2e * pscale;
        float sq = 0.f;
#pragma unroll
        for (int pp = 0; pp < P; ++pp) {
            const float lx = bf2f(pts[3 * pp]), ly = bf2f(pts[3 * pp + 1]), lz = bf2f(pts[3 * pp + 2]);
#pragma unroll
            for (int a = 0; a < 3; ++a) {
                float G = Rm[3 * a] * lx + Rm[3 * a + 1] * ly + Rm[3 * a + 2] * lz + tc[a];
                if (ROLE == 1) G *= kscale;
                const bf16_t hi = f2bf(G), lo = f2bf(G - bf2f(hi));
                const float eff = bf2f(hi) + bf2f(lo);
                sq += eff * eff;
                const int cc = 3 * pp + a;
                if (ROLE == 0) {
                    row[c + cc] = hi;
                    row[c + 3 * Pq + cc] = hi;
                    row[c + 6 * Pq + cc] = lo;
                    row[c + 9 * Pq + cc] = lo;
                } else if (ROLE == 1) {
                    row[c + cc] = hi;
                    row[c + 3 * Pq + cc] = lo;
                    row[c + 6 * Pq + cc] = hi;
                    row[c + 9 * Pq + cc] = lo;
                } else {
                    row[v_pt_col(c, Pv, pp, a, 0)] = hi;
                    row[v_pt_col(c, Pv, pp, a, 1)] = lo;
                }
            }
        }
        if (ROLE == 0) bias = 0.5f * pscale * sq;
        if (ROLE == 1) bias = kscale != 0.f ? -sq / (2.f * kscale) : 0.f;
    }
    static_assert(kDH == 64, "eight 16-byte chunks per row");
    const int lane = threadIdx.x & 63;
    bf16_t *dst = (ROLE == 0 ? p.Qh : (ROLE == 1 ? p.Kh : p.Vh)) + (bh * p.Lp + i) * kDH;
#pragma unroll
    for (int x = 0; x < 8; ++x)
        *reinterpret_cast<uint4 *>(stage + lane * 128 + 16 * ((x + lane) & 7)) = reinterpret_cast<const uint4 *>(row)[x];
    dst_of_row[lane] = active ? (unsigned long long)(uintptr_t)dst : 0ull;
    if (active) {
        if (ROLE == 0) p.qbias[bh * p.Lp + i] = bias;
        if (ROLE == 1) p.kbias[bh * p.Lp + i] = bias;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
        const int r = 8 * pass + (lane >> 3), c = lane & 7;
        const uint4 val = *reinterpret_cast<const uint4 *>(stage + r * 128 + 16 * ((c + r) & 7));
        const unsigned long long d = dst_of_row[r];
        if (d != 0ull) reinterpret_cast<uint4 *>((uintptr_t)d)[c] = val;
    }
}

// Reference point and key-loop bound of batch element b, computed by one wave (every wave that
// asks gets the same answer).  kvlen = 1 + index of the last valid residue.  The reference point
// only has to lie inside the structure (the result does not depend on it, Section 2; it keeps
// the coordinates that are split into bf16 pairs small): the mean translation of 64 valid
// residues spread evenly over [0, kvlen) stands in for the centroid of all of them.
__device__ __forceinline__ void batch_reference(const PackParams &p, int b, float (&cen)[3], int &kvlen)
{
    const int lane = threadIdx.x & 63;
    const int len = user_len(p, b);
    const size_t row0 = user_row(p, b, 0);
    int last = len;
    if (p.mask) {
        const uint8_t *m = p.mask + row0;
        last = 0;
        for (int i = lane; i < len; i += 64)
            if (m[i] != 0) last = i + 1;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) last = max(last, __shfl_xor(last, o));
    }
    kvlen = last;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (kvlen > 0) {
        const int i = (int)(((long long)lane * kvlen) >> 6);
        if (p.mask ? p.mask[row0 + i] != 0 : true) {
            const float *t = p.trans + (row0 + i) * 3;
            v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = 1.f;
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v[a] += __shfl_xor(v[a], o);
    const float n = v[3] > 0.f ? v[3] : 1.f;
#pragma unroll
    for (int a = 0; a < 3; ++a) cen[a] = v[a] / n;
}

// The launch covers the three roles (nbh workgroups each) and, after them, the z2 copy.
__global__ __launch_bounds__(256) void fipa_pack_heads_af2_bf16_kernel(PackParams p, unsigned nbh)
{
    const unsigned role = blockIdx.x / nbh;
    if (role >= 3) {
        pack_z2_chunk(p, (size_t)(blockIdx.x - 3 * nbh) * 256 + threadIdx.x);
        return;
    }
    const size_t per_batch = (size_t)p.Lp * p.H, total = (size_t)p.B * per_batch;
    const size_t idx0 = (size_t)(blockIdx.x - role * nbh) * 256;
    const size_t idx = idx0 + threadIdx.x;  // (b, i, h), h fastest
    float cen[3] = {0.f, 0.f, 0.f};
    if (p.cen_out) {
        if (role == 0)
            for (int i = (int)idx; i < p.n_counters; i += (int)nbh * 256) p.counters[i] = 0;
        // (wave-uniform control flow: the shuffles inside need all 64 lanes)
        const size_t w0 = idx0 + (threadIdx.x & ~63u);
        if (w0 >= total) return;
        const int b0 = (int)(w0 / per_batch), b1 = (int)(min(w0 + 63, total - 1) / per_batch);
        const int bmine = (int)(min(idx, total - 1) / per_batch);
        for (int bb = b0; bb <= b1; ++bb) {
            float cb[3];
            int kv;
            batch_reference(p, bb, cb, kv);
            if (bb == bmine)
#pragma unroll
                for (int a = 0; a < 3; ++a) cen[a] = cb[a];
            if (role == 0 && idx == (size_t)bb * per_batch) {  // the thread that packs (bb, 0, 0) publishes
                p.cen_out[4 * bb + 0] = cb[0];
                p.cen_out[4 * bb + 1] = cb[1];
                p.cen_out[4 * bb + 2] = cb[2];
                p.cen_out[4 * bb + 3] = 0.f;
                p.kvlen_out[bb] = kv;
            }
        }
    }
    // (whole waves stay together from here on: the rows leave through LDS, wave by wave)
    const bool active = idx < total;
    const size_t idc = active ? idx : total - 1;
    const int h = (int)(idc % p.H);
    const size_t bi = idc / p.H;
    const int i = (int)(bi % p.Lp), b = (int)(bi / p.Lp);
    if (!p.cen_out)
#pragma unroll
        for (int a = 0; a < 3; ++a) cen[a] = p.cen[4 * b + a];
    __shared__ __attribute__((aligned(16))) char stage[4][64 * 128];
    __shared__ unsigned long long dst_of_row[4][64];
    const int wv = threadIdx.x >> 6;
    if (role == 0)
        pack_head_row<0>(p, b, i, h, cen, active, stage[wv], dst_of_row[wv]);
    else if (role == 1)
        pack_head_row<1>(p, b, i, h, cen, active, stage[wv], dst_of_row[wv]);
    else
        pack_head_row<2>(p, b, i, h, cen, active, stage[wv], dst_of_row[wv]);
}

}  // namespace

hipError_t launch_pack_bf16(const PackParams &p, hipStream_t stream)
{
    hipError_t e;
    const size_t cpr = p.DZ / 8;
    const unsigned nbz = (unsigned)(((size_t)p.B * p.Lp * cpr + 255) / 256);
    if (p.c == 16 && p.Pq == 4 && p.Pv == 8) {
        const unsigned nbh = (unsigned)(((size_t)p.B * p.Lp * p.H + 255) / 256);
        hipLaunchKernelGGL(fipa_pack_heads_af2_bf16_kernel, dim3(3 * nbh + nbz), dim3(256), 0, stream, p, nbh);
    } else {
        const size_t lds_heads = (size_t)4 * 3 * 64 * kRowStride * sizeof(bf16_t);
        static LdsLimit lds_limit;
        e = raise_lds_limit(lds_limit, (const void *)fipa_pack_heads_bf16_kernel, (int)lds_heads);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(fipa_pack_heads_bf16_kernel, dim3(p.NT, (p.H + 3) / 4, p.B), dim3(256),
                           lds_heads, stream, p);
        hipLaunchKernelGGL(fipa_pack_z2_bf16_kernel, dim3(nbz), dim3(256), 0, stream, p);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (!p.skip_qz)
        hipLaunchKernelGGL(fipa_pack_qz_bf16_kernel,
                           dim3((unsigned)(((size_t)p.B * p.H * p.Lp * cpr + 255) / 256)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace fipa
