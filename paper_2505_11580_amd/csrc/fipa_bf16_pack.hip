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
    const bool ok = i < p.L && (p.mask ? p.mask[(size_t)b * p.L + i] != 0 : true);
    float kb = -INFINITY, qb = 0.f;
    if (ok) {
        const float *R = p.rot + ((size_t)b * p.L + i) * 9;
        const float *t = p.trans + ((size_t)b * p.L + i) * 3;
        float Rm[9], tc[3];
        for (int a = 0; a < 9; ++a) Rm[a] = R[a];
        for (int a = 0; a < 3; ++a) tc[a] = t[a] - p.cen[4 * b + a];
        const size_t row = ((size_t)b * p.L + i) * p.H + h;
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

// One workgroup per (batch, 64-residue tile): copies z2 (zeroing masked residues) and forms
// the query-side factor bias vectors b^{h1} = log2e * w_L * w_b[h] (.) z1 for every head
// (Algorithm 1 steps 2-3; Eq. 3 puts w_L on the bias, the log2e turns exp into exp2).
__global__ __launch_bounds__(256) void fipa_pack_pair_bf16_kernel(PackParams p)
{
    const int tile = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int DZ = p.DZ;
    const int chunks_per_row = DZ / 8;
    for (int idx = tid; idx < kTileK * chunks_per_row; idx += 256) {
        const int r_ = idx / chunks_per_row, cc = idx - r_ * chunks_per_row;
        const int i = tile * kTileK + r_;
        const bool ok = i < p.L && (p.mask ? p.mask[(size_t)b * p.L + i] != 0 : true);
        uint4 val = make_uint4(0, 0, 0, 0);
        if (ok) val = *reinterpret_cast<const uint4 *>(p.z2 + ((size_t)b * p.L + i) * DZ + cc * 8);
        *reinterpret_cast<uint4 *>(p.Z2 + ((size_t)b * p.Lp + i) * DZ + cc * 8) = val;
    }
    // Qz[b][h][i][x]
    const float bscale = kLog2e * p.w_L;
    for (int idx = tid; idx < p.H * kTileK * chunks_per_row; idx += 256) {
        const int cc = idx % chunks_per_row;
        const int rest = idx / chunks_per_row;
        const int r_ = rest % kTileK, h = rest / kTileK;
        const int i = tile * kTileK + r_;
        const bool ok = i < p.L && (p.mask ? p.mask[(size_t)b * p.L + i] != 0 : true);
        __attribute__((aligned(16))) bf16_t out[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (ok) {
            const uint4 val = *reinterpret_cast<const uint4 *>(p.z1 + ((size_t)b * p.L + i) * DZ + cc * 8);
            const bf16_t *e = reinterpret_cast<const bf16_t *>(&val);
            for (int x = 0; x < 8; ++x) {
                const int col = (cc * 8 + x) % p.cz;
                out[x] = f2bf(bscale * p.w_b[(size_t)h * p.cz + col] * bf2f(e[x]));
            }
        }
        *reinterpret_cast<uint4 *>(p.Qz + (((size_t)b * p.H + h) * p.Lp + i) * DZ + cc * 8) =
            *reinterpret_cast<const uint4 *>(out);
    }
}

}  // namespace

hipError_t launch_pack_bf16(const PackParams &p, hipStream_t stream)
{
    const size_t lds_heads = (size_t)4 * 3 * 64 * kRowStride * sizeof(bf16_t);
    hipError_t e = hipFuncSetAttribute((const void *)fipa_pack_heads_bf16_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_heads);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fipa_pack_heads_bf16_kernel, dim3(p.NT, (p.H + 3) / 4, p.B), dim3(256),
                       lds_heads, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fipa_pack_pair_bf16_kernel, dim3(p.NT, p.B), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace fipa
