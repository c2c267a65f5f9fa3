// Backward of the bf16 path: host orchestration and the memory-bound kernels around the MFMA
// kernels (lifting of the upstream gradients; chain rule through the packing back to the
// inputs).  The paper gives no backward; formulas follow from Eqs. 3-4 and z_ij = z1_i^T z2_j.
//
// Chain: forward pack -> forward attention (unfused, gives O^ and the log-sum-exp) -> lift the
// upstream gradients (dO^ = [d_o | R_i d_o_pts in the hi and lo columns | z1 (.) d_o_pair],
// D_i = dO^_i . O^_i) -> dQ^, dK^, dV^ (MFMA kernels) -> unpack.
#include "fipa_gfx950.h"

namespace fipa {

namespace {

// One wave per (batch, head, residue < Lp): lifted upstream gradient row, D_i, and -lse.
// Lane l takes head-specific column l and the four pair columns 4 l' .. 4 l' + 3 of each group of
// 256 (l' = l), so that the pair part moves in 16-byte (fp32) and 8-byte (bf16) pieces and all loads
// of a row are independent of each other.
__global__ __launch_bounds__(256) void fipa_bwd_pack_bf16_kernel(BwdPackParams p)
{
    const int lane = threadIdx.x & 63;
    const size_t row_id = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // over B*H*Lp, i fastest
    if (row_id >= (size_t)p.B * p.H * p.Lp) return;
    const int i = (int)(row_id % p.Lp);
    const size_t bh = row_id / p.Lp;
    const int h = (int)(bh % p.H), b = (int)(bh / p.H);
    const int c = p.c, D = kDH + p.DZ, PH = (p.Pv + 1) / 2;
    const size_t urow = user_row(p, b, i);  // (only used where i < the chain's length)
    const bool valid = i < user_len(p, b) && (p.mask ? p.mask[urow] != 0 : true);
    const size_t rec = valid ? urow * p.H + h : 0;
    const float *R = p.rot + (valid ? urow * 9 : 0);
    const float *oh = p.Ohat + row_id * D;
    bf16_t *dst = p.dOhat + row_id * D;
    float dsum = 0.f;
    // ---- pair part: columns kDH + 4 q, q = lane, lane + 64, ...
    for (int q = lane; 4 * q < p.DZ; q += 64) {
        const int x = 4 * q;
        f32x4 val = {0.f, 0.f, 0.f, 0.f}, o4 = {0.f, 0.f, 0.f, 0.f};
        if (valid) {
            const uint2 zr = *reinterpret_cast<const uint2 *>(p.z1 + urow * p.DZ + x);  // four bf16 values
            const f32x4 g4 = *reinterpret_cast<const f32x4 *>(p.d_o_pair + rec * p.cz + x % p.cz);  // (cz is a multiple of 8)
            o4 = *reinterpret_cast<const f32x4 *>(oh + kDH + x);
            val[0] = __uint_as_float(zr.x << 16) * g4[0];
            val[1] = __uint_as_float(zr.x & 0xFFFF0000u) * g4[1];
            val[2] = __uint_as_float(zr.y << 16) * g4[2];
            val[3] = __uint_as_float(zr.y & 0xFFFF0000u) * g4[3];
        }
        __attribute__((aligned(8))) bf16_t bv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            bv[e] = f2bf(val[e]);
            dsum += bf2f(bv[e]) * o4[e];  // D uses the rounded gradient the MFMAs will see
        }
        *reinterpret_cast<uint2 *>(dst + kDH + x) = *reinterpret_cast<const uint2 *>(bv);
    }
    // ---- head-specific part: column `lane`
    {
        const int col = lane;
        float val = 0.f;
        if (valid) {
            if (col < c) {
                val = p.d_o[rec * c + col];
            } else {
                // inverse of v_pt_col: which (point, axis) lives in this column, if any
                const int cp = col - c, within = cp & 7;
                const int gh = within >> 2, u = 4 * (cp >> 3) + (within & 3);
                const int lo = u / (3 * PH), u2 = u - lo * 3 * PH;
                const int pt = gh * PH + u2 / 3, ax = u2 % 3;
                if (lo < 2 && pt < p.Pv) {
                    const float *g = p.d_o_pts + (rec * p.Pv + pt) * 3;
                    val = R[3 * ax] * g[0] + R[3 * ax + 1] * g[1] + R[3 * ax + 2] * g[2];  // dG = R_i d_o_pts
                }
            }
        }
        const bf16_t bv = f2bf(val);
        dst[col] = bv;
        dsum += bf2f(bv) * (valid ? oh[col] : 0.f);
    }
    for (int off = 32; off > 0; off >>= 1) dsum += __shfl_xor(dsum, off);
    if (lane == 0) {
        const float l2 = p.lse2[row_id];
        p.Dvec[row_id] = dsum;
        p.nlse[row_id] = (valid && l2 > -INFINITY && l2 < INFINITY) ? -l2 : -INFINITY;
    }
}

// One wave per (batch, residue), four residues per workgroup: chain rule from dQ^, dK^, dV^ back to
// the inputs.  Nothing is exchanged between the waves, so there is no workgroup barrier: sums over
// the lanes of a wave go through shuffles in a fixed order.
//   first the per-head tasks -- 2 Pq + Pv point gradients and the three scalar rows of each head --
//   dealt to the lanes kind by kind (few bytes, many small scattered accesses);
//   then the pair factors (the bulk of the bytes): a lane owns four neighbouring lifted columns and
//   adds up the heads one after the other (16-byte loads of the four big arrays, all independent);
//   where the lifted width is below 256 the lanes form 64 / (DZ / 4) groups that take every
//   group-th head and are added at the end, above it a lane takes DZ / 256 sets of columns.
// Measured at B = 2, L = 4096, H = 12, r c_z = 256 (about 520 MB moved): 0.139 ms; the pair-factor part
// alone 0.099 ms (5.1 TB/s); the earlier form, one workgroup per residue with the sums of its threads
// meeting in LDS behind workgroup barriers, 0.191 ms.
__global__ __launch_bounds__(256) void fipa_bwd_unpack_bf16_kernel(BwdUnpackParams p)
{
    const int lane = threadIdx.x & 63;
    const long long rr = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);  // (b, i); uniform over the wave
    if (rr >= (long long)p.B * p.L) return;
    const int b = (int)(rr / p.L), i = (int)(rr - (long long)b * p.L);
    const int c = p.c, Pq = p.Pq, Pv = p.Pv, nq = 3 * Pq, D = kDH + p.DZ;
    if (i >= user_len(p, b)) return;  // (packed batch: the grid covers the longest chain)
    const size_t urow = user_row(p, b, i);
    const bool valid = p.mask ? p.mask[urow] != 0 : true;

    // ---- per-head tasks ----------------------------------------------------------------------------
    const float *R = p.rot + urow * 9;
    const float *t = p.trans + urow * 3;
    float Rm[9], tc[3];
    for (int a = 0; a < 9; ++a) Rm[a] = R[a];
    for (int a = 0; a < 3; ++a) tc[a] = t[a] - p.cen[4 * b + a];

    // frame gradients: every global-frame point gradient g of a point with local coordinates x
    // contributes g to d t_i and g x^T to d R_i (G = R_i x + t_i); the output points
    // o_pts = R_i^T (G - t_i) contribute -R_i d_o_pts and (G - t_i) d_o_pts^T
    float ft[3] = {0.f, 0.f, 0.f}, fr[9] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // Three kinds of task, each dealt to the lanes in passes of its own so that a pass runs one
    // piece of code: the 2 Pq query and key points of a head (whole heads per pass: their
    // contributions to d gamma are added across the head's lanes), the Pv value points, and the
    // scalar rows d_q, d_k, d_v in pieces of eight channels.
    {
        const int per = 2 * Pq, HP = 64 / per;
        for (int h0 = 0; h0 < p.H; h0 += HP) {
            float gpartial = 0.f;
            const int hl = lane / per;
            const bool active = hl < HP && h0 + hl < p.H;
            const int h = active ? h0 + hl : 0, tk = active ? lane - hl * per : 0;
            const size_t bh = (size_t)b * p.H + h;
            if (active) {
                const size_t rec = urow * p.H + h;
                const float pscale = p.gamma[h] * p.w_L * p.w_C;
                const bool isq = tk < Pq;
                const float sc = isq ? 1.f : kLog2e * pscale, inv_sc = sc != 0.f ? 1.f / sc : 0.f;
                const int pt = isq ? tk : tk - Pq;
                const float *dX = (isq ? p.dQhat : p.dKhat) + (bh * p.Lp + i) * D + c + 3 * pt;  // hi columns of this point
                const int lo_off = isq ? nq : 2 * nq;                                             // to its lo columns
                const float ws = (isq ? p.rowsum : p.colsum)[bh * p.Lp + i];
                const bf16_t *src = (isq ? p.q_pts : p.k_pts) + (rec * Pq + pt) * 3;
                const float lc[3] = {bf2f(src[0]), bf2f(src[1]), bf2f(src[2])};
                float grad[3];
                float gacc = 0.f;
#pragma unroll
                for (int a = 0; a < 3; ++a) {
                    const float G0 = Rm[3 * a] * lc[0] + Rm[3 * a + 1] * lc[1] + Rm[3 * a + 2] * lc[2] + tc[a];
                    const float X = dX[a] + dX[lo_off + a];  // sum over the other side of dS times its hi and lo coordinates
                    // the effective (hi + lo) global coordinate the kernels used: the query's as it is, the
                    // key's scaled by log2e gamma w_L w_C before the split
                    const float Gs = sc * G0;
                    const bf16_t hi = f2bf(Gs), lo = f2bf(Gs - bf2f(hi));
                    const float eff = sc != 0.f ? (bf2f(hi) + bf2f(lo)) * inv_sc : G0;
                    // query: d s / dQ = gamma w_L w_C (K - Q) summed with dS, and sum_j dS K^ sits in the Khi and
                    // Klo columns (in log2 units); key: the same with the sides exchanged
                    grad[a] = isq ? kLn2 * X - pscale * ws * eff : pscale * (X - ws * eff);
                    gacc += isq ? ws * eff * eff : ws * eff * eff - 2.f * eff * X;
                }
                gpartial = gacc;
#pragma unroll
                for (int x = 0; x < 3; ++x) {
                    ft[x] += grad[x];
#pragma unroll
                    for (int y = 0; y < 3; ++y) fr[3 * x + y] += grad[x] * lc[y];
                }
                bf16_t *dst = (isq ? p.d_q_pts : p.d_k_pts) + (rec * Pq + pt) * 3;
#pragma unroll
                for (int x = 0; x < 3; ++x) {
                    const float val = Rm[x] * grad[0] + Rm[3 + x] * grad[1] + Rm[6 + x] * grad[2];  // R^T
                    dst[x] = f2bf(valid ? val : 0.f);
                }
            }
            // d gamma: this residue's contribution, summed over the query and key points of a head in
            // a fixed order (they sit in the 2 Pq lanes from the head's first on)
            float gsum = 0.f;
            for (int x = 0; x < per; ++x) gsum += __shfl(gpartial, (lane + x) & 63);
            if (active && tk == 0) p.gpart[bh * p.Lp + i] = valid ? gsum : 0.f;
        }
    }
    for (int t0 = 0; t0 < p.H * Pv; t0 += 64) {
        const int tsk = t0 + lane;
        if (tsk < p.H * Pv) {
            const int h = tsk / Pv, pt = tsk - h * Pv;
            const size_t bh = (size_t)b * p.H + h;
            const size_t rec = urow * p.H + h;
            const float *dV = p.dVhat + (bh * p.Lp + i) * D;
            float grad[3];
#pragma unroll
            for (int a = 0; a < 3; ++a) grad[a] = dV[v_pt_col(c, Pv, pt, a, 0)];
            if (p.d_rot) {
                const bf16_t *vl = p.v_pts + (rec * Pv + pt) * 3;
                const float *gp = p.d_o_pts + (rec * Pv + pt) * 3;
                const float *oh = p.Ohat + (bh * p.Lp + i) * D;
                const bf16_t *dgh = p.dOhat + (bh * p.Lp + i) * D;
#pragma unroll
                for (int x = 0; x < 3; ++x) {
                    // R_i d_o_pts, in the rounded form that the gradient kernels used: it then cancels
                    // against the value-point term exactly where the mathematics says so (shift invariance)
                    const float dGx = bf2f(dgh[v_pt_col(c, Pv, pt, x, 0)]);
                    const float Gm = oh[v_pt_col(c, Pv, pt, x, 0)] + oh[v_pt_col(c, Pv, pt, x, 1)] - tc[x];
                    ft[x] += grad[x] - dGx;
#pragma unroll
                    for (int y = 0; y < 3; ++y) fr[3 * x + y] += grad[x] * bf2f(vl[y]) + Gm * gp[y];
                }
            }
            bf16_t *dst = p.d_v_pts + (rec * Pv + pt) * 3;
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                const float val = Rm[x] * grad[0] + Rm[3 + x] * grad[1] + Rm[6 + x] * grad[2];
                dst[x] = f2bf(valid ? val : 0.f);
            }
        }
    }
    {
        const int nchunk = c / 8, per = 3 * nchunk;  // (c is a multiple of 8; every piece is 16-byte aligned on both sides)
        for (int t0 = 0; t0 < p.H * per; t0 += 64) {
            const int tsk = t0 + lane;
            if (tsk < p.H * per) {
                const int h = tsk / per, rem = tsk - h * per;
                const int which = rem / nchunk, x = 8 * (rem - which * nchunk);  // 0: d_q, 1: d_k, 2: d_v
                const size_t row = (((size_t)b * p.H + h) * p.Lp + i) * D + x;
                const float *src = (which == 0 ? p.dQhat : (which == 1 ? p.dKhat : p.dVhat)) + row;
                const float scale = which == 0 ? kLn2 : (which == 1 ? p.w_L * p.qk_scale : 1.f);
                bf16_t *dst = (which == 0 ? p.d_q : (which == 1 ? p.d_k : p.d_v)) + (urow * p.H + h) * c + x;
                const f32x4 v0 = *reinterpret_cast<const f32x4 *>(src);
                const f32x4 v1 = *reinterpret_cast<const f32x4 *>(src + 4);
                uint4 o;
                o.x = (unsigned)f2bf(valid ? scale * v0[0] : 0.f) | ((unsigned)f2bf(valid ? scale * v0[1] : 0.f) << 16);
                o.y = (unsigned)f2bf(valid ? scale * v0[2] : 0.f) | ((unsigned)f2bf(valid ? scale * v0[3] : 0.f) << 16);
                o.z = (unsigned)f2bf(valid ? scale * v1[0] : 0.f) | ((unsigned)f2bf(valid ? scale * v1[1] : 0.f) << 16);
                o.w = (unsigned)f2bf(valid ? scale * v1[2] : 0.f) | ((unsigned)f2bf(valid ? scale * v1[3] : 0.f) << 16);
                *reinterpret_cast<uint4 *>(dst) = o;
            }
        }
    }

    // ---- pair factors: sums over heads -------------------------------------------------------------
    {
        const int NG = p.DZ >= 256 ? 64 : p.DZ / 4, HG = 64 / NG;  // lanes per set of columns, head groups
        const int grp = lane % NG, hg = lane / NG;
        for (int x0 = 4 * grp; x0 < p.DZ; x0 += 256) {
            const int d0 = x0 % p.cz;
            f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
            for (int h = hg; h < p.H; h += HG) {
                const size_t bh = (size_t)b * p.H + h;
                const size_t row = (bh * p.Lp + i) * D + kDH + x0;
                const size_t rec = urow * p.H + h;
                const f32x4 dq = *reinterpret_cast<const f32x4 *>(p.dQhat + row);
                const f32x4 dk = *reinterpret_cast<const f32x4 *>(p.dKhat + row);
                const f32x4 dv = *reinterpret_cast<const f32x4 *>(p.dVhat + row);
                const f32x4 oh = *reinterpret_cast<const f32x4 *>(p.Ohat + row);
                const f32x4 wb = *reinterpret_cast<const f32x4 *>(p.w_b + (size_t)h * p.cz + d0);
                const f32x4 dop = *reinterpret_cast<const f32x4 *>(p.d_o_pair + rec * p.cz + d0);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // z1: through the bias vector b^{h1} = w_L w_b z1, and through o~ = z1^T U
                    s1[e] += p.w_L * wb[e] * dq[e] + dop[e] * oh[e];
                    // z2: as key feature (the log2e sits on the query side) and as value feature
                    s2[e] += kLn2 * dk[e] + dv[e];
                }
            }
            for (int o = NG; o < 64; o <<= 1)  // (HG > 1: the head groups, added pairwise in a fixed order)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    s1[e] += __shfl_xor(s1[e], o);
                    s2[e] += __shfl_xor(s2[e], o);
                }
            if (hg == 0) {
                uint2 o1, o2;
                o1.x = (unsigned)f2bf(valid ? s1[0] : 0.f) | ((unsigned)f2bf(valid ? s1[1] : 0.f) << 16);
                o1.y = (unsigned)f2bf(valid ? s1[2] : 0.f) | ((unsigned)f2bf(valid ? s1[3] : 0.f) << 16);
                o2.x = (unsigned)f2bf(valid ? s2[0] : 0.f) | ((unsigned)f2bf(valid ? s2[1] : 0.f) << 16);
                o2.y = (unsigned)f2bf(valid ? s2[2] : 0.f) | ((unsigned)f2bf(valid ? s2[3] : 0.f) << 16);
                *reinterpret_cast<uint2 *>(p.d_z1 + urow * p.DZ + x0) = o1;
                *reinterpret_cast<uint2 *>(p.d_z2 + urow * p.DZ + x0) = o2;
            }
        }
    }

    // frame gradients of this residue: sum over the lanes in a fixed order
    if (p.d_rot) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
#pragma unroll
            for (int x = 0; x < 3; ++x) ft[x] += __shfl_xor(ft[x], o);
#pragma unroll
            for (int x = 0; x < 9; ++x) fr[x] += __shfl_xor(fr[x], o);
        }
        if (lane < 3) p.d_trans[urow * 3 + lane] = valid ? (lane == 0 ? ft[0] : (lane == 1 ? ft[1] : ft[2])) : 0.f;
        if (lane < 9) {
            float v = fr[0];
#pragma unroll
            for (int x = 1; x < 9; ++x) v = lane == x ? fr[x] : v;
            p.d_rot[urow * 9 + lane] = valid ? v : 0.f;
        }
    }
}

// d gamma^h = -(w_L w_C / 2) * sum over (batch, residue) of the partial sums, in a fixed order:
// one workgroup of 1024 threads per head, four independent chains of loads per thread.
// (cu: row offsets of a packed batch, whose chain b has cu[b+1] - cu[b] residues, or null.)
__global__ __launch_bounds__(1024) void fipa_bwd_gamma_kernel(const float *gpart, float *d_gamma, int B, int H,
                                                              int L, int Lp, const int *cu, float coef)
{
    __shared__ float red[1024];
    const int h = blockIdx.x, tid = threadIdx.x;
    float s4[4] = {0.f, 0.f, 0.f, 0.f};
    for (int b = 0; b < B; ++b) {
        const int len = cu ? cu[b + 1] - cu[b] : L;
        const float *g = gpart + ((size_t)b * H + h) * Lp;
        for (int i0 = tid; i0 < len; i0 += 4096)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + 1024 * u;
                s4[u] += i < len ? g[i] : 0.f;
            }
    }
    red[tid] = (s4[0] + s4[1]) + (s4[2] + s4[3]);
    __syncthreads();
    for (int st = 512; st > 0; st >>= 1) {
        if (tid < st) red[tid] += red[tid + st];
        __syncthreads();
    }
    if (tid == 0) d_gamma[h] = coef * red[0];
}

// d w_b[h, d] = w_L * sum over (batch, residue, rho) of z1[b,i,rho,d] * dQ^[b,h,i, 64 + rho*cz + d]
// (b^{h1} = w_L w_b (.) z1, Algorithm 1 step 2 with Eq. 3's w_L).  Two passes with a fixed
// summation order: per (head, chunk of 32 residues) partial sums per lifted column, then the
// sum over chunks and rho.
constexpr int kWbChunk = 32;

// One workgroup per (chunk, head): a thread takes four neighbouring lifted columns (16 bytes of
// dQ^, 8 of z1) of every NRG-th residue of the chunk, all loads independent; the NRG partial sums
// per column meet in LDS and are added in a fixed order.  r c_z <= 512 here, so NRG >= 2.
__global__ __launch_bounds__(256) void fipa_bwd_wb_partial_kernel(BwdUnpackParams p)
{
    __shared__ float red[256 * 4];  // [residue group][DZ], NRG * DZ = 1024 entries
    const int h = blockIdx.y, chunk = blockIdx.x, D = kDH + p.DZ;
    const int nres = p.total_rows;  // rows of the caller's tensors: B L, or the packed batch's total
    const int NG = p.DZ / 4, NRG = 256 / NG;
    const int cg = threadIdx.x % NG, rg = threadIdx.x / NG, x0 = 4 * cg;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int t = rg; t < kWbChunk; t += NRG) {
        const int bi = min(chunk * kWbChunk + t, nres - 1);
        int b, i;
        if (p.cu) {  // the chain that holds row bi: last b with cu[b] <= bi
            int lo = 0, hi = p.B - 1;
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (p.cu[mid] <= bi) lo = mid; else hi = mid - 1;
            }
            b = lo;
            i = bi - p.cu[b];
        } else {
            b = bi / p.L;
            i = bi - b * p.L;
        }
        const bool valid = chunk * kWbChunk + t < nres && (p.mask ? p.mask[bi] != 0 : true);
        const uint2 zr = *reinterpret_cast<const uint2 *>(p.z1 + (size_t)bi * p.DZ + x0);
        const f32x4 dq = *reinterpret_cast<const f32x4 *>(p.dQhat + (((size_t)b * p.H + h) * p.Lp + i) * D + kDH + x0);
        if (valid) {
            s[0] += __uint_as_float(zr.x << 16) * dq[0];
            s[1] += __uint_as_float(zr.x & 0xFFFF0000u) * dq[1];
            s[2] += __uint_as_float(zr.y << 16) * dq[2];
            s[3] += __uint_as_float(zr.y & 0xFFFF0000u) * dq[3];
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) red[rg * p.DZ + x0 + e] = s[e];
    __syncthreads();
    for (int x = threadIdx.x; x < p.DZ; x += 256) {
        float t = 0.f;
        for (int g = 0; g < NRG; ++g) t += red[g * p.DZ + x];
        p.wpart[((size_t)h * gridDim.x + chunk) * p.DZ + x] = t;
    }
}

// One workgroup of 1024 threads per head: the chunks are dealt to 1024 / DZ groups of threads
// (four independent chains of loads each); groups, then rho, are added in a fixed order.
__global__ __launch_bounds__(1024) void fipa_bwd_wb_reduce_kernel(BwdUnpackParams p, int nchunk)
{
    __shared__ float part[1024];  // [chunk group][DZ]
    __shared__ float col[512];    // per lifted pair column: sum over the chunks
    const int h = blockIdx.x;
    const int NCG = 1024 / p.DZ, x = threadIdx.x % p.DZ, cgp = threadIdx.x / p.DZ;
    float s4[4] = {0.f, 0.f, 0.f, 0.f};
    for (int ch0 = cgp; ch0 < nchunk; ch0 += 4 * NCG)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ch = ch0 + u * NCG;
            const float v = p.wpart[((size_t)h * nchunk + min(ch, nchunk - 1)) * p.DZ + x];
            s4[u] += ch < nchunk ? v : 0.f;
        }
    part[cgp * p.DZ + x] = (s4[0] + s4[1]) + (s4[2] + s4[3]);
    __syncthreads();
    if (threadIdx.x < p.DZ) {
        float t = 0.f;
        for (int g = 0; g < NCG; ++g) t += part[g * p.DZ + threadIdx.x];
        col[threadIdx.x] = t;
    }
    __syncthreads();
    for (int d = threadIdx.x; d < p.cz; d += 1024) {
        float t = 0.f;
        for (int rho = 0; rho < p.r; ++rho) t += col[rho * p.cz + d];
        p.d_w_b[(size_t)h * p.cz + d] = p.w_L * t;
    }
}

struct BwdLayout {
    Bf16Layout f;
    size_t dOhat, Dvec, nlse, dQhat, dKhat, dVhat, rowsum, colsum, gpart, wpart, total;
};

BwdLayout bwd_layout(const fipa_desc &d)
{
    BwdLayout w;
    w.f = bf16_layout(d, true, true);
    const size_t BHL = (size_t)d.B * d.H * w.f.Lp;
    const size_t D = kDH + w.f.DZ;
    size_t off = w.f.total;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    w.dOhat = take(BHL * D * 2);
    w.Dvec = take(BHL * 4);
    w.nlse = take(BHL * 4);
    w.dQhat = take(BHL * D * 4);
    w.dKhat = take(BHL * D * 4);
    w.dVhat = take(BHL * D * 4);
    w.rowsum = take(BHL * 4);
    w.colsum = take(BHL * 4);
    w.gpart = take(BHL * 4);
    w.wpart = take((size_t)d.H * (((size_t)d.B * d.L + kWbChunk - 1) / kWbChunk) * w.f.DZ * 4);
    w.total = off;
    return w;
}

}  // namespace

hipError_t launch_bwd_pack_bf16(const BwdPackParams &p, hipStream_t stream)
{
    const size_t rows = (size_t)p.B * p.H * p.Lp;
    hipLaunchKernelGGL(fipa_bwd_pack_bf16_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_bwd_unpack_bf16(const BwdUnpackParams &p, hipStream_t stream)
{
    hipLaunchKernelGGL(fipa_bwd_unpack_bf16_kernel, dim3((unsigned)(((long long)p.B * p.L + 3) / 4)), dim3(256), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(fipa_bwd_gamma_kernel, dim3(p.H), dim3(1024), 0, stream, p.gpart, p.d_gamma, p.B, p.H, p.L,
                       p.Lp, p.cu, -0.5f * p.w_L * p.w_C);
    if (p.d_w_b) {
        const int nchunk = (p.total_rows + kWbChunk - 1) / kWbChunk;
        hipLaunchKernelGGL(fipa_bwd_wb_partial_kernel, dim3(nchunk, p.H), dim3(256), 0, stream, p);
        hipLaunchKernelGGL(fipa_bwd_wb_reduce_kernel, dim3(p.H), dim3(1024), 0, stream, p, nchunk);
    }
    return hipGetLastError();
}

size_t bf16_backward_workspace(const fipa_desc &d) { return bwd_layout(d).total; }

namespace {

PackParams bwd_pack_params(const fipa_desc &d, const FwdArgs &f, const BwdLayout &w, char *base)
{
    PackParams pk;
    pk.q = (const bf16_t *)f.q; pk.k = (const bf16_t *)f.k; pk.v = (const bf16_t *)f.v;
    pk.q_pts = (const bf16_t *)f.q_pts; pk.k_pts = (const bf16_t *)f.k_pts;
    pk.v_pts = (const bf16_t *)f.v_pts;
    pk.z1 = (const bf16_t *)f.z1; pk.z2 = (const bf16_t *)f.z2;
    pk.rot = f.rot; pk.trans = f.trans; pk.w_b = f.w_b; pk.gamma = f.gamma;
    pk.cen = reinterpret_cast<float *>(base + w.f.cen);
    pk.mask = f.mask; pk.cu = f.cu;
    pk.Qh = (bf16_t *)(base + w.f.Qh); pk.Qz = (bf16_t *)(base + w.f.Qz);
    pk.Kh = (bf16_t *)(base + w.f.Kh); pk.Vh = (bf16_t *)(base + w.f.Vh); pk.Z2 = (bf16_t *)(base + w.f.Z2);
    pk.kbias = (float *)(base + w.f.kbias); pk.qbias = (float *)(base + w.f.qbias);
    pk.B = d.B; pk.L = d.L; pk.Lp = w.f.Lp; pk.NT = w.f.NT; pk.H = d.H; pk.c = d.c; pk.Pq = d.Pq;
    pk.Pv = d.Pv; pk.cz = d.cz; pk.r = d.r; pk.DZ = w.f.DZ;
    pk.w_L = d.w_L; pk.w_C = d.w_C; pk.qk_scale = d.qk_scale;
    pk.skip_qz = false;
    // (with the AlphaFold2 head shape the pack kernel finds the per-batch reference point and key-loop bound itself)
    const bool prep_in_pack = d.c == 16 && d.Pq == 4 && d.Pv == 8;
    pk.cen_out = prep_in_pack ? reinterpret_cast<float *>(base + w.f.cen) : nullptr;
    pk.kvlen_out = prep_in_pack ? reinterpret_cast<int *>(base + w.f.kvlen) : nullptr;
    pk.counters = nullptr; pk.n_counters = 0;
    return pk;
}

// Forward pack and (unfused) forward attention: leaves the lifted tensors, O^ and the log-sum-exp
// in the workspace; when f.o is set the core's outputs (steps 8-9) are produced from O^ as well.
hipError_t backward_forward_part(const fipa_desc &d, const FwdArgs &f, const BwdLayout &w, char *base, hipStream_t stream)
{
    float *cen = reinterpret_cast<float *>(base + w.f.cen);
    int *kvlen = reinterpret_cast<int *>(base + w.f.kvlen);
    const PackParams pk = bwd_pack_params(d, f, w, base);
    hipError_t e = hipSuccess;
    if (!pk.cen_out) {
        e = launch_prep(d, f.trans, f.mask, f.cu, cen, kvlen, nullptr, 0, stream);
        if (e != hipSuccess) return e;
    }
    e = launch_pack_bf16(pk, stream);
    if (e != hipSuccess) return e;

    AttnParams at;
    at.Qh = pk.Qh; at.Qz = pk.Qz; at.Kh = pk.Kh; at.Vh = pk.Vh; at.Z2 = pk.Z2;
    at.kbias = pk.kbias; at.qbias = pk.qbias; at.kvlen = kvlen;
    at.Ohat = (float *)(base + w.f.Ohat); at.lse2 = (float *)(base + w.f.lse2);
    at.rot = f.rot; at.trans = f.trans; at.cen = cen; at.z1 = pk.z1; at.mask = f.mask; at.cu = f.cu;
    at.o = nullptr; at.o_pts = nullptr; at.o_pair = nullptr; at.lse = nullptr;
    at.B = d.B; at.L = d.L; at.Lp = w.f.Lp; at.H = d.H; at.NT = w.f.NT;
    at.nQT = w.f.Lp / kTileQ; at.total_tiles = at.nQT * d.B * d.H; at.cz = d.cz; at.r = d.r; at.w_b = f.w_b; at.w_L = d.w_L;
    at.plan = w.f.plan; at.partial = nullptr; at.counters = nullptr;  // (unfused: never split)
    at.deal = f.mask != nullptr || f.cu != nullptr;
    // (width 576: the two-window kernel in its form that leaves O^ in the workspace)
    e = w.f.DZ > 256 ? launch_attn_fwd_wide_bf16(at, w.f.DZ, false, stream) : launch_attn_fwd_bf16(at, w.f.DZ, false, stream);
    if (e != hipSuccess || !f.o) return e;

    EpiParams ep;
    ep.Ohat = at.Ohat; ep.lse2 = at.lse2; ep.qbias = pk.qbias; ep.rot = f.rot; ep.trans = f.trans;
    ep.cen = cen; ep.z1 = pk.z1; ep.mask = f.mask; ep.cu = f.cu;
    ep.o = f.o; ep.o_pts = f.o_pts; ep.o_pair = f.o_pair; ep.lse = f.lse;
    ep.B = d.B; ep.L = d.L; ep.Lp = w.f.Lp; ep.H = d.H; ep.c = d.c; ep.Pv = d.Pv; ep.cz = d.cz;
    ep.r = d.r; ep.DZ = w.f.DZ;
    return launch_epilogue_bf16(ep, stream);
}

// Everything after the forward part: lifting of the upstream gradients, the three gradient
// kernels, and the way back to the inputs.
hipError_t backward_gradient_part(const fipa_desc &d, const BwdArgs &a, const BwdLayout &w, char *base, hipStream_t stream,
                                  StageTimer &timer)
{
    const int total_rows = a.f.cu ? a.f.total_rows : d.B * d.L;  // rows of the caller's tensors
    float *cen = reinterpret_cast<float *>(base + w.f.cen);
    int *kvlen = reinterpret_cast<int *>(base + w.f.kvlen);
    const PackParams pk = bwd_pack_params(d, a.f, w, base);
    float *Ohat = (float *)(base + w.f.Ohat);

    BwdPackParams bp;
    bp.d_o = a.d_o; bp.d_o_pts = a.d_o_pts; bp.d_o_pair = a.d_o_pair; bp.rot = a.f.rot;
    bp.Ohat = Ohat; bp.lse2 = (float *)(base + w.f.lse2); bp.z1 = pk.z1; bp.mask = a.f.mask; bp.cu = a.f.cu;
    bp.dOhat = (bf16_t *)(base + w.dOhat); bp.Dvec = (float *)(base + w.Dvec); bp.nlse = (float *)(base + w.nlse);
    bp.B = d.B; bp.L = d.L; bp.Lp = w.f.Lp; bp.H = d.H; bp.c = d.c; bp.Pv = d.Pv; bp.cz = d.cz; bp.r = d.r;
    bp.DZ = w.f.DZ;
    hipError_t e = launch_bwd_pack_bf16(bp, stream);
    if (e != hipSuccess) return e;
    timer.end(0);

    // ---- dQ^, dK^, dV^ --------------------------------------------------------------------------------
    timer.begin(1);
    BwdParams bw;
    bw.Qh = pk.Qh; bw.Qz = pk.Qz; bw.Kh = pk.Kh; bw.Vh = pk.Vh; bw.Z2 = pk.Z2; bw.dOhat = bp.dOhat;
    bw.kbias = pk.kbias; bw.nlse = bp.nlse; bw.Dvec = bp.Dvec; bw.kvlen = kvlen;
    bw.B = d.B; bw.L = d.L; bw.Lp = w.f.Lp; bw.H = d.H; bw.total_tiles = (w.f.Lp / kTileQ) * d.B * d.H;
    bw.deal = a.f.mask != nullptr || a.f.cu != nullptr;
    bw.out = (float *)(base + w.dQhat); bw.wsum = (float *)(base + w.rowsum);
    e = launch_bwd_bf16(bw, w.f.DZ, FIPA_BWD_DQ, stream);
    if (e != hipSuccess) return e;
    bw.out = (float *)(base + w.dKhat); bw.wsum = (float *)(base + w.colsum);
    e = launch_bwd_bf16(bw, w.f.DZ, FIPA_BWD_DK, stream);
    if (e != hipSuccess) return e;
    bw.out = (float *)(base + w.dVhat); bw.wsum = nullptr;
    e = launch_bwd_bf16(bw, w.f.DZ, FIPA_BWD_DV, stream);
    if (e != hipSuccess) return e;
    timer.end(1);

    // ---- back to the inputs ----------------------------------------------------------------------------
    timer.begin(2);
    BwdUnpackParams up;
    up.q_pts = pk.q_pts; up.k_pts = pk.k_pts; up.v_pts = pk.v_pts; up.z1 = pk.z1;
    up.d_o_pts = a.d_o_pts; up.d_rot = a.d_rot; up.d_trans = a.d_trans; up.dOhat = bp.dOhat;
    up.rot = a.f.rot; up.trans = a.f.trans; up.cen = cen; up.gamma = a.f.gamma; up.w_b = a.f.w_b;
    up.d_o_pair = a.d_o_pair; up.mask = a.f.mask; up.cu = a.f.cu;
    up.total_rows = total_rows;
    up.dQhat = (const float *)(base + w.dQhat); up.dKhat = (const float *)(base + w.dKhat);
    up.dVhat = (const float *)(base + w.dVhat); up.Ohat = Ohat;
    up.rowsum = (const float *)(base + w.rowsum); up.colsum = (const float *)(base + w.colsum);
    up.d_q = (bf16_t *)a.d_q; up.d_k = (bf16_t *)a.d_k; up.d_v = (bf16_t *)a.d_v;
    up.d_q_pts = (bf16_t *)a.d_q_pts; up.d_k_pts = (bf16_t *)a.d_k_pts; up.d_v_pts = (bf16_t *)a.d_v_pts;
    up.d_z1 = (bf16_t *)a.d_z1; up.d_z2 = (bf16_t *)a.d_z2;
    up.gpart = (float *)(base + w.gpart); up.d_gamma = a.d_gamma;
    up.d_w_b = a.d_w_b; up.wpart = (float *)(base + w.wpart);
    up.B = d.B; up.L = d.L; up.Lp = w.f.Lp; up.H = d.H; up.c = d.c; up.Pq = d.Pq; up.Pv = d.Pv; up.cz = d.cz;
    up.r = d.r; up.DZ = w.f.DZ;
    up.w_L = d.w_L; up.w_C = d.w_C; up.qk_scale = d.qk_scale;
    e = launch_bwd_unpack_bf16(up, stream);
    timer.end(2);
    return e;
}

}  // namespace

hipError_t bf16_backward(const fipa_desc &d, const BwdArgs &a, void *ws, hipStream_t stream)
{
    const BwdLayout w = bwd_layout(d);
    char *base = static_cast<char *>(ws);
    StageTimer timer(stream);
    timer.begin(0);
    FwdArgs f = a.f;
    f.o = nullptr;  // (the core's outputs are not needed here)
    const hipError_t e = backward_forward_part(d, f, w, base, stream);
    if (e != hipSuccess) return e;
    return backward_gradient_part(d, a, w, base, stream, timer);
}

// The same in two calls on one workspace, for a caller that needs the core's outputs before it
// can form the upstream gradients (the module's backward): the first call also writes f.o,
// f.o_pts, f.o_pair; the workspace must not be touched in between.
hipError_t bf16_backward_begin(const fipa_desc &d, const FwdArgs &f, void *ws, hipStream_t stream)
{
    if (!f.o || !f.o_pts || !f.o_pair) return hipErrorInvalidValue;
    return backward_forward_part(d, f, bwd_layout(d), static_cast<char *>(ws), stream);
}

hipError_t bf16_backward_finish(const fipa_desc &d, const BwdArgs &a, void *ws, hipStream_t stream)
{
    StageTimer timer;  // (not timed)
    return backward_gradient_part(d, a, bwd_layout(d), static_cast<char *>(ws), stream, timer);
}

}  // namespace fipa
