// Split of the lifted output, inverse frame on the point part (Eq. 4) and contraction of the
// pair part with z1 (Algorithm 1 steps 8-9).  Memory bound: one wave per (batch, head, row).
#include "fipa_gfx950.h"

namespace fipa {

namespace {

__global__ __launch_bounds__(256) void fipa_epilogue_bf16_kernel(EpiParams p)
{
    const int lane = threadIdx.x & 63;
    const size_t grid_id = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // over B*L*H, h fastest
    if (grid_id >= (size_t)p.B * p.L * p.H) return;
    const int h = (int)(grid_id % p.H);
    const size_t bi = grid_id / p.H;
    const int i = (int)(bi % p.L);
    const int b = (int)(bi / p.L);
    if (i >= user_len(p, b)) return;  // (packed batch: L is only an upper bound of the chain lengths)
    const size_t urow = user_row(p, b, i);
    const size_t row_id = urow * p.H + h;  // row of the outputs
    const int c = p.c, nv = 3 * p.Pv, DV = kDH + p.DZ;
    const size_t bh = (size_t)b * p.H + h;
    const float *oh = p.Ohat + (bh * p.Lp + i) * DV;
    const bool valid = p.mask ? p.mask[urow] != 0 : true;

    // (c and c_z are multiples of 8 on this path: 16-byte accesses throughout)
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    for (int d = 4 * lane; d < c; d += 256)
        *reinterpret_cast<f32x4 *>(p.o + row_id * c + d) = valid ? *reinterpret_cast<const f32x4 *>(oh + d) : zero4;

    const float *R = p.rot + urow * 9;
    const float *t = p.trans + urow * 3;
    for (int idx = lane; idx < nv; idx += 64) {
        const int pp = idx / 3, x = idx - 3 * pp;
        float val = 0.f;
        if (valid) {
            for (int y = 0; y < 3; ++y) {
                const float G = oh[v_pt_col(c, p.Pv, pp, y, 0)] + oh[v_pt_col(c, p.Pv, pp, y, 1)];
                val += R[3 * y + x] * (G - (t[y] - p.cen[4 * b + y]));
            }
        }
        p.o_pts[row_id * nv + idx] = val;
    }

    const bf16_t *z1 = p.z1 + urow * p.DZ;
    for (int d = 4 * lane; d < p.cz; d += 256) {
        f32x4 val = zero4;
        if (valid)
            for (int rho = 0; rho < p.r; ++rho) {
                const uint2 zr = *reinterpret_cast<const uint2 *>(z1 + rho * p.cz + d);  // four bf16 values
                const f32x4 u = *reinterpret_cast<const f32x4 *>(oh + kDH + rho * p.cz + d);
                val[0] += __uint_as_float(zr.x << 16) * u[0];
                val[1] += __uint_as_float(zr.x & 0xFFFF0000u) * u[1];
                val[2] += __uint_as_float(zr.y << 16) * u[2];
                val[3] += __uint_as_float(zr.y & 0xFFFF0000u) * u[3];
            }
        *reinterpret_cast<f32x4 *>(p.o_pair + row_id * p.cz + d) = val;
    }

    // natural log-sum-exp of Eq. 3's argument: undo the log2 scaling and put back the
    // per-query |Q|^2 term that was left out of the logits
    if (p.lse && lane == 0) {
        const float l2 = p.lse2[bh * p.Lp + i];
        p.lse[user_lse_index(p, b, h, i)] = (valid && l2 > -INFINITY) ? l2 * kLn2 - p.qbias[bh * p.Lp + i] : 0.f;
    }
}

}  // namespace

hipError_t launch_epilogue_bf16(const EpiParams &p, hipStream_t stream)
{
    const size_t rows = (size_t)p.B * p.L * p.H;
    hipLaunchKernelGGL(fipa_epilogue_bf16_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0,
                       stream, p);
    return hipGetLastError();
}

}  // namespace fipa
