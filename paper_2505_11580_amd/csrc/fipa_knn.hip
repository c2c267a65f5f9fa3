// k-nearest-neighbour distogram features (Section 2.5 of the paper): for every residue the k
// nearest valid residues of its chain by the distance of the frame origins, their squared
// distances and distogram bins -- [L, k] instead of the [L, L] distogram.  The paper gives one
// paragraph and no formula; the readings are stated in include/fipa.h.
//
// One wave per query residue.  The wave keeps its 64 best candidates so far as a sorted list, one
// entry per lane (lane s holds the s-th nearest), scans the chain 64 residues at a time, and
// inserts the few candidates that beat the current k-th entry one by one (a shift by one lane
// from the insertion point on); the scan starts at the residue's own block and moves outwards.
// Order is by (squared distance, index), a strict total order, so the result does not depend on
// the order of the scan.  Every decision is taken in float32 on
// ((dx*dx + dy*dy) + dz*dz) with one rounding per operation (no fused multiply-add).
#include "fipa_internal.h"

#include <climits>

// This file is compiled with -ffp-contract=off: the distance arithmetic is specified with one
// rounding per operation, and the compiler would otherwise contract a*b + c into a fused
// multiply-add (also through the __fmul_rn / __fadd_rn intrinsics, which are plain operators).

namespace fipa {

namespace {

__device__ __forceinline__ bool before(float ad, int aj, float bd, int bj) { return ad < bd || (ad == bd && aj < bj); }

__global__ __launch_bounds__(256) void fipa_knn_distogram_kernel(const float *__restrict__ trans,
                                                                 const uint8_t *__restrict__ mask, int B, int L, int k,
                                                                 int n_bins, float d_min, float w,
                                                                 int *__restrict__ nbr_idx, float *__restrict__ nbr_d2,
                                                                 int *__restrict__ nbr_bin)
{
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);  // (b, i); uniform over the wave
    if (row >= (long long)B * L) return;
    const int b = (int)(row / L), i = (int)(row - (long long)b * L);
    const float *t = trans + (size_t)b * L * 3;
    const uint8_t *m = mask ? mask + (size_t)b * L : nullptr;

    float best_d = INFINITY;  // lane s: the s-th nearest so far
    int best_j = INT_MAX;
    if (!m || m[i] != 0) {
        const float xi = t[3 * i], yi = t[3 * i + 1], zi = t[3 * i + 2];
        float thr_d = INFINITY;  // entry k - 1 of the list
        int thr_j = INT_MAX;
        // The blocks of 64 candidates are visited outwards from the residue's own: in a chain the
        // neighbours along the sequence are near in space, so the list fills with near residues at
        // once and few later candidates beat its k-th entry (in index order every residue before i
        // arrives nearer than the one before it and is inserted, one at a time).
        const int nblk = (L + 63) / 64, own = i / 64;
        for (int step = 0, up = own, down = own - 1; step < nblk; ++step) {
            // alternate above / below while both sides have blocks left
            const bool take_up = up < nblk && (down < 0 || ((step & 1) == 0));
            const int j0 = 64 * (take_up ? up : down);
            if (take_up) ++up; else --down;
            const int j = j0 + lane;
            const bool ok = j < L && j != i && (!m || m[j] != 0);
            float d2 = INFINITY;
            if (ok) {
                const float dx = __fsub_rn(t[3 * j], xi), dy = __fsub_rn(t[3 * j + 1], yi), dz = __fsub_rn(t[3 * j + 2], zi);
                d2 = __fadd_rn(__fadd_rn(__fmul_rn(dx, dx), __fmul_rn(dy, dy)), __fmul_rn(dz, dz));
            }
            unsigned long long todo = __ballot(ok && before(d2, j, thr_d, thr_j));
            while (todo) {
                const int l = __ffsll((long long)todo) - 1;
                todo &= todo - 1;
                const float nd = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, d2), l));
                const int nj = __builtin_amdgcn_readlane(j, l);
                if (!before(nd, nj, thr_d, thr_j)) continue;  // (the threshold has moved since the ballot)
                // insert: the entries behind the new one move one lane up
                const int behind = before(nd, nj, best_d, best_j) ? 1 : 0;
                const float prev_d = __shfl_up(best_d, 1);
                const int prev_j = __shfl_up(best_j, 1);
                const int up_behind = __shfl_up(behind, 1);  // (every lane takes part in the exchange)
                const int prev_behind = lane > 0 ? up_behind : 0;
                if (behind) {
                    best_d = prev_behind ? prev_d : nd;
                    best_j = prev_behind ? prev_j : nj;
                }
                thr_d = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, best_d), k - 1));
                thr_j = __builtin_amdgcn_readlane(best_j, k - 1);
            }
        }
    }
    if (lane < k) {
        const bool have = best_j != INT_MAX;
        int bin = -1;
        if (have) {
            bin = 0;
            for (int e = 0; e < n_bins - 1; ++e) {
                const float edge = __fadd_rn(d_min, __fmul_rn((float)e, w));
                bin += __fmul_rn(edge, edge) <= best_d ? 1 : 0;
            }
        }
        const size_t at = (size_t)row * k + lane;
        nbr_idx[at] = have ? best_j : -1;
        nbr_d2[at] = have ? best_d : INFINITY;
        nbr_bin[at] = bin;
    }
}

}  // namespace

}  // namespace fipa

extern "C" int fipa_knn_distogram(int32_t B, int32_t L, int32_t k, int32_t n_bins, float d_min, float d_max,
                                  const float *trans, const uint8_t *mask, int32_t *nbr_idx, float *nbr_d2,
                                  int32_t *nbr_bin, void *hip_stream)
{
    if (B <= 0 || L <= 0 || k <= 0 || n_bins < 2 || !(d_min >= 0.f) || !(d_max > d_min)) return FIPA_ERR_INVALID_ARG;
    if (!trans || !nbr_idx || !nbr_d2 || !nbr_bin) return FIPA_ERR_INVALID_ARG;
    if (k > 64 || n_bins > 4096 || (long long)B * L * k >= (1LL << 31)) return FIPA_ERR_UNSUPPORTED;
    const void *al[] = {trans, nbr_idx, nbr_d2, nbr_bin};
    for (const void *ptr : al)
        if ((reinterpret_cast<uintptr_t>(ptr) & 3u) != 0) return FIPA_ERR_ALIGNMENT;
    const float w = (d_max - d_min) / (float)(n_bins - 1);
    const long long rows = (long long)B * L;
    hipLaunchKernelGGL(fipa::fipa_knn_distogram_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), trans, mask, B, L, k, n_bins, d_min, w, nbr_idx, nbr_d2,
                       nbr_bin);
    return hipGetLastError() == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
}
