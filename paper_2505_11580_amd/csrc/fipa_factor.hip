// Pair pseudo-factors from k-nearest-neighbour features (Section 2.4 of the paper: each pair
// feature is represented by two [L, r, c_z] tensors obtained by linear projections; Section 2.5:
// the features are the distogram bins of the k nearest neighbours plus a positional encoding of
// the neighbours' indices).  The paper gives no formula; the readings are stated in include/fipa.h.
//
// A linear projection of concatenated one-hot vectors is a sum of table rows, so nothing is
// multiplied: z_i = bias + sum over the neighbour slots s of (e_bin[s][bin_is] + e_pos[s][code_is]).
// One thread per (residue, 8 output columns): the threads of a residue read the same k indices
// (one broadcast load each) and consecutive 16-byte pieces of the selected rows; the tables (a
// few MB at most) stay in L2, so the kernel is bound by L2 reads of 2 k n_out bf16 per residue,
// not by HBM (the algorithmic HBM traffic is the n_out bf16 written and 8 k index bytes read).
// Sums are float32 in slot order (bias, then per slot the bin row, then the position row), rounded
// to bf16 once at the end.
#include "fipa_bf16_common.h"
#include "fipa_internal.h"

namespace fipa {

namespace {

__device__ __forceinline__ void add_row(float (&acc)[8], const bf16_t *row, bool on)
{
    const uint4 v = *reinterpret_cast<const uint4 *>(row);
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        acc[2 * q] += on ? __uint_as_float(w[q] << 16) : 0.f;
        acc[2 * q + 1] += on ? __uint_as_float(w[q] & 0xffff0000u) : 0.f;
    }
}

template <bool HAS_POS>
__global__ __launch_bounds__(256) void fipa_factor_project_kernel(const int *__restrict__ nbr_idx, const int *__restrict__ nbr_bin,
                                                                  const bf16_t *__restrict__ e_bin, const bf16_t *__restrict__ e_pos,
                                                                  const float *__restrict__ bias, bf16_t *__restrict__ z,
                                                                  long long rows, int L, int k, int n_bins, int n_pos,
                                                                  int pos_mode, int nchunk)
{
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= rows * nchunk) return;
    const long long row = t / nchunk;
    const int ch = (int)(t - row * nchunk), i = (int)(row % L);
    const size_t n_out = (size_t)nchunk * 8;
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = bias ? bias[ch * 8 + q] : 0.f;
    const int *ji = nbr_idx + row * k, *bi = nbr_bin + row * k;
    const int half = (n_pos - 1) >> 1;
#pragma unroll 4
    for (int s = 0; s < k; ++s) {
        const int j = ji[s];
        const bool filled = j >= 0 && j < L;
        // an empty slot reads row 0 and adds nothing (no divergent branch around the loads); a bin
        // outside the table is clamped into it, so every address is inside the tables
        const bool on = filled;
        const int bn = filled ? min(max(bi[s], 0), n_bins - 1) : 0;
        add_row(acc, e_bin + ((size_t)s * n_bins + bn) * n_out + ch * 8, on);
        if constexpr (HAS_POS) {
            int code = pos_mode == 0 ? min(j, n_pos - 1) : min(max(j - i, -half), half) + half;
            code = filled ? code : 0;
            add_row(acc, e_pos + ((size_t)s * n_pos + code) * n_out + ch * 8, on);
        }
    }
    uint4 o;
    o.x = (unsigned)f2bf(acc[0]) | ((unsigned)f2bf(acc[1]) << 16);
    o.y = (unsigned)f2bf(acc[2]) | ((unsigned)f2bf(acc[3]) << 16);
    o.z = (unsigned)f2bf(acc[4]) | ((unsigned)f2bf(acc[5]) << 16);
    o.w = (unsigned)f2bf(acc[6]) | ((unsigned)f2bf(acc[7]) << 16);
    *reinterpret_cast<uint4 *>(z + row * n_out + ch * 8) = o;
}

}  // namespace
}  // namespace fipa

extern "C" int fipa_factor_project(int32_t B, int32_t L, int32_t k, int32_t n_bins, int32_t n_pos, int32_t pos_mode,
                                   int32_t n_out, const int32_t *nbr_idx, const int32_t *nbr_bin, const void *e_bin,
                                   const void *e_pos, const float *bias, void *z, void *hip_stream)
{
    if (B <= 0 || L <= 0 || k <= 0 || n_bins < 1 || n_out <= 0 || n_pos < 0) return FIPA_ERR_INVALID_ARG;
    if (!nbr_idx || !nbr_bin || !e_bin || !z) return FIPA_ERR_INVALID_ARG;
    if ((n_pos > 0) != (e_pos != nullptr)) return FIPA_ERR_INVALID_ARG;
    if (pos_mode != 0 && pos_mode != 1) return FIPA_ERR_INVALID_ARG;
    if (n_pos > 0 && pos_mode == 1 && n_pos % 2 == 0) return FIPA_ERR_INVALID_ARG;  // offsets -h .. +h
    if (n_out % 8 != 0 || k > 64 || (long long)B * L * k >= (1LL << 31)) return FIPA_ERR_UNSUPPORTED;
    const long long rows = (long long)B * L, threads = rows * (n_out / 8);
    if ((threads + 255) / 256 >= (1LL << 31)) return FIPA_ERR_UNSUPPORTED;
    const void *al16[] = {e_bin, e_pos, z, bias};
    for (const void *ptr : al16)
        if (ptr && !fipa::aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    if ((reinterpret_cast<uintptr_t>(nbr_idx) & 3u) != 0 || (reinterpret_cast<uintptr_t>(nbr_bin) & 3u) != 0) return FIPA_ERR_ALIGNMENT;
    const dim3 grid((unsigned)((threads + 255) / 256));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (n_pos > 0)
        hipLaunchKernelGGL(fipa::fipa_factor_project_kernel<true>, grid, dim3(256), 0, stream, nbr_idx, nbr_bin,
                           (const fipa::bf16_t *)e_bin, (const fipa::bf16_t *)e_pos, bias, (fipa::bf16_t *)z, rows, L, k,
                           n_bins, n_pos, pos_mode, n_out / 8);
    else
        hipLaunchKernelGGL(fipa::fipa_factor_project_kernel<false>, grid, dim3(256), 0, stream, nbr_idx, nbr_bin,
                           (const fipa::bf16_t *)e_bin, (const fipa::bf16_t *)nullptr, bias, (fipa::bf16_t *)z, rows, L, k,
                           n_bins, 1, pos_mode, n_out / 8);
    return hipGetLastError() == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
}
