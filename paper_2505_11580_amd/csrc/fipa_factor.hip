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

#include <algorithm>
#include <climits>

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


// Gradient with respect to the tables: d e_bin[s, m, :] is the sum of d_z[b, i, :] over the residues
// whose slot s is filled and holds bin m, likewise d e_pos by position code, d bias the sum over
// all residues -- a scatter of rows.  One workgroup per (slot, 64 output columns); each of its W
// working waves owns a private copy of the slot's table slice in LDS ([rows][64 columns], lane =
// column) and takes every W-th residue, adding the residue's 64 values into the rows its slot selects
// by plain LDS reads and writes: a wave's LDS instructions execute in the order issued and no other
// wave touches its copy, so every entry is summed in residue order and the result is the same on
// every run.  (LDS float atomics, which need no read, were three times slower: 8.6 against 2.6 ms at
// 32768 residues, 512 columns.)  At the end the copies are added in wave order.  A residue with mask 0
// adds nothing.  The residues arrive in tiles of 128 (their slot-s index and bin, mask, and 128 bytes
// of d_z each) that all 256 threads fetch with 16-byte loads into registers while the previous tile
// is being worked on, and hand over through LDS; one barrier per tile.
constexpr int kFbTile = 128;
constexpr int kFbStageBytes = kFbTile * 128 + 3 * kFbTile * 4;  // d_z rows, then index, bin, mask flag

template <bool HAS_POS>
__global__ __launch_bounds__(256) void fipa_factor_backward_kernel(const int *__restrict__ nbr_idx, const int *__restrict__ nbr_bin,
                                                                   const bf16_t *__restrict__ d_z, const uint8_t *__restrict__ mask,
                                                                   float *__restrict__ d_e_bin, float *__restrict__ d_e_pos,
                                                                   float *__restrict__ d_bias, int rows, int L, int k, int n_bins,
                                                                   int n_pos, int pos_mode, int n_out, int W)
{
    extern __shared__ __attribute__((aligned(16))) char fb_smem[];  // two stages, then tab[W][R][64]
    const int s = blockIdx.x, col0 = blockIdx.y * 64, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int R = n_bins + n_pos + 1;  // bin rows, position rows, one row for the bias (used by slot 0)
    float *tab = reinterpret_cast<float *>(fb_smem + 2 * kFbStageBytes);
    for (int x = tid; x < W * R * 64; x += 256) tab[x] = 0.f;
    float *t = tab + (size_t)wave * R * 64 + lane;
    const int half = (n_pos - 1) >> 1;
    const int ntiles = (rows + kFbTile - 1) / kFbTile;

    uint4 rz[4];
    int rmeta = 0;
    auto fetch = [&](int tile) {
        const int res0 = tile * kFbTile;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = tid + 256 * q, rr = c >> 3, part = c & 7;
            const int res = min(res0 + rr, rows - 1), col = col0 + 8 * part;
            rz[q] = col < n_out ? *reinterpret_cast<const uint4 *>(d_z + (size_t)res * n_out + col) : (uint4){0u, 0u, 0u, 0u};
        }
        // threads 0..127: index, 128..255: bin of residue tid % 128 (slot s); the mask flag rides in the index's thread
        const int rr = tid & (kFbTile - 1), res = min(res0 + rr, rows - 1);
        rmeta = tid < kFbTile ? nbr_idx[(size_t)res * k + s] : nbr_bin[(size_t)res * k + s];
        if (tid < kFbTile && (res0 + rr >= rows || (mask && mask[res] == 0))) rmeta = INT_MIN;  // nothing to add
    };
    fetch(0);
    for (int tile = 0; tile < ntiles; ++tile) {
        char *st = fb_smem + (tile & 1) * kFbStageBytes;
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<uint4 *>(st + (tid + 256 * q) * 16) = rz[q];
        reinterpret_cast<int *>(st + kFbTile * 128)[tid] = rmeta;  // [0, 128): index or INT_MIN; [128, 256): bin
        __syncthreads();  // (also orders the clearing of the tables before the first adds)
        if (tile + 1 < ntiles) fetch(tile + 1);
        if (wave < W) {
            const int *meta = reinterpret_cast<const int *>(st + kFbTile * 128);
            // the next residue's index, bin and value are read while this one's rows are updated; the (up to)
            // three rows of one residue are different rows, so their reads go out together
            int j = meta[wave], bn = meta[kFbTile + wave];
            float dz = bf2f(*reinterpret_cast<const bf16_t *>(st + wave * 128 + lane * 2));
            for (int rr = wave; rr < kFbTile; rr += W) {
                const int jc = j, bc = bn;
                const float dc = dz;
                const int nx = min(rr + W, kFbTile - 1);
                j = meta[nx];
                bn = meta[kFbTile + nx];
                dz = bf2f(*reinterpret_cast<const bf16_t *>(st + nx * 128 + lane * 2));
                if (jc == INT_MIN) continue;  // (uniform over the wave: all lanes look at the same residue)
                const bool filled = jc >= 0 && jc < L;
                float *p_bias = t + (R - 1) * 64;
                float *p_bin = t + min(max(bc, 0), n_bins - 1) * 64;
                float *p_pos = p_bin;
                if constexpr (HAS_POS) {
                    const int i = (tile * kFbTile + rr) % L;
                    const int code = pos_mode == 0 ? min(jc, n_pos - 1) : min(max(jc - i, -half), half) + half;
                    p_pos = t + (n_bins + (filled ? code : 0)) * 64;
                }
                const float v_bias = *p_bias, v_bin = *p_bin, v_pos = *p_pos;
                if (s == 0) *p_bias = v_bias + dc;
                if (filled) {
                    *p_bin = v_bin + dc;
                    if constexpr (HAS_POS) *p_pos = v_pos + dc;
                }
            }
        }
    }
    __syncthreads();
    const int col = col0 + lane;
    if (col >= n_out) return;
    for (int row = wave; row < R; row += 4) {
        float v = 0.f;
        for (int w = 0; w < W; ++w) v += tab[((size_t)w * R + row) * 64 + lane];
        if (row < n_bins)
            d_e_bin[((size_t)s * n_bins + row) * n_out + col] = v;
        else if (row < n_bins + n_pos)
            d_e_pos[((size_t)s * n_pos + (row - n_bins)) * n_out + col] = v;
        else if (s == 0 && d_bias)
            d_bias[col] = v;
    }
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

extern "C" int fipa_factor_project_backward(int32_t B, int32_t L, int32_t k, int32_t n_bins, int32_t n_pos, int32_t pos_mode,
                                            int32_t n_out, const int32_t *nbr_idx, const int32_t *nbr_bin, const void *d_z,
                                            const uint8_t *mask, float *d_e_bin, float *d_e_pos, float *d_bias,
                                            void *hip_stream)
{
    if (B <= 0 || L <= 0 || k <= 0 || n_bins < 1 || n_out <= 0 || n_pos < 0) return FIPA_ERR_INVALID_ARG;
    if (!nbr_idx || !nbr_bin || !d_z || !d_e_bin) return FIPA_ERR_INVALID_ARG;
    if ((n_pos > 0) != (d_e_pos != nullptr)) return FIPA_ERR_INVALID_ARG;
    if (pos_mode != 0 && pos_mode != 1) return FIPA_ERR_INVALID_ARG;
    if (n_pos > 0 && pos_mode == 1 && n_pos % 2 == 0) return FIPA_ERR_INVALID_ARG;
    if (n_out % 8 != 0 || k > 64 || (long long)B * L * k >= (1LL << 31)) return FIPA_ERR_UNSUPPORTED;
    // a wave's copy of a slot's table slice: (n_bins + n_pos + 1) rows of 64 floats; as many copies (waves
    // at work) as fit 120 KB of LDS beside the two stages of incoming residues, four at most
    const long long copy_bytes = ((long long)n_bins + n_pos + 1) * 64 * 4;
    const int W = (int)std::min<long long>(4, (120 * 1024) / copy_bytes);
    if (W < 1) return FIPA_ERR_UNSUPPORTED;
    const void *al16[] = {d_z, d_e_bin, d_e_pos, d_bias};
    for (const void *ptr : al16)
        if (ptr && !fipa::aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    if ((reinterpret_cast<uintptr_t>(nbr_idx) & 3u) != 0 || (reinterpret_cast<uintptr_t>(nbr_bin) & 3u) != 0) return FIPA_ERR_ALIGNMENT;
    const int lds = (int)(W * copy_bytes) + 2 * fipa::kFbStageBytes;
    const dim3 grid((unsigned)k, (unsigned)((n_out + 63) / 64));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int rows = B * L;
    hipError_t e;
    if (n_pos > 0) {
        static fipa::LdsLimit lim;
        e = fipa::raise_lds_limit(lim, (const void *)fipa::fipa_factor_backward_kernel<true>, lds);
        if (e != hipSuccess) return FIPA_ERR_LAUNCH;
        hipLaunchKernelGGL(fipa::fipa_factor_backward_kernel<true>, grid, dim3(256), lds, stream, nbr_idx, nbr_bin,
                           (const fipa::bf16_t *)d_z, mask, d_e_bin, d_e_pos, d_bias, rows, L, k, n_bins, n_pos, pos_mode, n_out, W);
    } else {
        static fipa::LdsLimit lim;
        e = fipa::raise_lds_limit(lim, (const void *)fipa::fipa_factor_backward_kernel<false>, lds);
        if (e != hipSuccess) return FIPA_ERR_LAUNCH;
        hipLaunchKernelGGL(fipa::fipa_factor_backward_kernel<false>, grid, dim3(256), lds, stream, nbr_idx, nbr_bin,
                           (const fipa::bf16_t *)d_z, mask, d_e_bin, (float *)nullptr, d_bias, rows, L, k, n_bins, 0, pos_mode, n_out, W);
    }
    return hipGetLastError() == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
}
