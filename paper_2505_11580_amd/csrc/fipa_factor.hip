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
#include "fipa_gfx950.h"
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
// all residues.  A scatter of rows -- but a scatter into shared sums either serialises on LDS
// round trips (per-wave table copies updated row by row: 2.1 ms at 32768 residues, 512 columns; with
// LDS float atomics 8.6 ms) or loses the fixed summation order.  Here it is the contraction it
// also is, over the residue axis: dE_s [rows, 64 columns] = X_s^T [rows, residues] . dZ [residues, 64],
// with X_s the one-hot features of slot s -- exact in bf16 -- on the matrix pipe with float32
// accumulation in a fixed order (the same bits on every run).  One workgroup per (slot, 64 output
// columns) walks the residues in tiles of 128: every thread fetches 64 bytes of d_z (16-byte loads, in
// flight while the two tiles before it are multiplied) and hands them over through LDS as they are
// ([residue][column]; the matrix operand is taken from there with the transposing read); one
// thread per residue marks that residue's (up to three) rows in the one-hot tile ([row][residue]) and
// takes back the marks it made two tiles earlier, so the tile never needs clearing as a whole; one
// barrier per tile; the 2 x ceil(rows / 32) output tiles are dealt to the four waves.  0.32 ms at 32768
// residues, 20 slots, 82 rows, 512 columns.
// rows = n_bins + n_pos + 1 (the last one collects the bias gradient, in slot 0's workgroups).
constexpr int kFbTile = 128;
constexpr int kFbStride = kFbTile * 2 + 16;  // bytes per row of the one-hot tile ([row][residue])
constexpr int kFbZStride = 64 * 2 + 16;      // bytes per row of the d_z tile ([residue][column])
constexpr int kFbMaxRowBlocks = 5, kFbMaxOwn = (2 * kFbMaxRowBlocks + 3) / 4;

template <bool HAS_POS>
__global__ __launch_bounds__(256) void fipa_factor_backward_kernel(const int *__restrict__ nbr_idx, const int *__restrict__ nbr_bin,
                                                                   const bf16_t *__restrict__ d_z, const uint8_t *__restrict__ mask,
                                                                   float *__restrict__ d_e_bin, float *__restrict__ d_e_pos,
                                                                   float *__restrict__ d_bias, int rows, int L, int k, int n_bins,
                                                                   int n_pos, int pos_mode, int n_out, int RB)
{
    extern __shared__ __attribute__((aligned(16))) char fb_smem[];  // d_z tiles [2][128][z stride], one-hot tiles [2][32 RB][stride]
    const int s = blockIdx.x, col0 = blockIdx.y * 64, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, li = lane & 31, g = lane >> 5;
    const int R = n_bins + n_pos + 1, Rpad = 32 * RB;
    char *const zt = fb_smem, *const xt = fb_smem + 2 * kFbTile * kFbZStride;
    for (int x = tid * 16; x < 2 * Rpad * kFbStride; x += 256 * 16) *reinterpret_cast<uint4 *>(xt + x) = (uint4){0u, 0u, 0u, 0u};
    const int half = (n_pos - 1) >> 1;
    const int ntiles = (rows + kFbTile - 1) / kFbTile;
    const int n_own = (2 * RB - wave + 3) / 4;  // output tiles wave, wave + 4, ... of the 2 RB (row block, column block) pairs

    f32x16 acc[kFbMaxOwn];
#pragma unroll
    for (int o = 0; o < kFbMaxOwn; ++o)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[o][r] = 0.f;

    // what a thread holds of a tile between its fetch and its hand-over: 64 bytes of d_z, and (threads
    // 128..255: the waves that own fewer output tiles when their number is not a multiple of four) one
    // residue's slot-s neighbour, bin and validity
    const int mr = tid - (256 - kFbTile);  // that residue
    struct Held {
        uint4 rz[4];
        int rj, rb;
        bool rv;
    };
    auto fetch = [&](int tile, Held &hd) {
        const int res0 = tile * kFbTile;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = tid + 256 * q, rr = c >> 3, part = c & 7;
            const int res = min(res0 + rr, rows - 1), col = col0 + 8 * part;
            const bool ok = res0 + rr < rows && col < n_out && (mask ? mask[res] != 0 : true);
            // (what a masked or missing residue holds never reaches the products: 0 x NaN would)
            hd.rz[q] = ok ? *reinterpret_cast<const uint4 *>(d_z + (size_t)res * n_out + col) : (uint4){0u, 0u, 0u, 0u};
        }
        if (tid >= 256 - kFbTile) {  // this thread's residue of the tile
            const int res = min(res0 + mr, rows - 1);
            hd.rj = nbr_idx[(size_t)res * k + s];
            hd.rb = nbr_bin[(size_t)res * k + s];
            hd.rv = res0 + mr < rows && (mask ? mask[res] != 0 : true);
        }
    };
    int marked[2][3] = {{-1, -1, -1}, {-1, -1, -1}};  // rows this thread marked in either one-hot tile
    // One tile: hand over what `hd` holds into stage b (= tile % 2, a literal at both call sites), fetch
    // the tile after next into `hd`, multiply.
    auto step = [&](int tile, int b, Held &hd) {
        char *zs = zt + b * kFbTile * kFbZStride, *xs = xt + b * Rpad * kFbStride;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = tid + 256 * q, rr = c >> 3, part = c & 7;
            *reinterpret_cast<uint4 *>(zs + rr * kFbZStride + 16 * part) = hd.rz[q];
        }
        if (tid >= 256 - kFbTile) {
            int now[3] = {-1, -1, -1};
            if (hd.rv) {
                if (s == 0) now[2] = R - 1;
                if (hd.rj >= 0 && hd.rj < L) {
                    now[0] = min(max(hd.rb, 0), n_bins - 1);
                    if constexpr (HAS_POS) {
                        const int i = (tile * kFbTile + mr) % L;
                        now[1] = n_bins + (pos_mode == 0 ? min(hd.rj, n_pos - 1) : min(max(hd.rj - i, -half), half) + half);
                    }
                }
            }
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                const int was = marked[b][x];
                if (was >= 0 && was != now[x]) *reinterpret_cast<bf16_t *>(xs + was * kFbStride + mr * 2) = 0;
                if (now[x] >= 0) *reinterpret_cast<bf16_t *>(xs + now[x] * kFbStride + mr * 2) = 0x3F80;  // bf16 1.0
                marked[b][x] = now[x];
            }
        }
        __syncthreads();
        if (tile + 2 < ntiles) fetch(tile + 2, hd);
#pragma unroll
        for (int o = 0; o < kFbMaxOwn; ++o) {
            if (o >= n_own) break;
            const int t = wave + 4 * o, mb = t >> 1, nb = t & 1;
            // The d_z operand comes through the transposing LDS read, which hands lane group g the residues
            // 16 ks + 4 g .. + 3 and 16 ks + 8 + 4 g .. + 3 of column 32 nb + li; the one-hot operand
            // takes the same residues of row 32 mb + li.
            const char *xa = xs + (32 * mb + li) * kFbStride + 8 * g;
            const char *zb = zs + (4 * g + ((lane & 15) >> 2)) * kFbZStride + (32 * nb + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
#pragma unroll
            for (int ks = 0; ks < kFbTile / 16; ++ks) {
                const bf16x4 alo = *reinterpret_cast<const bf16x4 *>(xa + 32 * ks);
                const bf16x4 ahi = *reinterpret_cast<const bf16x4 *>(xa + 32 * ks + 16);
                const bf16x4 zlo = lds_read_tr(zb + 16 * ks * kFbZStride);
                const bf16x4 zhi = lds_read_tr(zb + (16 * ks + 8) * kFbZStride);
                bf16x8 a, bz;
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    a[x] = alo[x];
                    a[4 + x] = ahi[x];
                    bz[x] = zlo[x];
                    bz[4 + x] = zhi[x];
                }
                acc[o] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bz, acc[o], 0, 0, 0);
            }
        }
    };
    Held h0 = {}, h1 = {};
    fetch(0, h0);
    if (ntiles > 1) fetch(1, h1);
    __syncthreads();  // (the one-hot tiles are clear)
    for (int tile = 0; tile < ntiles; tile += 2) {
        step(tile, 0, h0);
        if (tile + 1 < ntiles) step(tile + 1, 1, h1);
    }
    // accumulator register r of a lane: row 8 (r / 4) + 4 g + r % 4 of the row block, column li of the column block
#pragma unroll
    for (int o = 0; o < kFbMaxOwn; ++o) {
        if (o >= n_own) break;
        const int t = wave + 4 * o, mb = t >> 1, nb = t & 1;
        const int col = col0 + 32 * nb + li;
        if (col >= n_out) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 32 * mb + 8 * (r >> 2) + 4 * g + (r & 3);
            if (row < n_bins)
                d_e_bin[((size_t)s * n_bins + row) * n_out + col] = acc[o][r];
            else if (row < n_bins + n_pos)
                d_e_pos[((size_t)s * n_pos + (row - n_bins)) * n_out + col] = acc[o][r];
            else if (row == R - 1 && s == 0 && d_bias)
                d_bias[col] = acc[o][r];
        }
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
    // the one-hot tile holds 32-row blocks of the slot's rows (bins, position codes, one for the bias)
    const int RB = (n_bins + n_pos + 1 + 31) / 32;
    if (RB > fipa::kFbMaxRowBlocks) return FIPA_ERR_UNSUPPORTED;
    const void *al16[] = {d_z, d_e_bin, d_e_pos, d_bias};
    for (const void *ptr : al16)
        if (ptr && !fipa::aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    if ((reinterpret_cast<uintptr_t>(nbr_idx) & 3u) != 0 || (reinterpret_cast<uintptr_t>(nbr_bin) & 3u) != 0) return FIPA_ERR_ALIGNMENT;
    const int lds = 2 * fipa::kFbTile * fipa::kFbZStride + 2 * 32 * RB * fipa::kFbStride;
    const dim3 grid((unsigned)k, (unsigned)((n_out + 63) / 64));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int rows = B * L;
    hipError_t e;
    if (n_pos > 0) {
        static fipa::LdsLimit lim;
        e = fipa::raise_lds_limit(lim, (const void *)fipa::fipa_factor_backward_kernel<true>, lds);
        if (e != hipSuccess) return FIPA_ERR_LAUNCH;
        hipLaunchKernelGGL(fipa::fipa_factor_backward_kernel<true>, grid, dim3(256), lds, stream, nbr_idx, nbr_bin,
                           (const fipa::bf16_t *)d_z, mask, d_e_bin, d_e_pos, d_bias, rows, L, k, n_bins, n_pos, pos_mode, n_out, RB);
    } else {
        static fipa::LdsLimit lim;
        e = fipa::raise_lds_limit(lim, (const void *)fipa::fipa_factor_backward_kernel<false>, lds);
        if (e != hipSuccess) return FIPA_ERR_LAUNCH;
        hipLaunchKernelGGL(fipa::fipa_factor_backward_kernel<false>, grid, dim3(256), lds, stream, nbr_idx, nbr_bin,
                           (const fipa::bf16_t *)d_z, mask, d_e_bin, (float *)nullptr, d_bias, rows, L, k, n_bins, 0, pos_mode, n_out, RB);
    }
    return hipGetLastError() == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
}
