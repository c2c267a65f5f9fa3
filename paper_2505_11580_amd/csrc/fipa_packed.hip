// Packed batches: chains of different lengths stored back to back (the variable-length inputs of
// the experiments in Section 3, without padding).  fipa_forward_packed / fipa_backward_packed run
// them either as ONE set of launches -- the kernels of the padded path, which then address the
// caller's tensors through the row offsets (FwdArgs::cu) and skip the query tiles and key blocks
// past the end of each chain -- or chain by chain as B = 1 problems on offset pointers, whichever
// the lengths make cheaper (see packed_plan).
#include "fipa_internal.h"

using namespace fipa;

namespace {

constexpr int kChunk = 256;
struct IntChunk {
    int v[kChunk];
};

// The row offsets come as a host pointer; they travel to the device as kernel arguments, 256 at a
// time (no host-to-device copy, which would have to stage pageable memory: the library never
// synchronises and its calls can be captured into a graph).
__global__ __launch_bounds__(kChunk) void fipa_write_ints_kernel(IntChunk c, int n, int *__restrict__ dst)
{
    if ((int)threadIdx.x < n) dst[threadIdx.x] = c.v[threadIdx.x];
}

hipError_t upload_ints(const int32_t *src, int n, int *dst, hipStream_t stream)
{
    for (int i0 = 0; i0 < n; i0 += kChunk) {
        IntChunk c;
        const int m = n - i0 < kChunk ? n - i0 : kChunk;
        for (int i = 0; i < kChunk; ++i) c.v[i] = i < m ? src[i0 + i] : 0;
        hipLaunchKernelGGL(fipa_write_ints_kernel, dim3(1), dim3(kChunk), 0, stream, c, m, dst + i0);
    }
    return hipGetLastError();
}

// dst[x] = sum over the n_rows rows of src (row stride `stride`), in row order; n_rows may be 0.
__global__ __launch_bounds__(256) void fipa_sum_rows_kernel(const float *__restrict__ src, int n_rows, int stride,
                                                            int n, float *__restrict__ dst)
{
    const int x = blockIdx.x * 256 + threadIdx.x;
    if (x >= n) return;
    float s = 0.f;
    for (int j = 0; j < n_rows; ++j) s += src[(size_t)j * stride + x];
    dst[x] = s;
}

struct PackedPlan {
    bool one_launch;
    int total;       // rows of the packed tensors, cu_seqlens[B]
    int n_nonempty;  // chains with at least one residue
    fipa_desc d;     // what the kernels run with: one launch: B chains, L = longest chain; else B = 1, L = longest chain
    size_t fwd_bytes, bwd_bytes;
    size_t cu_fwd, cu_bwd;  // one launch: offset of the device copy of the row offsets
    size_t part_bwd;        // chain by chain: offset of the per-chain d_gamma | d_w_b partial sums
    int part_stride;        // floats per chain there
};

// One set of launches pays when the chains are many or short (a chain of 300 residues fills 36 of
// the chip's 256 compute units by itself), and costs a workspace padded to the longest chain:
// it is chosen when at most half of that workspace would be padding.  Otherwise -- one chain much
// longer than the rest -- the chains run one after the other and share a workspace sized for the
// longest (each long chain fills the chip by itself).  FIPA_FLAG_PACKED_PER_CHAIN forces the
// latter (smallest workspace); the fp32 mode always uses it.
int packed_plan(const fipa_desc *desc, const int32_t *cu, bool backward, PackedPlan &pl)
{
    int rc = check_desc(desc, backward);
    if (rc != FIPA_OK) return rc;
    if (backward && desc->dtype != FIPA_DTYPE_BF16) return FIPA_ERR_UNSUPPORTED;
    if (!cu || cu[0] != 0) return FIPA_ERR_INVALID_ARG;
    long long padded_sum = 0;
    int lmax = 0;
    pl.n_nonempty = 0;
    for (int b = 0; b < desc->B; ++b) {
        const long long len = (long long)cu[b + 1] - cu[b];
        if (len < 0 || len > desc->L) return FIPA_ERR_INVALID_ARG;
        if (len > lmax) lmax = (int)len;
        if (len > 0) pl.n_nonempty += 1;
        padded_sum += (len + 127) / 128 * 128;
    }
    pl.total = cu[desc->B];
    pl.d = *desc;
    pl.d.L = lmax > 0 ? lmax : 1;
    pl.d.flags &= ~(uint32_t)FIPA_FLAG_PACKED_PER_CHAIN;
    const long long padded_all = (long long)desc->B * (((long long)pl.d.L + 127) / 128 * 128);
    pl.one_launch = desc->dtype == FIPA_DTYPE_BF16 && !(desc->flags & FIPA_FLAG_PACKED_PER_CHAIN) &&
                    padded_all <= 2 * padded_sum && check_desc(&pl.d, backward) == FIPA_OK;
    if (!pl.one_launch) pl.d.B = 1;
    rc = fipa_workspace_bytes(&pl.d, &pl.fwd_bytes, backward ? &pl.bwd_bytes : nullptr);
    if (rc != FIPA_OK) return rc;
    if (!backward) pl.bwd_bytes = 0;
    pl.cu_fwd = pl.cu_bwd = pl.part_bwd = 0;
    pl.part_stride = (desc->H + desc->H * desc->cz + 3) / 4 * 4;
    if (pl.one_launch) {
        const size_t cu_bytes = align_up((size_t)(desc->B + 1) * sizeof(int), 256);
        pl.cu_fwd = align_up(pl.fwd_bytes, 256);
        pl.fwd_bytes = pl.cu_fwd + cu_bytes;
        if (backward) {
            pl.cu_bwd = align_up(pl.bwd_bytes, 256);
            pl.bwd_bytes = pl.cu_bwd + cu_bytes;
        }
    } else if (backward) {
        pl.part_bwd = align_up(pl.bwd_bytes, 256);
        pl.bwd_bytes = pl.part_bwd + align_up((size_t)(pl.n_nonempty > 0 ? pl.n_nonempty : 1) * pl.part_stride * sizeof(float), 256);
    }
    return FIPA_OK;
}

const void *at_row(const void *base, size_t row, size_t row_bytes)
{
    return static_cast<const char *>(base) + row * row_bytes;
}
void *at_row(void *base, size_t row, size_t row_bytes) { return static_cast<char *>(base) + row * row_bytes; }

}  // namespace

extern "C" {

int fipa_packed_workspace_bytes(const fipa_desc *desc, const int32_t *cu_seqlens, size_t *forward_bytes,
                                size_t *backward_bytes)
{
    if (forward_bytes) *forward_bytes = 0;
    if (backward_bytes) *backward_bytes = 0;
    PackedPlan pl;
    int rc = packed_plan(desc, cu_seqlens, false, pl);
    if (rc != FIPA_OK) return rc;
    if (forward_bytes) *forward_bytes = pl.fwd_bytes;
    if (backward_bytes && packed_plan(desc, cu_seqlens, true, pl) == FIPA_OK) *backward_bytes = pl.bwd_bytes;
    return FIPA_OK;
}

int fipa_forward_packed(const fipa_desc *desc, const int32_t *cu_seqlens, const void *q, const void *k, const void *v,
                        const void *q_pts, const void *k_pts, const void *v_pts, const float *rot,
                        const float *trans, const void *z1, const void *z2, const float *w_b,
                        const float *gamma, const uint8_t *mask, float *o, float *o_pts, float *o_pair,
                        float *lse, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    PackedPlan pl;
    const bool keep = desc && (desc->flags & FIPA_FLAG_KEEP_FORWARD);
    const int rc = packed_plan(desc, cu_seqlens, keep, pl);
    if (rc != FIPA_OK) return rc;
    if (keep) {  // one workspace for the whole batch, of the backward's size and layout
        if (!pl.one_launch && pl.total > 0) return FIPA_ERR_UNSUPPORTED;
        pl.fwd_bytes = pl.bwd_bytes;
        pl.cu_fwd = pl.cu_bwd;
    }
    const void *req[] = {q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, o, o_pts, o_pair, workspace};
    for (const void *ptr : req)
        if (!ptr) return FIPA_ERR_INVALID_ARG;
    const void *al[] = {q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, o, o_pts, o_pair, lse, workspace};
    for (const void *ptr : al)
        if (!aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    if (workspace_bytes < pl.fwd_bytes) return FIPA_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (pl.total == 0) return FIPA_OK;  // no residue, no output row

    if (pl.one_launch) {
        int *cu_dev = reinterpret_cast<int *>(static_cast<char *>(workspace) + pl.cu_fwd);
        if (upload_ints(cu_seqlens, desc->B + 1, cu_dev, stream) != hipSuccess) return FIPA_ERR_LAUNCH;
        FwdArgs a{q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask, o, o_pts, o_pair, lse};
        a.cu = cu_dev;
        a.total_rows = pl.total;
        const hipError_t e = keep ? bf16_backward_begin(pl.d, a, workspace, stream) : bf16_forward(pl.d, a, workspace, stream);
        return e == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
    }

    // chain by chain: bytes per residue of each tensor
    const size_t es = desc->dtype == FIPA_DTYPE_F32 ? 4 : 2;
    const size_t H = desc->H, n_s = H * desc->c, n_q = H * desc->Pq * 3, n_v = H * desc->Pv * 3,
                 n_z = (size_t)desc->r * desc->cz;
    fipa_desc one = pl.d;
    for (int b = 0; b < desc->B; ++b) {
        const size_t r0 = (size_t)cu_seqlens[b];
        one.L = cu_seqlens[b + 1] - cu_seqlens[b];
        if (one.L == 0) continue;
        const FwdArgs a{at_row(q, r0, n_s * es), at_row(k, r0, n_s * es), at_row(v, r0, n_s * es),
                        at_row(q_pts, r0, n_q * es), at_row(k_pts, r0, n_q * es), at_row(v_pts, r0, n_v * es),
                        rot + r0 * 9, trans + r0 * 3, at_row(z1, r0, n_z * es), at_row(z2, r0, n_z * es), w_b, gamma,
                        mask ? mask + r0 : nullptr,
                        o + r0 * n_s, o_pts + r0 * n_v, o_pair + r0 * H * desc->cz, lse ? lse + r0 * H : nullptr};
        if (enqueue_forward(one, a, workspace, stream) != hipSuccess) return FIPA_ERR_LAUNCH;
    }
    return FIPA_OK;
}

int fipa_backward_packed(const fipa_desc *desc, const int32_t *cu_seqlens, const void *q, const void *k, const void *v,
                         const void *q_pts, const void *k_pts, const void *v_pts, const float *rot,
                         const float *trans, const void *z1, const void *z2, const float *w_b,
                         const float *gamma, const uint8_t *mask, const float *d_o, const float *d_o_pts,
                         const float *d_o_pair, void *d_q, void *d_k, void *d_v, void *d_q_pts, void *d_k_pts,
                         void *d_v_pts, void *d_z1, void *d_z2, float *d_gamma, float *d_w_b, float *d_rot,
                         float *d_trans, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    PackedPlan pl;
    const int rc = packed_plan(desc, cu_seqlens, true, pl);
    if (rc != FIPA_OK) return rc;
    const bool keep = (desc->flags & FIPA_FLAG_KEEP_FORWARD) != 0;
    if (keep && !pl.one_launch && pl.total > 0) return FIPA_ERR_UNSUPPORTED;
    const void *req[] = {q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma,
                         d_o, d_o_pts, d_o_pair, d_q, d_k, d_v, d_q_pts, d_k_pts, d_v_pts, d_z1, d_z2,
                         d_gamma, workspace};
    for (const void *ptr : req) {
        if (!ptr) return FIPA_ERR_INVALID_ARG;
        if (!aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    }
    if (d_w_b && !aligned16(d_w_b)) return FIPA_ERR_ALIGNMENT;
    if ((d_rot == nullptr) != (d_trans == nullptr)) return FIPA_ERR_INVALID_ARG;
    if (d_rot && (!aligned16(d_rot) || !aligned16(d_trans))) return FIPA_ERR_ALIGNMENT;
    if (workspace_bytes < pl.bwd_bytes) return FIPA_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int H = desc->H, n_wb = H * desc->cz;

    BwdArgs a;
    a.f = FwdArgs{q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask, nullptr, nullptr, nullptr, nullptr};
    a.d_o = d_o; a.d_o_pts = d_o_pts; a.d_o_pair = d_o_pair;
    a.d_q = d_q; a.d_k = d_k; a.d_v = d_v; a.d_q_pts = d_q_pts; a.d_k_pts = d_k_pts;
    a.d_v_pts = d_v_pts; a.d_z1 = d_z1; a.d_z2 = d_z2; a.d_gamma = d_gamma; a.d_w_b = d_w_b;
    a.d_rot = d_rot; a.d_trans = d_trans;

    if (pl.one_launch && pl.total > 0) {
        int *cu_dev = reinterpret_cast<int *>(static_cast<char *>(workspace) + pl.cu_bwd);
        if (upload_ints(cu_seqlens, desc->B + 1, cu_dev, stream) != hipSuccess) return FIPA_ERR_LAUNCH;
        a.f.cu = cu_dev;
        a.f.total_rows = pl.total;
        const hipError_t e = keep ? bf16_backward_finish(pl.d, a, workspace, stream) : bf16_backward(pl.d, a, workspace, stream);
        return e == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
    }

    // chain by chain; gamma and w_b are shared by the chains, so each chain leaves its own sums in
    // the workspace and a last kernel adds them in chain order
    const size_t Hs = H, n_s = Hs * desc->c, n_q = Hs * desc->Pq * 3, n_v = Hs * desc->Pv * 3, n_z = (size_t)desc->r * desc->cz;
    float *part = reinterpret_cast<float *>(static_cast<char *>(workspace) + pl.part_bwd);
    fipa_desc one = pl.d;
    int j = 0;
    for (int b = 0; b < desc->B && pl.total > 0; ++b) {
        const size_t r0 = (size_t)cu_seqlens[b];
        one.L = cu_seqlens[b + 1] - cu_seqlens[b];
        if (one.L == 0) continue;
        BwdArgs c = a;
        c.f = FwdArgs{at_row(q, r0, n_s * 2), at_row(k, r0, n_s * 2), at_row(v, r0, n_s * 2),
                      at_row(q_pts, r0, n_q * 2), at_row(k_pts, r0, n_q * 2), at_row(v_pts, r0, n_v * 2),
                      rot + r0 * 9, trans + r0 * 3, at_row(z1, r0, n_z * 2), at_row(z2, r0, n_z * 2), w_b, gamma,
                      mask ? mask + r0 : nullptr, nullptr, nullptr, nullptr, nullptr};
        c.d_o = d_o + r0 * n_s; c.d_o_pts = d_o_pts + r0 * n_v; c.d_o_pair = d_o_pair + r0 * Hs * desc->cz;
        c.d_q = at_row(d_q, r0, n_s * 2); c.d_k = at_row(d_k, r0, n_s * 2); c.d_v = at_row(d_v, r0, n_s * 2);
        c.d_q_pts = at_row(d_q_pts, r0, n_q * 2); c.d_k_pts = at_row(d_k_pts, r0, n_q * 2);
        c.d_v_pts = at_row(d_v_pts, r0, n_v * 2);
        c.d_z1 = at_row(d_z1, r0, n_z * 2); c.d_z2 = at_row(d_z2, r0, n_z * 2);
        c.d_gamma = part + (size_t)j * pl.part_stride;
        c.d_w_b = d_w_b ? c.d_gamma + H : nullptr;
        c.d_rot = d_rot ? d_rot + r0 * 9 : nullptr;
        c.d_trans = d_trans ? d_trans + r0 * 3 : nullptr;
        if (bf16_backward(one, c, workspace, stream) != hipSuccess) return FIPA_ERR_LAUNCH;
        j += 1;
    }
    hipLaunchKernelGGL(fipa_sum_rows_kernel, dim3((H + 255) / 256), dim3(256), 0, stream, part, j, pl.part_stride, H, d_gamma);
    if (d_w_b)
        hipLaunchKernelGGL(fipa_sum_rows_kernel, dim3((n_wb + 255) / 256), dim3(256), 0, stream, part + H, j, pl.part_stride,
                           n_wb, d_w_b);
    return hipGetLastError() == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
}

}  // extern "C"
