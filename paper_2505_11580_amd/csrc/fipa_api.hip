// C ABI of libfipa: argument validation (host only, before anything is enqueued) and dispatch
// to the fp32 direct path or the bf16 MFMA path.
#include "fipa_internal.h"

using namespace fipa;

namespace fipa {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_desc(const fipa_desc *d, bool backward)
{
    if (!d) return FIPA_ERR_INVALID_ARG;
    if (d->B <= 0 || d->L <= 0 || d->H <= 0 || d->c <= 0 || d->Pq <= 0 || d->Pv <= 0 || d->cz <= 0 ||
        d->r <= 0)
        return FIPA_ERR_INVALID_ARG;
    if (d->dtype != FIPA_DTYPE_F32 && d->dtype != FIPA_DTYPE_BF16) return FIPA_ERR_INVALID_ARG;
    if ((d->flags & ~(uint32_t)(FIPA_FLAG_WAVE_SPECIALISED | FIPA_FLAG_PACKED_PER_CHAIN | FIPA_FLAG_KEEP_FORWARD)) != 0) return FIPA_ERR_INVALID_ARG;
    if (!(d->w_L == d->w_L) || !(d->w_C == d->w_C) || !(d->qk_scale == d->qk_scale))
        return FIPA_ERR_INVALID_ARG;
    const long long DZ = (long long)d->r * d->cz;
    if ((long long)d->B * d->H * ((long long)d->L + 128) >= (1LL << 31)) return FIPA_ERR_UNSUPPORTED;
    if (d->dtype == FIPA_DTYPE_F32) {
        if (backward) return FIPA_ERR_UNSUPPORTED;
        if (DZ > 512 || d->c + 3LL * d->Pv + DZ > 576) return FIPA_ERR_UNSUPPORTED;
    } else {
        const int PH = (d->Pv + 1) / 2;  // value points per lane half; see v_pt_col()
        if (d->c % 8 != 0 || d->cz % 8 != 0 || d->c + 12 * d->Pq > 64 ||
            d->c + 8 * ((6 * PH + 3) / 4) > 64)
            return FIPA_ERR_UNSUPPORTED;
        if (DZ != 32 && DZ != 64 && DZ != 128 && DZ != 256 && DZ != 512 && DZ != 1024) return FIPA_ERR_UNSUPPORTED;
        if (DZ > 512 && backward) return FIPA_ERR_UNSUPPORTED;
    }
    return FIPA_OK;
}

int check_forward_args(const fipa_desc *desc, const FwdArgs &a)
{
    const int rc = check_desc(desc, false);
    if (rc != FIPA_OK) return rc;
    const void *req[] = {a.q, a.k, a.v, a.q_pts, a.k_pts, a.v_pts, a.rot, a.trans, a.z1, a.z2, a.w_b, a.gamma,
                         a.o, a.o_pts, a.o_pair};
    for (const void *ptr : req)
        if (!ptr) return FIPA_ERR_INVALID_ARG;
    for (const void *ptr : req)
        if (!aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    if (!aligned16(a.lse)) return FIPA_ERR_ALIGNMENT;
    return FIPA_OK;
}

hipError_t enqueue_forward(const fipa_desc &desc, const FwdArgs &a, void *workspace, hipStream_t stream)
{
    return desc.dtype == FIPA_DTYPE_F32 ? f32_forward(desc, a, workspace, stream) : bf16_forward(desc, a, workspace, stream);
}

}  // namespace fipa

extern "C" {

int fipa_version(void) { return 100; }

const char *fipa_status_string(int status)
{
    switch (status) {
        case FIPA_OK: return "ok";
        case FIPA_ERR_INVALID_ARG: return "invalid argument (null pointer, non-positive size or bad dtype)";
        case FIPA_ERR_UNSUPPORTED: return "shape or mode not supported by the kernels";
        case FIPA_ERR_WORKSPACE: return "workspace too small";
        case FIPA_ERR_ALIGNMENT: return "tensor pointer not 16-byte aligned";
        case FIPA_ERR_LAUNCH: return "HIP error while enqueueing a kernel";
        default: return "unknown status";
    }
}

int fipa_workspace_bytes(const fipa_desc *desc, size_t *forward_bytes, size_t *backward_bytes)
{
    if (forward_bytes) *forward_bytes = 0;
    if (backward_bytes) *backward_bytes = 0;
    const int rc = check_desc(desc, false);
    if (rc != FIPA_OK) return rc;
    if (forward_bytes)
        *forward_bytes = desc->dtype == FIPA_DTYPE_F32 ? f32_forward_workspace(*desc)
                                                       : bf16_forward_workspace(*desc);
    if (backward_bytes)
        *backward_bytes = check_desc(desc, true) == FIPA_OK ? bf16_backward_workspace(*desc) : 0;
    return FIPA_OK;
}

int fipa_forward(const fipa_desc *desc, const void *q, const void *k, const void *v,
                 const void *q_pts, const void *k_pts, const void *v_pts, const float *rot,
                 const float *trans, const void *z1, const void *z2, const float *w_b,
                 const float *gamma, const uint8_t *mask, float *o, float *o_pts, float *o_pair,
                 float *lse, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const FwdArgs a{q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask, o, o_pts, o_pair, lse};
    const int rc = check_forward_args(desc, a);
    if (rc != FIPA_OK) return rc;
    if (!workspace) return FIPA_ERR_INVALID_ARG;
    if (!aligned16(workspace)) return FIPA_ERR_ALIGNMENT;
    size_t need = 0;
    if (desc->flags & FIPA_FLAG_KEEP_FORWARD) {
        // the forward part of the backward, which leaves the lifted operands, O^ and the
        // log-sum-exp in a workspace of the backward's size, gives the same outputs
        if (check_desc(desc, true) != FIPA_OK || desc->dtype != FIPA_DTYPE_BF16) return FIPA_ERR_UNSUPPORTED;
        fipa_workspace_bytes(desc, nullptr, &need);
        if (workspace_bytes < need) return FIPA_ERR_WORKSPACE;
        return bf16_backward_begin(*desc, a, workspace, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? FIPA_OK
                                                                                                           : FIPA_ERR_LAUNCH;
    }
    fipa_workspace_bytes(desc, &need, nullptr);
    if (workspace_bytes < need) return FIPA_ERR_WORKSPACE;
    return enqueue_forward(*desc, a, workspace, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? FIPA_OK
                                                                                                  : FIPA_ERR_LAUNCH;
}

int fipa_backward(const fipa_desc *desc, const void *q, const void *k, const void *v,
                  const void *q_pts, const void *k_pts, const void *v_pts, const float *rot,
                  const float *trans, const void *z1, const void *z2, const float *w_b,
                  const float *gamma, const uint8_t *mask, const float *o, const float *o_pts,
                  const float *o_pair, const float *lse, const float *d_o, const float *d_o_pts,
                  const float *d_o_pair, void *d_q, void *d_k, void *d_v, void *d_q_pts,
                  void *d_k_pts, void *d_v_pts, void *d_z1, void *d_z2, float *d_gamma, float *d_w_b,
                  float *d_rot, float *d_trans, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    int rc = check_desc(desc, true);
    if (rc != FIPA_OK) return rc;
    const void *req[] = {q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma,
                         d_o, d_o_pts, d_o_pair, d_q, d_k, d_v, d_q_pts, d_k_pts, d_v_pts, d_z1, d_z2,
                         d_gamma, workspace};
    for (const void *ptr : req) {
        if (!ptr) return FIPA_ERR_INVALID_ARG;
        if (!aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    }
    // (the saved forward results are not read: what the gradient needs is recomputed from the
    // inputs, or kept in the workspace by the forward call)
    const void *saved[] = {o, o_pts, o_pair, lse};
    for (const void *ptr : saved)
        if (ptr && !aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    if (d_w_b && !aligned16(d_w_b)) return FIPA_ERR_ALIGNMENT;
    if ((d_rot == nullptr) != (d_trans == nullptr)) return FIPA_ERR_INVALID_ARG;
    if (d_rot && (!aligned16(d_rot) || !aligned16(d_trans))) return FIPA_ERR_ALIGNMENT;
    size_t need = 0;
    fipa_workspace_bytes(desc, nullptr, &need);
    if (workspace_bytes < need) return FIPA_ERR_WORKSPACE;
    BwdArgs a;
    a.f = FwdArgs{q, k, v, q_pts, k_pts, v_pts, rot, trans, z1, z2, w_b, gamma, mask,
                  const_cast<float *>(o), const_cast<float *>(o_pts), const_cast<float *>(o_pair),
                  const_cast<float *>(lse)};
    a.d_o = d_o; a.d_o_pts = d_o_pts; a.d_o_pair = d_o_pair;
    a.d_q = d_q; a.d_k = d_k; a.d_v = d_v; a.d_q_pts = d_q_pts; a.d_k_pts = d_k_pts;
    a.d_v_pts = d_v_pts; a.d_z1 = d_z1; a.d_z2 = d_z2; a.d_gamma = d_gamma; a.d_w_b = d_w_b;
    a.d_rot = d_rot; a.d_trans = d_trans;
    // (with FIPA_FLAG_KEEP_FORWARD the workspace still holds what the forward call left there)
    const hipError_t e = (desc->flags & FIPA_FLAG_KEEP_FORWARD)
                             ? bf16_backward_finish(*desc, a, workspace, static_cast<hipStream_t>(hip_stream))
                             : bf16_backward(*desc, a, workspace, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
}

int fipa_module_workspace_bytes(const fipa_desc *desc, int32_t d_s, size_t *bytes)
{
    if (bytes) *bytes = 0;
    const int rc = check_desc(desc, false);
    if (rc != FIPA_OK) return rc;
    if (desc->dtype != FIPA_DTYPE_BF16 || !module_shape_supported(*desc, d_s)) return FIPA_ERR_UNSUPPORTED;
    if (bytes) *bytes = module_forward_workspace(*desc, d_s);
    return FIPA_OK;
}

int fipa_module_forward(const fipa_desc *desc, int32_t d_s, const void *s, const void *w_in, const float *b_in,
                        const float *rot, const float *trans, const void *z1, const void *z2, const float *w_b,
                        const float *gamma, const uint8_t *mask, const void *w_out, const float *b_out,
                        float *s_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    size_t need = 0;
    const bool keep = desc && (desc->flags & FIPA_FLAG_KEEP_FORWARD);  // runs in the backward's workspace
    const int rc = keep ? fipa_module_backward_workspace_bytes(desc, d_s, &need) : fipa_module_workspace_bytes(desc, d_s, &need);
    if (rc != FIPA_OK) return rc;
    const void *req[] = {s, w_in, rot, trans, z1, z2, w_b, gamma, w_out, s_out, workspace};
    for (const void *ptr : req) {
        if (!ptr) return FIPA_ERR_INVALID_ARG;
        if (!aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    }
    if (workspace_bytes < need) return FIPA_ERR_WORKSPACE;
    const ModuleArgs a{s, w_in, b_in, rot, trans, z1, z2, w_b, gamma, mask, w_out, b_out, s_out};
    const hipError_t e = module_forward(*desc, d_s, a, workspace, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
}

int fipa_module_backward_workspace_bytes(const fipa_desc *desc, int32_t d_s, size_t *bytes)
{
    if (bytes) *bytes = 0;
    const int rc = check_desc(desc, true);
    if (rc != FIPA_OK) return rc;
    if (!module_backward_shape_supported(*desc, d_s)) return FIPA_ERR_UNSUPPORTED;
    if (bytes) *bytes = module_backward_workspace(*desc, d_s);
    return FIPA_OK;
}

int fipa_module_backward(const fipa_desc *desc, int32_t d_s, const void *s, const void *w_in, const float *b_in,
                         const float *rot, const float *trans, const void *z1, const void *z2, const float *w_b,
                         const float *gamma, const uint8_t *mask, const void *w_out, const float *b_out,
                         const float *d_s_out, float *d_s_in, float *d_w_in, float *d_b_in, float *d_w_out,
                         float *d_b_out, void *d_z1, void *d_z2, float *d_gamma, float *d_w_b, float *d_rot,
                         float *d_trans, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    size_t need = 0;
    const int rc = fipa_module_backward_workspace_bytes(desc, d_s, &need);
    if (rc != FIPA_OK) return rc;
    const void *req[] = {s, w_in, rot, trans, z1, z2, w_b, gamma, w_out, d_s_out, d_s_in, d_w_in, d_w_out, d_z1, d_z2,
                         d_gamma, workspace};
    for (const void *ptr : req) {
        if (!ptr) return FIPA_ERR_INVALID_ARG;
        if (!aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    }
    if ((d_rot == nullptr) != (d_trans == nullptr)) return FIPA_ERR_INVALID_ARG;
    const void *opt[] = {b_in, b_out, d_b_in, d_b_out, d_w_b, d_rot, d_trans};
    for (const void *ptr : opt)
        if (ptr && !aligned16(ptr)) return FIPA_ERR_ALIGNMENT;
    if (workspace_bytes < need) return FIPA_ERR_WORKSPACE;
    const ModuleArgs a{s, w_in, b_in, rot, trans, z1, z2, w_b, gamma, mask, w_out, b_out, nullptr};
    const ModuleBwdArgs g{d_s_out, d_s_in, d_w_in, d_b_in, d_w_out, d_b_out, d_z1, d_z2, d_gamma, d_w_b, d_rot, d_trans};
    const hipError_t e = module_backward(*desc, d_s, a, g, workspace, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? FIPA_OK : FIPA_ERR_LAUNCH;
}

}  // extern "C"
