/*
 * fipa.h -- C ABI of the factorized Invariant Point Attention library for MI355X (gfx950).
 *
 * The library computes the attention core of FlashIPA (Algorithm 1, steps 2-9): frame
 * application and lifting of queries / keys / values, one softmax(Q^ K^T) V^ over the
 * concatenated scalar, point and pair-factor features, the split, the inverse frame on the
 * point output (Eq. 4) and the z1 contraction of the pair output -- without ever forming the
 * L x L x c_z pair tensor or the L x L attention matrix.  The result equals standard IPA
 * (Eqs. 2-4) evaluated on z_ij = z1_i^T z2_j (Section 2.4).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, contiguous, row-major and
 *     16-byte aligned.  `desc` is a HOST pointer.
 *   - The library allocates nothing, frees nothing and never synchronises: all work is
 *     enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - `workspace` is caller-owned device scratch of at least fipa_workspace_bytes(); its
 *     contents are undefined afterwards.  Forward and backward do not share state through it
 *     (unless FIPA_FLAG_KEEP_FORWARD asks for exactly that).
 *   - Outputs are fully overwritten.  Query rows whose mask byte is 0 receive zeros (and
 *     contribute nothing to any gradient); keys whose mask byte is 0 receive exactly zero
 *     weight, whatever finite values their slots hold.
 *   - Return value: FIPA_OK or a negative FIPA_ERR_* code.  Argument errors are detected on
 *     the host before anything is enqueued.
 *   - Calls on different streams with different workspaces may run concurrently.
 */
#ifndef FIPA_H
#define FIPA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FIPA_OK 0
#define FIPA_ERR_INVALID_ARG (-1) /* null pointer, non-positive size, bad dtype               */
#define FIPA_ERR_UNSUPPORTED (-2) /* shape outside what the kernels are built for (see below) */
#define FIPA_ERR_WORKSPACE (-3)   /* workspace_bytes smaller than fipa_workspace_bytes()      */
#define FIPA_ERR_ALIGNMENT (-4)   /* a tensor pointer is not 16-byte aligned                  */
#define FIPA_ERR_LAUNCH (-5)      /* HIP reported an error when a kernel was enqueued         */

#define FIPA_DTYPE_F32 0  /* q,k,v,points,z1,z2 float32; direct fp32 evaluation (no MFMA)      */
#define FIPA_DTYPE_BF16 1 /* q,k,v,points,z1,z2 bfloat16; bf16 MFMA with fp32 accumulation      */

/*
 * Problem description (symbols of Section 2.2 / Algorithm 1):
 *   B batch, L residues (padded length), H heads, c scalar q/k/v width, Pq = N_query,
 *   Pv = N_value, cz = d_z pair channels, r = factor rank.
 *   w_L, w_C: the constants of Eq. 3 (AlphaFold2 uses sqrt(1/3) and sqrt(2/(9*Pq))).
 *   qk_scale: the 1/sqrt(c) of Eq. 3.
 * Shapes supported:  FIPA_DTYPE_F32: c + 3*Pv + r*cz <= 576 and r*cz <= 512.
 *                    FIPA_DTYPE_BF16: c % 8 == 0, cz % 8 == 0, c + 12*Pq <= 64,
 *                    c + 8*ceil(3*ceil(Pv/2)/2) <= 64, r*cz in {32, 64, 128, 256, 512, 1024}
 *                    (1024, e.g. rank 8 at cz = 128 -- the larger lifted widths that Section 4.1 names as
 *                    the way to higher rank: forward only, a plain kernel that is not tuned).
 */
typedef struct fipa_desc {
    int32_t B, L, H, c, Pq, Pv, cz, r;
    int32_t dtype; /* FIPA_DTYPE_* : type of q,k,v,q_pts,k_pts,v_pts,z1,z2 and of their gradients */
    float w_L, w_C;
    float qk_scale;
    uint32_t flags; /* 0, or FIPA_FLAG_* bits; other bits are reserved and must be 0 */
} fipa_desc;

/*
 * fipa_forward, bf16, c = 16, Pv = 8, cz in {32, 64, 128, 256}, r*cz <= 256: run the fused attention
 * (Algorithm 1 step 7) with the variant of the kernel that gives every SIMD two waves -- one forming
 * S^T and the softmax, one accumulating P V -- instead of one wave doing both.  Same results within
 * the stated tolerance; slower than the default on every shape measured so far, kept as a measured
 * alternative.  Ignored where it does not apply.
 */
#define FIPA_FLAG_WAVE_SPECIALISED 1u

/*
 * Training steps (a forward call followed by the backward call on the same inputs), bf16, the shapes
 * the backward accepts: fipa_forward / fipa_forward_packed with this flag take a workspace of the
 * BACKWARD's size and leave in it what the gradient needs from the forward -- the lifted operands of
 * Algorithm 1 steps 2-6, the lifted output O^ and the log-sum-exp -- and
 * fipa_backward / fipa_backward_packed with this flag, the same descriptor, the same input tensors
 * and that workspace skip the recomputation (about a sixth of the backward's time at the headline
 * shape; the forward call is slower -- a separate epilogue pass, per-head query factors and O^ in memory,
 * no key-range split -- so the pair gains about a tenth, less at short lengths).
 * Outputs and gradients are the same as without the flag.  The caller keeps the workspace untouched
 * between the two calls; a backward call with the flag on a workspace that the matching forward call
 * did not fill returns gradients of garbage without an error.  Not for fipa_forward_static
 * (FIPA_ERR_UNSUPPORTED); packed batches only where they run as one launch (FIPA_ERR_UNSUPPORTED
 * with FIPA_FLAG_PACKED_PER_CHAIN or when the plan falls back to chain-by-chain).
 * fipa_module_forward / fipa_module_backward take it the same way: the forward call needs
 * fipa_module_backward_workspace_bytes and also leaves the projected inputs (Eq. 1) and the core's
 * outputs; the backward call then starts at Eq. 5's gradient.
 */
#define FIPA_FLAG_KEEP_FORWARD 4u

/* Library version, major*10000 + minor*100 + patch. */
int fipa_version(void);

/* Static, human-readable text for a return code. */
const char *fipa_status_string(int status);

/*
 * Scratch sizes in bytes for fipa_forward / fipa_backward with this description.  Both are
 * affine in L (the linear-memory property of Section 2.3).  Either output pointer may be
 * NULL.  Host-only, touches no device.
 */
int fipa_workspace_bytes(const fipa_desc *desc, size_t *forward_bytes, size_t *backward_bytes);

/*
 * Forward (Algorithm 1, steps 2-9, with Eq. 4's inverse frame).
 *   q, k, v          [B, L, H, c]        scalar queries / keys / values (desc->dtype)
 *   q_pts, k_pts     [B, L, H, Pq, 3]    query / key points, local frame (desc->dtype)
 *   v_pts            [B, L, H, Pv, 3]    value points, local frame (desc->dtype)
 *   rot, trans       [B, L, 3, 3], [B, L, 3]  frames T_i = (R_i, t_i), always float32:
 *                                        global = R_i * local + t_i
 *   z1, z2           [B, L, r, cz]       pair factors, z_ij[d] = sum_rho z1_i[rho,d] z2_j[rho,d]
 *   w_b              [H, cz] float32     weights of the pair-bias Linear of Eq. 2 (its additive
 *                                        constant cancels in the softmax and is not an input)
 *   gamma            [H] float32         per-head point weight gamma^h of Eq. 3, used as given
 *   mask             [B, L] bytes, 1 = valid residue; NULL = all valid
 *   o                [B, L, H, c]      float32   sum_j a_ij v_j
 *   o_pts            [B, L, H, Pv, 3]  float32   T_i^{-1} o sum_j a_ij (T_j o v_j), local frame of i
 *   o_pair           [B, L, H, cz]     float32   sum_j a_ij z_ij
 *   lse              [B, H, L] float32, or NULL: natural log-sum-exp over valid keys of the
 *                    softmax argument of Eq. 3 (0 for masked query rows).
 */
int fipa_forward(const fipa_desc *desc,
                 const void *q, const void *k, const void *v,
                 const void *q_pts, const void *k_pts, const void *v_pts,
                 const float *rot, const float *trans,
                 const void *z1, const void *z2,
                 const float *w_b, const float *gamma, const uint8_t *mask,
                 float *o, float *o_pts, float *o_pair, float *lse,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * fipa_forward without a workspace argument, for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, same kernels and same results as fipa_forward, with the scratch memory taken from an
 * array of FIPA_STATIC_SCRATCH_BYTES that is part of the library's device image (every GPU the
 * library is used on holds one copy until the process ends).  Calls nothing that allocates.
 *   - FIPA_ERR_WORKSPACE when fipa_workspace_bytes(desc) exceeds FIPA_STATIC_SCRATCH_BYTES
 *     (bf16, H = 12, c_z = 128, r = 2: up to about 8000 residues in total over the batch);
 *     FIPA_ERR_LAUNCH when the array's device address cannot be obtained.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 *     streams, or threads) race; calls enqueued one after the other on one stream are safe.  The
 *     array keeps the last call's contents; every call clears what it needs cleared itself.
 */
#define FIPA_STATIC_SCRATCH_BYTES (64u << 20)
int fipa_forward_static(const fipa_desc *desc,
                        const void *q, const void *k, const void *v,
                        const void *q_pts, const void *k_pts, const void *v_pts,
                        const float *rot, const float *trans,
                        const void *z1, const void *z2,
                        const float *w_b, const float *gamma, const uint8_t *mask,
                        float *o, float *o_pts, float *o_pair, float *lse,
                        void *hip_stream);

/*
 * Packed batches: chains of different lengths stored back to back (the variable-length inputs of
 * the experiments in Section 3, without padding).  The tensors of fipa_forward / fipa_backward
 * with the leading [B, L] replaced by [total], total = cu_seqlens[B], chain b occupying rows
 * cu_seqlens[b] .. cu_seqlens[b+1] - 1; residues attend within their chain only.
 *   desc->B          number of chains;  desc->L  an upper bound of the chain lengths
 *   cu_seqlens       HOST pointer, B + 1 int32, cu_seqlens[0] = 0, non-decreasing; a chain may be
 *                    empty; a chain longer than desc->L is FIPA_ERR_INVALID_ARG.  Read during the
 *                    call only.
 *   mask             [total] bytes or NULL
 *   lse              [H * total] float32 or NULL: chain b's block [H, len_b] starts at
 *                    H * cu_seqlens[b]
 *   workspace        at least what fipa_packed_workspace_bytes reports for the same desc and
 *                    cu_seqlens
 * Two ways of running, chosen from the lengths alone (so the workspace query and the call agree):
 *   - bf16, and padding every chain to the longest would at most double the 128-row tiles: ONE set
 *     of launches over all chains -- the kernels of fipa_forward / fipa_backward reading and
 *     writing the packed tensors through the row offsets, skipping query tiles and key blocks
 *     past each chain's end.  Workspace: that of a padded batch of B chains of the longest length,
 *     plus the offsets.  This is what fills the chip when chains are short or many.
 *   - otherwise (one chain much longer than the rest; fp32 mode; or FIPA_FLAG_PACKED_PER_CHAIN in
 *     desc->flags, which asks for the smallest workspace): chain after chain on the caller's
 *     stream, as B = 1 problems on offset pointers sharing a workspace sized for the longest
 *     chain; the backward adds the chains' d_gamma and d_w_b in chain order.
 * Nothing is computed for padding either way.  fipa_backward_packed: bf16, r*cz <= 512; gradient
 * tensors packed like their inputs, d_gamma [H] and d_w_b [H, cz] (or NULL) summed over all chains,
 * d_rot / d_trans [total, 3, 3] / [total, 3] (both or neither).
 */
#define FIPA_FLAG_PACKED_PER_CHAIN 2u
int fipa_packed_workspace_bytes(const fipa_desc *desc, const int32_t *cu_seqlens,
                                size_t *forward_bytes, size_t *backward_bytes);
int fipa_forward_packed(const fipa_desc *desc, const int32_t *cu_seqlens,
                        const void *q, const void *k, const void *v,
                        const void *q_pts, const void *k_pts, const void *v_pts,
                        const float *rot, const float *trans,
                        const void *z1, const void *z2,
                        const float *w_b, const float *gamma, const uint8_t *mask,
                        float *o, float *o_pts, float *o_pair, float *lse,
                        void *workspace, size_t workspace_bytes, void *hip_stream);
int fipa_backward_packed(const fipa_desc *desc, const int32_t *cu_seqlens,
                         const void *q, const void *k, const void *v,
                         const void *q_pts, const void *k_pts, const void *v_pts,
                         const float *rot, const float *trans,
                         const void *z1, const void *z2,
                         const float *w_b, const float *gamma, const uint8_t *mask,
                         const float *d_o, const float *d_o_pts, const float *d_o_pair,
                         void *d_q, void *d_k, void *d_v,
                         void *d_q_pts, void *d_k_pts, void *d_v_pts,
                         void *d_z1, void *d_z2, float *d_gamma, float *d_w_b,
                         float *d_rot, float *d_trans,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * k-nearest-neighbour distogram features (Section 2.5: only the distances to the k nearest
 * neighbours are kept, [L, k, n_bins] instead of [L, L, n_bins], with the neighbours' indices).
 * The paper gives no formula; this call fixes:
 *   - distance of residues i, j = Euclidean distance of the frame origins trans[b, i], trans[b, j];
 *   - candidates are the valid residues (mask, [B, L] bytes or NULL) of the same batch element other
 *     than i itself; an invalid residue has no neighbours; fewer than k candidates leave the last
 *     slots empty (index -1, squared distance +inf, bin -1);
 *   - neighbours are listed by increasing distance, equal distances by increasing index;
 *   - n_bins bins with edges e_m = d_min + m (d_max - d_min)/(n_bins - 1), m = 0 .. n_bins - 2;
 *     bin = number of edges e_m <= distance (bin 0: below d_min; bin n_bins - 1: at or above d_max);
 *   - all decisions in float32 on the squared distance ((dx*dx + dy*dy) + dz*dz) and the squared
 *     edges, one rounding per operation.
 * Outputs (device, 4-byte aligned, fully overwritten): nbr_idx [B, L, k] int32, nbr_d2 [B, L, k]
 * float32 (squared distances), nbr_bin [B, L, k] int32.  A one-hot distogram is
 * feat[b, i, s, nbr_bin[b, i, s]] = 1; the factors z1, z2 are linear projections of such features
 * (fipa_factor_project below).
 * 1 <= k <= 64, 2 <= n_bins <= 4096, 0 <= d_min < d_max; otherwise FIPA_ERR_INVALID_ARG /
 * FIPA_ERR_UNSUPPORTED.  No workspace; enqueued on hip_stream.
 */
int fipa_knn_distogram(int32_t B, int32_t L, int32_t k, int32_t n_bins, float d_min, float d_max,
                       const float *trans, const uint8_t *mask,
                       int32_t *nbr_idx, float *nbr_d2, int32_t *nbr_bin, void *hip_stream);

/*
 * Pair pseudo-factors from those features (Section 2.4: every pair feature is represented by two
 * [L, r, c_z] tensors obtained via linear projections; Section 2.5: the neighbours' identities
 * enter through a positional encoding of their indices).  The paper gives no formula; this call
 * fixes: the feature vector of residue i is the concatenation over its k neighbour slots s of
 * [one-hot(nbr_bin[b,i,s]) | one-hot(code(b,i,s))] with an empty slot (index < 0) all zero, and a
 * factor is one linear projection of it plus a bias.  A projection of one-hot vectors is a sum of
 * table rows, so the weights are passed as tables and nothing is multiplied:
 *   z[b, i, :] = bias + sum_s ( e_bin[s, nbr_bin[b,i,s], :] + e_pos[s, code(b,i,s), :] )
 *   pos_mode 0: code = min(j, n_pos - 1) with j = nbr_idx[b,i,s] (the neighbour's own index);
 *   pos_mode 1: code = clip(j - i, -(n_pos-1)/2, +(n_pos-1)/2) + (n_pos-1)/2 (its offset; n_pos odd).
 * A fixed encoding (sines and cosines of the code, say) followed by a linear map is the table
 * e_pos[s, code, :] = W_s enc(code) that the caller tabulates once.
 * nbr_idx, nbr_bin [B, L, k] int32 as fipa_knn_distogram writes them (device, 4-byte aligned; a bin
 * outside 0 .. n_bins - 1 in a filled slot is clamped into the table); e_bin [k, n_bins, n_out] and
 * e_pos [k, n_pos, n_out] bf16 (e_pos NULL exactly when n_pos = 0), bias [n_out] float32 or NULL,
 * z [B, L, n_out] bf16 fully overwritten (a residue without neighbours gets the bias) -- all device,
 * 16-byte aligned.  n_out = r c_z, so z is a z1 or z2 argument of fipa_forward as it stands; call
 * twice, with the two sets of tables.  Sums in float32, slot by slot, one rounding to bf16 at the end.
 * n_out a multiple of 8, 1 <= k <= 64; otherwise FIPA_ERR_INVALID_ARG / FIPA_ERR_UNSUPPORTED.
 * No workspace; enqueued on hip_stream.
 */
int fipa_factor_project(int32_t B, int32_t L, int32_t k, int32_t n_bins, int32_t n_pos, int32_t pos_mode,
                        int32_t n_out, const int32_t *nbr_idx, const int32_t *nbr_bin, const void *e_bin,
                        const void *e_pos, const float *bias, void *z, void *hip_stream);

/*
 * Gradient of fipa_factor_project with respect to its tables and bias, for training the producer of
 * the factors (d_z is fipa_backward's d_z1 or d_z2): the projection is linear, so
 *   d_e_bin[s, m, :] = sum of d_z[b, i, :] over the residues whose slot s is filled and holds bin m,
 *   d_e_pos[s, c, :] = the same by position code, d_bias = sum of d_z over all residues;
 * residues with mask[b, i] = 0 (mask [B, L] bytes or NULL) add nothing.  Same index arguments and
 * codes as the forward call; d_z [B, L, n_out] bf16; d_e_bin [k, n_bins, n_out], d_e_pos
 * [k, n_pos, n_out] (NULL exactly when n_pos = 0) and d_bias [n_out] (or NULL) float32, fully
 * overwritten (rows that nothing selects get 0) -- device, 16-byte aligned.  Sums are float32 in a
 * fixed order (a contraction over the residues on the matrix pipe; the one-hot operand is exact in
 * bf16): the same bits on every run.  n_bins + n_pos <= 159 (FIPA_ERR_UNSUPPORTED otherwise); the other
 * limits as in the forward call.  No workspace; enqueued on hip_stream.
 */
int fipa_factor_project_backward(int32_t B, int32_t L, int32_t k, int32_t n_bins, int32_t n_pos, int32_t pos_mode,
                                 int32_t n_out, const int32_t *nbr_idx, const int32_t *nbr_bin, const void *d_z,
                                 const uint8_t *mask, float *d_e_bin, float *d_e_pos, float *d_bias,
                                 void *hip_stream);

/*
 * Backward of fipa_forward: gradients of a scalar loss with respect to q, k, v, the three
 * point sets, z1, z2 (same shapes and dtype as the inputs), gamma ([H], float32) and, when the
 * pointers are not NULL, the pair-bias weights w_b (d_w_b [H, cz], float32) and the frames
 * (d_rot [B, L, 3, 3] and d_trans [B, L, 3], float32, both or neither; every entry of R_i is
 * taken as a free variable of R_i x + t_i in Eq. 3 and of R_i^T (. - t_i) in Eq. 4), given
 * the upstream gradients d_o, d_o_pts, d_o_pair (float32, shapes of o, o_pts, o_pair).
 * The forward results o, o_pts, o_pair, lse are accepted for callers that keep them but are not
 * read (the attention weights and outputs are recomputed from the inputs, or with
 * FIPA_FLAG_KEEP_FORWARD taken from the workspace the forward call filled); each may be NULL.
 * d_gamma, d_w_b, d_rot and d_trans are overwritten (not accumulated).  The paper gives no backward; it is the chain
 * rule through Eqs. 3-4 and z_ij = z1_i^T z2_j.
 * Supported for FIPA_DTYPE_BF16 with r*cz <= 512 (512, the rank-4 shape at cz = 128, on plain gradient
 * kernels that are not tuned); otherwise FIPA_ERR_UNSUPPORTED.
 */
int fipa_backward(const fipa_desc *desc,
                  const void *q, const void *k, const void *v,
                  const void *q_pts, const void *k_pts, const void *v_pts,
                  const float *rot, const float *trans,
                  const void *z1, const void *z2,
                  const float *w_b, const float *gamma, const uint8_t *mask,
                  const float *o, const float *o_pts, const float *o_pair, const float *lse,
                  const float *d_o, const float *d_o_pts, const float *d_o_pair,
                  void *d_q, void *d_k, void *d_v,
                  void *d_q_pts, void *d_k_pts, void *d_v_pts,
                  void *d_z1, void *d_z2, float *d_gamma, float *d_w_b,
                  float *d_rot, float *d_trans,
                  void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The whole IPA module around the core (Eq. 1 and Eq. 5; Algorithm 1 steps 1 and 10), for
 * FIPA_DTYPE_BF16 descriptions:
 *     q | k | v | q_pts | k_pts | v_pts = s W_in^T + b_in      (Eq. 1; results kept as bfloat16)
 *     o, o_pts, o_pair                  = fipa_forward(...)     (Eqs. 2-4)
 *     s_out = concat(o_pair, o, o_pts, |o_pts|_2) W_out^T + b_out                      (Eq. 5)
 *   s       [B, L, d_s] bfloat16        single representation
 *   w_in    [N_in, d_s] bfloat16        N_in = H*(3c + 3*(2Pq + Pv)); output features in the order
 *                                       q [H,c] | k | v | q_pts [H,Pq,3] | k_pts | v_pts [H,Pv,3]
 *   b_in    [N_in] float32 or NULL
 *   w_out   [d_s, N_cat] bfloat16       N_cat = H*(cz + c + 4*Pv); input features in the order
 *                                       o_pair [H,cz] | o [H,c] | o_pts [H,Pv,3] | norms [H,Pv]
 *   b_out   [d_s] float32 or NULL
 *   s_out   [B, L, d_s] float32         (rows of masked residues receive b_out)
 *   rot, trans, z1, z2, w_b, gamma, mask: as for fipa_forward.
 * Shapes: d_s % 16 == 0, H*Pv % 8 == 0, N_cat % 16 == 0, else FIPA_ERR_UNSUPPORTED.
 * The workspace holds the core's workspace, its six bfloat16 inputs and its float32 outputs
 * (affine in L).  Device pointers, caller's stream, nothing allocated, as for fipa_forward.
 */
int fipa_module_workspace_bytes(const fipa_desc *desc, int32_t d_s, size_t *bytes);
int fipa_module_forward(const fipa_desc *desc, int32_t d_s,
                        const void *s, const void *w_in, const float *b_in,
                        const float *rot, const float *trans,
                        const void *z1, const void *z2,
                        const float *w_b, const float *gamma, const uint8_t *mask,
                        const void *w_out, const float *b_out,
                        float *s_out,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward of fipa_module_forward: gradients of a scalar loss, given d_s_out [B, L, d_s] float32,
 * with respect to s (d_s_in [B, L, d_s] float32), the two Linear layers (d_w_in [N_in, d_s],
 * d_w_out [d_s, N_cat], float32; d_b_in [N_in], d_b_out [d_s], float32 or NULL) and, passed
 * through from fipa_backward, z1, z2 (bfloat16), gamma, w_b (or NULL) and the frames (d_rot,
 * d_trans, both or neither).  Everything is recomputed from the inputs: no forward results are
 * taken.  The bfloat16 rounding of Eq. 1's results is transparent to the gradient; the norm of a
 * zero vector contributes zero.  All outputs are overwritten.
 * Shapes: as fipa_module_forward, and r*cz <= 512, N_in % 8 == 0; else FIPA_ERR_UNSUPPORTED.
 */
int fipa_module_backward_workspace_bytes(const fipa_desc *desc, int32_t d_s, size_t *bytes);
int fipa_module_backward(const fipa_desc *desc, int32_t d_s,
                         const void *s, const void *w_in, const float *b_in,
                         const float *rot, const float *trans,
                         const void *z1, const void *z2,
                         const float *w_b, const float *gamma, const uint8_t *mask,
                         const void *w_out, const float *b_out,
                         const float *d_s_out,
                         float *d_s_in, float *d_w_in, float *d_b_in, float *d_w_out, float *d_b_out,
                         void *d_z1, void *d_z2, float *d_gamma, float *d_w_b,
                         float *d_rot, float *d_trans,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Optional stage timing for benchmarks.  Between fipa_profile_begin() and fipa_profile_end()
 * every fipa_forward / fipa_backward call on any stream additionally records HIP events around
 * its stages on that stream (up to `capacity` calls; later calls run untimed).  This is the only
 * process-wide state in the library and is not thread safe; do not use it with concurrent calls.
 *   stage 0: preparation + packing (frame application, lifting)     Algorithm 1 steps 2-6
 *   stage 1: fused attention                                        Algorithm 1 step 7
 *   stage 2: epilogue (split, inverse frame, z1 contraction)        Algorithm 1 steps 8-9
 * fipa_profile_end waits for the recorded events (it synchronises with them, nothing else),
 * writes the mean duration of each stage in milliseconds to stage_ms[FIPA_PROFILE_STAGES] and
 * the number of timed calls to *n_calls, and releases the events.  begin allocates the events
 * (host-side driver objects, no device memory).
 * The event records themselves cost GPU time (several microseconds per call, which is visible
 * next to a 150 us step): fipa_profile_begin_every times only every `every`-th call (the first,
 * the (every+1)-th, ...; every >= 1), so that a throughput measurement taken over the same calls
 * is hardly disturbed.  fipa_profile_begin(capacity) is fipa_profile_begin_every(capacity, 1).
 * Both return FIPA_ERR_INVALID_ARG for capacity outside 1..4096, every < 1, or when timing is
 * already active.
 */
#define FIPA_PROFILE_STAGES 3
int fipa_profile_begin(int capacity);
int fipa_profile_begin_every(int capacity, int every);
int fipa_profile_end(float *stage_ms, int *n_calls);

/*
 * Measured denominator for roofline figures: enqueues a kernel of `workgroups` x 4 waves that does
 * nothing but `iters` x 16 independent bf16 32x32x16 MFMAs per wave (operands in registers), and
 * writes the number of floating-point operations that launch performs to *flop (HOST pointer, may
 * be NULL).  out: device buffer of workgroups * 256 floats (receives a checksum).  The caller times
 * the launch.  A measuring aid, not part of the method: roofline fractions are quoted against the
 * published peak; this shows what the matrix pipes sustain at the clock they hold under load.
 */
int fipa_probe_mfma(int iters, int workgroups, float *out, void *hip_stream, double *flop);

#ifdef __cplusplus
}
#endif
#endif /* FIPA_H */
