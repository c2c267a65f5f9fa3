/*
 * ipa_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision CPU implementation of *standard* Invariant
 * Point Attention with a dense pair tensor z[L,L,c_z] and the explicit sum of
 * squared point distances (Section 2.2, Eqs. 2-4 of the FlashIPA paper).  It is
 * what the GPU library is checked against; the product never calls it.  Only
 * tests, the smoke check and the CPU-baseline leg of the benchmark use it.  It
 * shares no code, table or constant with the HIP path.
 *
 * Nothing here is blocked, fused or reordered: every quantity is computed by
 * the loop that its defining equation spells out.
 *
 * Layouts (one batch element per call, all row-major, all double):
 *   q, k, v        [L, H, c]
 *   q_pts, k_pts   [L, H, Pq, 3]   points in the local frame of their residue
 *   v_pts          [L, H, Pv, 3]
 *   rot            [L, 3, 3]       R_i, global = R_i * local + t_i
 *   trans          [L, 3]          t_i
 *   z (dense)      [L, L, cz]      or z_rows [n_rows, L, cz] for a row subset
 *   w_b            [H, cz]         weights of the pair-bias Linear (Eq. 2)
 *   gamma          [H]             per-head point weight, used as given
 *   mask           [L] bytes, 1 = valid residue, or NULL (all valid)
 *
 * Pins (tests/test_oracle_pins.py): brute force at L<=8, equality with the
 * factorized update rule (Algorithm 1) on rank-r pair tensors, SE(3)
 * invariance, closed forms, reduction to library softmax attention, and
 * central finite differences for the backward.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* global = R * local + t   (frame application T o x used in Eqs. 3 and 4) */
static void frame_apply(const double *R, const double *t, const double *x, double *y)
{
    for (int a = 0; a < 3; ++a)
        y[a] = R[3 * a + 0] * x[0] + R[3 * a + 1] * x[1] + R[3 * a + 2] * x[2] + t[a];
}

/* y = R^T * x  (rotation part of the inverse frame) */
static void rot_transpose_apply(const double *R, const double *x, double *y)
{
    for (int a = 0; a < 3; ++a)
        y[a] = R[0 + a] * x[0] + R[3 + a] * x[1] + R[6 + a] * x[2];
}

/* y = R * x */
static void rot_apply(const double *R, const double *x, double *y)
{
    for (int a = 0; a < 3; ++a)
        y[a] = R[3 * a + 0] * x[0] + R[3 * a + 1] * x[1] + R[3 * a + 2] * x[2];
}

int ipa_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of threads the row loops may use from now on (benchmark legs time the oracle on one core too). */
void ipa_oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0)
        omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * Dense pair rows from the factors (Section 2.4: z_ij = z1_i^T z2_j, the
 * contraction runs over the rank index):
 *   z_rows[a, j, d] = sum_rho z1[rows[a], rho, d] * z2[j, rho, d]
 * z1, z2: [L, r, cz].
 */
void ipa_oracle_pair_rows(int L, int r, int cz, const double *z1, const double *z2,
                          int n_rows, const int32_t *rows, double *z_rows)
{
#pragma omp parallel for schedule(static)
    for (int a = 0; a < n_rows; ++a) {
        const int i = rows[a];
        for (int j = 0; j < L; ++j)
            for (int d = 0; d < cz; ++d) {
                double s = 0.0;
                for (int rho = 0; rho < r; ++rho)
                    s += z1[((size_t)i * r + rho) * cz + d] * z2[((size_t)j * r + rho) * cz + d];
                z_rows[((size_t)a * L + j) * cz + d] = s;
            }
    }
}

/*
 * Logits of one (query row i, head h) against every key (argument of the
 * softmax in Eq. 3), with the pair bias of Eq. 2:
 *   s_j = w_L * ( q_i.k_j / sqrt(c) + sum_d w_b[h,d] z_ij[d]
 *                 - gamma_h * w_C / 2 * sum_p |T_i o q_ip - T_j o k_jp|^2 )
 * Also returns the squared-distance sums D_j when dist != NULL.
 */
static void logits_row(int L, int H, int c, int Pq, int cz, int i, int h,
                       const double *q, const double *k, const double *q_pts, const double *k_pts,
                       const double *rot, const double *trans, const double *z_i /* [L,cz] */,
                       const double *w_b, const double *gamma, double w_L, double w_C,
                       double *s, double *dist)
{
    for (int j = 0; j < L; ++j) {
        double qk = 0.0;
        for (int d = 0; d < c; ++d)
            qk += q[((size_t)i * H + h) * c + d] * k[((size_t)j * H + h) * c + d];
        double b = 0.0;
        for (int d = 0; d < cz; ++d)
            b += w_b[(size_t)h * cz + d] * z_i[(size_t)j * cz + d];
        double D = 0.0;
        for (int p = 0; p < Pq; ++p) {
            double Q[3], K[3];
            frame_apply(rot + 9 * (size_t)i, trans + 3 * (size_t)i,
                        q_pts + (((size_t)i * H + h) * Pq + p) * 3, Q);
            frame_apply(rot + 9 * (size_t)j, trans + 3 * (size_t)j,
                        k_pts + (((size_t)j * H + h) * Pq + p) * 3, K);
            for (int a = 0; a < 3; ++a)
                D += (Q[a] - K[a]) * (Q[a] - K[a]);
        }
        s[j] = w_L * (qk / sqrt((double)c) + b - gamma[h] * w_C / 2.0 * D);
        if (dist)
            dist[j] = D;
    }
}

/* softmax over valid keys with the maximum subtracted; masked keys get weight 0 */
static void softmax_row(int L, const uint8_t *mask, const double *s, double *a)
{
    double m = -INFINITY;
    for (int j = 0; j < L; ++j)
        if ((!mask || mask[j]) && s[j] > m)
            m = s[j];
    double sum = 0.0;
    for (int j = 0; j < L; ++j) {
        a[j] = (!mask || mask[j]) ? exp(s[j] - m) : 0.0;
        sum += a[j];
    }
    for (int j = 0; j < L; ++j)
        a[j] /= sum;
}

/*
 * Forward for a list of query rows against all keys (Eqs. 2-4).
 *   z_rows [n_rows, L, cz] : z_ij for i = rows[a]
 * Outputs (row a <-> query rows[a]):
 *   o      [n_rows, H, c]       sum_j a_ij v_j
 *   o_pts  [n_rows, H, Pv, 3]   T_i^{-1} o sum_j a_ij (T_j o v_jp)   (local frame of i)
 *   o_pair [n_rows, H, cz]      sum_j a_ij z_ij
 *   attn   [n_rows, H, L]       a_ij, or NULL
 * A query row whose own mask byte is 0 gives all-zero outputs.
 * Returns 0, or -1 when some valid query row has no valid key.
 */
int ipa_oracle_forward_rows(int L, int H, int c, int Pq, int Pv, int cz,
                            const double *q, const double *k, const double *v,
                            const double *q_pts, const double *k_pts, const double *v_pts,
                            const double *rot, const double *trans, const double *z_rows,
                            const double *w_b, const double *gamma, double w_L, double w_C,
                            const uint8_t *mask, int n_rows, const int32_t *rows,
                            double *o, double *o_pts, double *o_pair, double *attn)
{
    if (mask) {
        int any = 0;
        for (int j = 0; j < L; ++j)
            any |= mask[j];
        if (!any)
            return -1;
    }
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        double *a = (double *)malloc(sizeof(double) * (size_t)L);
#pragma omp for schedule(dynamic, 1)
        for (int r_ = 0; r_ < n_rows; ++r_) {
            const int i = rows[r_];
            const double *z_i = z_rows + (size_t)r_ * L * cz;
            for (int h = 0; h < H; ++h) {
                double *o_ih = o + ((size_t)r_ * H + h) * c;
                double *op_ih = o_pts + ((size_t)r_ * H + h) * Pv * 3;
                double *oz_ih = o_pair + ((size_t)r_ * H + h) * cz;
                double *at_ih = attn ? attn + ((size_t)r_ * H + h) * L : NULL;
                memset(o_ih, 0, sizeof(double) * c);
                memset(op_ih, 0, sizeof(double) * Pv * 3);
                memset(oz_ih, 0, sizeof(double) * cz);
                if (at_ih)
                    memset(at_ih, 0, sizeof(double) * L);
                if (mask && !mask[i])
                    continue;
                logits_row(L, H, c, Pq, cz, i, h, q, k, q_pts, k_pts, rot, trans, z_i, w_b, gamma,
                           w_L, w_C, s, NULL);
                softmax_row(L, mask, s, a);
                if (at_ih)
                    memcpy(at_ih, a, sizeof(double) * L);
                /* Eq. 4, scalar values and pair values */
                for (int j = 0; j < L; ++j) {
                    for (int d = 0; d < c; ++d)
                        o_ih[d] += a[j] * v[((size_t)j * H + h) * c + d];
                    for (int d = 0; d < cz; ++d)
                        oz_ih[d] += a[j] * z_i[(size_t)j * cz + d];
                }
                /* Eq. 4, value points: average in the global frame, then T_i^{-1} */
                for (int p = 0; p < Pv; ++p) {
                    double G[3] = {0.0, 0.0, 0.0};
                    for (int j = 0; j < L; ++j) {
                        double V[3];
                        frame_apply(rot + 9 * (size_t)j, trans + 3 * (size_t)j,
                                    v_pts + (((size_t)j * H + h) * Pv + p) * 3, V);
                        for (int x = 0; x < 3; ++x)
                            G[x] += a[j] * V[x];
                    }
                    double rel[3];
                    for (int x = 0; x < 3; ++x)
                        rel[x] = G[x] - trans[3 * (size_t)i + x];
                    rot_transpose_apply(rot + 9 * (size_t)i, rel, op_ih + 3 * p);
                }
            }
        }
        free(s);
        free(a);
    }
    return 0;
}

/*
 * Backward of the forward above for ALL query rows (dense z [L,L,cz]).
 * Upstream gradients d_o [L,H,c], d_o_pts [L,H,Pv,3], d_o_pair [L,H,cz]; rows
 * whose mask byte is 0 contribute nothing.  Outputs are overwritten:
 *   dq, dk, dv [L,H,c]; dq_pts, dk_pts [L,H,Pq,3]; dv_pts [L,H,Pv,3];
 *   dz [L,L,cz]; dgamma [H]; dw_b [H,cz].
 * Chain rule through Eq. 4 (values), the softmax, and Eq. 3 (logits); frames
 * are treated as constants.  Serial on purpose (gradients scatter into keys).
 */
int ipa_oracle_backward(int L, int H, int c, int Pq, int Pv, int cz,
                        const double *q, const double *k, const double *v,
                        const double *q_pts, const double *k_pts, const double *v_pts,
                        const double *rot, const double *trans, const double *z,
                        const double *w_b, const double *gamma, double w_L, double w_C,
                        const uint8_t *mask,
                        const double *d_o, const double *d_o_pts, const double *d_o_pair,
                        double *dq, double *dk, double *dv,
                        double *dq_pts, double *dk_pts, double *dv_pts,
                        double *dz, double *dgamma, double *dw_b,
                        double *drot, double *dtrans)
{
    /* drot [L,3,3], dtrans [L,3] (both may be NULL): gradients with respect to the frames, every
     * entry of R_i taken as a free variable of G = R_i x + t_i (Eq. 3) and of R_i^T (G - t_i) (Eq. 4). */
    const int frames = drot != NULL && dtrans != NULL;
    if (frames) {
        memset(drot, 0, sizeof(double) * (size_t)L * 9);
        memset(dtrans, 0, sizeof(double) * (size_t)L * 3);
    }
    double *Gacc = (double *)malloc(sizeof(double) * (size_t)Pv * 3);
    memset(dq, 0, sizeof(double) * (size_t)L * H * c);
    memset(dk, 0, sizeof(double) * (size_t)L * H * c);
    memset(dv, 0, sizeof(double) * (size_t)L * H * c);
    memset(dq_pts, 0, sizeof(double) * (size_t)L * H * Pq * 3);
    memset(dk_pts, 0, sizeof(double) * (size_t)L * H * Pq * 3);
    memset(dv_pts, 0, sizeof(double) * (size_t)L * H * Pv * 3);
    memset(dz, 0, sizeof(double) * (size_t)L * L * cz);
    memset(dgamma, 0, sizeof(double) * (size_t)H);
    memset(dw_b, 0, sizeof(double) * (size_t)H * cz);

    double *s = (double *)malloc(sizeof(double) * (size_t)L);
    double *a = (double *)malloc(sizeof(double) * (size_t)L);
    double *D = (double *)malloc(sizeof(double) * (size_t)L);
    double *da = (double *)malloc(sizeof(double) * (size_t)L);
    double *dG = (double *)malloc(sizeof(double) * (size_t)Pv * 3);

    for (int i = 0; i < L; ++i) {
        if (mask && !mask[i])
            continue;
        const double *z_i = z + (size_t)i * L * cz;
        double *dz_i = dz + (size_t)i * L * cz;
        for (int h = 0; h < H; ++h) {
            logits_row(L, H, c, Pq, cz, i, h, q, k, q_pts, k_pts, rot, trans, z_i, w_b, gamma,
                       w_L, w_C, s, D);
            softmax_row(L, mask, s, a);
            const double *go = d_o + ((size_t)i * H + h) * c;
            const double *gp = d_o_pts + ((size_t)i * H + h) * Pv * 3;
            const double *gz = d_o_pair + ((size_t)i * H + h) * cz;
            /* o_pts = R_i^T (G - t_i)  =>  dL/dG = R_i * dL/do_pts */
            for (int p = 0; p < Pv; ++p)
                rot_apply(rot + 9 * (size_t)i, gp + 3 * p, dG + 3 * p);

            for (int x = 0; x < 3 * Pv; ++x)
                Gacc[x] = 0.0;
            /* gradients of the three weighted sums of Eq. 4 */
            double dot = 0.0; /* sum_j a_ij * dL/da_ij */
            for (int j = 0; j < L; ++j) {
                double g = 0.0;
                for (int d = 0; d < c; ++d) {
                    g += go[d] * v[((size_t)j * H + h) * c + d];
                    dv[((size_t)j * H + h) * c + d] += a[j] * go[d];
                }
                for (int d = 0; d < cz; ++d) {
                    g += gz[d] * z_i[(size_t)j * cz + d];
                    dz_i[(size_t)j * cz + d] += a[j] * gz[d];
                }
                for (int p = 0; p < Pv; ++p) {
                    double V[3], aG[3], loc[3];
                    frame_apply(rot + 9 * (size_t)j, trans + 3 * (size_t)j,
                                v_pts + (((size_t)j * H + h) * Pv + p) * 3, V);
                    for (int x = 0; x < 3; ++x) {
                        g += dG[3 * p + x] * V[x];
                        aG[x] = a[j] * dG[3 * p + x];
                        Gacc[3 * p + x] += a[j] * V[x];
                    }
                    if (frames) { /* V_jp = R_j v_jp + t_j */
                        const double *vl = v_pts + (((size_t)j * H + h) * Pv + p) * 3;
                        for (int x = 0; x < 3; ++x) {
                            dtrans[3 * (size_t)j + x] += aG[x];
                            for (int y = 0; y < 3; ++y)
                                drot[9 * (size_t)j + 3 * x + y] += aG[x] * vl[y];
                        }
                    }
                    /* V_jp = R_j v_jp + t_j  =>  dL/dv_jp = R_j^T dL/dV_jp */
                    rot_transpose_apply(rot + 9 * (size_t)j, aG, loc);
                    for (int x = 0; x < 3; ++x)
                        dv_pts[(((size_t)j * H + h) * Pv + p) * 3 + x] += loc[x];
                }
                da[j] = g;
                dot += a[j] * g;
            }
            if (frames) { /* o_pts = R_i^T (G - t_i): dL/dt_i = -R_i g, dL/dR_i[x][y] = (G - t_i)[x] g[y] */
                for (int p = 0; p < Pv; ++p)
                    for (int x = 0; x < 3; ++x) {
                        dtrans[3 * (size_t)i + x] -= dG[3 * p + x];
                        for (int y = 0; y < 3; ++y)
                            drot[9 * (size_t)i + 3 * x + y] +=
                                (Gacc[3 * p + x] - trans[3 * (size_t)i + x]) * gp[3 * p + y];
                    }
            }
            /* softmax backward, then Eq. 3 term by term */
            for (int j = 0; j < L; ++j) {
                if (mask && !mask[j])
                    continue;
                const double ds = a[j] * (da[j] - dot);
                const double sc = w_L / sqrt((double)c);
                for (int d = 0; d < c; ++d) {
                    dq[((size_t)i * H + h) * c + d] += ds * sc * k[((size_t)j * H + h) * c + d];
                    dk[((size_t)j * H + h) * c + d] += ds * sc * q[((size_t)i * H + h) * c + d];
                }
                for (int d = 0; d < cz; ++d) {
                    dz_i[(size_t)j * cz + d] += ds * w_L * w_b[(size_t)h * cz + d];
                    dw_b[(size_t)h * cz + d] += ds * w_L * z_i[(size_t)j * cz + d];
                }
                dgamma[h] += ds * (-w_L * w_C / 2.0) * D[j];
                const double pc = w_L * gamma[h] * w_C; /* (w_L gamma w_C / 2) * 2 */
                for (int p = 0; p < Pq; ++p) {
                    double Qg[3], Kg[3], gQ[3], gK[3], loc[3];
                    frame_apply(rot + 9 * (size_t)i, trans + 3 * (size_t)i,
                                q_pts + (((size_t)i * H + h) * Pq + p) * 3, Qg);
                    frame_apply(rot + 9 * (size_t)j, trans + 3 * (size_t)j,
                                k_pts + (((size_t)j * H + h) * Pq + p) * 3, Kg);
                    for (int x = 0; x < 3; ++x) {
                        gQ[x] = -ds * pc * (Qg[x] - Kg[x]);
                        gK[x] = ds * pc * (Qg[x] - Kg[x]);
                    }
                    if (frames) {
                        const double *ql = q_pts + (((size_t)i * H + h) * Pq + p) * 3;
                        const double *kl = k_pts + (((size_t)j * H + h) * Pq + p) * 3;
                        for (int x = 0; x < 3; ++x) {
                            dtrans[3 * (size_t)i + x] += gQ[x];
                            dtrans[3 * (size_t)j + x] += gK[x];
                            for (int y = 0; y < 3; ++y) {
                                drot[9 * (size_t)i + 3 * x + y] += gQ[x] * ql[y];
                                drot[9 * (size_t)j + 3 * x + y] += gK[x] * kl[y];
                            }
                        }
                    }
                    rot_transpose_apply(rot + 9 * (size_t)i, gQ, loc);
                    for (int x = 0; x < 3; ++x)
                        dq_pts[(((size_t)i * H + h) * Pq + p) * 3 + x] += loc[x];
                    rot_transpose_apply(rot + 9 * (size_t)j, gK, loc);
                    for (int x = 0; x < 3; ++x)
                        dk_pts[(((size_t)j * H + h) * Pq + p) * 3 + x] += loc[x];
                }
            }
        }
    }
    free(s);
    free(a);
    free(D);
    free(da);
    free(dG);
    free(Gacc);
    return 0;
}

/*
 * Chain rule through z_ij[d] = sum_rho z1_i[rho,d] z2_j[rho,d]:
 *   dz1_i[rho,d] = sum_j dz_ij[d] z2_j[rho,d],  dz2_j[rho,d] = sum_i dz_ij[d] z1_i[rho,d]
 */
void ipa_oracle_pair_backward(int L, int r, int cz, const double *z1, const double *z2,
                              const double *dz, double *dz1, double *dz2)
{
    memset(dz1, 0, sizeof(double) * (size_t)L * r * cz);
    memset(dz2, 0, sizeof(double) * (size_t)L * r * cz);
    for (int i = 0; i < L; ++i)
        for (int j = 0; j < L; ++j)
            for (int rho = 0; rho < r; ++rho)
                for (int d = 0; d < cz; ++d) {
                    const double g = dz[((size_t)i * L + j) * cz + d];
                    dz1[((size_t)i * r + rho) * cz + d] += g * z2[((size_t)j * r + rho) * cz + d];
                    dz2[((size_t)j * r + rho) * cz + d] += g * z1[((size_t)i * r + rho) * cz + d];
                }
}

/*
 * Backward for sizes where the dense pair tensor does not fit: the same chain rule as
 * ipa_oracle_backward (Eq. 4 -> softmax -> Eq. 3 -> z_ij = z1_i^T z2_j of Section 2.4), walked
 * one query row at a time with that row's z_i [L, cz] formed on the spot from the factors
 * z1, z2 [L, r, cz].  Every query row is visited (the key-side gradients and the parameter
 * gradients are sums over all of them), but only the gradients of the n_s sampled residues
 * S[0..n_s) are kept; entry a of an output belongs to residue S[a]:
 *   dq, dk, dv [n_s,H,c]; dq_pts, dk_pts [n_s,H,Pq,3]; dv_pts [n_s,H,Pv,3];
 *   dz1, dz2 [n_s,r,cz]; drot [n_s,3,3]; dtrans [n_s,3]   (a residue's frame gradient needs both
 *   of its roles, as query row and as key column)
 * and in full dgamma [H], dw_b [H,cz].
 * Pinned by equality with ipa_oracle_backward + ipa_oracle_pair_backward at small L.
 * Rows are spread over threads; each thread sums into its own copy of the outputs and the
 * copies are added in thread order at the end.
 */
int ipa_oracle_backward_sampled(int L, int H, int c, int Pq, int Pv, int cz, int r,
                                const double *q, const double *k, const double *v,
                                const double *q_pts, const double *k_pts, const double *v_pts,
                                const double *rot, const double *trans,
                                const double *z1, const double *z2,
                                const double *w_b, const double *gamma, double w_L, double w_C,
                                const uint8_t *mask,
                                const double *d_o, const double *d_o_pts, const double *d_o_pair,
                                int n_s, const int32_t *S,
                                double *dq, double *dk, double *dv,
                                double *dq_pts, double *dk_pts, double *dv_pts,
                                double *dz1, double *dz2, double *drot, double *dtrans,
                                double *dgamma, double *dw_b)
{
    /* one flat buffer per thread holding all twelve outputs */
    const size_t n_sc = (size_t)n_s * H * c, n_qp = (size_t)n_s * H * Pq * 3, n_vp = (size_t)n_s * H * Pv * 3,
                 n_zf = (size_t)n_s * r * cz;
    const size_t o_dq = 0, o_dk = o_dq + n_sc, o_dv = o_dk + n_sc, o_dqp = o_dv + n_sc, o_dkp = o_dqp + n_qp,
                 o_dvp = o_dkp + n_qp, o_dz1 = o_dvp + n_vp, o_dz2 = o_dz1 + n_zf, o_drot = o_dz2 + n_zf,
                 o_dtr = o_drot + (size_t)n_s * 9, o_dg = o_dtr + (size_t)n_s * 3, o_dwb = o_dg + (size_t)H,
                 n_all = o_dwb + (size_t)H * cz;
    int *slot = (int *)malloc(sizeof(int) * (size_t)L); /* residue -> index in S, or -1 */
    for (int i = 0; i < L; ++i)
        slot[i] = -1;
    for (int a = 0; a < n_s; ++a)
        slot[S[a]] = a;
    const int nt = ipa_oracle_num_threads();
    double *all = (double *)calloc(n_all * (size_t)nt, sizeof(double));

#pragma omp parallel num_threads(nt)
    {
#ifdef _OPENMP
        double *acc = all + n_all * (size_t)omp_get_thread_num();
#else
        double *acc = all;
#endif
        double *z_i = (double *)malloc(sizeof(double) * (size_t)L * cz);
        double *dz_i = (double *)malloc(sizeof(double) * (size_t)L * cz);
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        double *a = (double *)malloc(sizeof(double) * (size_t)L);
        double *D = (double *)malloc(sizeof(double) * (size_t)L);
        double *da = (double *)malloc(sizeof(double) * (size_t)L);
        double *dG = (double *)malloc(sizeof(double) * (size_t)Pv * 3);
        double *Gacc = (double *)malloc(sizeof(double) * (size_t)Pv * 3);
#pragma omp for schedule(static)
        for (int i = 0; i < L; ++i) {
            if (mask && !mask[i])
                continue;
            const int ai = slot[i];
            /* z_i[j, d] = sum_rho z1_i[rho, d] z2_j[rho, d]   (Section 2.4) */
            for (int j = 0; j < L; ++j)
                for (int d = 0; d < cz; ++d) {
                    double zz = 0.0;
                    for (int rho = 0; rho < r; ++rho)
                        zz += z1[((size_t)i * r + rho) * cz + d] * z2[((size_t)j * r + rho) * cz + d];
                    z_i[(size_t)j * cz + d] = zz;
                    dz_i[(size_t)j * cz + d] = 0.0;
                }
            for (int h = 0; h < H; ++h) {
                logits_row(L, H, c, Pq, cz, i, h, q, k, q_pts, k_pts, rot, trans, z_i, w_b, gamma, w_L, w_C, s, D);
                softmax_row(L, mask, s, a);
                const double *go = d_o + ((size_t)i * H + h) * c;
                const double *gp = d_o_pts + ((size_t)i * H + h) * Pv * 3;
                const double *gz = d_o_pair + ((size_t)i * H + h) * cz;
                for (int p = 0; p < Pv; ++p)
                    rot_apply(rot + 9 * (size_t)i, gp + 3 * p, dG + 3 * p);
                for (int x = 0; x < 3 * Pv; ++x)
                    Gacc[x] = 0.0;
                /* Eq. 4: derivative with respect to the weights (da) and to the values of key j */
                double dot = 0.0;
                for (int j = 0; j < L; ++j) {
                    const int aj = slot[j];
                    double g = 0.0;
                    for (int d = 0; d < c; ++d)
                        g += go[d] * v[((size_t)j * H + h) * c + d];
                    for (int d = 0; d < cz; ++d) {
                        g += gz[d] * z_i[(size_t)j * cz + d];
                        dz_i[(size_t)j * cz + d] += a[j] * gz[d];
                    }
                    if (aj >= 0)
                        for (int d = 0; d < c; ++d)
                            acc[o_dv + ((size_t)aj * H + h) * c + d] += a[j] * go[d];
                    for (int p = 0; p < Pv; ++p) {
                        const double *vl = v_pts + (((size_t)j * H + h) * Pv + p) * 3;
                        double V[3], aG[3], loc[3];
                        frame_apply(rot + 9 * (size_t)j, trans + 3 * (size_t)j, vl, V);
                        for (int x = 0; x < 3; ++x) {
                            g += dG[3 * p + x] * V[x];
                            aG[x] = a[j] * dG[3 * p + x];
                            Gacc[3 * p + x] += a[j] * V[x];
                        }
                        if (aj >= 0) {
                            for (int x = 0; x < 3; ++x) {
                                acc[o_dtr + 3 * (size_t)aj + x] += aG[x];
                                for (int y = 0; y < 3; ++y)
                                    acc[o_drot + 9 * (size_t)aj + 3 * x + y] += aG[x] * vl[y];
                            }
                            rot_transpose_apply(rot + 9 * (size_t)j, aG, loc);
                            for (int x = 0; x < 3; ++x)
                                acc[o_dvp + (((size_t)aj * H + h) * Pv + p) * 3 + x] += loc[x];
                        }
                    }
                    da[j] = g;
                    dot += a[j] * g;
                }
                if (ai >= 0) /* o_pts = R_i^T (G - t_i) as a function of the frame of i */
                    for (int p = 0; p < Pv; ++p)
                        for (int x = 0; x < 3; ++x) {
                            acc[o_dtr + 3 * (size_t)ai + x] -= dG[3 * p + x];
                            for (int y = 0; y < 3; ++y)
                                acc[o_drot + 9 * (size_t)ai + 3 * x + y] +=
                                    (Gacc[3 * p + x] - trans[3 * (size_t)i + x]) * gp[3 * p + y];
                        }
                /* softmax, then Eq. 3 term by term */
                const double sc = w_L / sqrt((double)c);
                const double pc = w_L * gamma[h] * w_C;
                for (int j = 0; j < L; ++j) {
                    if (mask && !mask[j])
                        continue;
                    const int aj = slot[j];
                    const double ds = a[j] * (da[j] - dot);
                    if (ai >= 0)
                        for (int d = 0; d < c; ++d)
                            acc[o_dq + ((size_t)ai * H + h) * c + d] += ds * sc * k[((size_t)j * H + h) * c + d];
                    if (aj >= 0)
                        for (int d = 0; d < c; ++d)
                            acc[o_dk + ((size_t)aj * H + h) * c + d] += ds * sc * q[((size_t)i * H + h) * c + d];
                    for (int d = 0; d < cz; ++d) {
                        dz_i[(size_t)j * cz + d] += ds * w_L * w_b[(size_t)h * cz + d];
                        acc[o_dwb + (size_t)h * cz + d] += ds * w_L * z_i[(size_t)j * cz + d];
                    }
                    acc[o_dg + h] += ds * (-w_L * w_C / 2.0) * D[j];
                    if (ai < 0 && aj < 0)
                        continue;
                    for (int p = 0; p < Pq; ++p) {
                        const double *ql = q_pts + (((size_t)i * H + h) * Pq + p) * 3;
                        const double *kl = k_pts + (((size_t)j * H + h) * Pq + p) * 3;
                        double Qg[3], Kg[3], gQ[3], gK[3], loc[3];
                        frame_apply(rot + 9 * (size_t)i, trans + 3 * (size_t)i, ql, Qg);
                        frame_apply(rot + 9 * (size_t)j, trans + 3 * (size_t)j, kl, Kg);
                        for (int x = 0; x < 3; ++x) {
                            gQ[x] = -ds * pc * (Qg[x] - Kg[x]);
                            gK[x] = ds * pc * (Qg[x] - Kg[x]);
                        }
                        if (ai >= 0) {
                            for (int x = 0; x < 3; ++x) {
                                acc[o_dtr + 3 * (size_t)ai + x] += gQ[x];
                                for (int y = 0; y < 3; ++y)
                                    acc[o_drot + 9 * (size_t)ai + 3 * x + y] += gQ[x] * ql[y];
                            }
                            rot_transpose_apply(rot + 9 * (size_t)i, gQ, loc);
                            for (int x = 0; x < 3; ++x)
                                acc[o_dqp + (((size_t)ai * H + h) * Pq + p) * 3 + x] += loc[x];
                        }
                        if (aj >= 0) {
                            for (int x = 0; x < 3; ++x) {
                                acc[o_dtr + 3 * (size_t)aj + x] += gK[x];
                                for (int y = 0; y < 3; ++y)
                                    acc[o_drot + 9 * (size_t)aj + 3 * x + y] += gK[x] * kl[y];
                            }
                            rot_transpose_apply(rot + 9 * (size_t)j, gK, loc);
                            for (int x = 0; x < 3; ++x)
                                acc[o_dkp + (((size_t)aj * H + h) * Pq + p) * 3 + x] += loc[x];
                        }
                    }
                }
            }
            /* z_ij = z1_i^T z2_j: the row's dz_i [L, cz] goes to z1_i (if sampled) and to the sampled z2_j */
            for (int j = 0; j < L; ++j) {
                const int aj = slot[j];
                if (ai < 0 && aj < 0)
                    continue;
                for (int rho = 0; rho < r; ++rho)
                    for (int d = 0; d < cz; ++d) {
                        const double g = dz_i[(size_t)j * cz + d];
                        if (ai >= 0)
                            acc[o_dz1 + ((size_t)ai * r + rho) * cz + d] += g * z2[((size_t)j * r + rho) * cz + d];
                        if (aj >= 0)
                            acc[o_dz2 + ((size_t)aj * r + rho) * cz + d] += g * z1[((size_t)i * r + rho) * cz + d];
                    }
            }
        }
        free(z_i);
        free(dz_i);
        free(s);
        free(a);
        free(D);
        free(da);
        free(dG);
        free(Gacc);
    }
    for (int t = 1; t < nt; ++t)
        for (size_t x = 0; x < n_all; ++x)
            all[x] += all[n_all * (size_t)t + x];
    memcpy(dq, all + o_dq, sizeof(double) * n_sc);
    memcpy(dk, all + o_dk, sizeof(double) * n_sc);
    memcpy(dv, all + o_dv, sizeof(double) * n_sc);
    memcpy(dq_pts, all + o_dqp, sizeof(double) * n_qp);
    memcpy(dk_pts, all + o_dkp, sizeof(double) * n_qp);
    memcpy(dv_pts, all + o_dvp, sizeof(double) * n_vp);
    memcpy(dz1, all + o_dz1, sizeof(double) * n_zf);
    memcpy(dz2, all + o_dz2, sizeof(double) * n_zf);
    memcpy(drot, all + o_drot, sizeof(double) * (size_t)n_s * 9);
    memcpy(dtrans, all + o_dtr, sizeof(double) * (size_t)n_s * 3);
    memcpy(dgamma, all + o_dg, sizeof(double) * (size_t)H);
    memcpy(dw_b, all + o_dwb, sizeof(double) * (size_t)H * cz);
    free(all);
    free(slot);
    return 0;
}
