/*
 * CPU oracle for the ARL^2 hybrid attention step.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain definition of what the GPU library must compute,
 * written out as nested loops in fp64 (plus an all-fp32 twin for the
 * "fp32 throughout" configuration).  It shares no code, header, table or
 * helper with the HIP path and must never be linked into or called from it.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * What is computed, per stream b and head h (paper, Sec. 3.2 and 3.3, Alg. 1):
 *
 *   readout pass (state is read, never written):
 *     s_ij    = sm_scale * <q_i, k_j>                   softmax logits, Eq. (1) scale
 *     O_intra = softmax_j(s_ij) V                       intra-chunk branch, Eq. (2)
 *     q'_i    = q_i / sqrt(|q_i|^2 + eps)               L2Norm part of the feature map, Eq. (3)
 *     O_inter = q'_i S                                  same pre-update S for every token, Eq. (5), Eq. (7)
 *     out_i   = O_intra_i + g_i * O_inter_i             headwise gate broadcast over D, Eq. (6)
 *
 *   commit (once per chunk, after the last denoising pass, Sec. 3.3 "clean-pass update"):
 *     k'_i    = k_i / sqrt(|k_i|^2 + eps)               Eq. (3)
 *     S      <- gate * S + sum_i k'_i^T v_i             Eq. (4) with beta = 1 and the
 *                                                       delta-correction term dropped
 *   commit, delta-rule variant (Eq. (4) literally, frame level):
 *     S      <- alpha * S + beta * K'^T (V - K' S)
 *
 * Layouts (all contiguous, row-major):
 *   q [B][Lq][H][D], k,v [B][Lkv][H][D], g [B][Lq][H], out [B][nrows][H][D],
 *   S [B][H][D][D] indexed S[d_k][d_v], gate [B][H].
 * Inputs q,k,v,g are passed as float: both fp32 and bf16 stored values widen
 * to float exactly, so the oracle sees the very numbers the GPU reads.
 *
 * OpenMP only distributes independent (stream, head, row) triples; it does not
 * change any summation order.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- fp64 -- */

/* One query row i of one (b,h): Eq. (2) + Eq. (3) + Eq. (5) + Eq. (6). */
static void fwd_row_f64(int H, int Lkv, int D,
                        const float *q_row,            /* q[b][i][h][:]              */
                        const float *ql_row,           /* row the inter branch normalises: q_row, or
                                                          RoPE(phi_q(Q)) of Eq. (3) when given apart */
                        const float *k_bh,             /* k[b][0][h][:], stride H*D  */
                        const float *v_bh,             /* v[b][0][h][:], stride H*D  */
                        const double *S_bh,            /* S[b][h] or NULL            */
                        double g_i,                    /* headwise gate of this row, Eq. (6) */
                        const float *g_vec,            /* or one gate per output feature (the element-wise
                                                          granularity of the gate ablation); NULL: g_i */
                        double sm_scale, double l2_eps,
                        double *score,                 /* scratch, Lkv               */
                        double *out_row)               /* D                          */
{
    const size_t ts = (size_t)H * D;                   /* token stride of k and v    */

    /* logits and their maximum */
    double m = -INFINITY;
    for (int j = 0; j < Lkv; ++j) {
        double s = 0.0;
        for (int d = 0; d < D; ++d)
            s += (double)q_row[d] * (double)k_bh[j * ts + d];
        s *= sm_scale;
        score[j] = s;
        if (s > m) m = s;
    }
    /* stable softmax weights and normaliser */
    double Z = 0.0;
    for (int j = 0; j < Lkv; ++j) {
        score[j] = exp(score[j] - m);
        Z += score[j];
    }
    /* intra branch: each out_row[e] accumulates its terms in ascending j */
    for (int e = 0; e < D; ++e)
        out_row[e] = 0.0;
    for (int j = 0; j < Lkv; ++j)
        for (int e = 0; e < D; ++e)
            out_row[e] += score[j] * (double)v_bh[j * ts + e];
    for (int e = 0; e < D; ++e)
        out_row[e] /= Z;
    /* inter branch: normalised query times the shared state */
    if (S_bh) {
        double n2 = 0.0;
        for (int d = 0; d < D; ++d)
            n2 += (double)ql_row[d] * (double)ql_row[d];
        const double nq = sqrt(n2 + l2_eps);
        for (int e = 0; e < D; ++e) {
            double o = 0.0;
            for (int d = 0; d < D; ++d)
                o += ((double)ql_row[d] / nq) * S_bh[(size_t)d * D + e];
            out_row[e] += (g_vec ? (double)g_vec[e] : g_i) * o;
        }
    }
}

/*
 * Readout pass for a list of query rows.  rows == NULL means all Lq rows
 * (nrows must then equal Lq).  out is [B][nrows][H][D].
 * S == NULL: zero state (pure softmax).  g == NULL: gate of one.
 * Returns 0, or -1 on allocation failure.
 */
int arl2o_fwd_ex_f64(int B, int H, int Lq, int Lkv, int D,
                     const float *q, const float *k, const float *v, const float *q_lin,
                     const double *S, const float *g, int g_mode,
                     double sm_scale, double l2_eps,
                     const int32_t *rows, int nrows,
                     double *out);

int arl2o_fwd_f64(int B, int H, int Lq, int Lkv, int D,
                  const float *q, const float *k, const float *v,
                  const double *S, const float *g,
                  double sm_scale, double l2_eps,
                  const int32_t *rows, int nrows,
                  double *out)
{
    return arl2o_fwd_ex_f64(B, H, Lq, Lkv, D, q, k, v, NULL, S, g, 0, sm_scale, l2_eps, rows, nrows, out);
}

/*
 * The same pass with the inter branch's query given apart: q_lin [B][Lq][H][D] holds RoPE(phi_q(Q))
 * of Eq. (3), which the inter branch normalises and multiplies with S (Eq. (5)), while the intra
 * branch keeps q (Eq. (2)).  q_lin == NULL: the inter branch normalises q itself.
 * g_mode selects the gate granularity of the paper's gate ablation: 0 = headwise g [B][Lq][H] (Eq. (6)),
 * 1 = element-wise g [B][Lq][H][D] (one gate per output feature), 2 = scalar g [B][Lq] (one gate per
 * token, shared by the heads).
 */
int arl2o_fwd_ex_f64(int B, int H, int Lq, int Lkv, int D,
                     const float *q, const float *k, const float *v, const float *q_lin,
                     const double *S, const float *g, int g_mode,
                     double sm_scale, double l2_eps,
                     const int32_t *rows, int nrows,
                     double *out)
{
    int fail = 0;
    const long total = (long)B * H * nrows;
#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)(Lkv > 0 ? Lkv : 1));
        if (!score) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 4)
            for (long t = 0; t < total; ++t) {
                const int r = (int)(t % nrows);
                const int h = (int)((t / nrows) % H);
                const int b = (int)(t / ((long)nrows * H));
                const int i = rows ? rows[r] : r;
                const float *q_row = q + (((size_t)b * Lq + i) * H + h) * D;
                const float *k_bh = k + ((size_t)b * Lkv * H + h) * D;
                const float *v_bh = v + ((size_t)b * Lkv * H + h) * D;
                const double *S_bh = S ? S + ((size_t)b * H + h) * D * D : NULL;
                const size_t gi = ((size_t)b * Lq + i) * H + h;
                const double g_i = (g && g_mode == 0) ? (double)g[gi] : (g && g_mode == 2) ? (double)g[(size_t)b * Lq + i] : 1.0;
                const float *g_vec = (g && g_mode == 1) ? g + gi * D : NULL;
                double *out_row = out + (((size_t)b * nrows + r) * H + h) * D;
                const float *ql_row = q_lin ? q_lin + (((size_t)b * Lq + i) * H + h) * D : q_row;
                fwd_row_f64(H, Lkv, D, q_row, ql_row, k_bh, v_bh, S_bh, g_i, g_vec, sm_scale, l2_eps,
                            score, out_row);
            }
        }
        free(score);
    }
    return fail ? -1 : 0;
}

/*
 * Commit: S[b][h] <- gate[b][h] * S[b][h] + sum_i k'_i^T v_i, in place.
 * The gate multiplies the old state only; the new outer products enter un-gated.
 */
int arl2o_commit_f64(int B, int H, int L, int D,
                     const float *k, const float *v, const double *gate,
                     double l2_eps, double *S)
{
    const size_t ts = (size_t)H * D;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            double *S_bh = S + ((size_t)b * H + h) * D * D;
            const float *k_bh = k + ((size_t)b * L * H + h) * D;
            const float *v_bh = v + ((size_t)b * L * H + h) * D;
            /* acc[d][e] = sum_i k'_i[d] * v_i[e]; every element adds its terms in ascending i */
            double *acc = (double *)calloc((size_t)D * D + (size_t)D, sizeof(double));
            if (!acc) {
#pragma omp atomic write
                fail = 1;
                continue;
            }
            double *kp = acc + (size_t)D * D;          /* one normalised key row, Eq. (3) */
            for (int i = 0; i < L; ++i) {
                double n2 = 0.0;
                for (int d = 0; d < D; ++d)
                    n2 += (double)k_bh[i * ts + d] * (double)k_bh[i * ts + d];
                const double nk = sqrt(n2 + l2_eps);
                for (int d = 0; d < D; ++d)
                    kp[d] = (double)k_bh[i * ts + d] / nk;
                for (int d = 0; d < D; ++d)
                    for (int e = 0; e < D; ++e)
                        acc[(size_t)d * D + e] += kp[d] * (double)v_bh[i * ts + e];
            }
            const double a = gate[(size_t)b * H + h];
            for (int d = 0; d < D; ++d)
                for (int e = 0; e < D; ++e)
                    S_bh[(size_t)d * D + e] = a * S_bh[(size_t)d * D + e] + acc[(size_t)d * D + e];
            free(acc);
        }
    }
    return fail ? -1 : 0;
}

/*
 * Frame-level gated delta rule, Eq. (4) taken literally with one (alpha, beta) pair per
 * (stream, head):
 *     S_new = alpha * S_old + beta * K'^T (V - K' S_old)
 * Every token's correction term uses the same pre-update state S_old (frame-level access,
 * Sec. 3.3); the gate multiplies the old state only.  In place.
 */
int arl2o_commit_delta_f64(int B, int H, int L, int D,
                           const float *k, const float *v,
                           const double *alpha, const double *beta,
                           double l2_eps, double *S)
{
    const size_t ts = (size_t)H * D;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            double *S_bh = S + ((size_t)b * H + h) * D * D;
            const float *k_bh = k + ((size_t)b * L * H + h) * D;
            const float *v_bh = v + ((size_t)b * L * H + h) * D;
            /* acc[d][e] = sum_i k'_i[d] * u_i[e],  u_i = v_i - k'_i S_old */
            double *acc = (double *)calloc((size_t)D * D + 2 * (size_t)D, sizeof(double));
            if (!acc) {
#pragma omp atomic write
                fail = 1;
                continue;
            }
            double *kp = acc + (size_t)D * D;          /* normalised key row, Eq. (3) */
            double *u = kp + D;                        /* value minus what the old state predicts */
            for (int i = 0; i < L; ++i) {
                double n2 = 0.0;
                for (int d = 0; d < D; ++d)
                    n2 += (double)k_bh[i * ts + d] * (double)k_bh[i * ts + d];
                const double nk = sqrt(n2 + l2_eps);
                for (int d = 0; d < D; ++d)
                    kp[d] = (double)k_bh[i * ts + d] / nk;
                for (int e = 0; e < D; ++e) {
                    double pred = 0.0;
                    for (int d = 0; d < D; ++d)
                        pred += kp[d] * S_bh[(size_t)d * D + e];
                    u[e] = (double)v_bh[i * ts + e] - pred;
                }
                for (int d = 0; d < D; ++d)
                    for (int e = 0; e < D; ++e)
                        acc[(size_t)d * D + e] += kp[d] * u[e];
            }
            const double a = alpha[(size_t)b * H + h], bt = beta[(size_t)b * H + h];
            for (int d = 0; d < D; ++d)
                for (int e = 0; e < D; ++e)
                    S_bh[(size_t)d * D + e] = a * S_bh[(size_t)d * D + e] + bt * acc[(size_t)d * D + e];
            free(acc);
        }
    }
    return fail ? -1 : 0;
}

/*
 * Token-sequential gated delta rule: Eq. (4) applied to one token at a time, in token order, with
 * per-token gates (Sec. 3.2, the remark after Eq. (4); Alg. 1, clean pass).  For j = 1..L
 *     S_j = alpha_j * S_{j-1} + beta_j * k'_j^T (v_j - k'_j S_{j-1}),
 * the correction of token j reading the state as token j-1 left it.  alpha, beta: [B][L][H].
 * In place: S holds S_L on return.
 */
int arl2o_commit_gdn_f64(int B, int H, int L, int D,
                         const float *k, const float *v,
                         const double *alpha, const double *beta,
                         double l2_eps, double *S)
{
    const size_t ts = (size_t)H * D;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            double *S_bh = S + ((size_t)b * H + h) * D * D;
            const float *k_bh = k + ((size_t)b * L * H + h) * D;
            const float *v_bh = v + ((size_t)b * L * H + h) * D;
            double *kp = (double *)malloc(2 * (size_t)D * sizeof(double));
            if (!kp) {
#pragma omp atomic write
                fail = 1;
                continue;
            }
            double *u = kp + D;
            for (int j = 0; j < L; ++j) {
                const double a = alpha[((size_t)b * L + j) * H + h];
                const double bt = beta[((size_t)b * L + j) * H + h];
                double n2 = 0.0;
                for (int d = 0; d < D; ++d)
                    n2 += (double)k_bh[j * ts + d] * (double)k_bh[j * ts + d];
                const double nk = sqrt(n2 + l2_eps);
                for (int d = 0; d < D; ++d)
                    kp[d] = (double)k_bh[j * ts + d] / nk;
                for (int e = 0; e < D; ++e) {          /* u = v_j - k'_j S_{j-1} */
                    double pred = 0.0;
                    for (int d = 0; d < D; ++d)
                        pred += kp[d] * S_bh[(size_t)d * D + e];
                    u[e] = (double)v_bh[j * ts + e] - pred;
                }
                for (int d = 0; d < D; ++d)
                    for (int e = 0; e < D; ++e)
                        S_bh[(size_t)d * D + e] = a * S_bh[(size_t)d * D + e] + bt * kp[d] * u[e];
            }
            free(kp);
        }
    }
    return fail ? -1 : 0;
}

/*
 * Per-head feature map of Eq. (3) without its L2Norm (the readout and the commits normalise):
 *     y[b][l][h][:] = RoPE_l( W[h] x[b][l][h][:] )
 * W [H][D][D] holds, per head, the D x D matrix of the grouped 1 x 1 map, indexed [out][in].
 * RoPE rotates the pairs (y[2i], y[2i+1]) by the angle whose cosine and sine are cs[l][i], sn[l][i]
 * ([L][D/2]; which positions and frequencies they encode is the caller's choice).  cs == NULL: no
 * rotation (the value map phi_v).
 */
int arl2o_feature_map_f64(int B, int H, int L, int D,
                          const float *x, const float *W,
                          const double *cs, const double *sn,
                          double *y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int l = 0; l < L; ++l) {
            for (int h = 0; h < H; ++h) {
                const float *x_row = x + (((size_t)b * L + l) * H + h) * D;
                double *y_row = y + (((size_t)b * L + l) * H + h) * D;
                const float *W_h = W + (size_t)h * D * D;
                for (int e = 0; e < D; ++e) {
                    double acc = 0.0;
                    for (int d = 0; d < D; ++d)
                        acc += (double)W_h[(size_t)e * D + d] * (double)x_row[d];
                    y_row[e] = acc;
                }
                if (cs) {
                    for (int i = 0; i < D / 2; ++i) {
                        const double c = cs[(size_t)l * (D / 2) + i], s_ = sn[(size_t)l * (D / 2) + i];
                        const double y0 = y_row[2 * i], y1 = y_row[2 * i + 1];
                        y_row[2 * i] = y0 * c - y1 * s_;
                        y_row[2 * i + 1] = y0 * s_ + y1 * c;
                    }
                }
            }
        }
    }
    return 0;
}

/*
 * Headwise branch-mix gate, Eq. (6): G = sigmoid(x W_g), x [B][L][dm] the layer's hidden state
 * (dm = H * D), W_g given per head as Wg[H][dm] (column h of the paper's dm x H matrix), G [B][L][H].
 */
int arl2o_gate_proj_f64(int B, int L, int dm, int H,
                        const float *x, const float *Wg, double *G)
{
#pragma omp parallel for schedule(static)
    for (long t = 0; t < (long)B * L; ++t) {
        const float *x_row = x + (size_t)t * dm;
        for (int h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int j = 0; j < dm; ++j)
                acc += (double)x_row[j] * (double)Wg[(size_t)h * dm + j];
            G[(size_t)t * H + h] = 1.0 / (1.0 + exp(-acc));
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- fp32 -- */
/* The same two definitions with every operation in float: the reference for
 * the configuration that is specified as fp32 throughout.                    */

static void fwd_row_f32(int H, int Lkv, int D,
                        const float *q_row, const float *k_bh, const float *v_bh,
                        const float *S_bh, float g_i, float sm_scale, float l2_eps,
                        float *score, float *out_row)
{
    const size_t ts = (size_t)H * D;
    float m = -INFINITY;
    for (int j = 0; j < Lkv; ++j) {
        float s = 0.0f;
        for (int d = 0; d < D; ++d)
            s += q_row[d] * k_bh[j * ts + d];
        s *= sm_scale;
        score[j] = s;
        if (s > m) m = s;
    }
    float Z = 0.0f;
    for (int j = 0; j < Lkv; ++j) {
        score[j] = expf(score[j] - m);
        Z += score[j];
    }
    for (int e = 0; e < D; ++e)
        out_row[e] = 0.0f;
    for (int j = 0; j < Lkv; ++j)
        for (int e = 0; e < D; ++e)
            out_row[e] += score[j] * v_bh[j * ts + e];
    for (int e = 0; e < D; ++e)
        out_row[e] /= Z;
    if (S_bh) {
        float n2 = 0.0f;
        for (int d = 0; d < D; ++d)
            n2 += q_row[d] * q_row[d];
        const float nq = sqrtf(n2 + l2_eps);
        for (int e = 0; e < D; ++e) {
            float o = 0.0f;
            for (int d = 0; d < D; ++d)
                o += (q_row[d] / nq) * S_bh[(size_t)d * D + e];
            out_row[e] += g_i * o;
        }
    }
}

int arl2o_fwd_f32(int B, int H, int Lq, int Lkv, int D,
                  const float *q, const float *k, const float *v,
                  const float *S, const float *g,
                  float sm_scale, float l2_eps,
                  const int32_t *rows, int nrows,
                  float *out)
{
    int fail = 0;
    const long total = (long)B * H * nrows;
#pragma omp parallel
    {
        float *score = (float *)malloc(sizeof(float) * (size_t)(Lkv > 0 ? Lkv : 1));
        if (!score) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for schedule(dynamic, 4)
            for (long t = 0; t < total; ++t) {
                const int r = (int)(t % nrows);
                const int h = (int)((t / nrows) % H);
                const int b = (int)(t / ((long)nrows * H));
                const int i = rows ? rows[r] : r;
                const float *q_row = q + (((size_t)b * Lq + i) * H + h) * D;
                const float *k_bh = k + ((size_t)b * Lkv * H + h) * D;
                const float *v_bh = v + ((size_t)b * Lkv * H + h) * D;
                const float *S_bh = S ? S + ((size_t)b * H + h) * D * D : NULL;
                const float g_i = g ? g[((size_t)b * Lq + i) * H + h] : 1.0f;
                float *out_row = out + (((size_t)b * nrows + r) * H + h) * D;
                fwd_row_f32(H, Lkv, D, q_row, k_bh, v_bh, S_bh, g_i, sm_scale, l2_eps,
                            score, out_row);
            }
        }
        free(score);
    }
    return fail ? -1 : 0;
}

int arl2o_commit_f32(int B, int H, int L, int D,
                     const float *k, const float *v, const float *gate,
                     float l2_eps, float *S)
{
    const size_t ts = (size_t)H * D;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            float *S_bh = S + ((size_t)b * H + h) * D * D;
            const float *k_bh = k + ((size_t)b * L * H + h) * D;
            const float *v_bh = v + ((size_t)b * L * H + h) * D;
            /* acc[d][e] = sum_i k'_i[d] * v_i[e]; every element adds its terms in ascending i */
            float *acc = (float *)calloc((size_t)D * D + (size_t)D, sizeof(float));
            if (!acc) {
#pragma omp atomic write
                fail = 1;
                continue;
            }
            float *kp = acc + (size_t)D * D;          /* one normalised key row, Eq. (3) */
            for (int i = 0; i < L; ++i) {
                float n2 = 0.0;
                for (int d = 0; d < D; ++d)
                    n2 += (float)k_bh[i * ts + d] * (float)k_bh[i * ts + d];
                const float nk = sqrtf(n2 + l2_eps);
                for (int d = 0; d < D; ++d)
                    kp[d] = (float)k_bh[i * ts + d] / nk;
                for (int d = 0; d < D; ++d)
                    for (int e = 0; e < D; ++e)
                        acc[(size_t)d * D + e] += kp[d] * (float)v_bh[i * ts + e];
            }
            const float a = gate[(size_t)b * H + h];
            for (int d = 0; d < D; ++d)
                for (int e = 0; e < D; ++e)
                    S_bh[(size_t)d * D + e] = a * S_bh[(size_t)d * D + e] + acc[(size_t)d * D + e];
            free(acc);
        }
    }
    return fail ? -1 : 0;
}

int arl2o_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
