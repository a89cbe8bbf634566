/*
 * moe_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 CPU statement of what one Mixture-of-Experts layer with
 * top-k gating computes (FastMoE paper, Algorithm 1; Section 2.1 for the score
 * being the combine weight through which the gate is trained; Section 5.1 for
 * the expert being two linear layers d_m x d_h and d_h x d_m; Section 3.2 /
 * Figure "global operations" for counting the samples per expert and laying
 * the expert buffers out from those counts; Section 4 for scatter / gather).
 *
 * It is a literal per-token loop over the chosen experts.  It shares no code,
 * header, table or helper with the HIP library and must never be linked,
 * imported or called by the product path: only tests, the smoke check and the
 * cpu_baseline leg of the benchmark use it.
 *
 * Readings taken where the paper is silent:
 *   - G(x) is one fully-connected layer: l = x W_g + b_g (Section 5.2).
 *   - ArgMax_k ranks the raw logits; equal logits go to the lower expert id;
 *     slot j holds the j-th largest.
 *   - score_i is the softmax over the k selected logits (weights sum to 1); with score_all = 1 it is
 *     the softmax over all E logits taken at the selected experts (Algorithm 1 read literally).
 *   - the expert is W2^T GeLU(W1^T x + b1) + b2 with the exact erf GeLU; the
 *     biases are optional (the paper's expert is "an FFN": two linear layers).
 *   - inside an expert's contiguous segment rows keep assignment order
 *     a = t*k + j (a stable counting sort).
 *   - the backward is the ordinary gradient of L = <dY, Y> with the top-k
 *     indices held constant.
 *
 * Parity pins (tests/test_oracle_*.py): dense FFN for E=1,k=1 (numpy), dense
 * softmax mixture for k=E (scipy), identical experts, hand-worked example in
 * tests/golden, numpy stable argsort for top-k and the permutation, central
 * finite differences for every gradient.  No function here is unpinned.
 *
 * Storage types of the inputs: 0 = IEEE fp32, 1 = bfloat16 (upper 16 bits of an
 * fp32), 2 = fp64.  Every value is widened exactly to double before use; all
 * arithmetic is double, sums run in ascending index order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F64 = 2 };

typedef struct {
    int32_t N, d, h, E, k;
    int32_t dtype;        /* storage of X, Wg, W1, W2, dY                          */
    const void *X;        /* [N, d]                                               */
    const void *Wg;       /* [d, E]                                               */
    const double *bg;     /* [E] or NULL                                          */
    const void *W1;       /* [E, d, h]                                            */
    const void *W2;       /* [E, h, d]                                            */
    const void *dY;       /* [N, d] or NULL (forward only)                        */
    const double *b1;     /* [E, h] expert biases of the first layer, or NULL     */
    const double *b2;     /* [E, d] expert biases of the second layer, or NULL    */
    int32_t score_all;    /* 0: score = softmax over the k selected logits;
                             1: score = softmax over all E logits, taken at the selected experts
                                (Algorithm 1 read literally with G = softmax of the linear layer:
                                the scores of a token then sum to less than 1)           */
} orc_problem;

static inline double ld(const void *p, int dtype, size_t i)
{
    if (dtype == ORC_F64) return ((const double *)p)[i];
    if (dtype == ORC_F32) return (double)((const float *)p)[i];
    uint32_t u = ((uint32_t)((const uint16_t *)p)[i]) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* GeLU(z) = z * Phi(z), Phi the standard normal CDF. */
static inline double gelu(double z) { return 0.5 * z * (1.0 + erf(z * M_SQRT1_2)); }
/* d/dz [z Phi(z)] = Phi(z) + z phi(z). */
static inline double gelu_grad(double z)
{
    return 0.5 * (1.0 + erf(z * M_SQRT1_2)) + z * exp(-0.5 * z * z) * (M_2_SQRTPI * M_SQRT1_2 * 0.5);
}

/* Gate of one token: logits, the k selected experts, their combine weights
 * (Algorithm 1, first two steps). */
static void gate_token(const orc_problem *p, int t, double *logit /*[E]*/, int32_t *idx /*[k]*/,
                       double *w /*[k]*/)
{
    const int d = p->d, E = p->E, k = p->k;
    for (int e = 0; e < E; ++e) {
        double s = p->bg ? p->bg[e] : 0.0;
        for (int i = 0; i < d; ++i)
            s += ld(p->X, p->dtype, (size_t)t * d + i) * ld(p->Wg, p->dtype, (size_t)i * E + e);
        logit[e] = s;
    }
    for (int j = 0; j < k; ++j) {
        int best = -1;
        for (int e = 0; e < E; ++e) {
            int taken = 0;
            for (int q = 0; q < j; ++q) taken |= (idx[q] == e);
            if (taken) continue;
            if (best < 0 || logit[e] > logit[best]) best = e; /* strict: ties keep the lower id */
        }
        idx[j] = best;
    }
    double den = 0.0;
    for (int j = 0; j < k; ++j) {
        w[j] = exp(logit[idx[j]] - logit[idx[0]]);
        den += w[j];
    }
    if (p->score_all) {        /* the normaliser runs over every expert (idx[0] holds the largest logit) */
        den = 0.0;
        for (int e = 0; e < E; ++e) den += exp(logit[e] - logit[idx[0]]);
    }
    for (int j = 0; j < k; ++j) w[j] /= den;
}

/* Gate for every token.  logits may be NULL. */
int orc_gate(const orc_problem *p, double *logits /*[N,E]*/, int32_t *idx /*[N,k]*/, double *w /*[N,k]*/)
{
    if (p->k < 1 || p->k > p->E) return -1;
    int fail = 0;
#pragma omp parallel
    {
        double *l = (double *)malloc(sizeof(double) * (size_t)p->E);
        if (!l) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(static)
        for (int t = 0; t < p->N; ++t) {
            if (!l) continue;
            gate_token(p, t, l, idx + (size_t)t * p->k, w + (size_t)t * p->k);
            if (logits) memcpy(logits + (size_t)t * p->E, l, sizeof(double) * (size_t)p->E);
        }
        free(l);
    }
    return fail ? -2 : 0;
}

/* Counting and buffer layout (Section 3.2: count per expert, then offsets; Section 4:
 * samples of one expert are contiguous).  Literal stable loop over a = t*k + j. */
int orc_plan(int64_t M, int32_t E, const int32_t *idx /*[M]*/, int32_t *counts /*[E]*/,
             int32_t *offsets /*[E+1]*/, int32_t *pos /*[M]*/, int32_t *perm /*[M]*/)
{
    for (int e = 0; e < E; ++e) counts[e] = 0;
    for (int64_t a = 0; a < M; ++a) {
        if (idx[a] < 0 || idx[a] >= E) return -1;
        counts[idx[a]]++;
    }
    offsets[0] = 0;
    for (int e = 0; e < E; ++e) offsets[e + 1] = offsets[e] + counts[e];
    int32_t *seen = (int32_t *)calloc((size_t)(E > 0 ? E : 1), sizeof(int32_t));
    if (!seen) return -2;
    for (int64_t a = 0; a < M; ++a) {
        int e = idx[a];
        pos[a] = offsets[e] + seen[e]++;
        perm[pos[a]] = (int32_t)a;
    }
    free(seen);
    return 0;
}

/*
 * The layer on a list of tokens: Algorithm 1 per token, then its gradient.
 *
 *   tokens[n_tok]      token ids to process, in this order
 *   track[n_track]     expert ids whose weight gradients are wanted (dW1/dW2 rows
 *                      follow this list); NULL with n_track<0 means all experts
 *                      in natural order (dW1 is then [E,d,h])
 *   only_tracked != 0  slots whose expert is not tracked are skipped entirely;
 *                      Y, dX, dWg, dbg, dl are then NOT produced (must be NULL)
 *
 * Outputs (any may be NULL):
 *   Y[n_tok,d], dX[n_tok,d]           rows follow `tokens`
 *   idx[n_tok,k], w[n_tok,k], dl[n_tok,k]
 *   Zo[n_tok,k,h] pre-activation, Oo[n_tok,k,d] expert outputs E_i(x)
 *   Go[n_tok,k,h] GeLU(z), dOo[n_tok,k,d] dL/dE_i(x) = w_i dy, dZo[n_tok,k,h] dL/dz,
 *   dXo[n_tok,k,d] the expert's share of dL/dx (W1 dz): the values the loop holds per slot, copied out
 *   dW1[n_track,d,h], dW2[n_track,h,d] accumulated over the listed tokens (zeroed here)
 *   db1[n_track,h], db2[n_track,d]    likewise, gradients of the expert biases
 *   dWg[d,E], dbg[E]                  accumulated over the listed tokens (zeroed here)
 */
int orc_layer(const orc_problem *p, const int32_t *tokens, int32_t n_tok, const int32_t *track,
              int32_t n_track, int32_t only_tracked, double *Y, double *dX, int32_t *idx_out,
              double *w_out, double *dl_out, double *Zo, double *Oo, double *dW1, double *dW2,
              double *dWg, double *dbg, double *db1, double *db2, double *Go, double *dOo, double *dZo,
              double *dXo)
{
    const int d = p->d, h = p->h, E = p->E, k = p->k, dt = p->dtype;
    if (k < 1 || k > E) return -1;
    const int backward = p->dY != NULL;
    if (only_tracked && (Y || dX || dWg || dbg || dl_out)) return -1;

    /* slot of each expert in the dW arrays, -1 if untracked */
    int32_t *slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    if (!slot) return -2;
    int nslots;
    if (n_track < 0) {
        for (int e = 0; e < E; ++e) slot[e] = e;
        nslots = E;
    } else {
        for (int e = 0; e < E; ++e) slot[e] = -1;
        for (int s = 0; s < n_track; ++s) {
            if (track[s] < 0 || track[s] >= E) { free(slot); return -1; }
            slot[track[s]] = s;
        }
        nslots = n_track;
    }
    const size_t dh = (size_t)d * h;
    if (dW1) memset(dW1, 0, sizeof(double) * dh * (size_t)nslots);
    if (dW2) memset(dW2, 0, sizeof(double) * dh * (size_t)nslots);
    if (db1) memset(db1, 0, sizeof(double) * (size_t)h * (size_t)nslots);
    if (db2) memset(db2, 0, sizeof(double) * (size_t)d * (size_t)nslots);
    if (dWg) memset(dWg, 0, sizeof(double) * (size_t)d * E);
    if (dbg) memset(dbg, 0, sizeof(double) * (size_t)E);

    double *logit = (double *)malloc(sizeof(double) * (size_t)E);
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
    double *w = (double *)malloc(sizeof(double) * (size_t)k);
    double *dw = (double *)malloc(sizeof(double) * (size_t)k);
    double *dl = (double *)malloc(sizeof(double) * (size_t)k);
    double *x = (double *)malloc(sizeof(double) * (size_t)d);
    double *dy = (double *)malloc(sizeof(double) * (size_t)d);
    double *y = (double *)malloc(sizeof(double) * (size_t)d);
    double *dx = (double *)malloc(sizeof(double) * (size_t)d);
    double *dout = (double *)malloc(sizeof(double) * (size_t)d);
    double *z = (double *)malloc(sizeof(double) * (size_t)k * h);   /* z_j  = W1[e_j]^T x      */
    double *g = (double *)malloc(sizeof(double) * (size_t)k * h);   /* g_j  = GeLU(z_j)         */
    double *o = (double *)malloc(sizeof(double) * (size_t)k * d);   /* o_j  = W2[e_j]^T g_j     */
    double *dz = (double *)malloc(sizeof(double) * (size_t)h);
    if (!logit || !idx || !w || !dw || !dl || !x || !dy || !y || !dx || !dout || !z || !g || !o || !dz)
        return -2;

    for (int n = 0; n < n_tok; ++n) {
        const int t = tokens[n];
        if (t < 0 || t >= p->N) return -1;
        for (int i = 0; i < d; ++i) x[i] = ld(p->X, dt, (size_t)t * d + i);
        gate_token(p, t, logit, idx, w);
        if (idx_out) memcpy(idx_out + (size_t)n * k, idx, sizeof(int32_t) * (size_t)k);
        if (w_out) memcpy(w_out + (size_t)n * k, w, sizeof(double) * (size_t)k);

        /* ---- forward: y = sum_j w_j * E_{idx_j}(x)  (Algorithm 1 loop) ---- */
        for (int i = 0; i < d; ++i) y[i] = 0.0;
        for (int j = 0; j < k; ++j) {
            const int e = idx[j];
            if (only_tracked && slot[e] < 0) continue;
            const size_t w1o = (size_t)e * dh, w2o = (size_t)e * dh;
            double *zj = z + (size_t)j * h, *gj = g + (size_t)j * h, *oj = o + (size_t)j * d;
#pragma omp parallel for schedule(static)
            for (int c = 0; c < h; ++c) {
                double s = 0.0;
                for (int i = 0; i < d; ++i) s += x[i] * ld(p->W1, dt, w1o + (size_t)i * h + c);
                if (p->b1) s += p->b1[(size_t)e * h + c];
                zj[c] = s;
                gj[c] = gelu(s);
            }
#pragma omp parallel for schedule(static)
            for (int i = 0; i < d; ++i) {
                double s = 0.0;
                for (int c = 0; c < h; ++c) s += gj[c] * ld(p->W2, dt, w2o + (size_t)c * d + i);
                if (p->b2) s += p->b2[(size_t)e * d + i];
                oj[i] = s;
            }
            for (int i = 0; i < d; ++i) y[i] = w[j] * oj[i] + y[i];
            if (Zo) memcpy(Zo + ((size_t)n * k + j) * h, zj, sizeof(double) * (size_t)h);
            if (Oo) memcpy(Oo + ((size_t)n * k + j) * d, oj, sizeof(double) * (size_t)d);
            if (Go) memcpy(Go + ((size_t)n * k + j) * h, gj, sizeof(double) * (size_t)h);
        }
        if (Y) memcpy(Y + (size_t)n * d, y, sizeof(double) * (size_t)d);
        if (!backward) continue;

        /* ---- backward of L = <dY, Y>, indices constant ---- */
        for (int i = 0; i < d; ++i) dy[i] = ld(p->dY, dt, (size_t)t * d + i);
        for (int i = 0; i < d; ++i) dx[i] = 0.0;
        if (!only_tracked) {
            /* y = sum_j w_j o_j  =>  dL/dw_j = <dy, o_j>; w = softmax(l_sel) =>
             * dL/dl_j = w_j (dw_j - sum_i w_i dw_i). */
            double s = 0.0;
            for (int j = 0; j < k; ++j) {
                double acc = 0.0;
                for (int i = 0; i < d; ++i) acc += dy[i] * o[(size_t)j * d + i];
                dw[j] = acc;
                s += w[j] * acc;
            }
            /* (the same expression serves both score modes: with score_all the w_j are the softmax probabilities
             * p_e of the selected experts, d p_a / d l_b = p_a (delta_ab - p_b), so for a selected expert
             * dL/dl = w_j dw_j - w_j sum_i w_i dw_i; the experts that were not selected follow below) */
            for (int j = 0; j < k; ++j) dl[j] = w[j] * (dw[j] - s);
            if (dl_out) memcpy(dl_out + (size_t)n * k, dl, sizeof(double) * (size_t)k);
            if (p->score_all) {
                /* an expert b that was not selected: dL/dl_b = sum_j dw_j p_j (0 - p_b) = -p_b s */
                const double top = logit[idx[0]];
                double den = 0.0;
                for (int e = 0; e < E; ++e) den += exp(logit[e] - top);
                for (int e = 0; e < E; ++e) {
                    int sel = 0;
                    for (int j = 0; j < k; ++j) sel |= (idx[j] == e);
                    if (sel) continue;
                    const double dle = -(exp(logit[e] - top) / den) * s;
                    if (dbg) dbg[e] += dle;
                    for (int i = 0; i < d; ++i) {
                        if (dWg) dWg[(size_t)i * E + e] += dle * x[i];
                        dx[i] += dle * ld(p->Wg, dt, (size_t)i * E + e);
                    }
                }
            }
            /* l = x Wg + bg */
            for (int j = 0; j < k; ++j) {
                const int e = idx[j];
                if (dbg) dbg[e] += dl[j];
                for (int i = 0; i < d; ++i) {
                    if (dWg) dWg[(size_t)i * E + e] += dl[j] * x[i];
                    dx[i] += dl[j] * ld(p->Wg, dt, (size_t)i * E + e);
                }
            }
        }
        for (int j = 0; j < k; ++j) {
            const int e = idx[j];
            const int s = slot[e];
            if (only_tracked && s < 0) continue;
            const size_t w1o = (size_t)e * dh, w2o = (size_t)e * dh;
            const double *zj = z + (size_t)j * h, *gj = g + (size_t)j * h;
            for (int i = 0; i < d; ++i) dout[i] = w[j] * dy[i];       /* dL/do_j */
            if (dOo) memcpy(dOo + ((size_t)n * k + j) * d, dout, sizeof(double) * (size_t)d);
            if (db2 && s >= 0)                                        /* o = ... + b2 */
                for (int i = 0; i < d; ++i) db2[(size_t)s * d + i] += dout[i];
            /* o = W2^T g : dg = W2 dout ; dW2 += g (x) dout */
#pragma omp parallel for schedule(static)
            for (int c = 0; c < h; ++c) {
                double acc = 0.0;
                for (int i = 0; i < d; ++i) acc += ld(p->W2, dt, w2o + (size_t)c * d + i) * dout[i];
                dz[c] = acc * gelu_grad(zj[c]);                        /* g = GeLU(z) */
                if (dW2 && s >= 0) {
                    double *row = dW2 + (size_t)s * dh + (size_t)c * d;
                    for (int i = 0; i < d; ++i) row[i] += gj[c] * dout[i];
                }
            }
            if (dZo) memcpy(dZo + ((size_t)n * k + j) * h, dz, sizeof(double) * (size_t)h);
            if (db1 && s >= 0)                                        /* z = ... + b1 */
                for (int c = 0; c < h; ++c) db1[(size_t)s * h + c] += dz[c];
            /* z = W1^T x : dW1 += x (x) dz ; dx += W1 dz */
#pragma omp parallel for schedule(static)
            for (int i = 0; i < d; ++i) {
                double acc = 0.0;
                for (int c = 0; c < h; ++c) acc += ld(p->W1, dt, w1o + (size_t)i * h + c) * dz[c];
                dx[i] += acc;
                if (dXo) dXo[((size_t)n * k + j) * d + i] = acc;
                if (dW1 && s >= 0) {
                    double *row = dW1 + (size_t)s * dh + (size_t)i * h;
                    for (int c = 0; c < h; ++c) row[c] += x[i] * dz[c];
                }
            }
        }
        if (dX) memcpy(dX + (size_t)n * d, dx, sizeof(double) * (size_t)d);
    }
    free(slot); free(logit); free(idx); free(w); free(dw); free(dl); free(x); free(dy); free(y);
    free(dx); free(dout); free(z); free(g); free(o); free(dz);
    return 0;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
