/*
 * CPU oracle for the HGRN2 recurrence (paper Section 3.2, Eq. 3; multi-head variant;
 * Table 4 for the q/k/v/f naming).  TEST INFRASTRUCTURE ONLY: the product path never
 * links, loads or calls anything in this file.  It shares no code with the HIP kernels.
 *
 * Everything is fp64 and follows the defining recurrence one token at a time, per head:
 *
 *     S_t[a][b] = f_t[a] * S_{t-1}[a][b] + k_t[a] * v_t[b],     k_t = 1 - f_t   (tied gate)
 *     o_t[b]    = sum_a q_t[a] * S_t[a][b]                       (reads the UPDATED state)
 *
 * S is the transpose of the paper's h (the paper writes h = h * Diag{f} + i (x) (1-f),
 * y = h * o, so h is indexed [value dim][gate dim]); results are identical.
 * Heads and batch entries are independent recurrences.  There is no chunking, blocking or
 * reordering here: the chunkwise algorithm the GPU uses is an algebraic regrouping of this loop.
 *
 * Layouts (dense, row-major, last index fastest):
 *     q, f : [B][H][N][dk]      v, o : [B][H][N][dv]      h0, hT, state : [B][H][dk][dv]
 *
 * The backward pass is plain reverse-mode differentiation of the loop above (the paper gives
 * none).  It needs S_t and S_{t-1} at every step in reverse order; they come from a forward
 * sweep that stores a checkpoint every CKPT steps and replays the steps inside one block.
 *
 * Pins (tests/test_oracle_pins.py): brute-force quadratic (attention-like) form, f==1 and f==0
 * closed forms, constant-gate closed form, convexity invariant of the tied gate, split/hand-off,
 * linearity, a chunkwise fp64 regrouping, fp64 central finite differences and torch autograd.
 *
 * OpenMP parallelism is over the B*H independent sequences only.
 */
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define CKPT 64

int hgrn2_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One token of Eq. 3 for one head, with an explicit key vector k (tied callers pass 1-f). */
static void step_one(int dk, int dv, const double *q, const double *k, const double *f,
                     const double *v, double *S, double *o)
{
    for (int a = 0; a < dk; ++a) {
        double *row = S + (size_t)a * dv;
        for (int b = 0; b < dv; ++b) row[b] = f[a] * row[b] + k[a] * v[b];
    }
    if (o) {
        for (int b = 0; b < dv; ++b) o[b] = 0.0;
        for (int a = 0; a < dk; ++a) {
            const double *row = S + (size_t)a * dv;
            for (int b = 0; b < dv; ++b) o[b] += q[a] * row[b];
        }
    }
}

static int fwd_impl(int B, int H, int N, int dk, int dv, const double *q, const double *k_or_null,
                    const double *f, const double *v, const double *h0, double *o, double *hT)
{
    if (B < 0 || H < 0 || N < 0 || dk <= 0 || dv <= 0) return 2;
    if ((size_t)B * H * N > 0 && (!q || !f || !v || !o)) return 1;
    const long BH = (long)B * H;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long s = 0; s < BH; ++s) {
        double *S = (double *)malloc(sizeof(double) * dk * dv);
        double *k = (double *)malloc(sizeof(double) * dk);
        if (!S || !k) { fail = 1; free(S); free(k); continue; }
        if (h0) memcpy(S, h0 + (size_t)s * dk * dv, sizeof(double) * dk * dv);
        else    memset(S, 0, sizeof(double) * dk * dv);
        for (int t = 0; t < N; ++t) {
            const double *qt = q + ((size_t)s * N + t) * dk;
            const double *ft = f + ((size_t)s * N + t) * dk;
            const double *vt = v + ((size_t)s * N + t) * dv;
            if (k_or_null) {
                const double *kt = k_or_null + ((size_t)s * N + t) * dk;
                for (int a = 0; a < dk; ++a) k[a] = kt[a];
            } else {
                for (int a = 0; a < dk; ++a) k[a] = 1.0 - ft[a];
            }
            step_one(dk, dv, qt, k, ft, vt, S, o + ((size_t)s * N + t) * dv);
        }
        if (hT) memcpy(hT + (size_t)s * dk * dv, S, sizeof(double) * dk * dv);
        free(S); free(k);
    }
    return fail ? 6 : 0;
}

/* Forward pass, Eq. 3 with the tied input gate k = 1 - f.  h0 and hT may be NULL. */
int hgrn2_oracle_fwd(int B, int H, int N, int dk, int dv, const double *q, const double *f,
                     const double *v, const double *h0, double *o, double *hT)
{
    return fwd_impl(B, H, N, dk, dv, q, NULL, f, v, h0, o, hT);
}

/* Same loop with an independent key (the GLA column of Table 4).  Only used by the pins:
 * with f == 1 it must equal cumulative (causal) linear attention. */
int hgrn2_oracle_fwd_untied(int B, int H, int N, int dk, int dv, const double *q, const double *k,
                            const double *f, const double *v, const double *h0, double *o,
                            double *hT)
{
    if (!k) return 1;
    return fwd_impl(B, H, N, dk, dv, q, k, f, v, h0, o, hT);
}

/* Single-token recurrent step (Eq. 3 once): state is updated in place, o_t uses the new state.
 * q, f : [B][H][dk]   v, o : [B][H][dv]   state : [B][H][dk][dv] */
int hgrn2_oracle_step(int B, int H, int dk, int dv, const double *q, const double *f,
                      const double *v, double *state, double *o)
{
    if (B < 0 || H < 0 || dk <= 0 || dv <= 0) return 2;
    if ((size_t)B * H > 0 && (!q || !f || !v || !state || !o)) return 1;
    const long BH = (long)B * H;
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (long s = 0; s < BH; ++s) {
        double *k = (double *)malloc(sizeof(double) * dk);
        if (!k) { fail = 1; continue; }
        for (int a = 0; a < dk; ++a) k[a] = 1.0 - f[(size_t)s * dk + a];
        step_one(dk, dv, q + (size_t)s * dk, k, f + (size_t)s * dk, v + (size_t)s * dv,
                 state + (size_t)s * dk * dv, o + (size_t)s * dv);
        free(k);
    }
    return fail ? 6 : 0;
}

/* T consecutive single-token steps for the decode benchmark layout: tokens are
 * q, f : [T][B][H][dk], v, o : [T][B][H][dv].  Sequence-outer / token-inner so that one head's
 * state stays in cache; the arithmetic per token is exactly step_one. */
int hgrn2_oracle_steps(int T, int B, int H, int dk, int dv, const double *q, const double *f,
                       const double *v, double *state, double *o)
{
    if (T < 0 || B < 0 || H < 0 || dk <= 0 || dv <= 0) return 2;
    if ((size_t)T * B * H > 0 && (!q || !f || !v || !state || !o)) return 1;
    const long BH = (long)B * H;
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (long s = 0; s < BH; ++s) {
        double *k = (double *)malloc(sizeof(double) * dk);
        if (!k) { fail = 1; continue; }
        for (int t = 0; t < T; ++t) {
            const size_t r = (size_t)t * BH + s;
            for (int a = 0; a < dk; ++a) k[a] = 1.0 - f[r * dk + a];
            step_one(dk, dv, q + r * dk, k, f + r * dk, v + r * dv,
                     state + (size_t)s * dk * dv, o + r * dv);
        }
        free(k);
    }
    return fail ? 6 : 0;
}

/*
 * Backward pass: reverse-mode of the forward loop.  Given dO (and optionally dhT, the gradient
 * flowing into the final state), with dS the running gradient w.r.t. the state:
 *
 *     for t = N .. 1:
 *         dS     += q_t (x) do_t                          now dS = dL/dS_t
 *         dq_t[a] = sum_b S_t[a][b]   * do_t[b]
 *         dk_t[a] = sum_b dS[a][b]    * v_t[b]            gradient w.r.t. k_t as a free variable
 *         dv_t[b] = sum_a k_t[a]      * dS[a][b]
 *         dd_t[a] = sum_b dS[a][b]    * S_{t-1}[a][b]     gradient through the decay f_t * S_{t-1}
 *         df_t    = dd_t - dk_t                           because k_t = 1 - f_t
 *         dS      = Diag(f_t) dS                          now dS = dL/dS_{t-1} via the decay
 *     dh0 = dS
 *
 * dhT, dh0 and h0 may be NULL.
 */
int hgrn2_oracle_bwd(int B, int H, int N, int dk, int dv, const double *q, const double *f,
                     const double *v, const double *h0, const double *dO, const double *dhT,
                     double *dq, double *df, double *dvv, double *dh0)
{
    if (B < 0 || H < 0 || N < 0 || dk <= 0 || dv <= 0) return 2;
    if ((size_t)B * H * N > 0 && (!q || !f || !v || !dO || !dq || !df || !dvv)) return 1;
    const long BH = (long)B * H;
    const size_t SS = (size_t)dk * dv;
    const int nblk = (N + CKPT - 1) / CKPT;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long s = 0; s < BH; ++s) {
        /* ck[j] = state before token j*CKPT;  blk[i] = state before token (base + i), i = 0..len */
        double *ck  = (double *)malloc(sizeof(double) * SS * (size_t)(nblk + 1));
        double *blk = (double *)malloc(sizeof(double) * SS * (size_t)(CKPT + 1));
        double *dS  = (double *)malloc(sizeof(double) * SS);
        double *k   = (double *)malloc(sizeof(double) * dk);
        if (!ck || !blk || !dS || !k) { fail = 1; free(ck); free(blk); free(dS); free(k); continue; }

        if (h0) memcpy(ck, h0 + (size_t)s * SS, sizeof(double) * SS);
        else    memset(ck, 0, sizeof(double) * SS);
        for (int j = 0; j < nblk; ++j) {
            double *S = ck + SS * (size_t)(j + 1);
            memcpy(S, ck + SS * (size_t)j, sizeof(double) * SS);
            const int t1 = (j + 1) * CKPT < N ? (j + 1) * CKPT : N;
            for (int t = j * CKPT; t < t1; ++t) {
                const double *ft = f + ((size_t)s * N + t) * dk;
                for (int a = 0; a < dk; ++a) k[a] = 1.0 - ft[a];
                step_one(dk, dv, NULL, k, ft, v + ((size_t)s * N + t) * dv, S, NULL);
            }
        }

        if (dhT) memcpy(dS, dhT + (size_t)s * SS, sizeof(double) * SS);
        else     memset(dS, 0, sizeof(double) * SS);

        for (int j = nblk - 1; j >= 0; --j) {
            const int base = j * CKPT;
            const int len = (base + CKPT < N ? base + CKPT : N) - base;
            memcpy(blk, ck + SS * (size_t)j, sizeof(double) * SS);
            for (int i = 0; i < len; ++i) {
                double *S = blk + SS * (size_t)(i + 1);
                memcpy(S, blk + SS * (size_t)i, sizeof(double) * SS);
                const double *ft = f + ((size_t)s * N + base + i) * dk;
                for (int a = 0; a < dk; ++a) k[a] = 1.0 - ft[a];
                step_one(dk, dv, NULL, k, ft, v + ((size_t)s * N + base + i) * dv, S, NULL);
            }
            for (int i = len - 1; i >= 0; --i) {
                const size_t r = (size_t)s * N + base + i;
                const double *qt = q + r * dk, *ft = f + r * dk, *vt = v + r * dv, *dot = dO + r * dv;
                const double *St = blk + SS * (size_t)(i + 1);   /* S_t     */
                const double *Sp = blk + SS * (size_t)i;         /* S_{t-1} */
                for (int a = 0; a < dk; ++a) {
                    double *dSa = dS + (size_t)a * dv;
                    const double *Sta = St + (size_t)a * dv, *Spa = Sp + (size_t)a * dv;
                    double gq = 0.0, gk = 0.0, gd = 0.0;
                    for (int b = 0; b < dv; ++b) {
                        dSa[b] += qt[a] * dot[b];
                        gq += Sta[b] * dot[b];
                        gk += dSa[b] * vt[b];
                        gd += dSa[b] * Spa[b];
                    }
                    dq[r * dk + a] = gq;
                    df[r * dk + a] = gd - gk;
                }
                for (int b = 0; b < dv; ++b) {
                    double g = 0.0;
                    for (int a = 0; a < dk; ++a) g += (1.0 - ft[a]) * dS[(size_t)a * dv + b];
                    dvv[r * dv + b] = g;
                }
                for (int a = 0; a < dk; ++a) {
                    double *dSa = dS + (size_t)a * dv;
                    for (int b = 0; b < dv; ++b) dSa[b] *= ft[a];
                }
            }
        }
        if (dh0) memcpy(dh0 + (size_t)s * SS, dS, sizeof(double) * SS);
        free(ck); free(blk); free(dS); free(k);
    }
    return fail ? 6 : 0;
}
