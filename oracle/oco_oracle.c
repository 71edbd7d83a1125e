/*
 * oco_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, double-precision reference for the online learner of
 * Sec. 3.3: K projected online-gradient-descent base learners (Sec. 3.1
 * update, Assumption 2 domain), a Hedge meta learner over their cumulative
 * losses, and the dynamic regret of Eq. (2) against a piecewise-constant
 * comparator.  It follows the algorithm round by round in the paper's order
 * and notation with plain loops: no blocking, no fusion, no reordering.
 *
 * It shares no code with the GPU library and may be called only from tests,
 * the smoke check and the bench's reported CPU baseline.
 *
 * Readings of the paper taken here (each is listed in the design notes):
 *  - each base learner uses the gradient at ITS OWN iterate w_t^i (Sec. 3.3);
 *  - the Hedge exponent sums f_s(w_s^i) over s < t (the printed f_t inside
 *    the sum over s is read as f_s), so p_1 is uniform and round t's weights
 *    exclude round t's loss;
 *  - the domain is the L2 ball of RADIUS D; the projection rescales only
 *    when the norm exceeds D;
 *  - w_1^i = 0;
 *  - optimistic update (Eq. (3)): hint h_t = gradient of the previous round at
 *    the previously played iterate, h_1 = 0, w^_1 = 0; for K > 1 every learner
 *    runs it independently and Hedge weighs the played iterates;
 *  - optimism at both levels (appendix on combining optimism and ensemble; no
 *    update rule in the paper): base learners as above, Hedge on L_{t-1} + m_t
 *    with the last observed loss as hint m_t (m_1 = 0), no correction term;
 *  - Lemma 1 / Theorem 1: a negative regret is taken as 0.
 * Also here: the accepted-length / acceleration-rate bounds of Lemma 1 and
 * Theorem 1 (closed forms) and the optimistic two-step update of Eq. (3).
 * Every function is pinned by tests that do not call it to produce their
 * expectation (tests/test_oracle_pins.py, tests/test_oracle_pins_next.py),
 * the many-run wrappers and the sparse form of Eq. (3) included.
 *
 * Losses are generalised-linear: f_t(w) = phi(<w, x_t>; y_t), so the
 * gradient is phi'(z; y) x_t.  For the linear loss x_t is the gradient g_t.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { LOSS_LINEAR = 0, LOSS_SQUARED = 1, LOSS_LOGISTIC = 2 };

/* phi(z; y) */
double oco_oracle_loss(int loss, double z, double y)
{
    if (loss == LOSS_LINEAR) return z;
    if (loss == LOSS_SQUARED) return (z - y) * (z - y);
    /* logistic: log(1 + exp(-y z)), written so that exp never overflows */
    double m = y * z;
    return m > 0 ? log1p(exp(-m)) : -m + log1p(exp(m));
}

/* d phi / d z */
double oco_oracle_slope(int loss, double z, double y)
{
    if (loss == LOSS_LINEAR) return 1.0;
    if (loss == LOSS_SQUARED) return 2.0 * (z - y);
    double m = y * z;
    if (m > 0) { double e = exp(-m); return -y * e / (1.0 + e); }
    return -y / (1.0 + exp(m));
}

/* Euclidean projection of v[0..d) onto { ||w||_2 <= D }, in place (Sec. 3.1). */
void oco_oracle_project(double *v, int64_t d, double D)
{
    double s = 0.0;
    for (int64_t j = 0; j < d; ++j) s += v[j] * v[j];
    double nrm = sqrt(s);
    if (nrm > D) {
        double f = D / nrm;
        for (int64_t j = 0; j < d; ++j) v[j] *= f;
    }
}

/* Hedge weights p_i proportional to exp(-eps L_i) (Sec. 3.3), max-shifted. */
void oco_oracle_hedge(const double *L, int64_t K, double eps, double *p)
{
    double m = -eps * L[0];
    for (int64_t i = 1; i < K; ++i) if (-eps * L[i] > m) m = -eps * L[i];
    double s = 0.0;
    for (int64_t i = 0; i < K; ++i) { p[i] = exp(-eps * L[i] - m); s += p[i]; }
    for (int64_t i = 0; i < K; ++i) p[i] /= s;
}

typedef struct {
    /* all optional (NULL to skip); one entry per round */
    double *p;      /* [T][K] weights used at round t                     */
    double *z;      /* [T][K] <w_t^i, x_t>                                */
    double *loss;   /* [T][K] f_t(w_t^i)                                  */
    double *g2;     /* [T][K] ||grad f_t(w_t^i)||^2                       */
    double *f;      /* [T]    f_t(w_t), w_t = sum_i p_t^i w_t^i           */
    double *fu;     /* [T]    f_t(u_t)                                    */
    double *zmix;   /* [T]    sum_i p_t^i z_t^i (must equal <w_t, x_t>)   */
    double *wnorm;  /* [T][K] ||w_{t+1}^i|| after the projection          */
} oco_oracle_trace;

/*
 * One run.  Inputs are the float32 buffers the GPU path consumes, widened to
 * double.  Dense rounds: x[T][d].  Sparse rounds (nnz > 0): col/val[T][nnz],
 * x == NULL; the step touches nnz coordinates, the norm is over all d.
 *   norm_every == 0: the norm of the stepped vector is recomputed over all d
 *                    coordinates every round (the definition);
 *   norm_every  > 0: (sparse only) ||w||^2 is carried forward by adding
 *                    w'_j^2 - w_j^2 over the touched coordinates and is
 *                    recomputed over all d every norm_every rounds; the
 *                    largest relative gap seen at those checks is returned in
 *                    *max_drift.
 * Comparator: u[S][d], segment s active for rounds seg_start[s] <= t <
 * seg_start[s+1] (0-based rounds; the last segment runs to T).
 * Outputs: W[K][d] = w_{T+1}^i, L[K] cumulative losses, p[K] = p_{T+1},
 * wbar[d] = sum_i p_{T+1}^i w_{T+1}^i, *regret = Reg_T.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int oco_oracle_run(int64_t d, int64_t K, int64_t T, double D, const double *eta,
                   double eps, int loss,
                   const float *x, const int32_t *col, const float *val, int64_t nnz,
                   const float *y, const float *u, const int64_t *seg_start, int64_t S,
                   int64_t norm_every,
                   double *W, double *L, double *p, double *wbar, double *regret,
                   double *max_drift, const oco_oracle_trace *tr)
{
    if (d <= 0 || K <= 0 || T < 0 || S <= 0 || !eta || !u || !seg_start) return -1;
    if (nnz > 0 ? (!col || !val) : !x) return -1;
    if (loss != LOSS_LINEAR && !y) return -1;
    if (nnz == 0) norm_every = 0;

    double *z = malloc(sizeof(double) * K), *ell = malloc(sizeof(double) * K);
    double *c = malloc(sizeof(double) * K), *n2 = calloc(K, sizeof(double));
    double *wt = malloc(sizeof(double) * d);      /* the combined iterate w_t */
    double *xt = malloc(sizeof(double) * d);      /* x_t widened (dense rows) */
    if (!z || !ell || !c || !n2 || !wt || !xt) return -1;

    memset(W, 0, sizeof(double) * K * d);
    for (int64_t i = 0; i < K; ++i) L[i] = 0.0;
    double reg = 0.0, drift = 0.0;
    int64_t seg = 0;

    for (int64_t t = 0; t < T; ++t) {
        while (seg + 1 < S && t >= seg_start[seg + 1]) ++seg;
        const float *ut = u + seg * d;
        double yt = y ? (double)y[t] : 0.0;
        const int32_t *ct = nnz ? col + t * nnz : NULL;
        const float *vt = nnz ? val + t * nnz : NULL;

        /* meta weights from the losses of rounds < t */
        oco_oracle_hedge(L, K, eps, p);

        /* predictions of the base learners, their losses and slopes */
        double zu = 0.0, x2 = 0.0;
        if (nnz) {
            for (int64_t i = 0; i < K; ++i) {
                double s = 0.0;
                for (int64_t k = 0; k < nnz; ++k) s += W[i * d + ct[k]] * (double)vt[k];
                z[i] = s;
            }
            for (int64_t k = 0; k < nnz; ++k) {
                zu += (double)ut[ct[k]] * (double)vt[k];
                x2 += (double)vt[k] * (double)vt[k];
            }
        } else {
            for (int64_t j = 0; j < d; ++j) xt[j] = (double)x[t * d + j];
            for (int64_t i = 0; i < K; ++i) {
                double s = 0.0;
                for (int64_t j = 0; j < d; ++j) s += W[i * d + j] * xt[j];
                z[i] = s;
            }
            for (int64_t j = 0; j < d; ++j) { zu += (double)ut[j] * xt[j]; x2 += xt[j] * xt[j]; }
        }
        for (int64_t i = 0; i < K; ++i) {
            ell[i] = oco_oracle_loss(loss, z[i], yt);
            c[i] = oco_oracle_slope(loss, z[i], yt);
        }

        /* the combined iterate w_t = sum_i p_i w_t^i and its loss (Eq. (2)) */
        double zw = 0.0, zmix = 0.0;
        if (nnz) {
            for (int64_t k = 0; k < nnz; ++k) {
                double wj = 0.0;
                for (int64_t i = 0; i < K; ++i) wj += p[i] * W[i * d + ct[k]];
                zw += wj * (double)vt[k];
            }
        } else {
            for (int64_t j = 0; j < d; ++j) {
                double wj = 0.0;
                for (int64_t i = 0; i < K; ++i) wj += p[i] * W[i * d + j];
                wt[j] = wj;
            }
            for (int64_t j = 0; j < d; ++j) zw += wt[j] * xt[j];
        }
        for (int64_t i = 0; i < K; ++i) zmix += p[i] * z[i];
        double ft = oco_oracle_loss(loss, zw, yt);
        double fu = oco_oracle_loss(loss, zu, yt);
        reg += ft - fu;

        if (tr) {
            for (int64_t i = 0; i < K; ++i) {
                if (tr->p) tr->p[t * K + i] = p[i];
                if (tr->z) tr->z[t * K + i] = z[i];
                if (tr->loss) tr->loss[t * K + i] = ell[i];
                if (tr->g2) tr->g2[t * K + i] = c[i] * c[i] * x2;
            }
            if (tr->f) tr->f[t] = ft;
            if (tr->fu) tr->fu[t] = fu;
            if (tr->zmix) tr->zmix[t] = zmix;
        }

        /* gradient step and projection of every base learner */
        for (int64_t i = 0; i < K; ++i) {
            double *w = W + i * d;
            double a = eta[i] * c[i];
            double s2;
            if (nnz) {
                double delta = 0.0;
                for (int64_t k = 0; k < nnz; ++k) {
                    double old = w[ct[k]];
                    double nw = old - a * (double)vt[k];
                    w[ct[k]] = nw;
                    delta += nw * nw - old * old;
                }
                if (norm_every == 0) {
                    s2 = 0.0;
                    for (int64_t j = 0; j < d; ++j) s2 += w[j] * w[j];
                } else {
                    s2 = n2[i] + delta;
                    if ((t + 1) % norm_every == 0) {
                        double full = 0.0;
                        for (int64_t j = 0; j < d; ++j) full += w[j] * w[j];
                        double gap = fabs(full - s2) / (full > 1e-300 ? full : 1e-300);
                        if (full > 0 && gap > drift) drift = gap;
                        s2 = full;
                    }
                }
            } else {
                s2 = 0.0;
                for (int64_t j = 0; j < d; ++j) {
                    w[j] = w[j] - a * xt[j];
                    s2 += w[j] * w[j];
                }
            }
            double nrm = sqrt(s2);
            if (nrm > D) {
                double f = D / nrm;
                for (int64_t j = 0; j < d; ++j) w[j] *= f;
                s2 = D * D;
                nrm = D;
            }
            n2[i] = s2;
            if (tr && tr->wnorm) tr->wnorm[t * K + i] = nrm;
            L[i] += ell[i];
        }
    }

    oco_oracle_hedge(L, K, eps, p);
    for (int64_t j = 0; j < d; ++j) {
        double wj = 0.0;
        for (int64_t i = 0; i < K; ++i) wj += p[i] * W[i * d + j];
        wbar[j] = wj;
    }
    *regret = reg;
    if (max_drift) *max_drift = drift;
    free(z); free(ell); free(c); free(n2); free(wt); free(xt);
    return 0;
}

/*
 * R independent runs, one per thread at a time (OpenMP over runs, nothing
 * else is parallel).  Strides follow the GPU library's input layout:
 * x[T][d] when x_shared else x[R][T][d]; col/val[T][nnz] shared; y[R][T];
 * u[R][S][d].  Outputs W[R][K][d], L[R][K], p[R][K], wbar[R][d], regret[R].
 * Returns the number of runs that failed; *threads_used reports the team size.
 */
int oco_oracle_run_many(int64_t R, int64_t d, int64_t K, int64_t T, double D,
                        const double *eta, double eps, int loss, int x_shared,
                        const float *x, const int32_t *col, const float *val, int64_t nnz,
                        const float *y, const float *u, const int64_t *seg_start, int64_t S,
                        int64_t norm_every, int threads,
                        double *W, double *L, double *p, double *wbar, double *regret,
                        double *max_drift, int *threads_used)
{
    int bad = 0, used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
    if ((int64_t)used > R) used = (int)(R > 0 ? R : 1);
#else
    (void)threads;
#endif
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : bad)
    for (int64_t r = 0; r < R; ++r) {
        const float *xr = x ? (x_shared ? x : x + r * T * d) : NULL;
        double dr = 0.0;
        int rc = oco_oracle_run(d, K, T, D, eta, eps, loss, xr, col, val, nnz,
                                y ? y + r * T : NULL, u + r * S * d, seg_start, S, norm_every,
                                W + r * K * d, L + r * K, p + r * K, wbar + r * d, regret + r,
                                &dr, NULL);
        if (max_drift) max_drift[r] = dr;
        if (rc) bad += 1;
    }
    if (threads_used) *threads_used = used;
    return bad;
}

/*
 * Accepted-length and acceleration-rate bounds (Lemma 1, Theorem 1) for one run
 * with dynamic regret reg over T steps, candidate length k and draft/target
 * inference-time ratio alpha:
 *   out[0] = (k+1) T / (1 + (k+1) sqrt(reg / (2T)))   lower bound on E|x^|
 *   out[1] = (k+1) T                                   upper bound on E|x^|
 *   out[2] = out[0] / (T (alpha k + 1))                lower bound on gamma
 *   out[3] = (k+1) / (alpha k + 1)                     upper bound on gamma
 * Reading: the lemma's regret is a sum of KL divergences, hence >= 0; a
 * negative regret (possible against an arbitrary comparator) is taken as 0.
 */
void oco_oracle_accel_bounds(double reg, int64_t T, int64_t k, double alpha, double *out)
{
    double r = reg > 0.0 ? reg : 0.0;
    double k1 = (double)(k + 1);
    double denom = 1.0 + k1 * sqrt(r / (2.0 * (double)T));
    out[0] = k1 * (double)T / denom;
    out[1] = k1 * (double)T;
    out[2] = out[0] / ((double)T * (alpha * (double)k + 1.0));
    out[3] = k1 / (alpha * (double)k + 1.0);
}

/*
 * Optimistic online gradient descent, Eq. (3), with the last-round gradient as
 * the hint (Sec. 3.2), for K independent learners with steps eta[i] on a dense
 * round stream, combined by the same Hedge meta learner as oco_oracle_run.
 * Per learner:  h_1 = 0, w^_1 = 0;
 *   w_t      = Proj[w^_t - eta h_t]                 (the iterate that is played)
 *   g_t      = phi'(<w_t, x_t>; y_t) x_t            (gradient at the played iterate)
 *   w^_{t+1} = Proj[w^_t - eta g_t],   h_{t+1} = g_t.
 * With K = 1 this is the paper's optimistic update; for K > 1 every learner runs
 * it on its own and Hedge weighs the played iterates by their losses (the paper
 * names optimism inside the ensemble as future work and gives no algorithm).
 * Outputs: W[K][d] = w_{T+1} (played next), What[K][d] = w^_{T+1} (may be NULL),
 * L, p = p_{T+1}, wbar = sum_i p^i w_{T+1}^i, *regret; *delta (may be NULL) is
 * [K] sums of ||h_t - g_t||^2; tr->z / tr->loss / tr->p / tr->f / tr->fu /
 * tr->zmix as in oco_oracle_run (z of the played iterates).
 */
static int run_optimistic_impl(int meta_hint, int64_t d, int64_t K, int64_t T, double D, const double *eta,
                              double eps, int loss, const float *x, const float *y,
                              const float *u, const int64_t *seg_start, int64_t S,
                              double *W, double *What, double *L, double *p, double *wbar,
                              double *regret, double *delta, const oco_oracle_trace *tr)
{
    if (d <= 0 || K <= 0 || T < 0 || S <= 0 || !eta || !u || !seg_start || !x) return -1;
    if (loss != LOSS_LINEAR && !y) return -1;
    double *hat = calloc(K * d, sizeof(double));   /* w^_t */
    double *h = calloc(K * d, sizeof(double));     /* h_t */
    double *z = malloc(sizeof(double) * K), *ell = malloc(sizeof(double) * K);
    double *xt = malloc(sizeof(double) * d), *g = malloc(sizeof(double) * d);
    double *mh = calloc(K, sizeof(double));        /* meta hint m_t: the last observed loss (m_1 = 0) */
    double *Lh = malloc(sizeof(double) * K);       /* L_{t-1} + m_t */
    if (!hat || !h || !z || !ell || !xt || !g || !mh || !Lh) return -1;
    for (int64_t i = 0; i < K; ++i) { L[i] = 0.0; if (delta) delta[i] = 0.0; }
    double reg = 0.0;
    int64_t seg = 0;

    for (int64_t t = 0; t <= T; ++t) {
        /* the iterate to play in round t (for t == T: the state handed back) */
        for (int64_t i = 0; i < K; ++i) {
            double *w = W + i * d;
            for (int64_t j = 0; j < d; ++j) w[j] = hat[i * d + j] - eta[i] * h[i * d + j];
            oco_oracle_project(w, d, D);
        }
        if (t == T) break;
        while (seg + 1 < S && t >= seg_start[seg + 1]) ++seg;
        const float *ut = u + seg * d;
        double yt = y ? (double)y[t] : 0.0;
        for (int64_t j = 0; j < d; ++j) xt[j] = (double)x[t * d + j];
        for (int64_t i = 0; i < K; ++i) Lh[i] = L[i] + (meta_hint ? mh[i] : 0.0);
        oco_oracle_hedge(Lh, K, eps, p);

        double zu = 0.0, zw = 0.0, zmix = 0.0;
        for (int64_t j = 0; j < d; ++j) zu += (double)ut[j] * xt[j];
        for (int64_t i = 0; i < K; ++i) {
            double sdot = 0.0;
            for (int64_t j = 0; j < d; ++j) sdot += W[i * d + j] * xt[j];
            z[i] = sdot;
            ell[i] = oco_oracle_loss(loss, z[i], yt);
            zmix += p[i] * z[i];
        }
        for (int64_t j = 0; j < d; ++j) {
            double wj = 0.0;
            for (int64_t i = 0; i < K; ++i) wj += p[i] * W[i * d + j];
            zw += wj * xt[j];
        }
        double ft = oco_oracle_loss(loss, zw, yt), fu = oco_oracle_loss(loss, zu, yt);
        reg += ft - fu;
        if (tr) {
            for (int64_t i = 0; i < K; ++i) {
                if (tr->p) tr->p[t * K + i] = p[i];
                if (tr->z) tr->z[t * K + i] = z[i];
                if (tr->loss) tr->loss[t * K + i] = ell[i];
            }
            if (tr->f) tr->f[t] = ft;
            if (tr->fu) tr->fu[t] = fu;
            if (tr->zmix) tr->zmix[t] = zmix;
        }
        for (int64_t i = 0; i < K; ++i) {
            double c = oco_oracle_slope(loss, z[i], yt);
            double dsum = 0.0;
            for (int64_t j = 0; j < d; ++j) {
                g[j] = c * xt[j];
                double df = h[i * d + j] - g[j];
                dsum += df * df;
            }
            if (delta) delta[i] += dsum;
            for (int64_t j = 0; j < d; ++j) {
                hat[i * d + j] -= eta[i] * g[j];
                h[i * d + j] = g[j];
            }
            oco_oracle_project(hat + i * d, d, D);
            L[i] += ell[i];
            mh[i] = ell[i];
        }
    }
    for (int64_t i = 0; i < K; ++i) Lh[i] = L[i] + (meta_hint ? mh[i] : 0.0);
    oco_oracle_hedge(Lh, K, eps, p);
    for (int64_t j = 0; j < d; ++j) {
        double wj = 0.0;
        for (int64_t i = 0; i < K; ++i) wj += p[i] * W[i * d + j];
        wbar[j] = wj;
    }
    if (What) memcpy(What, hat, sizeof(double) * K * d);
    *regret = reg;
    free(hat); free(h); free(z); free(ell); free(xt); free(g); free(mh); free(Lh);
    return 0;
}

int oco_oracle_run_optimistic(int64_t d, int64_t K, int64_t T, double D, const double *eta,
                              double eps, int loss, const float *x, const float *y,
                              const float *u, const int64_t *seg_start, int64_t S,
                              double *W, double *What, double *L, double *p, double *wbar,
                              double *regret, double *delta, const oco_oracle_trace *tr)
{
    return run_optimistic_impl(0, d, K, T, D, eta, eps, loss, x, y, u, seg_start, S, W, What, L, p, wbar, regret, delta, tr);
}

/* Optimism at both levels of the ensemble (appendix, "Combining Optimistic Online Learning and
 * Ensemble Learning": base learners and meta learner both optimistic; the paper gives no update
 * rule).  Reading: the base learners run Eq. (3) as above; the meta learner is Hedge on the
 * cumulative losses plus a hint for the coming loss, p_t^i ~ exp(-eps (L_{t-1}^i + m_t^i)), with
 * the last observed loss as hint, m_t^i = f_{t-1}(w_{t-1}^i), m_1 = 0 -- the same reuse of the
 * last feedback that Sec. 3.2 makes for the gradient.  The weights handed back are those of
 * round T + 1.  meta_hint == 0 is oco_oracle_run_optimistic. */
int oco_oracle_run_optimistic_meta(int64_t d, int64_t K, int64_t T, double D, const double *eta,
                                   double eps, int loss, const float *x, const float *y,
                                   const float *u, const int64_t *seg_start, int64_t S,
                                   double *W, double *What, double *L, double *p, double *wbar,
                                   double *regret, double *delta, const oco_oracle_trace *tr, int meta_hint)
{
    return run_optimistic_impl(meta_hint != 0, d, K, T, D, eta, eps, loss, x, y, u, seg_start, S, W, What, L, p, wbar, regret,
                               delta, tr);
}

/*
 * The same optimistic update (Eq. (3), last-gradient hint) on SPARSE rounds:
 * col/val[T][nnz], columns distinct within a round.  The intermediate model w^
 * is kept as a dense double vector per learner; the hint h_t is the previous
 * round's row times that learner's previous slope, so it is held as
 * (column, value) of the previous round plus one slope per learner.
 *   norm_every == 0: the definition.  Every round the played iterate
 *                    w_t = Proj[w^_t - eta h_t] is formed over all d
 *                    coordinates and projected by its recomputed norm, and the
 *                    norm of the stepped w^ is recomputed over all d.
 *   norm_every  > 0: ||w^||^2 is carried forward by adding w'_j^2 - w_j^2 over
 *                    the touched coordinates and recomputed over all d every
 *                    norm_every rounds (largest relative gap -> *max_drift); the
 *                    norm of w^_t - eta h_t is ||w^_t||^2 plus the same kind of
 *                    difference over the hint's coordinates, and the played
 *                    iterate is only evaluated at the coordinates round t reads.
 * Outputs as oco_oracle_run_optimistic.
 */
static int run_optimistic_sparse_impl(int meta_hint, int64_t d, int64_t K, int64_t T, double D, const double *eta,
                                     double eps, int loss, const int32_t *col, const float *val,
                                     int64_t nnz, const float *y, const float *u,
                                     const int64_t *seg_start, int64_t S, int64_t norm_every,
                                     double *W, double *What, double *L, double *p, double *wbar,
                                     double *regret, double *delta, double *max_drift,
                                     const oco_oracle_trace *tr)
{
    if (d <= 0 || K <= 0 || T < 0 || S <= 0 || nnz <= 0 || !eta || !u || !seg_start || !col || !val)
        return -1;
    if (loss != LOSS_LINEAR && !y) return -1;
    double *hat = calloc(K * d, sizeof(double));       /* w^_t, dense */
    double *cprev = calloc(K, sizeof(double));         /* slope of the previous round: h_t = cprev x_{t-1} */
    double *n2 = calloc(K, sizeof(double));            /* carried ||w^_t||^2 */
    double *z = malloc(sizeof(double) * K), *ell = malloc(sizeof(double) * K);
    double *wc = malloc(sizeof(double) * K * nnz);     /* played iterates at round t's columns */
    double *saved = malloc(sizeof(double) * nnz);
    double *tmp = calloc(d, sizeof(double));           /* dense scratch, all zero between uses */
    double *mh = calloc(K, sizeof(double));            /* meta hint m_t: the last observed loss (m_1 = 0) */
    double *Lh = malloc(sizeof(double) * K);           /* L_{t-1} + m_t */
    if (!hat || !cprev || !n2 || !z || !ell || !wc || !saved || !tmp || !mh || !Lh) return -1;
    for (int64_t i = 0; i < K; ++i) { L[i] = 0.0; if (delta) delta[i] = 0.0; }
    double reg = 0.0, drift = 0.0;
    int64_t seg = 0;

    for (int64_t t = 0; t < T; ++t) {
        while (seg + 1 < S && t >= seg_start[seg + 1]) ++seg;
        const float *ut = u + seg * d;
        double yt = y ? (double)y[t] : 0.0;
        const int32_t *ct = col + t * nnz, *cp = t > 0 ? col + (t - 1) * nnz : NULL;
        const float *vt = val + t * nnz, *vp = t > 0 ? val + (t - 1) * nnz : NULL;
        for (int64_t i = 0; i < K; ++i) Lh[i] = L[i] + (meta_hint ? mh[i] : 0.0);
        oco_oracle_hedge(Lh, K, eps, p);

        /* the played iterates w_t^i = Proj[w^_t - eta_i h_t] and their predictions */
        for (int64_t i = 0; i < K; ++i) {
            double *hi = hat + i * d;
            double a = eta[i] * cprev[i];
            double f = 1.0;
            if (norm_every == 0) {
                double *w = W + i * d;
                memcpy(w, hi, sizeof(double) * d);
                if (cp) for (int64_t k = 0; k < nnz; ++k) w[cp[k]] -= a * (double)vp[k];
                oco_oracle_project(w, d, D);
                for (int64_t k = 0; k < nnz; ++k) wc[i * nnz + k] = w[ct[k]];
            } else {
                double m2 = n2[i];
                if (cp) for (int64_t k = 0; k < nnz; ++k) {     /* w^ - eta h, in place for now */
                    saved[k] = hi[cp[k]];
                    double nw = saved[k] - a * (double)vp[k];
                    hi[cp[k]] = nw;
                    m2 += nw * nw - saved[k] * saved[k];
                }
                double nrm = sqrt(m2 > 0.0 ? m2 : 0.0);
                if (nrm > D) f = D / nrm;
                for (int64_t k = 0; k < nnz; ++k) wc[i * nnz + k] = f * hi[ct[k]];
                if (cp) for (int64_t k = 0; k < nnz; ++k) hi[cp[k]] = saved[k];   /* back to w^ */
            }
            double sdot = 0.0;
            for (int64_t k = 0; k < nnz; ++k) sdot += wc[i * nnz + k] * (double)vt[k];
            z[i] = sdot;
            ell[i] = oco_oracle_loss(loss, z[i], yt);
        }
        double zu = 0.0, zw = 0.0, zmix = 0.0;
        for (int64_t k = 0; k < nnz; ++k) {
            zu += (double)ut[ct[k]] * (double)vt[k];
            double wj = 0.0;
            for (int64_t i = 0; i < K; ++i) wj += p[i] * wc[i * nnz + k];
            zw += wj * (double)vt[k];
        }
        for (int64_t i = 0; i < K; ++i) zmix += p[i] * z[i];
        double ft = oco_oracle_loss(loss, zw, yt), fu = oco_oracle_loss(loss, zu, yt);
        reg += ft - fu;
        if (tr) {
            for (int64_t i = 0; i < K; ++i) {
                if (tr->p) tr->p[t * K + i] = p[i];
                if (tr->z) tr->z[t * K + i] = z[i];
                if (tr->loss) tr->loss[t * K + i] = ell[i];
            }
            if (tr->f) tr->f[t] = ft;
            if (tr->fu) tr->fu[t] = fu;
            if (tr->zmix) tr->zmix[t] = zmix;
        }

        /* w^_{t+1} = Proj[w^_t - eta g_t], g_t = c x_t at the played iterate; h_{t+1} = g_t */
        for (int64_t i = 0; i < K; ++i) {
            double *hi = hat + i * d;
            double c = oco_oracle_slope(loss, z[i], yt);
            if (delta) {                                   /* ||h_t - g_t||^2 over the union of columns */
                double dsum = 0.0;
                if (cp) for (int64_t k = 0; k < nnz; ++k) tmp[cp[k]] += cprev[i] * (double)vp[k];
                for (int64_t k = 0; k < nnz; ++k) tmp[ct[k]] -= c * (double)vt[k];
                if (cp) for (int64_t k = 0; k < nnz; ++k) { dsum += tmp[cp[k]] * tmp[cp[k]]; tmp[cp[k]] = 0.0; }
                for (int64_t k = 0; k < nnz; ++k) { dsum += tmp[ct[k]] * tmp[ct[k]]; tmp[ct[k]] = 0.0; }
                delta[i] += dsum;
            }
            double a = eta[i] * c, dl = 0.0, s2;
            for (int64_t k = 0; k < nnz; ++k) {
                double old = hi[ct[k]];
                double nw = old - a * (double)vt[k];
                hi[ct[k]] = nw;
                dl += nw * nw - old * old;
            }
            if (norm_every == 0) {
                s2 = 0.0;
                for (int64_t j = 0; j < d; ++j) s2 += hi[j] * hi[j];
            } else {
                s2 = n2[i] + dl;
                if ((t + 1) % norm_every == 0) {
                    double full = 0.0;
                    for (int64_t j = 0; j < d; ++j) full += hi[j] * hi[j];
                    double gap = fabs(full - s2) / (full > 1e-300 ? full : 1e-300);
                    if (full > 0 && gap > drift) drift = gap;
                    s2 = full;
                }
            }
            double nrm = sqrt(s2 > 0.0 ? s2 : 0.0);
            if (nrm > D) {
                double f = D / nrm;
                for (int64_t j = 0; j < d; ++j) hi[j] *= f;
                s2 = D * D;
            }
            n2[i] = s2;
            cprev[i] = c;
            L[i] += ell[i];
            mh[i] = ell[i];
        }
    }

    /* the iterates that would be played next, formed over all d coordinates */
    for (int64_t i = 0; i < K; ++i) {
        double *w = W + i * d;
        memcpy(w, hat + i * d, sizeof(double) * d);
        if (T > 0) {
            const int32_t *cp = col + (T - 1) * nnz;
            const float *vp = val + (T - 1) * nnz;
            for (int64_t k = 0; k < nnz; ++k) w[cp[k]] -= eta[i] * cprev[i] * (double)vp[k];
        }
        oco_oracle_project(w, d, D);
    }
    for (int64_t i = 0; i < K; ++i) Lh[i] = L[i] + (meta_hint ? mh[i] : 0.0);
    oco_oracle_hedge(Lh, K, eps, p);
    for (int64_t j = 0; j < d; ++j) {
        double wj = 0.0;
        for (int64_t i = 0; i < K; ++i) wj += p[i] * W[i * d + j];
        wbar[j] = wj;
    }
    if (What) memcpy(What, hat, sizeof(double) * K * d);
    *regret = reg;
    if (max_drift) *max_drift = drift;
    free(hat); free(cprev); free(n2); free(z); free(ell); free(wc); free(saved); free(tmp); free(mh); free(Lh);
    return 0;
}

int oco_oracle_run_optimistic_sparse(int64_t d, int64_t K, int64_t T, double D, const double *eta,
                                     double eps, int loss, const int32_t *col, const float *val,
                                     int64_t nnz, const float *y, const float *u,
                                     const int64_t *seg_start, int64_t S, int64_t norm_every,
                                     double *W, double *What, double *L, double *p, double *wbar,
                                     double *regret, double *delta, double *max_drift,
                                     const oco_oracle_trace *tr)
{
    return run_optimistic_sparse_impl(0, d, K, T, D, eta, eps, loss, col, val, nnz, y, u, seg_start, S, norm_every, W, What, L, p,
                                      wbar, regret, delta, max_drift, tr);
}

/* The sparse form with the meta learner's hint (see oco_oracle_run_optimistic_meta). */
int oco_oracle_run_optimistic_sparse_meta(int64_t d, int64_t K, int64_t T, double D, const double *eta,
                                          double eps, int loss, const int32_t *col, const float *val,
                                          int64_t nnz, const float *y, const float *u,
                                          const int64_t *seg_start, int64_t S, int64_t norm_every,
                                          double *W, double *What, double *L, double *p, double *wbar,
                                          double *regret, double *delta, double *max_drift,
                                          const oco_oracle_trace *tr, int meta_hint)
{
    return run_optimistic_sparse_impl(meta_hint != 0, d, K, T, D, eta, eps, loss, col, val, nnz, y, u, seg_start, S, norm_every, W,
                                      What, L, p, wbar, regret, delta, max_drift, tr);
}

/* R independent optimistic runs, one per thread at a time; layout as oco_oracle_run_many
 * (dense x[T][d] shared or x[R][T][d]; or, with nnz > 0, shared col/val[T][nnz] and x == NULL). */
static int run_many_optimistic_impl(int meta_hint, int64_t R, int64_t d, int64_t K, int64_t T, double D,
                                   const double *eta, double eps, int loss, int x_shared,
                                   const float *x, const int32_t *col, const float *val, int64_t nnz,
                                   const float *y, const float *u,
                                   const int64_t *seg_start, int64_t S, int64_t norm_every, int threads,
                                   double *W, double *L, double *p, double *wbar, double *regret,
                                   double *max_drift, int *threads_used)
{
    int bad = 0, used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    used = omp_get_max_threads();
    if ((int64_t)used > R) used = (int)(R > 0 ? R : 1);
#else
    (void)threads;
#endif
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : bad)
    for (int64_t r = 0; r < R; ++r) {
        int rc;
        double dr = 0.0;
        if (nnz > 0)
            rc = run_optimistic_sparse_impl(meta_hint, d, K, T, D, eta, eps, loss, col, val, nnz,
                                                  y ? y + r * T : NULL, u + r * S * d, seg_start, S,
                                                  norm_every, W + r * K * d, NULL, L + r * K, p + r * K,
                                                  wbar + r * d, regret + r, NULL, &dr, NULL);
        else
            rc = run_optimistic_impl(meta_hint, d, K, T, D, eta, eps, loss, x_shared ? x : x + r * T * d,
                                           y ? y + r * T : NULL, u + r * S * d, seg_start, S,
                                           W + r * K * d, NULL, L + r * K, p + r * K, wbar + r * d,
                                           regret + r, NULL, NULL);
        if (max_drift) max_drift[r] = dr;
        if (rc) bad += 1;
    }
    if (threads_used) *threads_used = used;
    return bad;
}

int oco_oracle_run_many_optimistic(int64_t R, int64_t d, int64_t K, int64_t T, double D,
                                   const double *eta, double eps, int loss, int x_shared,
                                   const float *x, const int32_t *col, const float *val, int64_t nnz,
                                   const float *y, const float *u,
                                   const int64_t *seg_start, int64_t S, int64_t norm_every, int threads,
                                   double *W, double *L, double *p, double *wbar, double *regret,
                                   double *max_drift, int *threads_used)
{
    return run_many_optimistic_impl(0, R, d, K, T, D, eta, eps, loss, x_shared, x, col, val, nnz, y, u, seg_start, S, norm_every,
                                    threads, W, L, p, wbar, regret, max_drift, threads_used);
}

/* ... with the meta learner's hint (see oco_oracle_run_optimistic_meta). */
int oco_oracle_run_many_optimistic_meta(int64_t R, int64_t d, int64_t K, int64_t T, double D,
                                        const double *eta, double eps, int loss, int x_shared,
                                        const float *x, const int32_t *col, const float *val, int64_t nnz,
                                        const float *y, const float *u,
                                        const int64_t *seg_start, int64_t S, int64_t norm_every, int threads,
                                        double *W, double *L, double *p, double *wbar, double *regret,
                                        double *max_drift, int *threads_used, int meta_hint)
{
    return run_many_optimistic_impl(meta_hint != 0, R, d, K, T, D, eta, eps, loss, x_shared, x, col, val, nnz, y, u, seg_start, S,
                                    norm_every, threads, W, L, p, wbar, regret, max_drift, threads_used);
}
