/*
 * CPU oracle for one CoCoA round on an L2-regularised generalised linear model.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, double-precision
 * statement of what the GPU library must compute.  It shares no code with that library
 * and is called only by the tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * What the paper fixes (Section 2.2 "CoCoA", Eq. 1 and Eq. 2, Section 5.1 "CoCoA"):
 *   - K workers each solve a local subproblem on their partition D_k from the shared model,
 *     the results are combined into the model of the next iteration;
 *   - the local solver is stochastic coordinate descent with L = 1 (strictly sequential
 *     coordinate steps) and H = number of local samples (one pass per iteration);
 *   - the subproblem parameter sigma equals the number of tasks K.
 * The paper prints no formula for the step, the combination constant or the duality gap; the
 * ones below follow from Fenchel duality of
 *        P(w) = lambda/2 |w|^2 + 1/n sum_i loss_i(x_i . w),
 *        D(a) = -lambda/2 |w(a)|^2 - 1/n sum_i loss_i^*(-a_i),   w(a) = 1/(lambda n) sum_i a_i s_i x_i
 * with   hinge:   loss_i(z) = max(0, 1 - y_i z),  s_i = y_i,  a_i in [0,1],  -loss_i^*(-a_i) = a_i
 *        squared: loss_i(z) = (z - y_i)^2 / 2,     s_i = 1,    a_i real,     loss_i^*(-a_i) = a_i^2/2 - a_i y_i
 *        logistic: loss_i(z) = log(1 + exp(-y_i z)), s_i = y_i,  a_i in [0,1],
 *                  loss_i^*(-a_i) = a_i log a_i + (1 - a_i) log(1 - a_i)   (0 log 0 = 0)
 * (Section 2.2 speaks of generalised linear models in general; the evaluation trains the hinge case.)
 * and the "adding" combination (gamma = 1) that sigma = K makes safe.
 *
 * All state (a, w, v) is double; data (values, labels) are the caller's float arrays.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>

enum { ORACLE_HINGE = 0, ORACLE_SQUARED = 1, ORACLE_LOGISTIC = 2 };

/* One exact coordinate step of the local subproblem.
 * z = x_i . v where v = w + sigma * (Delta w_k so far); q = |x_i|^2; c = lambda n / sigma.
 * Returns the change delta of the dual variable that maximises, over delta,
 *    -1/n loss_i^*(-(a + delta)) - delta s_i z / n - sigma q delta^2 / (2 lambda n^2).          */
static double dual_step(int loss, double a, double y, double z, double q, double c)
{
    if (loss == ORACLE_HINGE) {
        double a_new = a + c * (1.0 - y * z) / q;
        if (a_new < 0.0) a_new = 0.0;
        if (a_new > 1.0) a_new = 1.0;
        return a_new - a;
    }
    if (loss == ORACLE_LOGISTIC) {
        /* a' = a + delta maximises H(a') - (a' - a) y z - (q / 2c) (a' - a)^2 with the entropy
         * H(a') = -a' log a' - (1 - a') log(1 - a').  With a' = 1 / (1 + exp(-s)) the stationarity
         * condition reads f(s) = -s - y z - (q/c) (a'(s) - a) = 0; f decreases strictly and its root
         * lies within q/c of -y z because |a' - a| <= 1.  Plain bisection. */
        const double r = q / c, m = -y * z;
        double lo = m - r, hi = m + r;
        for (int it = 0; it < 200; ++it) {
            const double s = 0.5 * (lo + hi);
            const double ap = s >= 0.0 ? 1.0 / (1.0 + exp(-s)) : exp(s) / (1.0 + exp(s));
            const double f = -s + m - r * (ap - a);
            if (f > 0.0) lo = s; else hi = s;
        }
        const double s = 0.5 * (lo + hi);
        const double ap = s >= 0.0 ? 1.0 / (1.0 + exp(-s)) : exp(s) / (1.0 + exp(s));
        return ap - a;
    }
    return (y - z - a) / (1.0 + q / c);
}

static double xlogx(double x) { return x > 0.0 ? x * log(x) : 0.0; }

/* Local solver of one worker, sparse rows (Section 2.2: sequential coordinate steps, one pass).
 *   rows[t]      global row id of the worker's t-th local row (t = 0 .. n_local-1)
 *   perm[t]      visiting order: the t-th step works on local row perm[t]
 *   row_ptr/col/val  CSR of the whole training set (row_ptr has n_total + 1 entries)
 *   alpha        dual variables of the whole training set, updated in place
 *   v            in: the shared vector w; out: w + sigma * Delta w_k
 */
void oracle_local_epoch_csr(int loss, int64_t n_local, const int64_t *rows, const int32_t *perm,
                            const int64_t *row_ptr, const int32_t *col, const float *val,
                            const float *y, double *alpha, double *v,
                            double lambda, int64_t n_total, double sigma)
{
    const double c = lambda * (double)n_total / sigma;
    for (int64_t t = 0; t < n_local; ++t) {
        const int64_t i = rows[perm[t]];
        const int64_t b = row_ptr[i], e = row_ptr[i + 1];
        double z = 0.0, q = 0.0;
        for (int64_t p = b; p < e; ++p) {
            const double x = (double)val[p];
            z += x * v[col[p]];
            q += x * x;
        }
        if (q == 0.0) continue;
        const double delta = dual_step(loss, alpha[i], (double)y[i], z, q, c);
        alpha[i] += delta;
        const double s = (loss == ORACLE_SQUARED) ? 1.0 : (double)y[i];
        const double coef = delta * s / c;
        for (int64_t p = b; p < e; ++p) v[col[p]] += coef * (double)val[p];
    }
}

/* Same, rows stored densely: X is row-major n_total x d. */
void oracle_local_epoch_dense(int loss, int64_t n_local, const int64_t *rows, const int32_t *perm,
                              const float *X, int64_t d, const float *y, double *alpha, double *v,
                              double lambda, int64_t n_total, double sigma)
{
    const double c = lambda * (double)n_total / sigma;
    for (int64_t t = 0; t < n_local; ++t) {
        const int64_t i = rows[perm[t]];
        const float *x = X + i * d;
        double z = 0.0, q = 0.0;
        for (int64_t j = 0; j < d; ++j) {
            z += (double)x[j] * v[j];
            q += (double)x[j] * (double)x[j];
        }
        if (q == 0.0) continue;
        const double delta = dual_step(loss, alpha[i], (double)y[i], z, q, c);
        alpha[i] += delta;
        const double s = (loss == ORACLE_SQUARED) ? 1.0 : (double)y[i];
        const double coef = delta * s / c;
        for (int64_t j = 0; j < d; ++j) v[j] += coef * (double)x[j];
    }
}

/* Primal value, dual value and their difference at (w, alpha); also the per-row
 * Fenchel-Young form of the gap, which equals P - D whenever w = w(alpha).
 *   out[0] = P, out[1] = D, out[2] = P - D, out[3] = 1/n sum_i g_i
 * with hinge g_i = max(0, 1 - y_i z_i) - a_i + a_i y_i z_i, squared g_i = (z_i - y_i + a_i)^2 / 2 and
 * logistic g_i = log(1 + exp(-y_i z_i)) + a_i log a_i + (1 - a_i) log(1 - a_i) + a_i y_i z_i.
 * Pass X != NULL for dense rows, else the CSR arrays.
 * Elastic-net regulariser lambda (|w|^2 / 2 + l1 |w|_1): w is the soft-thresholded dual image
 * (see oracle_soft_threshold); the conjugate of the regulariser at the dual image is |w|^2 / 2, so only the
 * primal value gains a term. */
void oracle_gap(int loss, int64_t n_total, int64_t d, const float *X, const int64_t *row_ptr,
                const int32_t *col, const float *val, const float *y, const double *alpha,
                const double *w, double lambda, double l1, double *out)
{
    double wsq = 0.0, wabs = 0.0;
    for (int64_t j = 0; j < d; ++j) { wsq += w[j] * w[j]; wabs += fabs(w[j]); }
    double loss_sum = 0.0, conj_sum = 0.0, fy_sum = 0.0;
    for (int64_t i = 0; i < n_total; ++i) {
        double z = 0.0;
        if (X) {
            const float *x = X + i * d;
            for (int64_t j = 0; j < d; ++j) z += (double)x[j] * w[j];
        } else {
            for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) z += (double)val[p] * w[col[p]];
        }
        const double yi = (double)y[i], a = alpha[i];
        if (loss == ORACLE_HINGE) {
            const double h = 1.0 - yi * z;
            const double l = h > 0.0 ? h : 0.0;
            loss_sum += l;
            conj_sum += -a;                      /* loss^*(-a) = -a on [0,1] */
            fy_sum += l - a + a * yi * z;
        } else if (loss == ORACLE_LOGISTIC) {
            const double m = -yi * z;
            const double l = m > 0.0 ? m + log1p(exp(-m)) : log1p(exp(m));
            const double cj = xlogx(a) + xlogx(1.0 - a);
            loss_sum += l;
            conj_sum += cj;
            fy_sum += l + cj + a * yi * z;
        } else {
            const double r = z - yi;
            loss_sum += 0.5 * r * r;
            conj_sum += 0.5 * a * a - a * yi;
            fy_sum += 0.5 * (r + a) * (r + a);
        }
    }
    const double nn = (double)n_total;
    out[0] = lambda * (0.5 * wsq + l1 * wabs) + loss_sum / nn;
    out[1] = -0.5 * lambda * wsq - conj_sum / nn;
    out[2] = out[0] - out[1];
    out[3] = fy_sum / nn;
}

/* Greedy chunk-to-solver assignment on integers (longest processing time first).
 * Chunks are taken by (load descending, id ascending); each goes to the solver that would finish
 * it earliest, (L_k + load) / speed_k, compared exactly by cross-multiplication; ties go to the
 * smallest solver index.  speed == NULL means all speeds equal.  Returns 0, or -1 on bad input. */
int oracle_assign_greedy(const int64_t *load, int32_t n_chunks, int32_t K, const int32_t *speed,
                         int32_t *chunk_to_solver, int32_t *order_scratch, int64_t *L_scratch)
{
    if (K <= 0 || n_chunks < 0) return -1;
    for (int32_t k = 0; k < K; ++k) {
        if (speed && speed[k] <= 0) return -1;
        L_scratch[k] = 0;
    }
    for (int32_t c = 0; c < n_chunks; ++c) order_scratch[c] = c;
    /* insertion sort: plain and stable, so equal loads keep ascending id */
    for (int32_t a = 1; a < n_chunks; ++a) {
        int32_t cur = order_scratch[a];
        int32_t b = a - 1;
        while (b >= 0 && load[order_scratch[b]] < load[cur]) {
            order_scratch[b + 1] = order_scratch[b];
            --b;
        }
        order_scratch[b + 1] = cur;
    }
    for (int32_t o = 0; o < n_chunks; ++o) {
        const int32_t c = order_scratch[o];
        int32_t best = 0;
        for (int32_t k = 1; k < K; ++k) {
            /* (L_k + load)/s_k < (L_best + load)/s_best  <=>  (L_k + load) s_best < (L_best + load) s_k */
            const __int128 lhs = (__int128)(L_scratch[k] + load[c]) * (speed ? speed[best] : 1);
            const __int128 rhs = (__int128)(L_scratch[best] + load[c]) * (speed ? speed[k] : 1);
            if (lhs < rhs) best = k;
        }
        chunk_to_solver[c] = best;
        L_scratch[best] += load[c];
    }
    return 0;
}

/* Elastic net: the primal vector that belongs to a dual image v under the regulariser
 * g(w) = |w|^2 / 2 + l1 |w|_1 is the gradient of g's conjugate, w_j = sign(v_j) max(|v_j| - l1, 0). */
void oracle_soft_threshold(int64_t d, const double *v, double l1, double *w)
{
    for (int64_t j = 0; j < d; ++j) {
        const double a = fabs(v[j]) - l1;
        w[j] = a > 0.0 ? (v[j] > 0.0 ? a : -a) : 0.0;
    }
}

