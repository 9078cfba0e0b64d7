// Partition-count cost model of Parallax Sec. 3.2 (host code, no device work).
//
//   iter_time(P) = theta0 + theta1 / P + theta2 * P                       (Eq. 1)
// theta0: cost that does not depend on the number of partitions P; theta1: work that
// partitioning parallelises; theta2: per-partition overhead (stitching, bookkeeping).
// The model is fitted to sampled iteration times by least squares.  Samples are taken
// at P = start, 2*start, 4*start, ... until the time goes up, then at start/2, start/4, ...
// until it goes up again; Eq. 1 is convex, so its minimum lies inside the sampled range
// and is read off the fit without extrapolating.
#include <math.h>

#include "px_internal.h"

namespace {

// Solves the 3x3 system a x = b in place (partial pivoting).  False if singular.
bool solve3(double a[3][3], double b[3], double x[3]) {
    for (int c = 0; c < 3; ++c) {
        int piv = c;
        for (int r = c + 1; r < 3; ++r)
            if (fabs(a[r][c]) > fabs(a[piv][c])) piv = r;
        if (fabs(a[piv][c]) < 1e-300) return false;
        for (int k = 0; k < 3; ++k) {
            double t = a[c][k];
            a[c][k] = a[piv][k];
            a[piv][k] = t;
        }
        double t = b[c];
        b[c] = b[piv];
        b[piv] = t;
        for (int r = c + 1; r < 3; ++r) {
            const double f = a[r][c] / a[c][c];
            for (int k = c; k < 3; ++k) a[r][k] -= f * a[c][k];
            b[r] -= f * b[c];
        }
    }
    for (int r = 2; r >= 0; --r) {
        double s = b[r];
        for (int k = r + 1; k < 3; ++k) s -= a[r][k] * x[k];
        x[r] = s / a[r][r];
    }
    return true;
}

double model(const double* theta, double p) { return theta[0] + theta[1] / p + theta[2] * p; }

// Time measured at partition count p, or a negative number if p was not sampled.
double sampled(const double* p, const double* t, int n, double want) {
    for (int i = 0; i < n; ++i)
        if (p[i] == want) return t[i];
    return -1.0;
}

}  // namespace

extern "C" px_status px_partition_cost_fit(const double* p, const double* t, int n, double* theta) {
    if (!p || !t || !theta || n < 3) return PX_ERR_INVALID_ARG;
    // Three parameters need three distinct partition counts: with fewer the normal equations are
    // singular, which round-off can hide from a pivot test, so count them first.
    double seen[3];
    int n_seen = 0;
    for (int i = 0; i < n && n_seen < 3; ++i) {
        if (!(p[i] > 0)) return PX_ERR_INVALID_ARG;
        bool is_new = true;
        for (int j = 0; j < n_seen; ++j)
            if (seen[j] == p[i]) is_new = false;
        if (is_new) seen[n_seen++] = p[i];
    }
    if (n_seen < 3) return PX_ERR_INVALID_ARG;
    double a[3][3] = {{0, 0, 0}, {0, 0, 0}, {0, 0, 0}}, b[3] = {0, 0, 0};
    for (int i = 0; i < n; ++i) {
        if (!(p[i] > 0)) return PX_ERR_INVALID_ARG;
        const double f[3] = {1.0, 1.0 / p[i], p[i]};
        for (int r = 0; r < 3; ++r) {
            for (int c = 0; c < 3; ++c) a[r][c] += f[r] * f[c];
            b[r] += f[r] * t[i];
        }
    }
    return solve3(a, b, theta) ? PX_OK : PX_ERR_INVALID_ARG;      // singular: fewer than 3 distinct P
}

extern "C" px_status px_partition_cost_argmin(const double* theta, int64_t p_lo, int64_t p_hi,
                                              int64_t* best_p, double* best_time) {
    if (!theta || !best_p || p_lo < 1 || p_hi < p_lo) return PX_ERR_INVALID_ARG;
    int64_t cand[4] = {p_lo, p_hi, p_lo, p_lo};
    int n_cand = 2;
    if (theta[1] > 0 && theta[2] > 0) {                            // convex: critical point sqrt(theta1 / theta2)
        const double crit = sqrt(theta[1] / theta[2]);
        const double lo = floor(crit), hi = ceil(crit);
        if (lo >= (double) p_lo && lo <= (double) p_hi) cand[n_cand++] = (int64_t) lo;
        if (hi >= (double) p_lo && hi <= (double) p_hi) cand[n_cand++] = (int64_t) hi;
    }
    int64_t best = cand[0];
    for (int i = 1; i < n_cand; ++i)
        if (model(theta, (double) cand[i]) < model(theta, (double) best)) best = cand[i];
    *best_p = best;
    if (best_time) *best_time = model(theta, (double) best);
    return PX_OK;
}

extern "C" px_status px_partition_search_next(const double* p, const double* t, int n, int64_t p_start,
                                              int64_t p_max, int64_t* next_p) {
    if (!next_p || p_start < 1 || p_max < p_start || n < 0 || (n > 0 && (!p || !t))) return PX_ERR_INVALID_ARG;
    *next_p = 0;
    double prev = sampled(p, t, n, (double) p_start);
    if (prev < 0) {
        *next_p = p_start;
        return PX_OK;
    }
    // upwards: double until the time goes up
    for (int64_t q = p_start * 2; q <= p_max; q *= 2) {
        const double cur = sampled(p, t, n, (double) q);
        if (cur < 0) {
            *next_p = q;
            return PX_OK;
        }
        if (cur > prev) break;
        prev = cur;
    }
    // downwards: halve until the time goes up
    prev = sampled(p, t, n, (double) p_start);
    for (int64_t q = p_start / 2; q >= 1; q /= 2) {
        const double cur = sampled(p, t, n, (double) q);
        if (cur < 0) {
            *next_p = q;
            return PX_OK;
        }
        if (cur > prev) break;
        prev = cur;
    }
    return PX_OK;                                                  // *next_p == 0: sampling is complete
}
