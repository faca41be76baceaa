/*
 * CPU oracle for SVD-Attention -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 * See solar_oracle.h for the contract.  Plain loops in double precision.
 */
#include "solar_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#define JACOBI_MAX_SWEEPS 60

static int valid_len(const int32_t* lengths, int b, int N) {
    return lengths ? (int)lengths[b] : N;
}

int solar_oracle_gram(const double* X, const int32_t* lengths, int B, int N, int d,
                      double* G) {
    if (!X || !G || B <= 0 || N <= 0 || d <= 0) return -1;
    for (int b = 0; b < B; ++b) {
        int len = valid_len(lengths, b, N);
        if (len < 0 || len > N) return -2;
        const double* x = X + (size_t)b * N * d;
        double* g = G + (size_t)b * d * d;
        for (int i = 0; i < d; ++i)
            for (int j = 0; j < d; ++j) {
                double acc = 0.0;
                for (int n = 0; n < len; ++n) acc += x[(size_t)n * d + i] * x[(size_t)n * d + j];
                g[(size_t)i * d + j] = acc;
            }
    }
    return 0;
}

/* One-sided Jacobi on the len x d matrix held column by column in a (column j at
 * a + j*len); w (d x d, column j at w + j*d) accumulates the rotations, so that on
 * exit  X w_j = a_j  with the a_j mutually orthogonal.  Returns sweeps used or -1. */
static int hestenes_jacobi(double* a, double* w, int len, int d) {
    const double tol = 2.220446049250313e-16 * sqrt((double)(len > 1 ? len : 1));
    for (int sweep = 1; sweep <= JACOBI_MAX_SWEEPS; ++sweep) {
        int rotations = 0;
        for (int p = 0; p < d - 1; ++p) {
            for (int q = p + 1; q < d; ++q) {
                double* ap = a + (size_t)p * len;
                double* aq = a + (size_t)q * len;
                double alpha = 0.0, beta = 0.0, gamma = 0.0;
                for (int i = 0; i < len; ++i) {
                    alpha += ap[i] * ap[i];
                    beta += aq[i] * aq[i];
                    gamma += ap[i] * aq[i];
                }
                if (alpha == 0.0 || beta == 0.0) continue;
                if (fabs(gamma) <= tol * sqrt(alpha * beta)) continue;
                ++rotations;
                double zeta = (beta - alpha) / (2.0 * gamma);
                double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                double c = 1.0 / sqrt(1.0 + t * t);
                double s = c * t;
                for (int i = 0; i < len; ++i) {
                    double x = ap[i], y = aq[i];
                    ap[i] = c * x - s * y;
                    aq[i] = s * x + c * y;
                }
                double* wp = w + (size_t)p * d;
                double* wq = w + (size_t)q * d;
                for (int i = 0; i < d; ++i) {
                    double x = wp[i], y = wq[i];
                    wp[i] = c * x - s * y;
                    wq[i] = s * x + c * y;
                }
            }
        }
        if (rotations == 0) return sweep;
    }
    return -1;
}

int solar_oracle_svd_factorize(const double* X, const int32_t* lengths, int B, int N,
                               int d, int r, double* S, double* V, double* U,
                               double* S_full, int32_t* info) {
    if (!X || !S || !V || B <= 0 || N <= 0 || d <= 0 || r <= 0 || r > d) return -1;
    int status = 0;
    for (int b = 0; b < B; ++b) {
        int len = valid_len(lengths, b, N);
        if (len < r || len > N) return -2;
        const double* x = X + (size_t)b * N * d;
        double* a = (double*)malloc(sizeof(double) * (size_t)len * d);
        double* w = (double*)calloc((size_t)d * d, sizeof(double));
        double* sig = (double*)malloc(sizeof(double) * d);
        int* order = (int*)malloc(sizeof(int) * d);
        if (!a || !w || !sig || !order) { free(a); free(w); free(sig); free(order); return -3; }
        for (int j = 0; j < d; ++j) {
            for (int i = 0; i < len; ++i) a[(size_t)j * len + i] = x[(size_t)i * d + j];
            w[(size_t)j * d + j] = 1.0;
        }
        int sweeps = hestenes_jacobi(a, w, len, d);
        if (sweeps < 0) status = 1;
        if (info) info[b] = sweeps;
        for (int j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int i = 0; i < len; ++i) acc += a[(size_t)j * len + i] * a[(size_t)j * len + i];
            sig[j] = sqrt(acc);
            order[j] = j;
        }
        /* stable insertion sort, descending singular value */
        for (int i = 1; i < d; ++i) {
            int oi = order[i];
            int k = i - 1;
            while (k >= 0 && sig[order[k]] < sig[oi]) { order[k + 1] = order[k]; --k; }
            order[k + 1] = oi;
        }
        if (S_full) for (int k = 0; k < d; ++k) S_full[(size_t)b * d + k] = sig[order[k]];
        for (int k = 0; k < r; ++k) {
            int j = order[k];
            const double* wj = w + (size_t)j * d;
            int imax = 0;
            for (int i = 1; i < d; ++i) if (fabs(wj[i]) > fabs(wj[imax])) imax = i;
            double sign = (wj[imax] < 0.0) ? -1.0 : 1.0;
            S[(size_t)b * r + k] = sig[j];
            for (int i = 0; i < d; ++i) V[((size_t)b * d + i) * r + k] = sign * wj[i];
            if (U) {
                double inv = sig[j] > 0.0 ? sign / sig[j] : 0.0;
                for (int i = 0; i < len; ++i) U[((size_t)b * N + i) * r + k] = a[(size_t)j * len + i] * inv;
                for (int i = len; i < N; ++i) U[((size_t)b * N + i) * r + k] = 0.0;
            }
        }
        free(a); free(w); free(sig); free(order);
    }
    return status;
}

/* softmax_n(scale * q K^T) K for one query row over len key/value rows. */
static void attend_row(const double* q, const double* kv, int len, int d, double scale,
                       double* scores, double* out) {
    double mx = -INFINITY;
    for (int n = 0; n < len; ++n) {
        double s = 0.0;
        for (int j = 0; j < d; ++j) s += q[j] * kv[(size_t)n * d + j];
        s *= scale;
        scores[n] = s;
        if (s > mx) mx = s;
    }
    double denom = 0.0;
    for (int n = 0; n < len; ++n) { scores[n] = exp(scores[n] - mx); denom += scores[n]; }
    for (int j = 0; j < d; ++j) out[j] = 0.0;
    for (int n = 0; n < len; ++n) {
        double wgt = scores[n] / denom;
        for (int j = 0; j < d; ++j) out[j] += wgt * kv[(size_t)n * d + j];
    }
}

int solar_oracle_dense_attention(const double* Q, const double* X, const int32_t* lengths,
                                 int B, int N, int d, int M, double scale, double* O) {
    if (!Q || !X || !O || B <= 0 || N <= 0 || d <= 0 || M <= 0) return -1;
    double* scores = (double*)malloc(sizeof(double) * N);
    if (!scores) return -3;
    for (int b = 0; b < B; ++b) {
        int len = valid_len(lengths, b, N);
        if (len < 1 || len > N) { free(scores); return -2; }
        for (int m = 0; m < M; ++m)
            attend_row(Q + ((size_t)b * M + m) * d, X + (size_t)b * N * d, len, d, scale,
                       scores, O + ((size_t)b * M + m) * d);
    }
    free(scores);
    return 0;
}

int solar_oracle_svd_attention(const double* Q, const double* X, const int32_t* lengths,
                               const double* S, const double* V, int B, int N, int d,
                               int r, int M, double scale, int mode, double* O) {
    if (!Q || !S || !V || !O || B <= 0 || N <= 0 || d <= 0 || M <= 0 || r <= 0 || r > d) return -1;
    if (mode < 0 || mode > 2) return -1;
    if (mode == 0 && !X) return -1;
    for (int b = 0; b < B; ++b) {
        const double* v = V + (size_t)b * d * r;
        const double* q = Q + (size_t)b * M * d;
        double* o = O + (size_t)b * M * d;
        if (mode == 0) {
            int len = valid_len(lengths, b, N);
            if (len < 1 || len > N) return -2;
            const double* x = X + (size_t)b * N * d;
            /* P = X V (len x r), then X_r = P V^T (len x d), then dense attention on X_r */
            double* p = (double*)malloc(sizeof(double) * (size_t)len * r);
            double* xr = (double*)malloc(sizeof(double) * (size_t)len * d);
            double* scores = (double*)malloc(sizeof(double) * len);
            if (!p || !xr || !scores) { free(p); free(xr); free(scores); return -3; }
            for (int n = 0; n < len; ++n)
                for (int k = 0; k < r; ++k) {
                    double acc = 0.0;
                    for (int j = 0; j < d; ++j) acc += x[(size_t)n * d + j] * v[(size_t)j * r + k];
                    p[(size_t)n * r + k] = acc;
                }
            for (int n = 0; n < len; ++n)
                for (int j = 0; j < d; ++j) {
                    double acc = 0.0;
                    for (int k = 0; k < r; ++k) acc += p[(size_t)n * r + k] * v[(size_t)j * r + k];
                    xr[(size_t)n * d + j] = acc;
                }
            for (int m = 0; m < M; ++m)
                attend_row(q + (size_t)m * d, xr, len, d, scale, scores, o + (size_t)m * d);
            free(p); free(xr); free(scores);
        } else {
            /* T = diag(S) V^T : r eigen-tokens of width d */
            double* t = (double*)malloc(sizeof(double) * (size_t)r * d);
            double* sc = (double*)malloc(sizeof(double) * r);
            if (!t || !sc) { free(t); free(sc); return -3; }
            for (int k = 0; k < r; ++k)
                for (int j = 0; j < d; ++j) t[(size_t)k * d + j] = S[(size_t)b * r + k] * v[(size_t)j * r + k];
            for (int m = 0; m < M; ++m) {
                if (mode == 1) {
                    attend_row(q + (size_t)m * d, t, r, d, scale, sc, o + (size_t)m * d);
                } else {
                    for (int j = 0; j < d; ++j) o[(size_t)m * d + j] = 0.0;
                    for (int k = 0; k < r; ++k) {
                        double s = 0.0;
                        for (int j = 0; j < d; ++j) s += q[(size_t)m * d + j] * t[(size_t)k * d + j];
                        s *= scale;
                        for (int j = 0; j < d; ++j) o[(size_t)m * d + j] += s * t[(size_t)k * d + j];
                    }
                }
            }
            free(t); free(sc);
        }
    }
    return 0;
}
