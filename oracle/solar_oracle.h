/*
 * CPU oracle for SVD-Attention -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * Plain double-precision C with no blocking, fusion or reordering, written so it
 * can be checked against the paper by eye.  It shares no code with the GPU
 * library and must only be used by the tests, the smoke check and the benchmark's
 * CPU-baseline leg.
 *
 * All pointers are HOST pointers owned by the caller.  Arrays are row-major with
 * the last index contiguous.  B users, N rows per (padded) sequence, d embedding
 * columns, r rank, M candidates.  lengths[b] (or N when lengths == NULL) is the
 * number of valid rows of user b; rows past it are ignored everywhere.
 *
 * Every function returns 0 on success and a negative number on invalid
 * arguments; the factorization returns +1 if some user's Jacobi iteration did
 * not converge within the sweep cap (its info[] entry says which).
 */
#ifndef SOLAR_ORACLE_H
#define SOLAR_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Gram matrix of the valid rows, G_b = X_b^T X_b  (the contraction over the
 * sequence axis that the power iteration of Algorithm 1 applies to Omega).
 * G: out [B,d,d]. */
int solar_oracle_gram(const double* X, const int32_t* lengths, int B, int N, int d,
                      double* G);

/* Rank-r truncated SVD of each user's valid rows, X_b = U S V^T with U^T U = I
 * (Section "SVD-Attention", the truncated-SVD equation), computed by the plain
 * one-sided (Hestenes) Jacobi method.  This is the exact object that Algorithm 1
 * (randomized SVD) approximates; its outputs s, R are S and V here.
 *   S      out [B,r]   singular values, descending
 *   V      out [B,d,r] right singular vectors; each column's largest-magnitude
 *                      entry is made positive (lowest index wins ties)
 *   U      out [B,N,r] left singular vectors (rows >= length are zero); may be NULL
 *   S_full out [B,d]   all min(len,d) singular values (zero padded); may be NULL
 *   info   out [B]     number of sweeps used, or -1 if the cap of 60 was hit;
 *                      may be NULL
 */
int solar_oracle_svd_factorize(const double* X, const int32_t* lengths, int B, int N,
                               int d, int r, double* S, double* V, double* U,
                               double* S_full, int32_t* info);

/* SVD-Attention, three readings of the operator Attn_SVD (Section
 * "SVD-Attention", equations for Key_r / Value_r and Attn_SVD), W_Q=W_K=W_V=I:
 *   mode 0: softmax over the sequence axis evaluated on the rank-r projection
 *           X_r = (X V) V^T :  O = softmax_n(scale * Q X_r^T) X_r
 *           (equals dense softmax attention whenever rank(X) <= r)
 *   mode 1: the literal r-token form, T = diag(S) V^T (r x d):
 *           O = softmax_k(scale * Q T^T) T
 *   mode 2: the same without softmax: O = scale * (Q T^T) T
 * Q [B,M,d], X [B,N,d] (mode 0 only; may be NULL otherwise), S [B,r], V [B,d,r],
 * O out [B,M,d].
 */
int solar_oracle_svd_attention(const double* Q, const double* X, const int32_t* lengths,
                               const double* S, const double* V, int B, int N, int d,
                               int r, int M, double scale, int mode, double* O);

/* Dense softmax attention of the candidates over the raw sequence
 * (Preliminaries, Attn_sm with Key = Value = X):
 *   O = softmax_n(scale * Q X^T) X  over the valid rows.  O out [B,M,d]. */
int solar_oracle_dense_attention(const double* Q, const double* X, const int32_t* lengths,
                                 int B, int N, int d, int M, double scale, double* O);

#ifdef __cplusplus
}
#endif
#endif
