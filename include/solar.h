/*
 * solar.h -- C ABI of the MI355X (gfx950) SVD-Attention library.
 *
 * SVD-Attention (Section "SVD-Attention" of the SOLAR paper): each user's N x d
 * behaviour-sequence matrix X is given a rank-r truncated SVD, X = U S V^T, and M
 * candidate items attend to the sequence through the factors, so that the cost is
 * O(N d r) instead of the O(N^2 d) of dense softmax attention.
 *
 * Conventions shared by every entry point
 *   - Every array pointer is a DEVICE pointer owned by the caller (for example a
 *     torch tensor's data_ptr()).  The library never allocates or frees device
 *     memory and never synchronizes: all work is enqueued on `stream`, a
 *     hipStream_t passed as void* (NULL = the default stream).
 *   - Arrays are row-major with the last index contiguous and start on a 16-byte
 *     boundary.  B users, N rows per (padded) sequence, d embedding columns, r rank,
 *     M candidates.
 *   - `lengths` ([B] int32, device) holds the number of valid rows of each user;
 *     NULL means every user has N valid rows.  Rows at or past the valid length
 *     are never read as data: they are left out of the factorization and masked
 *     out of every softmax, whatever they contain.
 *   - X and Q have element type `t` (float or bf16 bit patterns); every output
 *     is float.
 *   - Supported shapes: d in {64, 128, 256}; 1 <= r <= min(d, 64) (r <= 32 when
 *     d = 256); N, M, B >= 1.  Anything else returns SOLAR_ERR_UNSUPPORTED.
 *   - Errors: a status code is returned, nothing is printed and nothing aborts.
 *     Arguments are validated on the host before any launch; on an argument
 *     error no kernel runs and the outputs are untouched.  Conditions that only
 *     the device can see (a bad entry of `lengths`, an eigen-iteration that did
 *     not converge) are reported per user through `info`.
 *   - `workspace` is caller-owned device scratch of at least
 *     solar_workspace_bytes(...) bytes, 256-byte aligned.  Its contents are
 *     undefined on return.  Two calls that share a workspace must be ordered on
 *     one stream.
 */
#ifndef SOLAR_H
#define SOLAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SOLAR_OK = 0,
    SOLAR_ERR_INVALID_ARG = 1,
    SOLAR_ERR_UNSUPPORTED = 2,
    SOLAR_ERR_WORKSPACE = 3,
    SOLAR_ERR_HIP = 4,
    SOLAR_ERR_NOT_CONVERGED = 5,  /* never returned by the asynchronous calls (they do not wait for
                                     the device): solar_info_status() derives it from `info` */
    SOLAR_ERR_SCRATCH_LIMIT = 6   /* solar_svd_factorize_static only: see SOLAR_STATIC_SCRATCH_BYTES */
} solar_status;

typedef enum { SOLAR_F32 = 0, SOLAR_BF16 = 1 } solar_dtype;

/* Where the softmax of Attn_SVD sits (the paper's formula omits it; see the
 * operator definitions in Section "SVD-Attention" and the "without Softmax" row
 * of the attention-ablation table). */
typedef enum {
    SOLAR_ATTN_SEQ_SOFTMAX = 0,   /* softmax over the N sequence positions, evaluated in
                                     factor space; equals dense softmax attention when
                                     rank(X) <= r                                          */
    SOLAR_ATTN_EIGEN_SOFTMAX = 1, /* literal form: softmax over the r rows of (V S)^T       */
    SOLAR_ATTN_LINEAR = 2         /* the same without softmax: scale * Q (V S^2 V^T)        */
} solar_attn_mode;

/* Human-readable name of a status code (static string, host memory). */
const char* solar_status_string(solar_status s);

/*
 * Verdict over the per-user `info` array of a factorization, after the caller has waited for
 * the stream and copied `info` to HOST memory: SOLAR_OK if every entry is 0,
 * SOLAR_ERR_INVALID_ARG if any entry is negative (a bad length), else
 * SOLAR_ERR_NOT_CONVERGED (some user's eigen-iteration reached its cap; that user's factors
 * are the best available and finite).
 */
solar_status solar_info_status(const int32_t* info_host, int B);

/*
 * Debug switches, process-wide, for tests that must reach a rarely taken path from the host
 * without an input built to provoke it.  Not for production use; both are off (0) at start.
 *   SOLAR_DEBUG_EIG_MAX_ITER        value > 0 caps the power steps of the eigen-iteration in
 *                                   solar_svd_factorize (users that hit the cap report it in
 *                                   `info`); 0 restores the default cap of 40
 *   SOLAR_DEBUG_FORCE_GUARDED_PASS  nonzero makes the fp16 attention kernel of mode 0 skip its
 *                                   optimistic pass and walk the sequence with the guarded pass
 *                                   (the one that moves the softmax reference) straight away
 */
typedef enum { SOLAR_DEBUG_EIG_MAX_ITER = 0, SOLAR_DEBUG_FORCE_GUARDED_PASS = 1 } solar_debug_key;
solar_status solar_debug_option(solar_debug_key key, int value);

/* Bytes of device scratch that any of the calls below needs for these sizes. */
size_t solar_workspace_bytes(int B, int N, int d, int r, int M, solar_dtype t);

/*
 * Factorization step: rank-r truncated SVD of every user's valid rows
 * (truncated-SVD equation of Section "SVD-Attention"; Algorithm 1, "Randomized
 * SVD with Power Iteration", whose outputs s and R are S and V here).
 *
 * The power iteration Omega <- X^T (X Omega) of Algorithm 1 is applied through
 * the Gram matrix G = X^T X, formed in one pass over X; the subspace iteration
 * and the small decomposition then run on G, one workgroup per user.  U is never
 * formed (Section "SVD-Attention" eliminates it from Key^T Value); the projection
 * P = X V (= U S) is returned instead.
 *
 *   X        in  [B,N,d] of type t
 *   lengths  in  [B] or NULL
 *   S        out [B,r]   singular values, descending
 *   V        out [B,d,r] right singular vectors; each column's largest-magnitude
 *                        entry is positive.
 *                        Resolution: the factors come from the float Gram matrix, whose
 *                        eigenvalues are the squared singular values, so the direction
 *                        of component k is resolved to about 2^-24 (s_1/s_k)^2 (7e-5
 *                        at s_k = 5e-3 s_1); S and the attention outputs stay within
 *                        the 1e-4 contract of the float path for every component that
 *                        is returned.  A component below 3.2e-3 of s_1 (1e-5 of the
 *                        largest eigenvalue of G) is treated as rank deficiency: it
 *                        comes back as S = 0 with a zero column of V, which is how
 *                        the caller sees that it was dropped; the 1e-4 contract then
 *                        holds against the factorization without it.
 *   P        out [B,N,r] = X V, rows at or past the valid length are zero; may be
 *                        NULL if only modes 1 and 2 or solar_svd_attention_from_x
 *                        will be used
 *   info     out [B] or NULL: 0 converged; k > 0 iteration cap reached after k
 *                        steps (results are the best available); -1 bad length
 *                        (not in [r, N]; that user's outputs are zero)
 */
solar_status solar_svd_factorize(const void* X, const int32_t* lengths, int B, int N, int d,
                                 int r, solar_dtype t, float* S, float* V, float* P,
                                 int32_t* info, void* workspace, size_t workspace_bytes,
                                 void* stream);

/*
 * solar_svd_factorize for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * The same kernels run with their scratch (the split-N partial blocks of the Gram contraction
 * and G) in an array built into the library's device code, SOLAR_STATIC_SCRATCH_BYTES long;
 * every device the library is used on holds one copy of it until the process ends.  The call
 * allocates and frees nothing, on the device or through any library.  The array's device address
 * is looked up on the first call made with a given device current; the stream must belong to the
 * current device.
 *   - Arguments, outputs, info and return codes as for solar_svd_factorize, minus the workspace.
 *   - Sizes for which solar_workspace_bytes(B, N, d, r, 0, t) exceeds SOLAR_STATIC_SCRATCH_BYTES
 *     return SOLAR_ERR_SCRATCH_LIMIT; nothing is launched.  (The five benchmark workloads need
 *     0.1 to 42 MB.)
 *   - All calls on one device share that device's array, and it keeps the last call's contents.
 *     Nothing in it has to start at zero (every partial block and G is written before it is
 *     read), so nothing is cleared.  Calls whose work overlaps in time on one device (different
 *     streams, or several host threads) race on it: order them on one stream or with events.
 *   - Per-phase timing (solar_phase_timing_begin) does not cover this call.
 */
#define SOLAR_STATIC_SCRATCH_BYTES (48u * 1024u * 1024u)
solar_status solar_svd_factorize_static(const void* X, const int32_t* lengths, int B, int N, int d,
                                        int r, solar_dtype t, float* S, float* V, float* P,
                                        int32_t* info, void* stream);

/*
 * Attention step, Attn_SVD = MatMul(MatMul(Query, Key_r^T), Value_r) with
 * W_Q = W_K = W_V = I (fold W_Q W_K^T into Q before the call and apply W_V to O
 * after it).
 *
 *   mode 0:  O = softmax_n(scale * (Q V) P^T) P V^T      (needs P, lengths)
 *   mode 1:  O = softmax_k(scale * Q T^T) T,  T = diag(S) V^T   (r <= 64)
 *   mode 2:  O = scale * (Q T^T) T
 *
 *   Q        in  [B,M,d] of type t
 *   S, V, P  in  as written by solar_svd_factorize (P may be NULL for modes 1, 2)
 *   O        out [B,M,d]
 *
 * Mode 0 on bf16 inputs multiplies 16-bit softmax weights on the matrix unit (2e-2 contract).
 * A weight more than 25 log2 units below the softmax reference rounds to zero; the reference
 * sits at most 4 log2 units above the largest score up to N = 16384, 2 up to 65536 and 0 up to
 * 262144 (beyond that, and whenever a score would leave the 16-bit range, the reference follows
 * the running maximum), so a flat tail of N rows loses at most N * 2^-21 ... N * 2^-25 of the
 * softmax mass, under one percent at every N up to 262144 and 1.6 % at 524288.  Longer sequences
 * (and float inputs, S == NULL, r not a multiple of 4) are evaluated in float arithmetic.
 */
solar_status solar_svd_attention(const void* Q, const float* S, const float* V, const float* P,
                                 const int32_t* lengths, int B, int N, int d, int r, int M,
                                 float scale, solar_attn_mode mode, solar_dtype t, float* O,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Mode 0 of the attention step with the projection fused into it: P = X V (Section
 * "SVD-Attention", the product U Sigma that replaces U) is formed tile by tile inside the attention
 * kernel and never written, so solar_svd_factorize can be called with P = NULL:
 *   O = softmax_n(scale * (Q V) (X V)^T) (X V) V^T   over the rows n < lengths[b].
 * Every workgroup of a user repeats that user's projection (ceil(M/256) times in all); the call
 * pays when the factors are used for one candidate set, solar_svd_attention with a stored P when
 * they are used for many.
 *   Q  in [B,M,d] bf16     X  in [B,N,d] bf16     S, V  in  as written by solar_svd_factorize
 *   O  out [B,M,d] float
 * Supported: t = SOLAR_BF16, d in {64, 128, 256}, r a multiple of 4, r <= 64 (r <= 32 when d = 256),
 * N <= 524288; anything else returns SOLAR_ERR_UNSUPPORTED.  No workspace is used.
 */
solar_status solar_svd_attention_from_x(const void* Q, const void* X, const float* S, const float* V,
                                        const int32_t* lengths, int B, int N, int d, int r, int M,
                                        float scale, solar_dtype t, float* O, void* workspace,
                                        size_t workspace_bytes, void* stream);

/*
 * Dense softmax attention over the raw sequence (Preliminaries, Attn_sm with
 * Key = Value = X): O = softmax_n(scale * Q X^T) X over the valid rows.  A
 * straightforward float kernel kept as the on-device reference for what
 * SVD-Attention replaces; it is not tuned.
 */
solar_status solar_dense_attention_ref(const void* Q, const void* X, const int32_t* lengths,
                                       int B, int N, int d, int M, float scale, solar_dtype t,
                                       float* O, void* workspace, size_t workspace_bytes,
                                       void* stream);

/*
 * Linear attention of the Preliminaries, Attn_lin = Query (Key^T Value) with Key = Value = X:
 * O_b = scale * Q_b (X_b^T X_b) over the valid rows of X_b, no softmax.  It is the operator the
 * paper compares against in its forward-latency figure, and what the literal r-token mode
 * (SOLAR_ATTN_LINEAR) truncates to rank r.  Workspace: solar_workspace_bytes(...).
 *   O        out [B,M,d] float
 */
solar_status solar_linear_attention(const void* Q, const void* X, const int32_t* lengths, int B, int N,
                                    int d, int M, float scale, solar_dtype t, float* O,
                                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * The learnable projections of the Preliminaries (Query = C W_Q, Key = H W_K, Value = H W_V)
 * folded around an operator that works on H itself: Out = In * W for every row, W a d x d float
 * matrix shared by all rows.  With Wfold = W_Q W_K^T applied to the candidates before
 * solar_svd_attention and W_V applied to its output, every mode equals the operator with the
 * projections inside, because Key and Value share H.
 *   In       [rows, d]   element type t_in
 *   W        [d, d] float, row-major
 *   Out      [rows, d]   element type t_out (bf16 output is rounded to nearest even)
 */
solar_status solar_apply_weights(const void* In, const float* W, int rows, int d, solar_dtype t_in,
                                 solar_dtype t_out, void* Out, void* stream);

/*
 * Gradient through the truncated SVD with respect to X ("Backward Pass Through SVD", the form
 * with U-bar = 0, U being eliminated from the forward pass):
 *   dX_b = U_b [diag(S_bar_b) + 2 S_b sym(F_b o (V_b^T V_bar_b))] V_b^T,  U_b = P_b S_b^-1,
 * sym(A) = (A + A^T)/2, F_ij = 1/(s_j^2 - s_i^2) for i != j (the orientation confirmed by finite
 * differences; the printed F is its transpose), F_ij = 0 on the diagonal and wherever
 * |s_i^2 - s_j^2| <= gap_rel * s_1^2 (the paper states no guard; pass 0 for none).  Only the part
 * of V_bar inside span(V) contributes (the truncated form of "Backward Pass Through SVD").
 *   S, V, P        from solar_svd_factorize (P is required)
 *   S_bar  in  [B,r]      dL/dS          V_bar  in  [B,d,r]   dL/dV
 *   dX     out [B,N,d] float; rows >= lengths[b] are zero
 * Supported: d in {64, 128, 256}, r in {16, 32, 48, 64}.  Workspace: B*r*d floats
 * (solar_workspace_bytes(...) is enough), 256-byte aligned.
 */
solar_status solar_svd_backward(const float* S, const float* V, const float* P, const float* S_bar,
                                const float* V_bar, int B, int N, int d, int r, float gap_rel,
                                float* dX, void* workspace, size_t workspace_bytes, void* stream);

/*
 * First phase of the factorization on its own, exported so that it can be checked
 * and profiled in isolation: G_b = X_b^T X_b over the valid rows, the contraction
 * over the sequence axis that Algorithm 1's power iteration applies to Omega.
 *   G        out [B,d,d]
 */
solar_status solar_gram(const void* X, const int32_t* lengths, int B, int N, int d,
                        solar_dtype t, float* G, void* workspace, size_t workspace_bytes,
                        void* stream);

/*
 * The factorization by Algorithm 1 ("Randomized SVD with Power Iteration") with the passes
 * over X that it prints, instead of the Gram matrix: Y = X Omega; n_iter times
 * Omega <- X^T Y, Y = X Omega; Q R = Y; s and R = singular values and right singular vectors
 * of Q^T X.  One step is added to the printed ones: after every power step Omega is replaced
 * by an orthonormal basis of its range.  Every output of the algorithm depends on Omega only
 * through that range, so the result is the printed algorithm's; in float arithmetic the
 * printed form loses the trailing directions (cond(X Omega) grows by (s_1/s_r)^2 per power
 * step), this one does not.  The QR step is carried by the Cholesky factor of Y^T Y (Q is
 * never formed: Q^T X = R^-T (X^T Y)^T), the small SVD by a one-sided Jacobi.  X is read
 * 2*n_iter + 2 times (plus once for P).
 *   Omega    in  [B,d,r] float   the Gaussian start blocks (the caller draws them)
 *   n_iter   power iterations, >= 0
 *   S, V, P, info   as for solar_svd_factorize; info[b] = -2 when Y^T Y is not numerically
 *            positive definite (X Omega has fewer than r independent columns: rank(X) < r, or
 *            a degenerate Omega)
 * Supported: d in {64, 128}, r in {16, 32, 48, 64}, r <= d.  Workspace:
 * solar_rsvd_workspace_bytes(B, N, d, r) bytes, 256-byte aligned.
 */
size_t solar_rsvd_workspace_bytes(int B, int N, int d, int r);
solar_status solar_svd_factorize_rsvd(const void* X, const int32_t* lengths, int B, int N, int d,
                                      int r, solar_dtype t, const float* Omega, int n_iter,
                                      float* S, float* V, float* P, int32_t* info,
                                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * Per-phase timing of solar_svd_factorize, for benchmarks.  After
 * solar_phase_timing_begin() every factorize call records HIP
 * events on its stream around its three phases: the Gram contraction, the
 * eigen-iteration and the projection (Algorithm 1's power-iteration product, its
 * basis/small-SVD steps, and P = X V).  solar_phase_timing_end() waits for the
 * last of them, stores the summed milliseconds of each phase in ms_sum[0..2]
 * (HOST memory, may be NULL), switches the timing off and returns the number of
 * calls that were timed.  Not thread-safe; one stream at a time.
 */
void solar_phase_timing_begin(void);
int solar_phase_timing_end(float* ms_sum);

#ifdef __cplusplus
}
#endif
#endif
