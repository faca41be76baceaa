// Host-side launchers of the gfx950 kernels (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace solar {

// api.hip: raises a kernel's limit of dynamic LDS to `bytes`.  The limit is sticky per device
// and kernel, so the runtime is asked only when a launch needs more than was granted before.
hipError_t allow_dynamic_lds(const void* kernel, size_t bytes);
// api.hip: the debug switches of solar_debug_option (0 = off)
int debug_eig_max_iter();
bool debug_force_guarded_pass();

// gram.hip
int gram_nsplit(int B, int N);
size_t gram_partial_floats(int B, int N, int d);
// finalize = false leaves the split-N partial blocks unreduced (G is not written) for a consumer
// that sums them itself; only honoured where gram_partials_consumable(d)
bool gram_partials_consumable(int d);
hipError_t launch_gram(const void* X, const int32_t* lengths, int B, int N, int d, bool bf16,
                       float* partials, float* G, bool finalize, hipStream_t stream);

// eig.hip
struct EigParams {
    float tol_res;      // residual tolerance relative to the largest Ritz value
    float tol_orth;     // a sweep whose largest |cos| is below this ends the Jacobi phase
    int max_iter;       // cap on power steps
    int sweeps;         // cap on Jacobi sweeps per power step
    int mgs_steps;      // leading power steps that use a Gram-Schmidt pass instead of Jacobi
};
EigParams eig_default_params();
int eig_block_columns(int d, int r);
size_t eig_lds_bytes(int d, int r);
// partials != nullptr (with nsplit blocks per user, the layout gram_partial_kernel writes):
// G is not read, the kernel sums the partial blocks itself
hipError_t launch_eig(const float* G, const float* partials, int nsplit, const int32_t* lengths, int B, int N,
                      int d, int r, float* S, float* V, int32_t* info, const EigParams& prm, hipStream_t stream);

// W [B][d][r] <- an orthonormal basis of the range of each user's block (rsvd shapes only)
hipError_t launch_orthonormalize_block(float* W, int B, int d, int r, hipStream_t stream);
hipError_t launch_rsvd_small(const float* W, const float* Gy, const int32_t* lengths, int B, int N, int d,
                             int r, float* S, float* V, int32_t* info, hipStream_t stream);

// rsvd.hip
bool rsvd_supported(int d, int r);
size_t xty_partial_floats(int B, int N, int d, int r);
hipError_t launch_xty(const void* X, const float* Y, const int32_t* lengths, int B, int N, int d, int r,
                      bool bf16, float* partials, float* W, float* Gy, hipStream_t stream);

// project.hip
hipError_t launch_project(const void* X, const int32_t* lengths, const float* V,
                          const int32_t* info, int B, int N, int d, int r, bool bf16, float* P,
                          hipStream_t stream);

// attention.hip
hipError_t launch_attention_seq(const void* Q, const float* V, const float* P,
                                const int32_t* lengths, int B, int N, int d, int r, int M,
                                float scale, bool bf16, float* O, hipStream_t stream);
hipError_t launch_attention_tokens(const void* Q, const float* S, const float* V, int B, int d,
                                   int r, int M, float scale, bool softmax, bool bf16, float* O,
                                   hipStream_t stream);

// attention_x32.hip
bool attention_seq_x32_supported(int d, int r);
bool attention_seq_x32_from_x_supported(int d, int r);
hipError_t launch_attention_seq_x32(const void* Q, const float* S, const float* V, const float* P,
                                    const int32_t* lengths, int B, int N, int d, int r, int M,
                                    float scale, float* O, hipStream_t stream);

// the same kernel with P = X V formed inside it (X and Q bf16)
hipError_t launch_attention_seq_x32_from_x(const void* Q, const float* S, const float* V, const void* X,
                                           const int32_t* lengths, int B, int N, int d, int r, int M,
                                           float scale, float* O, hipStream_t stream);

// linear.hip
hipError_t launch_rowgemm(const void* In, const float* W, size_t w_stride, int B, int rows, int d, float scale,
                          bool in_bf16, bool out_bf16, void* Out, hipStream_t stream);

// backward.hip
bool svd_backward_supported(int d, int r);
hipError_t launch_svd_backward(const float* S, const float* V, const float* P, const float* S_bar,
                               const float* V_bar, int B, int N, int d, int r, float gap_rel, float* Mt,
                               float* dX, hipStream_t stream);

// dense_ref.hip
hipError_t launch_dense_ref(const void* Q, const void* X, const int32_t* lengths, int B, int N,
                            int d, int M, float scale, bool bf16, float* O, hipStream_t stream);

}  // namespace solar
