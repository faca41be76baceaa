// Dense softmax attention over the raw sequence (Preliminaries, Attn_sm with
// Key = Value = X):  O = softmax_n(scale * Q X^T) X  over the valid rows.
//
// Deliberately plain: float FMA arithmetic on LDS tiles with an online softmax, no
// matrix unit and no tuning.  It is the on-device statement of what SVD-Attention
// replaces and an independent check of the factored kernels.
#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kDM = 16;   // queries per workgroup
constexpr int kDN = 64;   // rows of X per tile

template <bool BF16>
__global__ __launch_bounds__(256) void dense_ref_kernel(
    const void* __restrict__ Qv, const void* __restrict__ Xv, const int32_t* __restrict__ lengths,
    int N, int d, int M, float scale, float* __restrict__ O) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int LDX = d + 1;
    float* qs = smem;                 // [kDM][d]
    float* xs = qs + kDM * d;         // [kDN][LDX]
    float* ws = xs + kDN * LDX;       // [kDM][kDN]
    const int b = blockIdx.y;
    const int m0 = blockIdx.x * kDM;
    const int tid = threadIdx.x;
    const int len = user_len(lengths, b, N);

    auto load_elem = [&](const void* base, size_t idx) -> float {
        if constexpr (BF16)
            return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(base)[idx] << 16);
        else
            return reinterpret_cast<const float*>(base)[idx];
    };

    for (int e = tid; e < kDM * d; e += 256) {
        const int mm = e / d, j = e % d;
        qs[e] = (m0 + mm < M) ? load_elem(Qv, ((size_t)b * M + m0 + mm) * d + j) : 0.f;
    }
    const int mm = tid >> 4;      // query of this thread (16 threads per query)
    const int sub = tid & 15;
    float acc[16];                // output columns sub, sub+16, ... (d <= 256)
#pragma unroll
    for (int c = 0; c < 16; ++c) acc[c] = 0.f;
    float mrun = -INFINITY, lrun = 0.f;
    const float c2 = scale * 1.4426950408889634f;

    for (int n0 = 0; n0 < len; n0 += kDN) {
        __syncthreads();
        for (int e = tid; e < kDN * d; e += 256) {
            const int nn = e / d, j = e % d;
            xs[nn * LDX + j] = (n0 + nn < len) ? load_elem(Xv, ((size_t)b * N + n0 + nn) * d + j) : 0.f;
        }
        __syncthreads();
        float sc[4];
        float mt = -INFINITY;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int nn = sub + 16 * i;
            float s = 0.f;
            for (int j = 0; j < d; ++j) s += qs[mm * d + j] * xs[nn * LDX + j];
            sc[i] = (n0 + nn < len) ? s * c2 : -INFINITY;
            mt = fmaxf(mt, sc[i]);
        }
        for (int msk = 1; msk < 16; msk <<= 1) mt = fmaxf(mt, __shfl_xor(mt, msk));
        const float mnew = fmaxf(mrun, mt);
        const float alpha = exp2f(mrun - mnew);
        mrun = mnew;
        float lsum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float w = exp2f(sc[i] - mnew);
            ws[mm * kDN + sub + 16 * i] = w;
            lsum += w;
        }
        for (int msk = 1; msk < 16; msk <<= 1) lsum += __shfl_xor(lsum, msk);
        lrun = lrun * alpha + lsum;
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const int j = sub + 16 * c;
            if (j < d) {
                float a = acc[c] * alpha;
                for (int nn = 0; nn < kDN; ++nn) a += ws[mm * kDN + nn] * xs[nn * LDX + j];
                acc[c] = a;
            }
        }
    }
    const float inv = lrun > 0.f ? 1.f / lrun : 0.f;
    if (m0 + mm < M) {
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const int j = sub + 16 * c;
            if (j < d) O[((size_t)b * M + m0 + mm) * d + j] = acc[c] * inv;
        }
    }
}

}  // namespace

hipError_t launch_dense_ref(const void* Q, const void* X, const int32_t* lengths, int B, int N,
                            int d, int M, float scale, bool bf16, float* O, hipStream_t stream) {
    if (d > 256) return hipErrorInvalidValue;
    const size_t lds = sizeof(float) * ((size_t)kDM * d + (size_t)kDN * (d + 1) + kDM * kDN);
    dim3 grid(ceil_div(M, kDM), B), block(256);
    if (bf16) {
        auto kern = dense_ref_kernel<true>;
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, Q, X, lengths, N, d, M, scale, O);
    } else {
        auto kern = dense_ref_kernel<false>;
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, Q, X, lengths, N, d, M, scale, O);
    }
    return hipGetLastError();
}

}  // namespace solar
