// Row-times-matrix products around the attention operators:
//   * linear attention Attn_lin = Query (Key^T Value) (Preliminaries) with Key = Value = X:
//     O_b = scale * Q_b G_b, G_b = X_b^T X_b from the Gram kernel;
//   * the learnable projections W_Q, W_K, W_V of the Preliminaries, folded around an operator
//     that works on H itself: Q' = C (W_Q W_K^T) before it and O' = O W_V after it.
// Both are Out[rows x d] = scale * In[rows x d] * W[d x d] with a float matrix W (per user or
// shared) held in LDS and the float 16x16x4 MFMA (G has the dynamic range of squared singular
// values; the products are tiny next to the attention itself).  A wave owns 16 rows; its A
// operand is a contiguous quarter of each row per lane group (contraction slot (ks, g) is
// column g*d/4 + ks, which both operands agree on).
#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kRowWaves = 4;
constexpr int kColChunk = 64;   // output columns per pass over the rows (bounds the LDS image of W)

template <int D, bool IN_BF16, bool OUT_BF16>
__global__ __launch_bounds__(kRowWaves * 64) void rowgemm_kernel(
    const void* __restrict__ In, const float* __restrict__ W, size_t w_stride, int rows, float scale,
    void* __restrict__ Out) {
    constexpr int LDW = kColChunk + 1;
    extern __shared__ __attribute__((aligned(16))) float smem[];   // [D][LDW]
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    const int row0 = (blockIdx.x * kRowWaves + wave) * 16;
    const int row = row0 + i16;
    const bool valid = row < rows;
    const float* Wb = W + (size_t)b * w_stride;
    // this lane's quarter of its row, as floats
    float a[D / 4];
    {
        const size_t off = ((size_t)b * rows + (valid ? row : 0)) * D + (size_t)g * (D / 4);
        if constexpr (IN_BF16) {
            const uint16_t* p = reinterpret_cast<const uint16_t*>(In) + off;
#pragma unroll
            for (int q = 0; q < D / 16; ++q) {
                const uint2 v = *reinterpret_cast<const uint2*>(p + 4 * q);
                a[4 * q + 0] = bf16_lo(v.x); a[4 * q + 1] = bf16_hi(v.x);
                a[4 * q + 2] = bf16_lo(v.y); a[4 * q + 3] = bf16_hi(v.y);
            }
        } else {
            const float* p = reinterpret_cast<const float*>(In) + off;
#pragma unroll
            for (int q = 0; q < D / 16; ++q) {
                const v4f v = *reinterpret_cast<const v4f*>(p + 4 * q);
                a[4 * q + 0] = v.x; a[4 * q + 1] = v.y; a[4 * q + 2] = v.z; a[4 * q + 3] = v.w;
            }
        }
        if (!valid) {
#pragma unroll
            for (int k = 0; k < D / 4; ++k) a[k] = 0.f;
        }
    }
    for (int c0 = 0; c0 < D; c0 += kColChunk) {
        __syncthreads();
        for (int e = threadIdx.x; e < D * kColChunk; e += kRowWaves * 64) {
            const int k = e / kColChunk, c = e % kColChunk;
            smem[k * LDW + c] = Wb[(size_t)k * D + c0 + c];
        }
        __syncthreads();
#pragma unroll
        for (int cb = 0; cb < kColChunk / 16; ++cb) {
            v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
            const float* wcol = smem + (g * (D / 4)) * LDW + 16 * cb + i16;
#pragma unroll
            for (int ks = 0; ks < D / 4; ++ks) acc = mfma16x16x4(a[ks], wcol[ks * LDW], acc);
            // element t of the accumulator is row 4*g + t of the wave's block, column i16
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int orow = row0 + 4 * g + t;
                if (orow < rows) {
                    const size_t o = ((size_t)b * rows + orow) * D + c0 + 16 * cb + i16;
                    const float v = scale * acc[t];
                    if constexpr (OUT_BF16) reinterpret_cast<__bf16*>(Out)[o] = (__bf16)v;
                    else reinterpret_cast<float*>(Out)[o] = v;
                }
            }
        }
    }
}

template <int D>
hipError_t launch_d(const void* In, const float* W, size_t w_stride, int B, int rows, float scale, bool in_bf16,
                    bool out_bf16, void* Out, hipStream_t stream) {
    const size_t lds = sizeof(float) * (size_t)D * (kColChunk + 1);
    dim3 grid(ceil_div(rows, kRowWaves * 16), B), block(kRowWaves * 64);
#define SOLAR_ROWGEMM(IB, OB)                                                                        \
    do {                                                                                             \
        auto kern = rowgemm_kernel<D, IB, OB>;                                                       \
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);    \
        if (e != hipSuccess) return e;                                                               \
        hipLaunchKernelGGL(kern, grid, block, lds, stream, In, W, w_stride, rows, scale, Out);       \
    } while (0)
    if (in_bf16 && out_bf16) SOLAR_ROWGEMM(true, true);
    else if (in_bf16) SOLAR_ROWGEMM(true, false);
    else if (out_bf16) SOLAR_ROWGEMM(false, true);
    else SOLAR_ROWGEMM(false, false);
#undef SOLAR_ROWGEMM
    return hipGetLastError();
}

}  // namespace

// Out[b] = scale * In[b] * W[b * w_stride ...]; w_stride = 0 shares one matrix among the users.
hipError_t launch_rowgemm(const void* In, const float* W, size_t w_stride, int B, int rows, int d, float scale,
                          bool in_bf16, bool out_bf16, void* Out, hipStream_t stream) {
    switch (d) {
        case 64: return launch_d<64>(In, W, w_stride, B, rows, scale, in_bf16, out_bf16, Out, stream);
        case 128: return launch_d<128>(In, W, w_stride, B, rows, scale, in_bf16, out_bf16, Out, stream);
        case 256: return launch_d<256>(In, W, w_stride, B, rows, scale, in_bf16, out_bf16, Out, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace solar
