// Projection of the sequence onto the rank-r factors, P_b = X_b V_b (= U_b S_b: the
// left factor never has to be formed once U is eliminated, Section "SVD-Attention").
//
// Evaluated transposed, P^T = V^T X^T, with the float 16x16x4 MFMA so that the
// streamed operand X needs no re-layout: a lane loads four consecutive columns of
// one row (16 lanes = 16 rows of the tile, 4 lane groups = 4 column quads) and the
// four values are the B operand of four successive MFMAs; the matching rows of V
// come from LDS.  The result tile leaves the matrix unit with four consecutive
// rank indices per lane, i.e. as one 16-byte store into the row-major P.
#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kProjThreads = 256;
constexpr int kProjTilesPerWave = 8;  // 16-row tiles handled by one wave

template <int D, bool BF16>
__global__ __launch_bounds__(kProjThreads) void project_kernel(
    const void* __restrict__ Xv, const int32_t* __restrict__ lengths, const float* __restrict__ V,
    int N, int r, int RP, float* __restrict__ P) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int LDV = RP + 4;
    float* Vs = smem;  // [D][LDV], columns >= r are zero
    const int b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    const int len = user_len(lengths, b, N);
    const int RB = RP / 16;

    for (int e = tid; e < D * RP; e += kProjThreads) {
        const int k = e / RP, c = e % RP;
        Vs[k * LDV + c] = (c < r) ? V[((size_t)b * D + k) * r + c] : 0.f;
    }
    __syncthreads();

    const int rows_per_block = 16 * 4 * kProjTilesPerWave;
    const int block_row0 = blockIdx.x * rows_per_block;
    float* Pb = P + (size_t)b * N * r;
    for (int tile = 0; tile < kProjTilesPerWave; ++tile) {
        const int n0 = block_row0 + (tile * 4 + wave) * 16;
        if (n0 >= N) break;
        const int n = n0 + i16;
        if (n0 >= len) {
            // rows past the valid length: P is defined to be zero there
            for (int e = lane; e < 16 * r; e += 64) {
                const int rr = n0 + e / r;
                if (rr < N) Pb[(size_t)rr * r + e % r] = 0.f;
            }
            continue;
        }
        // one row per lane: D/16 quads of columns
        v4f x[D / 16];
        const bool valid = n < len;
        if constexpr (BF16) {
            const uint2* src = reinterpret_cast<const uint2*>(
                reinterpret_cast<const uint16_t*>(Xv) + ((size_t)b * N + (valid ? n : 0)) * D);
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk) {
                uint2 w = src[4 * kk + g];
                x[kk] = valid ? v4f{bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y)}
                              : v4f{0.f, 0.f, 0.f, 0.f};
            }
        } else {
            const v4f* src = reinterpret_cast<const v4f*>(
                reinterpret_cast<const float*>(Xv) + ((size_t)b * N + (valid ? n : 0)) * D);
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk) {
                v4f w = src[4 * kk + g];
                x[kk] = valid ? w : v4f{0.f, 0.f, 0.f, 0.f};
            }
        }
        for (int rb = 0; rb < RB; ++rb) {
            v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float a = Vs[(16 * kk + 4 * g + t) * LDV + 16 * rb + i16];
                    acc = mfma16x16x4(a, x[kk][t], acc);
                }
            }
            // acc[t] = P[n0 + i16][16*rb + 4*g + t]
            if (n < N) {
                const int c0 = 16 * rb + 4 * g;
                float* dst = Pb + (size_t)n * r + c0;
                if (c0 + 3 < r && (r % 4) == 0) {
                    *reinterpret_cast<v4f*>(dst) = acc;
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if (c0 + t < r) dst[t] = acc[t];
                }
            }
        }
    }
}

}  // namespace

template <int D>
static hipError_t launch_project_d(const void* X, const int32_t* lengths, const float* V, int B,
                                   int N, int r, bool bf16, float* P, hipStream_t stream) {
    const int RP = 16 * ((r + 15) / 16);
    const size_t lds = sizeof(float) * (size_t)D * (RP + 4);
    dim3 grid(ceil_div(N, 16 * 4 * kProjTilesPerWave), B), block(kProjThreads);
    if (bf16) {
        auto kern = project_kernel<D, true>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, X, lengths, V, N, r, RP, P);
    } else {
        auto kern = project_kernel<D, false>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, X, lengths, V, N, r, RP, P);
    }
    return hipGetLastError();
}

hipError_t launch_project(const void* X, const int32_t* lengths, const float* V,
                          const int32_t* /*info*/, int B, int N, int d, int r, bool bf16, float* P,
                          hipStream_t stream) {
    switch (d) {
        case 64: return launch_project_d<64>(X, lengths, V, B, N, r, bf16, P, stream);
        case 128: return launch_project_d<128>(X, lengths, V, B, N, r, bf16, P, stream);
        case 256: return launch_project_d<256>(X, lengths, V, B, N, r, bf16, P, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace solar
