// Projection of the sequence onto the rank-r factors, P_b = X_b V_b (= U_b S_b: the
// left factor never has to be formed once U is eliminated, Section "SVD-Attention").
//
// Evaluated transposed, P^T = V^T X^T, with the float 16x16x4 MFMA so that the
// streamed operand X needs no re-layout: a lane loads four consecutive columns of
// one row (16 lanes = 16 rows of the tile, 4 lane groups = 4 column quads) and the
// four values are the B operand of four successive MFMAs; the matching rows of V
// come from LDS.  The result tile leaves the matrix unit with four consecutive
// rank indices per lane, i.e. as one 16-byte store into the row-major P.
#include <cstdlib>

#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kProjThreads = 256;
constexpr int kProjTilesPerWave = 8;  // 16-row tiles handled by one wave (fewer in small launches)

// The 16 rows from n0 on (as far as they exist) of one user's P set to zero by one wave: the rows
// are contiguous in memory, so the wave fills them with 16-byte stores when r is a multiple of 4.
__device__ __forceinline__ void zero_rows(float* Pb, int n0, int N, int r, int lane) {
    const int rows = min(16, N - n0);
    float* dst = Pb + (size_t)n0 * r;
    if ((r & 3) == 0) {
        for (int e = lane; e < rows * (r >> 2); e += 64) reinterpret_cast<v4f*>(dst)[e] = v4f{0.f, 0.f, 0.f, 0.f};
    } else {
        for (int e = lane; e < rows * r; e += 64) dst[e] = 0.f;
    }
}

template <int D, bool BF16>
__global__ __launch_bounds__(kProjThreads) void project_kernel(
    const void* __restrict__ Xv, const int32_t* __restrict__ lengths, const float* __restrict__ V,
    int N, int r, int RP, int tiles_per_wave, float* __restrict__ P) {
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

    const int rows_per_block = 16 * 4 * tiles_per_wave;
    const int block_row0 = blockIdx.x * rows_per_block;
    float* Pb = P + (size_t)b * N * r;
    for (int tile = 0; tile < tiles_per_wave; ++tile) {
        const int n0 = block_row0 + (tile * 4 + wave) * 16;
        if (n0 >= N) break;
        const int n = n0 + i16;
        if (n0 >= len) {
            // rows past the valid length: P is defined to be zero there
            zero_rows(Pb, n0, N, r, lane);
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

// bf16 inputs: the rows of X are bf16 already, so a lane's 16-byte load (eight consecutive
// columns of its row) is the B operand of the 16x16x32 bf16 MFMA as it stands.  V is float:
// it is split once per wave into a bf16 head and tail (V = hi + lo to 16 bits) that stay in
// registers as the A operands, and each k-chunk costs two MFMAs.  The next tile of X is
// fetched while the current one is in the matrix unit.
template <int D, int RB>
__global__ __launch_bounds__(kProjThreads) void project_bf16_kernel(
    const uint16_t* __restrict__ X, const int32_t* __restrict__ lengths, const float* __restrict__ V,
    int N, int r, int tiles_per_wave, float* __restrict__ P) {
    constexpr int KK = D / 32;
    const int b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    const int len = user_len(lengths, b, N);
    const float* Vb = V + (size_t)b * D * r;

    // A operands: slot (g, u) of chunk kk is column 32*kk + 8*g + u; row i16 is rank 16*rb + i16
    v4u ahi[KK][RB], alo[KK][RB];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int rank = 16 * rb + i16;
            uint32_t hw[4], lw[4];
#pragma unroll
            for (int u2 = 0; u2 < 4; ++u2) {
                float v0 = 0.f, v1 = 0.f;
                if (rank < r) {
                    v0 = Vb[(size_t)(32 * kk + 8 * g + 2 * u2) * r + rank];
                    v1 = Vb[(size_t)(32 * kk + 8 * g + 2 * u2 + 1) * r + rank];
                }
                typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
                const v2bf h = {(__bf16)v0, (__bf16)v1};
                const v2bf l = {(__bf16)(v0 - (float)h[0]), (__bf16)(v1 - (float)h[1])};
                hw[u2] = __builtin_bit_cast(uint32_t, h);
                lw[u2] = __builtin_bit_cast(uint32_t, l);
            }
            ahi[kk][rb] = v4u{hw[0], hw[1], hw[2], hw[3]};
            alo[kk][rb] = v4u{lw[0], lw[1], lw[2], lw[3]};
        }

    const int rows_per_block = 16 * 4 * tiles_per_wave;
    const int block_row0 = blockIdx.x * rows_per_block;
    const uint16_t* Xb = X + (size_t)b * N * D;
    float* Pb = P + (size_t)b * N * r;
    auto fetch = [&](v4u (&x)[KK], int n0) __attribute__((always_inline)) {
        const int n = n0 + i16;
        const bool valid = n < len;
        const v4u* src = reinterpret_cast<const v4u*>(Xb + (size_t)(valid ? n : 0) * D);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            x[kk] = src[4 * kk + g];
            if (!valid) x[kk] = v4u{0u, 0u, 0u, 0u};
        }
    };
    v4u cur[KK], nxt[KK];
    int n0 = block_row0 + wave * 16;
    if (n0 < len) fetch(cur, n0);
    for (int tile = 0; tile < tiles_per_wave; ++tile) {
        if (n0 >= N) break;
        const int n_next = n0 + 64;
        const bool have_next = tile + 1 < tiles_per_wave && n_next < len;
        if (have_next) fetch(nxt, n_next);
        const int n = n0 + i16;
        if (n0 >= len) {
            // rows past the valid length: P is defined to be zero there
            zero_rows(Pb, n0, N, r, lane);
        } else {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
                v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    acc = mfma16x16x32bf16(ahi[kk][rb], cur[kk], acc);
                    acc = mfma16x16x32bf16(alo[kk][rb], cur[kk], acc);
                }
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
        if (have_next) {
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) cur[kk] = nxt[kk];
        }
        n0 = n_next;
    }
}

}  // namespace

template <int D>
static hipError_t launch_project_d(const void* X, const int32_t* lengths, const float* V, int B,
                                   int N, int r, bool bf16, float* P, hipStream_t stream) {
    const int RP = 16 * ((r + 15) / 16);
    const size_t lds = sizeof(float) * (size_t)D * (RP + 4);
    // A wave takes eight 16-row tiles when that still gives every SIMD four waves (float
    // kernel, which has no prefetch and hides its loads behind other waves) or every compute
    // unit a workgroup (bf16 kernel, where a wave first builds its operands of V and wants
    // many tiles to spread that over); smaller launches take fewer tiles per wave.
    const long long want = bf16 ? 256 : 1024;
    int tiles = kProjTilesPerWave;
    while (tiles > 1 && (long long)B * ceil_div(N, 64 * tiles) < want) tiles /= 2;
    dim3 grid(ceil_div(N, 16 * 4 * tiles), B), block(kProjThreads);
    if (bf16) {
        const uint16_t* Xh = reinterpret_cast<const uint16_t*>(X);
        switch (RP / 16) {
            case 1: hipLaunchKernelGGL((project_bf16_kernel<D, 1>), grid, block, 0, stream, Xh, lengths, V, N, r, tiles, P); break;
            case 2: hipLaunchKernelGGL((project_bf16_kernel<D, 2>), grid, block, 0, stream, Xh, lengths, V, N, r, tiles, P); break;
            case 3: hipLaunchKernelGGL((project_bf16_kernel<D, 3>), grid, block, 0, stream, Xh, lengths, V, N, r, tiles, P); break;
            case 4:
                if constexpr (D <= 128) {
                    hipLaunchKernelGGL((project_bf16_kernel<D, 4>), grid, block, 0, stream, Xh, lengths, V, N, r, tiles, P);
                    break;
                }
                [[fallthrough]];
            default: {
                auto kern = project_kernel<D, true>;
                hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL(kern, grid, block, lds, stream, X, lengths, V, N, r, RP, tiles, P);
            }
        }
    } else {
        auto kern = project_kernel<D, false>;
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, X, lengths, V, N, r, RP, tiles, P);
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
