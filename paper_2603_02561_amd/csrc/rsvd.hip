// The two contractions over the sequence axis that Algorithm 1 ("Randomized SVD with Power
// Iteration") needs beside Y = H Omega, when it is run as printed, with passes over H:
//   W  = H^T Y   (d x r): the power iteration Omega <- H^T (H Omega), and, after the last
//                          pass, the factor of Q^T H = R^-T (H^T Y)^T for Y = Q R;
//   Gy = Y^T Y   (r x r): the Gram matrix whose Cholesky factor is the R of that QR.
// H is the row-major X (bf16 or float), Y is float [N][r].  As in the Gram kernel the
// sequence axis is the contraction axis of the MFMA and both operands of a product come from
// the same rows: a wave streams 16 rows per step with 16 lanes per row, lane j holding CPL =
// d/16 consecutive columns of X and CY = r/16 consecutive columns of Y; fragment pair (s, c)
// yields the 16x16 block {W[CPL*i+s][CY*j+c]}, pair (c1 <= c2) of Y fragments the block
// {Gy[CY*i+c1][CY*j+c2]}.  Y is a float quantity of unbounded dynamic range (no
// normalisation between power steps in the printed algorithm), so the float 16x16x4 MFMA is
// used for both input types; bf16 values of X are widened exactly.
// Split-N with a fixed-order reduction (waves in LDS, chunks in the finalize kernel): results
// are bitwise reproducible.
#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kWaves = 4;

template <int CPL, int CY>
__host__ __device__ constexpr int xty_blocks() { return CPL * CY + CY * (CY + 1) / 2; }

template <int CPL, int CY, bool BF16>
__global__ __launch_bounds__(kWaves * 64) void xty_partial_kernel(
    const void* __restrict__ Xv, const float* __restrict__ Y, const int32_t* __restrict__ lengths, int N,
    int nsplit, float* __restrict__ partials) {
    constexpr int D = 16 * CPL, R = 16 * CY;
    constexpr int NB = xty_blocks<CPL, CY>();
    constexpr int STEP = 16;
    const int b = blockIdx.y, split = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, h = lane >> 4;
    const int len = user_len(lengths, b, N);
    const int chunk = ceil_div(ceil_div(len, nsplit), STEP) * STEP;
    const int r0 = split * chunk;
    const int r1 = min(len, r0 + chunk);
    const float* Yb = Y + (size_t)b * N * R;

    v4f acc[NB];
#pragma unroll
    for (int p = 0; p < NB; ++p) acc[p] = v4f{0.f, 0.f, 0.f, 0.f};

    struct Rows { float x[4][CPL]; float y[4][CY]; };
    auto load = [&](Rows& dst, int base) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int row = base + 4 * t + h;
            if (row < r1) {
                if constexpr (BF16) {
                    const uint16_t* p = reinterpret_cast<const uint16_t*>(Xv) + ((size_t)b * N + row) * D + CPL * j;
#pragma unroll
                    for (int q = 0; q < CPL / 4; ++q) {
                        const uint2 v = *reinterpret_cast<const uint2*>(p + 4 * q);
                        dst.x[t][4 * q + 0] = bf16_lo(v.x); dst.x[t][4 * q + 1] = bf16_hi(v.x);
                        dst.x[t][4 * q + 2] = bf16_lo(v.y); dst.x[t][4 * q + 3] = bf16_hi(v.y);
                    }
                } else {
                    const float* p = reinterpret_cast<const float*>(Xv) + ((size_t)b * N + row) * D + CPL * j;
#pragma unroll
                    for (int q = 0; q < CPL / 4; ++q) {
                        const v4f v = *reinterpret_cast<const v4f*>(p + 4 * q);
                        dst.x[t][4 * q + 0] = v.x; dst.x[t][4 * q + 1] = v.y;
                        dst.x[t][4 * q + 2] = v.z; dst.x[t][4 * q + 3] = v.w;
                    }
                }
                const float* py = Yb + (size_t)row * R + CY * j;
#pragma unroll
                for (int c = 0; c < CY; ++c) dst.y[t][c] = py[c];
            } else {
#pragma unroll
                for (int s = 0; s < CPL; ++s) dst.x[t][s] = 0.f;
#pragma unroll
                for (int c = 0; c < CY; ++c) dst.y[t][c] = 0.f;
            }
        }
    };
    Rows cur, nxt;
    int base = r0 + wave * STEP;
    if (base < r1) load(cur, base);
    while (base < r1) {
        const int nbase = base + kWaves * STEP;
        if (nbase < r1) load(nxt, nbase);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
#pragma unroll
            for (int s = 0; s < CPL; ++s)
#pragma unroll
                for (int c = 0; c < CY; ++c)
                    acc[s * CY + c] = mfma16x16x4(cur.x[t][s], cur.y[t][c], acc[s * CY + c]);
            int p = CPL * CY;
#pragma unroll
            for (int c1 = 0; c1 < CY; ++c1)
#pragma unroll
                for (int c2 = c1; c2 < CY; ++c2) {
                    acc[p] = mfma16x16x4(cur.y[t][c1], cur.y[t][c2], acc[p]);
                    ++p;
                }
        }
        if (nbase < r1) cur = nxt;
        base = nbase;
    }

    // Fixed-order sum over the waves of the workgroup, then one coalesced store.
    __shared__ v4f red[NB * 64];
    for (int w = 0; w < kWaves; ++w) {
        if (wave == w) {
#pragma unroll
            for (int p = 0; p < NB; ++p) {
                if (w == 0) red[p * 64 + lane] = acc[p];
                else red[p * 64 + lane] += acc[p];
            }
        }
        __syncthreads();
    }
    v4f* out = reinterpret_cast<v4f*>(partials) + ((size_t)b * nsplit + split) * (NB * 64);
    for (int i = threadIdx.x; i < NB * 64; i += kWaves * 64) out[i] = red[i];
}

// W[b][a][c] and Gy[b][u][v] = sums over the chunks of the partial-block element that holds
// them (register q of lane l of a block is element (4*(l/16)+q, l%16)).
template <int CPL, int CY>
__global__ __launch_bounds__(256) void xty_finalize_kernel(const float* __restrict__ partials, int nsplit,
                                                           float* __restrict__ W, float* __restrict__ Gy) {
    constexpr int D = 16 * CPL, R = 16 * CY;
    constexpr int NB = xty_blocks<CPL, CY>();
    const int b = blockIdx.y;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= D * R + R * R) return;
    int blk, i, jj;
    float* dst;
    if (e < D * R) {
        const int a = e / R, c = e % R;
        i = a / CPL; jj = c / CY;
        blk = (a % CPL) * CY + (c % CY);
        dst = W + (size_t)b * D * R + e;
    } else {
        const int g = e - D * R;
        int u = g / R, v = g % R;
        int c1 = u % CY, c2 = v % CY;
        i = u / CY; jj = v / CY;
        if (c1 > c2) {
            int t = c1; c1 = c2; c2 = t;
            t = i; i = jj; jj = t;
        }
        blk = CPL * CY + c1 * CY - (c1 * (c1 - 1)) / 2 + (c2 - c1);
        dst = Gy + (size_t)b * R * R + g;
    }
    const int off = blk * 256 + (jj + 16 * (i / 4)) * 4 + (i % 4);
    const float* p = partials + (size_t)b * nsplit * (NB * 256) + off;
    float acc = 0.f;
    for (int s = 0; s < nsplit; ++s) acc += p[(size_t)s * (NB * 256)];
    *dst = acc;
}

template <int CPL, int CY>
hipError_t launch_t(const void* X, const float* Y, const int32_t* lengths, int B, int N, bool bf16,
                    float* partials, float* W, float* Gy, hipStream_t stream) {
    constexpr int D = 16 * CPL, R = 16 * CY;
    const int nsplit = gram_nsplit(B, N);
    dim3 grid(nsplit, B), block(kWaves * 64);
    if (bf16) hipLaunchKernelGGL((xty_partial_kernel<CPL, CY, true>), grid, block, 0, stream, X, Y, lengths, N, nsplit, partials);
    else hipLaunchKernelGGL((xty_partial_kernel<CPL, CY, false>), grid, block, 0, stream, X, Y, lengths, N, nsplit, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 fgrid(ceil_div(D * R + R * R, 256), B);
    hipLaunchKernelGGL((xty_finalize_kernel<CPL, CY>), fgrid, dim3(256), 0, stream, partials, nsplit, W, Gy);
    return hipGetLastError();
}

template <int CPL>
hipError_t launch_c(const void* X, const float* Y, const int32_t* lengths, int B, int N, int r, bool bf16,
                    float* partials, float* W, float* Gy, hipStream_t stream) {
    switch (r) {
        case 16: return launch_t<CPL, 1>(X, Y, lengths, B, N, bf16, partials, W, Gy, stream);
        case 32: return launch_t<CPL, 2>(X, Y, lengths, B, N, bf16, partials, W, Gy, stream);
        case 48: return launch_t<CPL, 3>(X, Y, lengths, B, N, bf16, partials, W, Gy, stream);
        case 64: return launch_t<CPL, 4>(X, Y, lengths, B, N, bf16, partials, W, Gy, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool rsvd_supported(int d, int r) { return (d == 64 || d == 128) && r >= 16 && r <= 64 && r % 16 == 0 && r <= d; }

size_t xty_partial_floats(int B, int N, int d, int r) {
    const int cpl = d / 16, cy = r / 16;
    return (size_t)B * gram_nsplit(B, N) * (cpl * cy + cy * (cy + 1) / 2) * 256;
}

hipError_t launch_xty(const void* X, const float* Y, const int32_t* lengths, int B, int N, int d, int r,
                      bool bf16, float* partials, float* W, float* Gy, hipStream_t stream) {
    switch (d) {
        case 64: return launch_c<4>(X, Y, lengths, B, N, r, bf16, partials, W, Gy, stream);
        case 128: return launch_c<8>(X, Y, lengths, B, N, r, bf16, partials, W, Gy, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace solar
