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
// are bitwise reproducible.  A wave keeps a ring of three row blocks, two of them as loads in
// flight (the scheme of the Gram kernel).
#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kWaves = 4;

template <int CPL, int CY>
__host__ __device__ constexpr int xty_blocks() { return CPL * CY + CY * (CY + 1) / 2; }

// Partial blocks of more than kParallelReduceBlocks fragment pairs do not fit the LDS four times
// over; their waves are added one after another into one region instead.
constexpr int kParallelReduceBlocks = 36;

template <int CPL, int CY, bool BF16>
__global__ __launch_bounds__(kWaves * 64) void xty_partial_kernel(
    const void* __restrict__ Xv, const float* __restrict__ Y, const int32_t* __restrict__ lengths, int N,
    int nsplit, float* __restrict__ partials) {
    constexpr int D = 16 * CPL, R = 16 * CY;
    constexpr int NB = xty_blocks<CPL, CY>();
    constexpr int STEP = 16;
    constexpr int XW = BF16 ? CPL / 2 : CPL;   // 32-bit words of X per lane and row
    const int b = blockIdx.y, split = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, h = lane >> 4;
    const int len = user_len(lengths, b, N);
    const int chunk = ceil_div(ceil_div(len, nsplit), STEP) * STEP;
    const int r0 = split * chunk;
    const int r1 = min(len, r0 + chunk);
    const float* Yb = Y + (size_t)b * N * R + CY * j;
    const uint32_t* Xb = reinterpret_cast<const uint32_t*>(Xv) + (size_t)b * N * (XW * 16) + XW * j;

    v4f acc[NB];
#pragma unroll
    for (int p = 0; p < NB; ++p) acc[p] = v4f{0.f, 0.f, 0.f, 0.f};

    // A block is 16 rows: lane (j, h) holds rows 4t + h, t = 0..3, as loaded (bf16 pairs or floats
    // of X, floats of Y).  Loads carry no predicate and sit behind no branch: the row index is
    // clamped to the chunk's last row and the rows of Y past it count as zero when a ragged
    // block is multiplied (a zero row of Y contributes to neither W nor Gy).  With a branch
    // around a prefetch the compiler waits for all outstanding loads before every block.
    struct Rows { uint32_t x[4][XW]; float y[4][CY]; };
    const int row_max = max(r1 - 1, 0);
    auto load = [&](Rows& dst, int base) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const size_t row = (size_t)min(base + 4 * t + h, row_max);
            const uint32_t* px = Xb + row * (XW * 16);
            if constexpr (XW % 4 == 0) {
#pragma unroll
                for (int q = 0; q < XW / 4; ++q) {
                    const v4u v = *reinterpret_cast<const v4u*>(px + 4 * q);
                    dst.x[t][4 * q + 0] = v.x; dst.x[t][4 * q + 1] = v.y;
                    dst.x[t][4 * q + 2] = v.z; dst.x[t][4 * q + 3] = v.w;
                }
            } else {
                static_assert(XW == 2, "d = 64 in bf16: one 8-byte load");
                const uint2 v = *reinterpret_cast<const uint2*>(px);
                dst.x[t][0] = v.x; dst.x[t][1] = v.y;
            }
            const float* py = Yb + row * R;
            if constexpr (CY == 4) {
                const v4f v = *reinterpret_cast<const v4f*>(py);
                dst.y[t][0] = v.x; dst.y[t][1] = v.y; dst.y[t][2] = v.z; dst.y[t][3] = v.w;
            } else if constexpr (CY == 2) {
                const float2 v = *reinterpret_cast<const float2*>(py);
                dst.y[t][0] = v.x; dst.y[t][1] = v.y;
            } else {
#pragma unroll
                for (int c = 0; c < CY; ++c) dst.y[t][c] = py[c];
            }
        }
    };
    auto compute = [&](const Rows& src) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float x[CPL];
#pragma unroll
            for (int s = 0; s < CPL; ++s) {
                if constexpr (BF16) x[s] = (s & 1) ? bf16_hi(src.x[t][s / 2]) : bf16_lo(src.x[t][s / 2]);
                else x[s] = __uint_as_float(src.x[t][s]);
            }
#pragma unroll
            for (int s = 0; s < CPL; ++s)
#pragma unroll
                for (int c = 0; c < CY; ++c)
                    acc[s * CY + c] = mfma16x16x4(x[s], src.y[t][c], acc[s * CY + c]);
            int p = CPL * CY;
#pragma unroll
            for (int c1 = 0; c1 < CY; ++c1)
#pragma unroll
                for (int c2 = c1; c2 < CY; ++c2) {
                    acc[p] = mfma16x16x4(src.y[t][c1], src.y[t][c2], acc[p]);
                    ++p;
                }
        }
    };
    auto compute_tail = [&](Rows& src, int base) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (base + 4 * t + h >= r1) {
#pragma unroll
                for (int c = 0; c < CY; ++c) src.y[t][c] = 0.f;
            }
        compute(src);
    };
    // ring of kRing row blocks per wave: kRing - 1 blocks of loads stay in flight while one block
    // is multiplied; the steady-state loop takes kRing whole blocks per trip and has no branch in
    // its body, at most kRing - 1 whole blocks and one ragged block are left for the tail
    constexpr int kRing = 3;
    Rows ring[kRing];
    constexpr int stride = kWaves * STEP;
    const int base0 = r0 + wave * STEP;
    const int nblk = base0 < r1 ? ceil_div(r1 - base0, stride) : 0;
    const int nwhole = r1 - base0 >= STEP ? (r1 - base0 - STEP) / stride + 1 : 0;
#pragma unroll
    for (int k = 0; k < kRing - 1; ++k) load(ring[k], base0 + k * stride);
    int i = 0;
    for (; i + kRing <= nwhole; i += kRing) {
#pragma unroll
        for (int k = 0; k < kRing; ++k) {
            load(ring[(k + kRing - 1) % kRing], base0 + (i + k + kRing - 1) * stride);
            __builtin_amdgcn_sched_barrier(0);   // the prefetch is issued before the block is used
            compute(ring[k]);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int k = 0; k < kRing; ++k) {
        if (i + k < nblk) {
            if (i + k + kRing - 1 < nblk) load(ring[(k + kRing - 1) % kRing], base0 + (i + k + kRing - 1) * stride);
            compute_tail(ring[k], base0 + (i + k) * stride);
        }
    }

    // Fixed-order sum over the waves of the workgroup (wave 0 + 1 + 2 + 3), then one coalesced store.
    extern __shared__ __attribute__((aligned(16))) v4f red[];
    v4f* out = reinterpret_cast<v4f*>(partials) + ((size_t)b * nsplit + split) * (NB * 64);
    if constexpr (NB <= kParallelReduceBlocks) {
        // every wave parks its blocks in its own region: one barrier
#pragma unroll
        for (int p = 0; p < NB; ++p) red[(wave * NB + p) * 64 + lane] = acc[p];
        __syncthreads();
        for (int e = threadIdx.x; e < NB * 64; e += kWaves * 64) {
            v4f v = red[e];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) v += red[w * NB * 64 + e];
            out[e] = v;
        }
    } else {
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
        for (int e = threadIdx.x; e < NB * 64; e += kWaves * 64) out[e] = red[e];
    }
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
    constexpr int NB = xty_blocks<CPL, CY>();
    constexpr size_t lds = sizeof(v4f) * 64 * NB * (NB <= kParallelReduceBlocks ? kWaves : 1);
    const int nsplit = gram_nsplit(B, N);
    dim3 grid(nsplit, B), block(kWaves * 64);
    hipError_t e = bf16 ? allow_dynamic_lds(reinterpret_cast<const void*>(xty_partial_kernel<CPL, CY, true>), lds)
                        : allow_dynamic_lds(reinterpret_cast<const void*>(xty_partial_kernel<CPL, CY, false>), lds);
    if (e != hipSuccess) return e;
    if (bf16) hipLaunchKernelGGL((xty_partial_kernel<CPL, CY, true>), grid, block, lds, stream, X, Y, lengths, N, nsplit, partials);
    else hipLaunchKernelGGL((xty_partial_kernel<CPL, CY, false>), grid, block, lds, stream, X, Y, lengths, N, nsplit, partials);
    e = hipGetLastError();
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
