// Gradient through the truncated SVD with respect to X ("Backward Pass Through SVD", the form
// with U-bar = 0):
//   dL/dX = U [diag(S_bar) + 2 S sym(F o (V^T V_bar))] V^T,   U = P S^-1,  P = X V,
// F_ij = 1/(s_j^2 - s_i^2) off the diagonal (the orientation that finite differences of the
// decomposition confirm; the printed F is its transpose), 0 on it and for pairs of singular
// values closer than gap_rel * s_1^2.  Two kernels:
//   * svd_backward_small_kernel, one workgroup per user: A = V^T V_bar (r x r),
//     K = diag(S_bar) + S (F o A + (F o A)^T), Mt = S^-1 K V^T (r x d) into the workspace;
//   * backproject_kernel: dX = P Mt, rows of P (float, r values) times the r x d matrix held in
//     LDS, float 32x32x2 MFMA, 32 rows per wave at a time; it writes N*d floats for N*r read
//     (HBM-bound; the float contraction, 2 N r d flops, takes about two thirds as long).  Rows past the valid length are zero in P, hence in dX.
#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kSmallThreads = 512;

// V of one user is staged in LDS with an odd row stride (V_bar too when both fit, stage_g; else
// it is read from global memory), and both small products run on the float 16x16x4 MFMA, one
// 16 x 16 tile of the result per wave at a time: V^T V_bar contracts over the d rows, K V^T over
// the r columns.  All strides are odd, so operand reads are free of bank conflicts.
__global__ __launch_bounds__(kSmallThreads) void svd_backward_small_kernel(
    const float* __restrict__ S, const float* __restrict__ V, const float* __restrict__ S_bar,
    const float* __restrict__ V_bar, int d, int r, float gap_rel, int stage_g, float* __restrict__ Mt) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int ld = r + 1;
    float* Vs = smem;                 // [d][ld]
    float* Gs = Vs + d * ld;          // [d][ld] when stage_g
    float* A = Gs + (stage_g ? d * ld : 0);   // [r][ld]  V^T V_bar
    float* Kt = A + r * ld;           // [r][ld]  K
    float* Ss = Kt + r * ld;          // [r]
    const int b = blockIdx.x, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, i16 = lane & 15, g = lane >> 4;
    constexpr int kWaves = kSmallThreads / 64;
    const float* Vb = V + (size_t)b * d * r;
    const float* Gb = V_bar + (size_t)b * d * r;
    for (int e = tid; e < d * r; e += kSmallThreads) {
        const int c = e / r, j = e % r;
        Vs[c * ld + j] = Vb[e];
        if (stage_g) Gs[c * ld + j] = Gb[e];
    }
    if (tid < r) Ss[tid] = S[(size_t)b * r + tid];
    __syncthreads();
    const int rt = r / 16;
    for (int tile = wave; tile < rt * rt; tile += kWaves) {
        const int ti = tile / rt, tj = tile % rt;
        v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
        if (stage_g) {
            for (int c0 = 0; c0 < d; c0 += 4)
                acc = mfma16x16x4(Vs[(c0 + g) * ld + 16 * ti + i16], Gs[(c0 + g) * ld + 16 * tj + i16], acc);
        } else {
            for (int c0 = 0; c0 < d; c0 += 4)
                acc = mfma16x16x4(Vs[(c0 + g) * ld + 16 * ti + i16], Gb[(size_t)(c0 + g) * r + 16 * tj + i16], acc);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) A[(16 * ti + 4 * g + t) * ld + 16 * tj + i16] = acc[t];
    }
    __syncthreads();
    const float s1sq = Ss[0] * Ss[0];
    for (int e = tid; e < r * r; e += kSmallThreads) {
        const int i = e / r, j = e % r;
        const float si = Ss[i], sj = Ss[j];
        float k = 0.f;
        if (i == j) {
            k = S_bar[(size_t)b * r + i];
        } else {
            const float diff = sj * sj - si * si;            // F_ij = 1/diff, F_ji = -1/diff
            if (fabsf(diff) > gap_rel * s1sq) k = si * (A[i * ld + j] - A[j * ld + i]) / diff;
        }
        Kt[i * ld + j] = k;
    }
    __syncthreads();
    const int dt = d / 16;
    for (int tile = wave; tile < rt * dt; tile += kWaves) {
        const int ti = tile / dt, tc = tile % dt;
        v4f acc = v4f{0.f, 0.f, 0.f, 0.f};
        for (int j0 = 0; j0 < r; j0 += 4)
            acc = mfma16x16x4(Kt[(16 * ti + i16) * ld + j0 + g], Vs[(16 * tc + i16) * ld + j0 + g], acc);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int i = 16 * ti + 4 * g + t;
            const float si = Ss[i];
            Mt[(size_t)b * r * d + (size_t)i * d + 16 * tc + i16] = si > 0.f ? acc[t] / si : 0.f;
        }
    }
}

constexpr int kRowWaves = 4;

// Out[b][rows][D] = In[b][rows][KR] * W[b][KR][D] with the 32x32x2 float MFMA: a wave owns 32
// rows at a time; lane l supplies row l%32 of In, and since the contraction order is free as long
// as both operands agree, lane half h = l/32 takes the contiguous columns h*KR/2 .. (h+1)*KR/2 of
// its row (plain 16-byte loads).  The result register t of a 32-column block holds row
// 8(t/4) + 4h + t%4 and column l%32, so every store covers two full 128-byte lines.  The rows of
// the next block are fetched before the current one is multiplied.
template <int KR, int D>
__global__ __launch_bounds__(kRowWaves * 64) void backproject_kernel(
    const float* __restrict__ In, const float* __restrict__ W, int rows, float* __restrict__ Out) {
    constexpr int LDW = D + 1;
    constexpr int KH = KR / 2;
    extern __shared__ __attribute__((aligned(16))) float smem[];   // [KR][LDW]
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i32 = lane & 31, h = lane >> 5;
    for (int e = threadIdx.x; e < KR * D; e += kRowWaves * 64) smem[(e / D) * LDW + e % D] = W[(size_t)b * KR * D + e];
    __syncthreads();
    const int nblocks = ceil_div(rows, 32);
    const int stride = gridDim.x * kRowWaves;
    const float* in_b = In + (size_t)b * rows * KR + h * KH;
    float* out_b = Out + (size_t)b * rows * D;
    v4f nxt[KH / 4];
    auto fetch = [&](int blk) {
        int row = blk * 32 + i32;
        row = row < rows ? row : rows - 1;          // clamped: rows past the end are never stored
        const v4f* p = reinterpret_cast<const v4f*>(in_b + (size_t)row * KR);
#pragma unroll
        for (int q = 0; q < KH / 4; ++q) nxt[q] = p[q];
    };
    int blk = blockIdx.x * kRowWaves + wave;
    if (blk < nblocks) fetch(blk);
    for (; blk < nblocks; blk += stride) {
        float a[KH];
#pragma unroll
        for (int q = 0; q < KH / 4; ++q) {
            a[4 * q + 0] = nxt[q].x; a[4 * q + 1] = nxt[q].y; a[4 * q + 2] = nxt[q].z; a[4 * q + 3] = nxt[q].w;
        }
        if (blk + stride < nblocks) fetch(blk + stride);
        const int row0 = blk * 32 + 4 * h;
        const bool full = blk * 32 + 32 <= rows;
#pragma unroll
        for (int cb = 0; cb < D / 32; ++cb) {
            v16f acc;
#pragma unroll
            for (int t = 0; t < 16; ++t) acc[t] = 0.f;
            const float* wcol = smem + (h * KH) * LDW + 32 * cb + i32;
#pragma unroll
            for (int ks = 0; ks < KH; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ks], wcol[ks * LDW], acc, 0, 0, 0);
            float* o = out_b + (size_t)row0 * D + 32 * cb + i32;
            if (full) {
#pragma unroll
                for (int t = 0; t < 16; ++t)
                    __builtin_nontemporal_store(acc[t], o + (size_t)(8 * (t / 4) + (t % 4)) * D);
            } else {
#pragma unroll
                for (int t = 0; t < 16; ++t)
                    if (row0 + 8 * (t / 4) + (t % 4) < rows) o[(size_t)(8 * (t / 4) + (t % 4)) * D] = acc[t];
            }
        }
    }
}

template <int KR, int D>
hipError_t launch_bp(const float* In, const float* W, int B, int rows, float* Out, hipStream_t stream) {
    const size_t lds = sizeof(float) * (size_t)KR * (D + 1);
    // about four workgroups per compute unit in total, each walking several 64-row groups
    int gx = ceil_div(1024, B);
    const int maxgx = ceil_div(rows, kRowWaves * 32);
    if (gx > maxgx) gx = maxgx;
    if (gx < 1) gx = 1;
    auto kern = backproject_kernel<KR, D>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(gx, B), dim3(kRowWaves * 64), lds, stream, In, W, rows, Out);
    return hipGetLastError();
}

template <int D>
hipError_t launch_bp_d(const float* In, const float* W, int B, int rows, int r, float* Out, hipStream_t stream) {
    switch (r) {
        case 16: return launch_bp<16, D>(In, W, B, rows, Out, stream);
        case 32: return launch_bp<32, D>(In, W, B, rows, Out, stream);
        case 48: return launch_bp<48, D>(In, W, B, rows, Out, stream);
        case 64: return launch_bp<64, D>(In, W, B, rows, Out, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool svd_backward_supported(int d, int r) {
    return (d == 64 || d == 128 || d == 256) && r >= 16 && r <= 64 && r % 16 == 0 && r <= d;
}

hipError_t launch_svd_backward(const float* S, const float* V, const float* P, const float* S_bar,
                               const float* V_bar, int B, int N, int d, int r, float gap_rel, float* Mt,
                               float* dX, hipStream_t stream) {
    const size_t base = sizeof(float) * ((size_t)d * (r + 1) + 2 * (size_t)r * (r + 1) + r);
    const size_t extra = sizeof(float) * (size_t)d * (r + 1);
    const int stage_g = base + extra <= 128 * 1024;
    const size_t lds = base + (stage_g ? extra : 0);
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(svd_backward_small_kernel), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(svd_backward_small_kernel, dim3(B), dim3(kSmallThreads), lds, stream, S, V, S_bar, V_bar,
                       d, r, gap_rel, stage_g, Mt);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    switch (d) {
        case 64: return launch_bp_d<64>(P, Mt, B, N, r, dX, stream);
        case 128: return launch_bp_d<128>(P, Mt, B, N, r, dX, stream);
        case 256: return launch_bp_d<256>(P, Mt, B, N, r, dX, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace solar
