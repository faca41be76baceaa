// Gram contraction over the sequence axis, G_b = X_b^T X_b (the product that the
// power iteration of Algorithm 1 applies to Omega), for gfx950.
//
// The sequence axis is the slow memory axis of the row-major X, so it is the
// contraction (K) axis of the MFMA while both operands come from the same rows.
// A wave streams whole rows with 16 lanes per row and CPL = d/16 consecutive
// columns per lane; column CPL*j + s of lane j becomes "fragment s", and fragment
// pair (s1 <= s2) yields the 16x16 block {G[CPL*i+s1][CPL*j+s2]}.  Only the upper
// triangle of fragment pairs is formed.  For bf16 the eight rows a lane loads are
// transposed in registers into the k-contiguous operand the 16x16x32 MFMA wants;
// for float the 16x16x4 MFMA takes the loaded values as they are.  No LDS is used
// in the streaming loop: every byte of X is read from HBM once, by one wave.
//
// The sequence is cut into `nsplit` chunks per user (one workgroup each); the
// waves of a workgroup add their accumulators in LDS in a fixed order, the
// per-chunk partial blocks go to the workspace, and gram_finalize_kernel adds them
// in a fixed order and undoes the fragment permutation.  Results are therefore
// bitwise reproducible.
#include <cstdlib>

#include "common.h"
#include "kernels.h"

namespace solar {

template <int CPL>
__host__ __device__ constexpr int gram_pairs() { return CPL * (CPL + 1) / 2; }

constexpr int kGramWaves = 4;
// Sum of the accumulators of the workgroup's waves in a fixed order (wave 0 + 1 + 2 + 3, so the
// result does not depend on timing), then one coalesced store.  Every wave parks its block in its
// own LDS region (dynamic LDS, kGramWaves * NP KiB), so a single barrier separates the writes
// from the sums; adding the waves one after another into one region cost four barriers and a
// quarter of the kernel's time.
template <int NP>
__device__ __forceinline__ void reduce_waves_and_store(const v4f (&acc)[NP], v4f* __restrict__ out) {
    extern __shared__ __attribute__((aligned(16))) v4f red[];   // [kGramWaves][NP * 64]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int p = 0; p < NP; ++p) red[(wave * NP + p) * 64 + lane] = acc[p];
    __syncthreads();
    for (int i = threadIdx.x; i < NP * 64; i += kGramWaves * 64) {
        v4f v = red[i];
#pragma unroll
        for (int w = 1; w < kGramWaves; ++w) v += red[w * NP * 64 + i];
        out[i] = v;
    }
}

template <int NP>
constexpr size_t gram_reduce_lds() { return sizeof(v4f) * kGramWaves * NP * 64; }

template <typename K>
static hipError_t gram_allow_lds(K kern, size_t bytes) {
    return allow_dynamic_lds(reinterpret_cast<const void*>(kern), bytes);
}

#ifndef SOLAR_GRAM_RING
#define SOLAR_GRAM_RING 3
#endif

template <int CPL, bool BF16>
__global__ __launch_bounds__(kGramWaves * 64) void gram_partial_kernel(
    const void* __restrict__ Xv, const int32_t* __restrict__ lengths, int N, int nsplit,
    float* __restrict__ partials) {
    constexpr int D = 16 * CPL;
    constexpr int NP = gram_pairs<CPL>();
    constexpr int STEP = BF16 ? 32 : 16;  // rows a wave consumes per step
    const int b = blockIdx.y;
    const int split = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int j = lane & 15;
    const int h = lane >> 4;
    const int len = user_len(lengths, b, N);
    int chunk = ceil_div(ceil_div(len, nsplit), STEP) * STEP;
    const int r0 = split * chunk;
    const int r1 = min(len, r0 + chunk);

    v4f acc[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) acc[p] = v4f{0.f, 0.f, 0.f, 0.f};

    if constexpr (BF16) {
        constexpr int W = CPL / 2;  // 32-bit words per lane per row
        const uint32_t* X = reinterpret_cast<const uint32_t*>(Xv) + (size_t)b * N * (D / 2);
        auto load_row = [&](uint32_t (&dst)[W], const uint32_t* p) __attribute__((always_inline)) {
            if constexpr (W == 2) {
                uint2 v = *reinterpret_cast<const uint2*>(p);
                dst[0] = v.x; dst[1] = v.y;
            } else {
#pragma unroll
                for (int q = 0; q < W / 4; ++q) {
                    v4u v = *reinterpret_cast<const v4u*>(p + 4 * q);
                    dst[4 * q + 0] = v.x; dst[4 * q + 1] = v.y;
                    dst[4 * q + 2] = v.z; dst[4 * q + 3] = v.w;
                }
            }
        };
        // Loads carry no predicate and sit behind no branch: the row index is clamped to the
        // chunk's last row (rows past it are zeroed when a ragged block is multiplied).  With a
        // branch around a prefetch the compiler cannot count the loads that are younger than the
        // block it is about to use and waits for all of them, which undoes the prefetch.
        const int row_max = max(r1 - 1, 0);
        auto load = [&](uint32_t (&dst)[8][W], int base) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < 8; ++t)
                load_row(dst[t], X + (size_t)min(base + 8 * h + t, row_max) * (D / 2) + W * j);
        };
        auto compute = [&](const uint32_t (&src)[8][W]) __attribute__((always_inline)) {
            // 8x(2W) transpose of 16-bit elements: fragment s holds column CPL*j+s of the
            // lane's eight rows, two rows per word (one byte-permute per word).
            v4u frag[CPL];
#pragma unroll
            for (int s = 0; s < CPL; ++s) {
                uint32_t o[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    o[u] = __builtin_amdgcn_perm(src[2 * u + 1][s / 2], src[2 * u][s / 2],
                                                 (s & 1) ? 0x07060302u : 0x05040100u);
                frag[s] = v4u{o[0], o[1], o[2], o[3]};
            }
            int p = 0;
#pragma unroll
            for (int s1 = 0; s1 < CPL; ++s1)
#pragma unroll
                for (int s2 = s1; s2 < CPL; ++s2) {
                    acc[p] = mfma16x16x32bf16(frag[s1], frag[s2], acc[p]);
                    ++p;
                }
        };
        // a block of the tail: rows at or past the end of the chunk count as zero
        auto compute_tail = [&](uint32_t (&src)[8][W], int base) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < 8; ++t)
                if (base + 8 * h + t >= r1) {
#pragma unroll
                    for (int w = 0; w < W; ++w) src[t][w] = 0u;
                }
            compute(src);
        };
        // ring of kRing row blocks per wave: kRing-1 blocks of loads stay in flight while one
        // block is multiplied, with the ring index fixed at compile time by the unrolling.  The
        // steady-state loop takes kRing whole blocks per trip and has no branch in its body; at
        // most kRing - 1 whole blocks and one ragged block are left for the tail.
        constexpr int kRing = SOLAR_GRAM_RING;
        uint32_t ring[kRing][8][W];
        constexpr int stride = kGramWaves * STEP;
        const int base0 = r0 + wave * STEP;
        const int nblk = base0 < r1 ? ceil_div(r1 - base0, stride) : 0;              // blocks of this wave
        const int nwhole = r1 - base0 >= STEP ? (r1 - base0 - STEP) / stride + 1 : 0;  // of which whole
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
    } else {
        // float inputs: the same ring of row blocks (16 rows per block: lane (j, h) holds rows
        // 4t + h, t = 0..3, and the loaded values are the MFMA operands as they stand)
        const float* X = reinterpret_cast<const float*>(Xv) + (size_t)b * N * D + CPL * j;
        const int row_max = max(r1 - 1, 0);
        auto load = [&](float (&dst)[4][CPL], int base) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float* p = X + (size_t)min(base + 4 * t + h, row_max) * D;
#pragma unroll
                for (int q = 0; q < CPL / 4; ++q) {
                    const v4f v = *reinterpret_cast<const v4f*>(p + 4 * q);
                    dst[t][4 * q + 0] = v.x; dst[t][4 * q + 1] = v.y;
                    dst[t][4 * q + 2] = v.z; dst[t][4 * q + 3] = v.w;
                }
            }
        };
        auto compute = [&](const float (&src)[4][CPL]) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                int p = 0;
#pragma unroll
                for (int s1 = 0; s1 < CPL; ++s1)
#pragma unroll
                    for (int s2 = s1; s2 < CPL; ++s2) {
                        acc[p] = mfma16x16x4(src[t][s1], src[t][s2], acc[p]);
                        ++p;
                    }
            }
        };
        auto compute_tail = [&](float (&src)[4][CPL], int base) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (base + 4 * t + h >= r1) {
#pragma unroll
                    for (int s = 0; s < CPL; ++s) src[t][s] = 0.f;
                }
            compute(src);
        };
        constexpr int kRing = SOLAR_GRAM_RING;
        float ring[kRing][4][CPL];
        constexpr int stride = kGramWaves * STEP;
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
                __builtin_amdgcn_sched_barrier(0);
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
    }

    v4f* out = reinterpret_cast<v4f*>(partials) + ((size_t)b * nsplit + split) * (NP * 64);
    reduce_waves_and_store<NP>(acc, out);
}

// G[b][a][c] = sum over chunks of the partial block element that holds (a, c) or,
// below the diagonal of fragment pairs, its mirror image (c, a).
template <int CPL>
__global__ __launch_bounds__(256) void gram_finalize_kernel(const float* __restrict__ partials,
                                                            int nsplit, float* __restrict__ G) {
    constexpr int D = 16 * CPL;
    constexpr int NP = gram_pairs<CPL>();
    const int b = blockIdx.y;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= D * D) return;
    int a = e / D, c = e % D;
    int s1 = a % CPL, i1 = a / CPL, s2 = c % CPL, i2 = c / CPL;
    if (s1 > s2) {
        int t = s1; s1 = s2; s2 = t;
        t = i1; i1 = i2; i2 = t;
    }
    const int pair = s1 * CPL - (s1 * (s1 - 1)) / 2 + (s2 - s1);
    const int off = pair * 256 + (i2 + 16 * (i1 / 4)) * 4 + (i1 % 4);
    const float* p = partials + (size_t)b * nsplit * (NP * 256) + off;
    float acc = 0.f;
#pragma unroll 8
    for (int s = 0; s < nsplit; ++s) acc += p[(size_t)s * (NP * 256)];
    G[(size_t)b * D * D + e] = acc;
}

// ---- d = 256 ---------------------------------------------------------------------------
// 136 fragment pairs do not fit one wave's accumulators, so G is cut into the four 128 x 128
// blocks of its 2 x 2 block form and a workgroup (blockIdx.z = job) forms one of
//   job 0: G00 = X0^T X0 (36 symmetric pairs)     job 1: G11 = X1^T X1 (36 pairs)
//   job 2: G01 = X0^T X1, fragments s1 = 0..3 of X0 against all 8 of X1 (32 pairs)
//   job 3: the same for s1 = 4..7
// with X0, X1 the left and right 128 columns.  G10 is the mirror image of G01.
constexpr int kGram256Pairs = 36;   // partial slots per job (jobs 2, 3 use 32 of them)

template <bool BF16>
__global__ __launch_bounds__(kGramWaves * 64) void gram256_partial_kernel(
    const void* __restrict__ Xv, const int32_t* __restrict__ lengths, int N, int nsplit,
    float* __restrict__ partials) {
    constexpr int D = 256, CPL = 8, NP = kGram256Pairs;
    constexpr int STEP = BF16 ? 32 : 16;
    const int b = blockIdx.y, split = blockIdx.x, job = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, h = lane >> 4;
    const int len = user_len(lengths, b, N);
    const int chunk = ceil_div(ceil_div(len, nsplit), STEP) * STEP;
    const int r0 = split * chunk;
    const int r1 = min(len, r0 + chunk);
    const bool cross = job >= 2;
    const int colA = (job == 1) ? 128 : 0;          // half that supplies the A fragments
    const int colB = (job == 0) ? 0 : 128;          // half that supplies the B fragments
    const int sa0 = (job == 3) ? 4 : 0;             // first A fragment of a cross job

    v4f acc[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) acc[p] = v4f{0.f, 0.f, 0.f, 0.f};

    auto mma = [&](auto& fa, auto& fb) __attribute__((always_inline)) {
        // fa, fb: the eight fragments of the A half and of the B half for this k-step
        if (!cross) {
            int p = 0;
#pragma unroll
            for (int s1 = 0; s1 < CPL; ++s1)
#pragma unroll
                for (int s2 = s1; s2 < CPL; ++s2) {
                    if constexpr (BF16) acc[p] = mfma16x16x32bf16(fa[s1], fa[s2], acc[p]);
                    else acc[p] = mfma16x16x4(fa[s1], fa[s2], acc[p]);
                    ++p;
                }
        } else {
#pragma unroll
            for (int s1 = 0; s1 < 4; ++s1)
#pragma unroll
                for (int s2 = 0; s2 < CPL; ++s2) {
                    if constexpr (BF16) {
                        const v4u a = sa0 ? fa[s1 + 4] : fa[s1];
                        acc[s1 * CPL + s2] = mfma16x16x32bf16(a, fb[s2], acc[s1 * CPL + s2]);
                    } else {
                        const float a = sa0 ? fa[s1 + 4] : fa[s1];
                        acc[s1 * CPL + s2] = mfma16x16x4(a, fb[s2], acc[s1 * CPL + s2]);
                    }
                }
        }
    };

    if constexpr (BF16) {
        const uint32_t* X = reinterpret_cast<const uint32_t*>(Xv) + (size_t)b * N * (D / 2);
        auto load_frags = [&](v4u (&frag)[CPL], int base, int col0) __attribute__((always_inline)) {
            uint32_t in[8][4];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const int row = base + 8 * h + t;
                v4u v = v4u{0u, 0u, 0u, 0u};
                if (row < r1) v = *reinterpret_cast<const v4u*>(X + (size_t)row * (D / 2) + col0 / 2 + 4 * j);
                in[t][0] = v.x; in[t][1] = v.y; in[t][2] = v.z; in[t][3] = v.w;
            }
#pragma unroll
            for (int s = 0; s < CPL; ++s) {
                uint32_t o[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t a = in[2 * u][s / 2], c = in[2 * u + 1][s / 2];
                    o[u] = (s & 1) ? ((a >> 16) | (c & 0xffff0000u)) : ((a & 0xffffu) | (c << 16));
                }
                frag[s] = v4u{o[0], o[1], o[2], o[3]};
            }
        };
        for (int base = r0 + wave * STEP; base < r1; base += kGramWaves * STEP) {
            v4u fa[CPL], fb[CPL];
            load_frags(fa, base, colA);
            if (cross) load_frags(fb, base, colB);
            mma(fa, fb);
        }
    } else {
        const float* X = reinterpret_cast<const float*>(Xv) + (size_t)b * N * D;
        for (int base = r0 + wave * STEP; base < r1; base += kGramWaves * STEP) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int row = base + 4 * t + h;
                float fa[CPL], fb[CPL];
#pragma unroll
                for (int q = 0; q < CPL / 4; ++q) {
                    v4f va = v4f{0.f, 0.f, 0.f, 0.f}, vb = va;
                    if (row < r1) {
                        va = *reinterpret_cast<const v4f*>(X + (size_t)row * D + colA + CPL * j + 4 * q);
                        if (cross) vb = *reinterpret_cast<const v4f*>(X + (size_t)row * D + colB + CPL * j + 4 * q);
                    }
                    fa[4 * q + 0] = va.x; fa[4 * q + 1] = va.y; fa[4 * q + 2] = va.z; fa[4 * q + 3] = va.w;
                    fb[4 * q + 0] = vb.x; fb[4 * q + 1] = vb.y; fb[4 * q + 2] = vb.z; fb[4 * q + 3] = vb.w;
                }
                mma(fa, fb);
            }
        }
    }

    v4f* out = reinterpret_cast<v4f*>(partials) + (((size_t)b * nsplit + split) * 4 + job) * (NP * 64);
    reduce_waves_and_store<NP>(acc, out);
}

// bf16 inputs: the four jobs are the four waves of one workgroup and share every row block through
// LDS, so X is read from HBM once.  Wave w loads columns 64w .. 64w+63 of a 32-row block (16 lanes
// per row, four columns per lane), transposes them in registers into the four MFMA operand
// fragments 4w .. 4w+3 (fragment f, lane j: column 64 (f/4) + 4j + f%4) and parks them in LDS; after
// one barrier every wave reads the 8 or 12 fragments of its job.  Fragments 0..7 are the left half
// X0, 8..15 the right half X1, so the jobs and the partial slots are those of the layout above.
// The fragment buffer is double: a wave that writes block i+2 has passed the barrier of block
// i+1, which every wave reaches only after its reads of block i.  Loads run kGram256Ring - 1
// blocks ahead in registers (16 registers per block and lane), unconditional and clamped to the
// chunk's last row as in gram_partial_kernel.
constexpr int kGram256Ring = 4;

__global__ __launch_bounds__(kGramWaves * 64) void gram256_shared_kernel(
    const void* __restrict__ Xv, const int32_t* __restrict__ lengths, int N, int nsplit,
    float* __restrict__ partials) {
    constexpr int D = 256, NP = kGram256Pairs, STEP = 32, kRing = kGram256Ring;
    static_assert(kRing % 2 == 0, "the LDS buffer index follows the ring slot's parity");
    __shared__ __attribute__((aligned(16))) v4u fragbuf[2][16][64];
    const int b = blockIdx.y, split = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 15, h = lane >> 4;
    const int len = user_len(lengths, b, N);
    const int chunk = ceil_div(ceil_div(len, nsplit), STEP) * STEP;
    const int r0 = split * chunk;
    const int r1 = min(len, r0 + chunk);
    const int nblk = r1 > r0 ? ceil_div(r1 - r0, STEP) : 0;   // the same for all four waves
    const int nwhole = r1 > r0 ? (r1 - r0) / STEP : 0;
    const int row_max = max(r1 - 1, 0);
    const uint32_t* X = reinterpret_cast<const uint32_t*>(Xv) + (size_t)b * N * (D / 2) + 32 * wave + 2 * j;

    v4f acc[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) acc[p] = v4f{0.f, 0.f, 0.f, 0.f};

    auto load = [&](uint2 (&dst)[8], int blk) __attribute__((always_inline)) {
        const int base = r0 + blk * STEP + 8 * h;
#pragma unroll
        for (int t = 0; t < 8; ++t)
            dst[t] = *reinterpret_cast<const uint2*>(X + (size_t)min(base + t, row_max) * (D / 2));
    };
    auto stage = [&](const uint2 (&src)[8], int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            uint32_t o[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t lo = (s / 2) ? src[2 * u].y : src[2 * u].x;
                const uint32_t hi = (s / 2) ? src[2 * u + 1].y : src[2 * u + 1].x;
                o[u] = __builtin_amdgcn_perm(hi, lo, (s & 1) ? 0x07060302u : 0x05040100u);
            }
            fragbuf[buf][4 * wave + s][lane] = v4u{o[0], o[1], o[2], o[3]};
        }
    };
    auto stage_tail = [&](uint2 (&src)[8], int blk, int buf) __attribute__((always_inline)) {
        const int base = r0 + blk * STEP + 8 * h;
#pragma unroll
        for (int t = 0; t < 8; ++t)
            if (base + t >= r1) src[t] = uint2{0u, 0u};
        stage(src, buf);
    };
    auto consume = [&](int buf) __attribute__((always_inline)) {
        if (wave < 2) {
            v4u f[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) f[s] = fragbuf[buf][8 * wave + s][lane];
            int p = 0;
#pragma unroll
            for (int s1 = 0; s1 < 8; ++s1)
#pragma unroll
                for (int s2 = s1; s2 < 8; ++s2) {
                    acc[p] = mfma16x16x32bf16(f[s1], f[s2], acc[p]);
                    ++p;
                }
        } else {
            v4u fa[4], fb[8];
#pragma unroll
            for (int s = 0; s < 4; ++s) fa[s] = fragbuf[buf][4 * (wave - 2) + s][lane];
#pragma unroll
            for (int s = 0; s < 8; ++s) fb[s] = fragbuf[buf][8 + s][lane];
#pragma unroll
            for (int s1 = 0; s1 < 4; ++s1)
#pragma unroll
                for (int s2 = 0; s2 < 8; ++s2)
                    acc[s1 * 8 + s2] = mfma16x16x32bf16(fa[s1], fb[s2], acc[s1 * 8 + s2]);
        }
    };

    uint2 ring[kRing][8];
#pragma unroll
    for (int k = 0; k < kRing - 1; ++k) load(ring[k], k);
    int i = 0;
    for (; i + kRing <= nwhole; i += kRing) {
#pragma unroll
        for (int k = 0; k < kRing; ++k) {
            load(ring[(k + kRing - 1) % kRing], i + k + kRing - 1);
            __builtin_amdgcn_sched_barrier(0);   // the prefetch is issued before the block is used
            stage(ring[k], k & 1);
            __syncthreads();
            consume(k & 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int k = 0; k < kRing; ++k) {
        if (i + k < nblk) {
            if (i + k + kRing - 1 < nblk) load(ring[(k + kRing - 1) % kRing], i + k + kRing - 1);
            stage_tail(ring[k], i + k, k & 1);
            __syncthreads();
            consume(k & 1);
        }
    }

    v4f* out = reinterpret_cast<v4f*>(partials) + (((size_t)b * nsplit + split) * 4 + wave) * (NP * 64);
#pragma unroll
    for (int p = 0; p < NP; ++p) out[p * 64 + lane] = acc[p];
}

// Sum over the chunks and undo the fragment permutation of gram256_shared_kernel.  A workgroup
// owns one 64 x 64 block (q1 <= q2) of G's 4 x 4 block form, i.e. the 4 x 4 fragment pairs
// (4 q1 + s1, 4 q2 + s2): wave s1 reads the partial blocks of its four pairs as they were stored
// (one 16-byte element per lane and chunk, consecutive lanes consecutive addresses), adds the
// chunks in a fixed order, and drops the sums into an LDS tile at (4 i1 + s1, 4 i2 + s2); the tile
// then goes out row by row, and transposed into the mirror block when q1 < q2.  On the diagonal
// only the pairs s1 <= s2 exist; their mirror images fill the rest of the tile.
__global__ __launch_bounds__(256) void gram256_gather_kernel(const float* __restrict__ partials, int nsplit,
                                                             float* __restrict__ G) {
    constexpr int D = 256, NP = kGram256Pairs, T = 64, LDT = T + 1;
    __shared__ float tile[T * LDT];
    const int b = blockIdx.y;
    int q1 = 0, q2 = blockIdx.x;                       // blockIdx.x enumerates the pairs q1 <= q2
    while (q2 >= 4 - q1) { q2 -= 4 - q1; ++q1; }
    q2 += q1;
    const int lane = threadIdx.x & 63, s1 = threadIdx.x >> 6;
    const bool diag = q1 == q2;
    const bool same_half = q1 / 2 == q2 / 2;
    const int fl1 = 4 * (q1 % 2) + s1;
    const int job = same_half ? q1 / 2 : 2 + q1 % 2;
    const v4f* base = reinterpret_cast<const v4f*>(partials) + ((size_t)b * nsplit * 4 + job) * (NP * 64) + lane;
    const size_t split_stride = (size_t)4 * NP * 64;
    v4f sum[4];
    int pair[4];
    const int row_start = fl1 * 8 - (fl1 * (fl1 - 1)) / 2;   // slot of the pair (fl1, fl1)
#pragma unroll
    for (int s2 = 0; s2 < 4; ++s2) {
        const int fl2 = 4 * (q2 % 2) + s2;
        // a pair below the diagonal is not stored: it reads the slot (fl1, fl1) and drops the value
        pair[s2] = same_half ? row_start + max(fl2 - fl1, 0) : s1 * 8 + fl2;
        sum[s2] = v4f{0.f, 0.f, 0.f, 0.f};
    }
    // four chunks (16 loads) are in flight before the first is added; the order of the additions is
    // that of the chunks either way
    int s = 0;
    for (; s + 4 <= nsplit; s += 4) {
        v4f part[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2) part[u][s2] = base[(size_t)(s + u) * split_stride + pair[s2] * 64];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2) sum[s2] += part[u][s2];
    }
    for (; s < nsplit; ++s) {
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2) sum[s2] += base[(size_t)s * split_stride + pair[s2] * 64];
    }
    const int i2 = lane & 15;
#pragma unroll
    for (int s2 = 0; s2 < 4; ++s2) {
        if (diag && s2 < s1) continue;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int i1 = 4 * (lane >> 4) + k;
            const int row = 4 * i1 + s1, col = 4 * i2 + s2;
            tile[row * LDT + col] = sum[s2][k];
            if (diag && s2 > s1) tile[col * LDT + row] = sum[s2][k];
        }
    }
    __syncthreads();
    float* Gb = G + (size_t)b * D * D;
    for (int e = threadIdx.x; e < T * T; e += 256) {
        const int row = e / T, col = e % T;
        Gb[(size_t)(T * q1 + row) * D + T * q2 + col] = tile[row * LDT + col];
        if (!diag) Gb[(size_t)(T * q2 + row) * D + T * q1 + col] = tile[col * LDT + row];
    }
}

__global__ __launch_bounds__(256) void gram256_finalize_kernel(const float* __restrict__ partials,
                                                               int nsplit, float* __restrict__ G) {
    constexpr int D = 256, CPL = 8, NP = kGram256Pairs;
    const int b = blockIdx.y;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= D * D) return;
    int a = e / D, c = e % D;
    if (a / 128 > c / 128) { const int t = a; a = c; c = t; }   // lower-left block: mirror
    const int ha = a / 128, hc = c / 128;
    int s1 = (a % 128) % CPL, i1 = (a % 128) / CPL, s2 = (c % 128) % CPL, i2 = (c % 128) / CPL;
    int job, pair;
    if (ha == hc) {
        job = ha;
        if (s1 > s2) {
            int t = s1; s1 = s2; s2 = t;
            t = i1; i1 = i2; i2 = t;
        }
        pair = s1 * CPL - (s1 * (s1 - 1)) / 2 + (s2 - s1);
    } else {
        job = 2 + (s1 >= 4 ? 1 : 0);
        pair = (s1 % 4) * CPL + s2;
    }
    const int off = pair * 256 + (i2 + 16 * (i1 / 4)) * 4 + (i1 % 4);
    const float* p = partials + ((size_t)b * nsplit * 4 + job) * (NP * 256) + off;
    float acc = 0.f;
    for (int s = 0; s < nsplit; ++s) acc += p[(size_t)s * 4 * (NP * 256)];
    G[(size_t)b * D * D + e] = acc;
}

int gram_nsplit(int B, int N) {
    // One workgroup per compute unit (its accumulators leave room for one wave per SIMD, so a
    // second round of workgroups would only queue behind the first), at least 512 rows per
    // chunk.
    constexpr int target = 256;
    int want = ceil_div(target, B);
    int cap = ceil_div(N, 512);
    int n = want < cap ? want : cap;
    if (n < 1) n = 1;
    if (n > 64) n = 64;
    return n;
}

size_t gram_partial_floats(int B, int N, int d) {
    if (d == 256) return (size_t)B * gram_nsplit(B, N) * 4 * kGram256Pairs * 256;
    const int cpl = d / 16;
    return (size_t)B * gram_nsplit(B, N) * (cpl * (cpl + 1) / 2) * 256;
}

template <int CPL>
static hipError_t launch_gram_t(const void* X, const int32_t* lengths, int B, int N, bool bf16,
                                float* partials, float* G, bool finalize, hipStream_t stream) {
    const int nsplit = gram_nsplit(B, N);
    dim3 grid(nsplit, B), block(kGramWaves * 64);
    constexpr size_t lds = gram_reduce_lds<gram_pairs<CPL>()>();
    hipError_t e = bf16 ? gram_allow_lds(gram_partial_kernel<CPL, true>, lds)
                        : gram_allow_lds(gram_partial_kernel<CPL, false>, lds);
    if (e != hipSuccess) return e;
    if (bf16)
        hipLaunchKernelGGL((gram_partial_kernel<CPL, true>), grid, block, lds, stream, X, lengths, N,
                           nsplit, partials);
    else
        hipLaunchKernelGGL((gram_partial_kernel<CPL, false>), grid, block, lds, stream, X, lengths, N,
                           nsplit, partials);
    if (finalize) {
        constexpr int D = 16 * CPL;
        dim3 g2(ceil_div(D * D, 256), B);
        hipLaunchKernelGGL((gram_finalize_kernel<CPL>), g2, dim3(256), 0, stream, partials, nsplit, G);
    }
    return hipGetLastError();
}

bool gram_partials_consumable(int d) { return d == 64 || d == 128; }

hipError_t launch_gram(const void* X, const int32_t* lengths, int B, int N, int d, bool bf16,
                       float* partials, float* G, bool finalize, hipStream_t stream) {
    if (!gram_partials_consumable(d)) finalize = true;
    switch (d) {
        case 64: return launch_gram_t<4>(X, lengths, B, N, bf16, partials, G, finalize, stream);
        case 128: return launch_gram_t<8>(X, lengths, B, N, bf16, partials, G, finalize, stream);
        case 256: {
            const int nsplit = gram_nsplit(B, N);
            dim3 block(kGramWaves * 64), g2(256 * 256 / 256, B);
            if (bf16) {
                hipLaunchKernelGGL(gram256_shared_kernel, dim3(nsplit, B), block, 0, stream, X, lengths, N, nsplit,
                                   partials);
                hipLaunchKernelGGL(gram256_gather_kernel, dim3(10, B), dim3(256), 0, stream, partials, nsplit, G);
                return hipGetLastError();
            }
            dim3 grid(nsplit, B, 4);
            constexpr size_t lds = gram_reduce_lds<kGram256Pairs>();
            hipError_t e = bf16 ? gram_allow_lds(gram256_partial_kernel<true>, lds)
                                : gram_allow_lds(gram256_partial_kernel<false>, lds);
            if (e != hipSuccess) return e;
            if (bf16)
                hipLaunchKernelGGL((gram256_partial_kernel<true>), grid, block, lds, stream, X, lengths, N,
                                   nsplit, partials);
            else
                hipLaunchKernelGGL((gram256_partial_kernel<false>), grid, block, lds, stream, X, lengths, N,
                                   nsplit, partials);
            hipLaunchKernelGGL(gram256_finalize_kernel, g2, dim3(256), 0, stream, partials, nsplit, G);
            return hipGetLastError();
        }
        default: return hipErrorInvalidValue;
    }
}

}  // namespace solar
