// SVD-Attention in its sequence-softmax form, O = softmax_n(scale * Qt P^T) P V^T
// (Section "SVD-Attention"; Qt = Q V, P = X V), fast path for bf16 inputs on the
// bf16 matrix unit of gfx950.
//
// P and Qt are float quantities derived from the factorization, and the scores are
// exponentiated, so they are not simply rounded to bf16: each is split into a bf16
// head and a bf16 tail (x = hi + lo, |lo| <= 2^-9 |hi|) and the score product uses
// the three leading cross terms, hi*hi + lo*hi + hi*lo, accumulated in float by the
// 16x16x32 MFMA: the scores carry about 16 mantissa bits.  The softmax weights are
// rounded to bf16 once and multiplied into hi + lo of P (two MFMAs); the row sum of
// the *rounded* weights is produced by one more MFMA against a tile of ones, so the
// normalization is consistent with the weights actually used and needs neither a
// VALU add per score nor a cross-lane reduction.
//
// A second, faster variant (PREC = 1) rounds P, Qt and the weights to fp16 once (11-bit
// significands; P is first scaled by 1/S[0] so that it lies in [-1, 1]) and needs one MFMA
// where the split variant needs three or two.  Its scores carry about 2^-11 relative error
// (<= ~1e-2 absolute at scores of 20), which stays inside the 2e-2 contract for bf16 inputs;
// it is the default for bf16 inputs when S is supplied.
//
// As in the float kernel the products are evaluated transposed (S^T = P Qt^T,
// Z^T = P^T W^T) so that a query is a lane: accumulators of one product are the B
// operand of the next without any data movement, because the contraction index can
// be enumerated in any order as long as both operands agree.  The A operands come
// from two LDS images of the current tile of P that the loader writes while it
// splits the tile: row-major (contraction over the rank index, for the scores) and
// transposed (contraction over the sequence index, for Z).
//
// The kernel is bound by the vector ALU: per score half a max3, one exp2 (transcendental
// rate) and half a pack instruction, against 5/16 of a 16-cycle MFMA.  The subtraction of
// the row maximum is folded into the accumulator start value of the score MFMA.
// Eight waves per workgroup (two per SIMD) let the matrix unit of one wave run
// under the exponentials of the other.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

#ifndef SOLAR_ATTN_THREADS
#define SOLAR_ATTN_THREADS 512
#endif
#ifndef SOLAR_ATTN_NT
#define SOLAR_ATTN_NT 128
#endif
constexpr int kThreads = SOLAR_ATTN_THREADS;
constexpr int kWaves = kThreads / 64;
constexpr int kQB = 2;    // 16-query blocks per wave
// rows of P per tile; the split variant (two images per layout) and ranks above 32 take half the
// rows so that three tile buffers fit the LDS and the operands fit the registers
template <int PREC, int RB2>
constexpr int tile_rows() { return (PREC == 0 || RB2 > 1) ? 64 : SOLAR_ATTN_NT; }
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    // round to nearest even; inputs are finite
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    v2bf v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ void split_bf16(float x, float& hi, float& lo) {
    hi = (float)(__bf16)x;
    lo = x - hi;
}

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

__device__ __forceinline__ v4f mfma16x16x32f16(v4u a, v4u b, v4f c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c,
                                                  0, 0, 0);
}

// two floats -> packed fp16, round to nearest even (operands that are prepared once)
__device__ __forceinline__ uint32_t pack_f16(float a, float b) {
    v2h v = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(uint32_t, v);
}

// two floats -> packed fp16 in one instruction, round toward zero (softmax weights; their
// row sum is taken from the rounded values, so the rounding direction cancels)
__device__ __forceinline__ uint32_t pack_f16_rtz(float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}

// transposing 64-bit LDS read of 16-bit elements (see load_zops for the lane mapping)
__device__ __forceinline__ uint2 lds_read_tr16(const uint16_t* p) {
    typedef short v4s __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;
    const v4s v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(p));
    return __builtin_bit_cast(uint2, v);
}

template <int PREC>
__device__ __forceinline__ uint32_t pack_w(float a, float b);

template <int PREC>
__device__ __forceinline__ v4f mma(v4u a, v4u b, v4f c) {
    if constexpr (PREC == 0) return mfma16x16x32bf16(a, b, c);
    else return mfma16x16x32f16(a, b, c);
}

template <>
__device__ __forceinline__ uint32_t pack_w<0>(float a, float b) { return pack_bf16(a, b); }
template <>
__device__ __forceinline__ uint32_t pack_w<1>(float a, float b) { return pack_f16_rtz(a, b); }

template <int D, int RB2, bool BF16, int PREC>
__global__ __launch_bounds__(kThreads) void attention_seq_bf16_kernel(
    const void* __restrict__ Qv, const float* __restrict__ S, const float* __restrict__ V,
    const float* __restrict__ P, const int32_t* __restrict__ lengths, int B, int N, int r, int M,
    float scale, float* __restrict__ O) {
    constexpr int NIMG = PREC == 0 ? 2 : 1;   // images per layout: head (+ tail)
    constexpr int kNT = tile_rows<PREC, RB2>();
    constexpr float kBig = PREC == 0 ? 65536.f : 1024.f;   // a tile row sum above this moves the reference
    constexpr int RP = 32 * RB2;          // padded rank
    constexpr int RB = RP / 16;
    constexpr int LDV = RP + 4;           // floats
#ifndef SOLAR_ATTN_RPAD
#define SOLAR_ATTN_RPAD 4
#endif
    constexpr int LDR = RP + SOLAR_ATTN_RPAD;   // bf16 elements, row-major image  [kNT][LDR]
    constexpr int kImg = kNT * LDR;       // elements of one image
    constexpr int kBuf = NIMG * kImg;     // head (, tail)
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* Vs = smem;                                             // [D][LDV]
    uint16_t* tiles = reinterpret_cast<uint16_t*>(Vs + D * LDV);  // [3][kBuf]
    // Workgroups are dealt to the 8 XCDs round-robin by linear id.  All M-tiles of a user
    // get ids that agree modulo 8, so they share one XCD and its L2 holds that user's P once.
    const int mtiles = ceil_div(M, kWaves * kQB * 16);
    const int slot = blockIdx.x >> 3;
    const int b = (slot / mtiles) * 8 + (blockIdx.x & 7);
    if (b >= B) return;   // uniform over the workgroup
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    const int len = user_len(lengths, b, N);
    const int m_wave = (slot % mtiles) * (kWaves * kQB * 16) + wave * (kQB * 16);
    const float* Pb = P + (size_t)b * N * r;
    // PREC 1: P is scaled into [-1, 1] by the largest singular value before it is rounded
    // when it lies outside [1, 2^13]; inside that range fp16 holds P as it is
    float pscale = 1.f, punscale = 1.f;
    bool rescale = false;
    if constexpr (PREC == 1) {
        const float s0 = S[(size_t)b * r];
        rescale = s0 > 0.f && !(s0 >= 1.f && s0 <= 8192.f);
        if (rescale) { pscale = 1.f / s0; punscale = s0; }
    }

    for (int e = tid; e < D * RP; e += kThreads) {
        const int k = e / RP, c = e % RP;
        Vs[k * LDV + c] = (c < r) ? V[((size_t)b * D + k) * r + c] : 0.f;
    }
    // zero the tile buffers once: padded rank columns / rows stay zero for ever
    for (int e = tid; e < 3 * kBuf / 2; e += kThreads) reinterpret_cast<uint32_t*>(tiles)[e] = 0u;
    __syncthreads();

    // ---- prologue: Qt^T = V^T Q^T in float, scaled by scale*log2(e), split hi/lo ------
    // accumulator (lane group g, register t) of block ib is rank 16*ib + 4*g + t
    v4u qhi[kQB][RB2], qlo[kQB][RB2];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
        v4f qt[RB];
#pragma unroll
        for (int ib = 0; ib < RB; ++ib) qt[ib] = v4f{0.f, 0.f, 0.f, 0.f};
        const int m = m_wave + 16 * qb + i16;
        const bool valid = m < M;
        const size_t row = ((size_t)b * M + (valid ? m : 0)) * D;
        for (int kk = 0; kk < D / 16; ++kk) {
            v4f q4;
            if constexpr (BF16) {
                uint2 w = reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(Qv) + row)[4 * kk + g];
                q4 = v4f{bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y)};
            } else {
                q4 = reinterpret_cast<const v4f*>(reinterpret_cast<const float*>(Qv) + row)[4 * kk + g];
            }
            if (!valid) q4 = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float* vrow = Vs + (16 * kk + 4 * g + t) * LDV;
#pragma unroll
                for (int ib = 0; ib < RB; ++ib) qt[ib] = mfma16x16x4(vrow[16 * ib + i16], q4[t], qt[ib]);
            }
        }
        // B operand of the score MFMA, chunk kk of 32 ranks: slot (g, u) is rank
        // 32*kk + 16*(u/4) + 4*g + u%4, i.e. registers of blocks 2*kk and 2*kk+1
#pragma unroll
        for (int kk = 0; kk < RB2; ++kk) {
            if constexpr (PREC == 0) {
                float h[8], l[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) split_bf16(qt[2 * kk + u / 4][u % 4] * (scale * kLog2e), h[u], l[u]);
                qhi[qb][kk] = v4u{pack_bf16(h[0], h[1]), pack_bf16(h[2], h[3]), pack_bf16(h[4], h[5]), pack_bf16(h[6], h[7])};
                qlo[qb][kk] = v4u{pack_bf16(l[0], l[1]), pack_bf16(l[2], l[3]), pack_bf16(l[4], l[5]), pack_bf16(l[6], l[7])};
            } else {
                float h[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    h[u] = fminf(fmaxf(qt[2 * kk + u / 4][u % 4] * (scale * kLog2e * punscale), -6.0e4f), 6.0e4f);
                qhi[qb][kk] = v4u{pack_f16(h[0], h[1]), pack_f16(h[2], h[3]), pack_f16(h[4], h[5]), pack_f16(h[6], h[7])};
                qlo[qb][kk] = qhi[qb][kk];
            }
        }
    }

    v4f z[kQB][RB], lacc[kQB];
    float mref[kQB];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
        mref[qb] = -INFINITY;
        lacc[qb] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ib = 0; ib < RB; ++ib) z[qb][ib] = v4f{0.f, 0.f, 0.f, 0.f};
    }
    const uint32_t one2 = PREC == 0 ? 0x3f803f80u : 0x3c003c00u;   // two ones (bf16 / fp16)
    const v4u ones = v4u{one2, one2, one2, one2};

    // ---- tile loader: float P -> 16-bit image(s) [kNT][LDR] ------------------------------
    // A thread owns two consecutive rows and four consecutive ranks of a tile.  The loads carry
    // no predicate (rows and ranks are clamped into the user's P instead), so that nothing but
    // the loads themselves sits between their issue and the conversion a stage later; rows past
    // the valid length are zeroed when a ragged tile is converted.
    constexpr int kQuads = RP / 4;
    constexpr int kTasks = (kNT / 2) * kQuads;
    constexpr int kMaxLoads = (kTasks + kThreads - 1) / kThreads;
    v4f stage[kMaxLoads][2];
    auto fetch = [&](int tile) __attribute__((always_inline)) {
        const int n0 = tile * kNT;
#pragma unroll
        for (int i = 0; i < kMaxLoads; ++i) {
            const int e = tid + i * kThreads;
            const int np = e / kQuads, c4 = min(e % kQuads, (r >> 2) - 1);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int n = min(n0 + 2 * np + h, len - 1);
                stage[i][h] = *reinterpret_cast<const v4f*>(Pb + (size_t)n * r + 4 * c4);
            }
        }
    };
    auto commit = [&](uint16_t* buf, int tile, auto masked_tag) __attribute__((always_inline)) {
        uint16_t* rhi = buf;
        const int n0 = tile * kNT;
#pragma unroll
        for (int i = 0; i < kMaxLoads; ++i) {
            const int e = tid + i * kThreads;
            const int np = e / kQuads, c4 = e % kQuads;
            if ((kTasks % kThreads == 0 || e < kTasks) && 4 * c4 < r) {
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    uint16_t* dst = rhi + (2 * np + hh) * LDR + 4 * c4;
                    v4f x = stage[i][hh];
                    if constexpr (decltype(masked_tag)::value) {
                        if (n0 + 2 * np + hh >= len) x = v4f{0.f, 0.f, 0.f, 0.f};
                    }
                    if constexpr (PREC == 0) {
                        float h[4], l[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) split_bf16(x[c], h[c], l[c]);
                        *reinterpret_cast<uint2*>(dst) = uint2{pack_bf16(h[0], h[1]), pack_bf16(h[2], h[3])};
                        *reinterpret_cast<uint2*>(dst + (NIMG - 1) * kImg) =
                            uint2{pack_bf16(l[0], l[1]), pack_bf16(l[2], l[3])};
                    } else {
                        if (rescale) x *= pscale;   // uniform over the workgroup
                        *reinterpret_cast<uint2*>(dst) = uint2{pack_f16(x[0], x[1]), pack_f16(x[2], x[3])};
                    }
                }
            }
        }
    };

    // ---- per-tile building blocks -------------------------------------------------------
    // A operands of the score product: 16 rows of P per block, slot (g, u) = rank
    // 32*kk + 16*(u/4) + 4*g + u%4 (row-major image).
    v4u sah[kNT / 16][RB2], sal[kNT / 16][RB2];
    auto load_sops = [&](const uint16_t* buf) __attribute__((always_inline)) {
        const uint16_t* rhi = buf;
        const uint16_t* rlo = buf + (NIMG - 1) * kImg;
#pragma unroll
        for (int nb = 0; nb < kNT / 16; ++nb)
#pragma unroll
            for (int kk = 0; kk < RB2; ++kk) {
                const int off = (16 * nb + i16) * LDR + 32 * kk + 4 * g;
                const uint2 h0 = *reinterpret_cast<const uint2*>(rhi + off);
                const uint2 h1 = *reinterpret_cast<const uint2*>(rhi + off + 16);
                sah[nb][kk] = v4u{h0.x, h0.y, h1.x, h1.y};
                if constexpr (PREC == 0) {
                    const uint2 l0 = *reinterpret_cast<const uint2*>(rlo + off);
                    const uint2 l1 = *reinterpret_cast<const uint2*>(rlo + off + 16);
                    sal[nb][kk] = v4u{l0.x, l0.y, l1.x, l1.y};
                }
            }
    };
    // A operands of Z^T += P^T W^T: 16 ranks per block, 32 rows of the tile per chunk, slot
    // (g, u) = row 32*kb + 16*(u/4) + 4*g + u%4.  They come out of the same row-major image
    // through the transposing LDS read: within a group of 16 lanes, lane i passes the address
    // of four consecutive 16-bit elements and receives element i%4 of the lanes i/4, 4 + i/4,
    // 8 + i/4, 12 + i/4.  So lane i points at row 4*g + i/4, ranks 16*ib + 4*(i%4) ..+3, and
    // gets rank 16*ib + i of rows 4*g .. 4*g+3.
    v4u zah[kNT / 32][RB], zal[kNT / 32][RB];
    auto load_zops = [&](const uint16_t* buf) __attribute__((always_inline)) {
        const uint16_t* rhi = buf;
        const uint16_t* rlo = buf + (NIMG - 1) * kImg;
#pragma unroll
        for (int kb = 0; kb < kNT / 32; ++kb)
#pragma unroll
            for (int ib = 0; ib < RB; ++ib) {
                const int off = (32 * kb + 4 * g + (i16 >> 2)) * LDR + 16 * ib + 4 * (i16 & 3);
                const uint2 h0 = lds_read_tr16(rhi + off);
                const uint2 h1 = lds_read_tr16(rhi + off + 16 * LDR);
                zah[kb][ib] = v4u{h0.x, h0.y, h1.x, h1.y};
                if constexpr (PREC == 0) {
                    const uint2 l0 = lds_read_tr16(rlo + off);
                    const uint2 l1 = lds_read_tr16(rlo + off + 16 * LDR);
                    zal[kb][ib] = v4u{l0.x, l0.y, l1.x, l1.y};
                }
            }
    };
    // S(q): scores of query block q relative to its reference value: the accumulators start at
    // -mref (before the first tile: 0), so what leaves the matrix unit is s - mref.  The masked
    // form, which sets rows past the valid length to -inf, is only instantiated for a ragged
    // last tile (register t of block nb is row 16*nb + 4*g + t).
    v4f s[kQB][kNT / 16];
    auto scores = [&](int qb, int n0, auto masked_tag) __attribute__((always_inline)) {
        const float c0 = (mref[qb] == -INFINITY) ? 0.f : -mref[qb];
        const v4f cinit = v4f{c0, c0, c0, c0};
#pragma unroll
        for (int nb = 0; nb < kNT / 16; ++nb)
#pragma unroll
            for (int kk = 0; kk < RB2; ++kk) {
                s[qb][nb] = mma<PREC>(sah[nb][kk], qhi[qb][kk], kk == 0 ? cinit : s[qb][nb]);
                if constexpr (PREC == 0) {
                    s[qb][nb] = mma<PREC>(sal[nb][kk], qhi[qb][kk], s[qb][nb]);
                    s[qb][nb] = mma<PREC>(sah[nb][kk], qlo[qb][kk], s[qb][nb]);
                }
            }
        if constexpr (decltype(masked_tag)::value) {
#pragma unroll
            for (int nb = 0; nb < kNT / 16; ++nb)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (n0 + 16 * nb + 4 * g + t >= len) s[qb][nb][t] = -INFINITY;
        }
    };
    // one 16-row block of S(q)
    auto score_block = [&](int qb, int nb, int n0, auto masked_tag) __attribute__((always_inline)) {
        const float c0 = (mref[qb] == -INFINITY) ? 0.f : -mref[qb];
        const v4f cinit = v4f{c0, c0, c0, c0};
#pragma unroll
        for (int kk = 0; kk < RB2; ++kk) {
            s[qb][nb] = mma<PREC>(sah[nb][kk], qhi[qb][kk], kk == 0 ? cinit : s[qb][nb]);
            if constexpr (PREC == 0) {
                s[qb][nb] = mma<PREC>(sal[nb][kk], qhi[qb][kk], s[qb][nb]);
                s[qb][nb] = mma<PREC>(sah[nb][kk], qlo[qb][kk], s[qb][nb]);
            }
        }
        if constexpr (decltype(masked_tag)::value) {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (n0 + 16 * nb + 4 * g + t >= len) s[qb][nb][t] = -INFINITY;
        }
    };
    // E(q): weights rounded to 16 bits and packed as the B operand of the next product: slot
    // (g, u) of chunk kb is row 32*kb + 16*(u/4) + 4*g + u%4.  The row sums 1^T W^T of the
    // rounded weights are added to lacc (one MFMA against a tile of ones per chunk); lold keeps
    // the value from before the tile (all four registers of lacc are equal).
    v4u wp[kQB][kNT / 32];
    float lold[kQB];
    auto weights = [&](int qb) __attribute__((always_inline)) {
#pragma unroll
        for (int kb = 0; kb < kNT / 32; ++kb) {
            float w[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) w[u] = __builtin_amdgcn_exp2f(s[qb][2 * kb + u / 4][u % 4]);
            if constexpr (PREC == 0)
                wp[qb][kb] = v4u{pack_bf16(w[0], w[1]), pack_bf16(w[2], w[3]), pack_bf16(w[4], w[5]),
                                 pack_bf16(w[6], w[7])};
            else
                wp[qb][kb] = v4u{pack_f16_rtz(w[0], w[1]), pack_f16_rtz(w[2], w[3]),
                                 pack_f16_rtz(w[4], w[5]), pack_f16_rtz(w[6], w[7])};
            lacc[qb] = mma<PREC>(ones, wp[qb][kb], lacc[qb]);
        }
    };
    // the weights of one 16-row block (four per lane), or of one half of it (two per lane)
    auto weight_half = [&](int qb, int nb, int half) __attribute__((always_inline)) {
        const float w0 = __builtin_amdgcn_exp2f(s[qb][nb][2 * half]);
        const float w1 = __builtin_amdgcn_exp2f(s[qb][nb][2 * half + 1]);
        wp[qb][nb / 2][2 * (nb & 1) + half] = PREC == 0 ? pack_bf16(w0, w1) : pack_f16_rtz(w0, w1);
    };
    auto weight_block = [&](int qb, int nb) __attribute__((always_inline)) {
        weight_half(qb, nb, 0);
        weight_half(qb, nb, 1);
    };
    // C(q): online softmax with a lazily updated reference: weights are exp2(s - mref) and may
    // exceed one.  No maximum is taken on the common path: a weight above kBig shows in the
    // tile's row sum, which the matrix unit delivers anyway, so the row sum is what is
    // tested.  Only when it exceeds kBig (or is not finite), or on the first tile, is the
    // tile maximum formed, mref moved there, Z and l rescaled and the weights recomputed.
    // Every accepted weight is below kBig, far inside the range of the 16-bit formats, and
    // kBig times the sequence length is far inside the float range.
    auto settle = [&](int qb) __attribute__((always_inline)) {
        const bool first = mref[qb] == -INFINITY;
        const bool big = !(lacc[qb][0] - lold[qb] <= kBig);
        if (__any(first || big)) {   // uniform over the wave, rare
            float v = -INFINITY;
#pragma unroll
            for (int nb = 0; nb < kNT / 16; ++nb)
#pragma unroll
                for (int t = 0; t < 4; ++t) v = fmaxf(v, s[qb][nb][t]);
            v = wave_xor_max(v, 16);
            v = wave_xor_max(v, 32);   // tile maximum relative to mref; finite: a tile has a valid row
            const float shift = (first || big) ? v : 0.f;
            const float alpha = first ? 0.f : __builtin_amdgcn_exp2f(-shift);
            mref[qb] = (first ? 0.f : mref[qb]) + shift;
#pragma unroll
            for (int nb = 0; nb < kNT / 16; ++nb) s[qb][nb] -= shift;
            const float l0 = lold[qb] * alpha;
            lacc[qb] = v4f{l0, l0, l0, l0};
#pragma unroll
            for (int ib = 0; ib < RB; ++ib) z[qb][ib] *= alpha;
            weights(qb);
        }
    };
    // Z(q): Z^T += P^T W^T
    auto accumulate = [&](int qb) __attribute__((always_inline)) {
#pragma unroll
        for (int kb = 0; kb < kNT / 32; ++kb) {
#pragma unroll
            for (int ib = 0; ib < RB; ++ib) {
                z[qb][ib] = mma<PREC>(zah[kb][ib], wp[qb][kb], z[qb][ib]);
                if constexpr (PREC == 0) z[qb][ib] = mma<PREC>(zal[kb][ib], wp[qb][kb], z[qb][ib]);
            }
        }
    };
    constexpr int kSMfma = (kNT / 16) * RB2 * (PREC == 0 ? 3 : 1);   // MFMAs of one S(q)
    constexpr int kZMfma = (kNT / 32) * (NIMG * RB);                 // MFMAs of one Z(q)
    constexpr int kLMfma = kNT / 32;                                 // MFMAs of the row sums of one E(q)

    // ---- the sequence loop, software-pipelined over tiles ---------------------------------
    // Three tile buffers rotate: tile t is multiplied while tile t+1 already sits complete in
    // the second buffer and tile t+2 is converted into the third.  That lets the scores of
    // query block 0 of tile t+1 be issued inside tile t, so that every stage of the loop has
    // work for the matrix unit and for the vector ALU side by side:
    //   S(t,1) + E(t,0) | C(t,0) | Z(t,0) + S(t+1,0) + E(t,1) | C(t,1) | Z(t,1) + convert(t+2)
    // NEXT: 0 = no following tile, 1 = a full one, 2 = the ragged last one.
    const int ntiles = ceil_div(len, kNT);
    const int nfull = len / kNT;
    auto do_tile = [&](int tile, auto cur_masked, auto next_tag) __attribute__((always_inline)) {
        constexpr int NEXT = decltype(next_tag)::value;
        const uint16_t* bufc = tiles + (tile % 3) * kBuf;
        const uint16_t* bufn = tiles + ((tile + 1) % 3) * kBuf;
        uint16_t* bufw = tiles + ((tile + 2) % 3) * kBuf;
        const bool ahead = tile + 2 < ntiles;
        if (ahead) fetch(tile + 2);

        // The order of issue is written out by hand and fenced, because the instruction
        // scheduler otherwise bunches the matrix and the vector work of a stage.  A stage is
        // kNB slots; a slot issues its share of the stage's matrix units, the four
        // exponentials of one 16-row block and the two packs of the block before (a pack right
        // behind its exponentials would wait for them; issued a slot later it does not).
        constexpr int kNB = kNT / 16;
        constexpr int kUZ = (kNT / 32) * RB;   // Z units of a query block
        auto z_unit = [&](int qb, int u) __attribute__((always_inline)) {
            const int kb = u / RB, ib = u % RB;
            z[qb][ib] = mma<PREC>(zah[kb][ib], wp[qb][kb], z[qb][ib]);
            if constexpr (PREC == 0) z[qb][ib] = mma<PREC>(zal[kb][ib], wp[qb][kb], z[qb][ib]);
        };
        auto stage_of = [&](int qe, auto nunits_tag, auto&& unit) __attribute__((always_inline)) {
            constexpr int nunits = decltype(nunits_tag)::value;
            float wprev[4], wcur[4];
            lold[qe] = lacc[qe][0];
#pragma unroll
            for (int nb = 0; nb < kNB; ++nb) {
                // the row sums of a chunk whose second pack was issued one slot ago
                if (nb >= 3 && (nb & 1) == 1) lacc[qe] = mma<PREC>(ones, wp[qe][(nb - 3) / 2], lacc[qe]);
#pragma unroll
                for (int u = nb * nunits / kNB; u < (nb + 1) * nunits / kNB; ++u) unit(u);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 4; ++t) wcur[t] = __builtin_amdgcn_exp2f(s[qe][nb][t]);
                if (nb > 0) {
                    wp[qe][(nb - 1) / 2][2 * ((nb - 1) & 1)] = pack_w<PREC>(wprev[0], wprev[1]);
                    wp[qe][(nb - 1) / 2][2 * ((nb - 1) & 1) + 1] = pack_w<PREC>(wprev[2], wprev[3]);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < 4; ++t) wprev[t] = wcur[t];
            }
            wp[qe][(kNB - 1) / 2][2 * ((kNB - 1) & 1)] = pack_w<PREC>(wprev[0], wprev[1]);
            wp[qe][(kNB - 1) / 2][2 * ((kNB - 1) & 1) + 1] = pack_w<PREC>(wprev[2], wprev[3]);
            lacc[qe] = mma<PREC>(ones, wp[qe][kNB / 2 - 1], lacc[qe]);
            __builtin_amdgcn_sched_barrier(0);
        };
        // stage 1: E(t,0) next to S(t,1), then Z(t-1,1); the Z operands of this tile are read
        // once the last product with the previous tile's operands is issued
        stage_of(0, std::integral_constant<int, kUZ + kNB>{}, [&](int u) __attribute__((always_inline)) {
            if (u < kNB) score_block(1, u, tile * kNT, cur_masked);
            else z_unit(1, u - kNB);
        });
        load_zops(bufc);
        if (tile + 2 < nfull) commit(bufw, tile + 2, std::false_type{});
        else if (ahead) commit(bufw, tile + 2, std::true_type{});
        settle(0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (NEXT != 0) load_sops(bufn);
        // stage 2: E(t,1) next to Z(t,0), then S(t+1,0)
        stage_of(1, std::integral_constant<int, kUZ + (NEXT != 0 ? kNB : 0)>{}, [&](int u) __attribute__((always_inline)) {
            if (u < kUZ) z_unit(0, u);
            else score_block(0, u - kUZ, (tile + 1) * kNT, std::integral_constant<bool, NEXT == 2>{});
        });
        settle(1);
        __syncthreads();
    };
    // Z(t,1) trails its tile by one stage; before the first tile its operands are zero
#pragma unroll
    for (int kb = 0; kb < kNT / 32; ++kb) {
        wp[1][kb] = v4u{0u, 0u, 0u, 0u};
#pragma unroll
        for (int ib = 0; ib < RB; ++ib) {
            zah[kb][ib] = v4u{0u, 0u, 0u, 0u};
            zal[kb][ib] = v4u{0u, 0u, 0u, 0u};
        }
    }
    if (ntiles > 0) { fetch(0); commit(tiles, 0, std::true_type{}); }
    if (ntiles > 1) { fetch(1); commit(tiles + kBuf, 1, std::true_type{}); }
    __syncthreads();
    if (ntiles > 0) {
        load_sops(tiles);
        if (nfull == 0) scores(0, 0, std::true_type{});
        else scores(0, 0, std::false_type{});
    }
    using tag0 = std::integral_constant<int, 0>;
    using tag1 = std::integral_constant<int, 1>;
    using tag2 = std::integral_constant<int, 2>;
    // full tiles followed by a full tile
    for (int tile = 0; tile + 1 < nfull; ++tile) do_tile(tile, std::false_type{}, tag1{});
    if (nfull > 0) {
        if (nfull < ntiles) do_tile(nfull - 1, std::false_type{}, tag2{});
        else do_tile(nfull - 1, std::false_type{}, tag0{});
    }
    if (nfull < ntiles) do_tile(nfull, std::true_type{}, tag0{});
    if (ntiles > 0) accumulate(1);

    // ---- epilogue in float: O^T = V (Z / l)^T ------------------------------------------
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
        const float l = lacc[qb][0];
        const float inv = l > 0.f ? punscale / l : 0.f;
#pragma unroll
        for (int ib = 0; ib < RB; ++ib) z[qb][ib] *= inv;
        const int m = m_wave + 16 * qb + i16;
        for (int cb = 0; cb < D / 16; ++cb) {
            v4f o = v4f{0.f, 0.f, 0.f, 0.f};
            const float* vrow = Vs + (16 * cb + i16) * LDV;
#pragma unroll
            for (int ib = 0; ib < RB; ++ib)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    o = mfma16x16x4(vrow[16 * ib + 4 * g + t], z[qb][ib][t], o);
            if (m < M) *reinterpret_cast<v4f*>(O + ((size_t)b * M + m) * D + 16 * cb + 4 * g) = o;
        }
    }
}

template <int D, int RB2, int PREC>
hipError_t launch_t(const void* Q, const float* S, const float* V, const float* P,
                    const int32_t* lengths, int B, int N, int r, int M, float scale, float* O,
                    hipStream_t stream) {
    constexpr int RP = 32 * RB2;
    constexpr int NIMG = PREC == 0 ? 2 : 1;
    constexpr int kNT = tile_rows<PREC, RB2>();
    const size_t lds = sizeof(float) * (size_t)D * (RP + 4) +
                       sizeof(uint16_t) * 3 * NIMG * ((size_t)kNT * (RP + SOLAR_ATTN_RPAD));
    dim3 grid(ceil_div(M, kWaves * kQB * 16) * 8 * ceil_div(B, 8)), block(kThreads);
    auto kern = attention_seq_bf16_kernel<D, RB2, true, PREC>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, lds, stream, Q, S, V, P, lengths, B, N, r, M, scale, O);
    return hipGetLastError();
}

template <int D, int PREC>
hipError_t launch_d(const void* Q, const float* S, const float* V, const float* P,
                    const int32_t* lengths, int B, int N, int r, int M, float scale, float* O,
                    hipStream_t stream) {
    if (r <= 32) return launch_t<D, 1, PREC>(Q, S, V, P, lengths, B, N, r, M, scale, O, stream);
    if constexpr (D < 256) {
        if (r <= 64) return launch_t<D, 2, PREC>(Q, S, V, P, lengths, B, N, r, M, scale, O, stream);
    }
    return hipErrorInvalidValue;
}

template <int PREC>
hipError_t launch_p(const void* Q, const float* S, const float* V, const float* P,
                    const int32_t* lengths, int B, int N, int d, int r, int M, float scale, float* O,
                    hipStream_t stream) {
    switch (d) {
        case 64: return launch_d<64, PREC>(Q, S, V, P, lengths, B, N, r, M, scale, O, stream);
        case 128: return launch_d<128, PREC>(Q, S, V, P, lengths, B, N, r, M, scale, O, stream);
        case 256: return launch_d<256, PREC>(Q, S, V, P, lengths, B, N, r, M, scale, O, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool attention_seq_bf16_supported(int d, int r) {
    return (d == 64 || d == 128 || d == 256) && r >= 4 && r <= (d == 256 ? 32 : 64) && (r % 4) == 0;
}

// Q is bf16.  split == true: bf16 head + tail operands (about 16 mantissa bits in the scores);
// split == false: single fp16 operands scaled by S[.][0] (S must not be null).
hipError_t launch_attention_seq_bf16(const void* Q, const float* S, const float* V, const float* P,
                                     const int32_t* lengths, int B, int N, int d, int r, int M,
                                     float scale, bool split, float* O, hipStream_t stream) {
    if (split || !S) return launch_p<0>(Q, S, V, P, lengths, B, N, d, r, M, scale, O, stream);
    return launch_p<1>(Q, S, V, P, lengths, B, N, d, r, M, scale, O, stream);
}

}  // namespace solar
