// SVD-Attention, Attn_SVD = MatMul(MatMul(Query, Key_r^T), Value_r) (Section
// "SVD-Attention"), on gfx950.
//
// attention_seq_kernel -- softmax over the N sequence positions, evaluated in
// factor space:   O = softmax_n(scale * Qt P^T) P V^T,   Qt = Q V,  P = X V.
// The M x N score matrix is never stored: the kernel walks over tiles of P with an
// online softmax (running row maximum and row sum), keeps Z = sum_n w_n P_n in the
// matrix-unit accumulators and only at the end maps Z / l back to d columns with
// V^T.  Key and value are the same tile of P, so one LDS tile feeds both products.
// All three products use the float 16x16x4 MFMA, whose operands are single values
// per lane; the transposed forms S^T = P Qt^T and Z^T = P^T W^T are used so that a
// query is a lane (column l%16 of every accumulator): the softmax statistics of a
// query are then combined over 4 lane groups only, and the accumulator of one
// product is directly the B operand of the next with no data movement (the
// contraction index may be enumerated in any order as long as A and B agree).
//
// attention_tokens_kernel -- the literal r-token form, with or without softmax:
//   O = softmax_k(scale * Q T^T) T   or   O = scale * (Q T^T) T,   T = diag(S) V^T.
#include <cstdlib>

#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kAttnThreads = 256;
constexpr int kNT = 64;   // rows of P per tile
constexpr float kLog2e = 1.4426950408889634f;

// Accumulator component (lane group g, register t) of a 16-row output block is
// bound to rank index g + 4*t of the block instead of 4*g + t: with this choice the
// four lane groups read four consecutive floats of an LDS row when the accumulator
// is reused as a B operand, which keeps those reads free of bank conflicts.
__device__ __forceinline__ int rank_perm(int i) { return (i >> 2) + 4 * (i & 3); }

// NS > 1: the workgroup has NS groups of four waves; group sp takes every NS-th tile of the
// sequence for the same queries and the groups' partial results (reference, row sum, Z) are
// merged in a fixed order at the end.  It gives a small batch, whose workgroups do not fill the
// GPU's wave slots, NS independent chains of products and exponentials per SIMD.
template <int D, int RB, bool BF16, int QB, int NS>
__global__ __launch_bounds__(kAttnThreads * NS) void attention_seq_kernel(
    const void* __restrict__ Qv, const float* __restrict__ V, const float* __restrict__ P,
    const int32_t* __restrict__ lengths, int B, int N, int r, int M, float scale, float* __restrict__ O) {
    constexpr int RP = 16 * RB;
    constexpr int LDV = RP + 4;
    constexpr int LDP = RP + 4;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* Vs = smem;                       // [D][LDV]
    float* Ps = Vs + D * LDV;               // [2][NS][kNT][LDP]
    constexpr int NTHR = kAttnThreads * NS;
    // Workgroups are dealt to the 8 XCDs round-robin by linear id.  All M-tiles of a user
    // get ids that agree modulo 8, so they share one XCD and its L2 holds that user's P once.
    const int mtiles = ceil_div(M, 4 * QB * 16);
    const int slot = blockIdx.x >> 3;
    const int b = (slot / mtiles) * 8 + (blockIdx.x & 7);
    if (b >= B) return;   // uniform over the workgroup
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = (tid >> 6) & 3;        // query group of the wave
    const int sp = tid >> 8;                // its share of the sequence (0 when NS == 1)
    const int i16 = lane & 15, g = lane >> 4;
    const int len = user_len(lengths, b, N);
    const int m_wave = (slot % mtiles) * (4 * QB * 16) + wave * (QB * 16);
    const float* Pb = P + (size_t)b * N * r;

    for (int e = tid; e < D * RP; e += NTHR) {
        const int k = e / RP, c = e % RP;
        Vs[k * LDV + c] = (c < r) ? V[((size_t)b * D + k) * r + c] : 0.f;
    }
    // zero both P tiles once so that the padded rank columns stay zero
    for (int e = tid; e < 2 * NS * kNT * LDP; e += NTHR) Ps[e] = 0.f;
    __syncthreads();

    // ---- prologue: Qt^T = V^T Q^T, scaled by scale*log2(e) -------------------------
    v4f qt[QB][RB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
        for (int ib = 0; ib < RB; ++ib) qt[qb][ib] = v4f{0.f, 0.f, 0.f, 0.f};
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
                for (int ib = 0; ib < RB; ++ib)
                    qt[qb][ib] = mfma16x16x4(vrow[16 * ib + rank_perm(i16)], q4[t], qt[qb][ib]);
            }
        }
#pragma unroll
        for (int ib = 0; ib < RB; ++ib) qt[qb][ib] *= scale * kLog2e;
    }

    // ---- main loop over tiles of P -------------------------------------------------
    v4f z[QB][RB];
    float mrun[QB], lrun[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        mrun[qb] = -INFINITY;
        lrun[qb] = 0.f;
#pragma unroll
        for (int ib = 0; ib < RB; ++ib) z[qb][ib] = v4f{0.f, 0.f, 0.f, 0.f};
    }

    const int ntiles = ceil_div(ceil_div(len, kNT), NS);   // steps of NS tiles
    constexpr int kRows = NS * kNT;                        // rows loaded per step
    // A step is kRows*r consecutive floats of P; a thread moves float4 (r % 4 == 0) or falls
    // back to scalars.
    auto load_tile = [&](int tile, float* dst) {
        const int n0 = tile * kRows;
        if ((r & 3) == 0) {
            const int quads_per_row = r >> 2;
            for (int e = tid; e < kRows * quads_per_row; e += NTHR) {
                const int nn = e / quads_per_row, c4 = e % quads_per_row;
                v4f v = v4f{0.f, 0.f, 0.f, 0.f};
                if (n0 + nn < len) v = *reinterpret_cast<const v4f*>(Pb + (size_t)(n0 + nn) * r + 4 * c4);
                *reinterpret_cast<v4f*>(dst + nn * LDP + 4 * c4) = v;
            }
        } else {
            for (int e = tid; e < kRows * r; e += NTHR) {
                const int nn = e / r, c = e % r;
                dst[nn * LDP + c] = (n0 + nn < len) ? Pb[(size_t)(n0 + nn) * r + c] : 0.f;
            }
        }
    };
    if (ntiles > 0) load_tile(0, Ps);
    __syncthreads();

    for (int tile = 0; tile < ntiles; ++tile) {
        const float* pt = Ps + ((tile & 1) * NS + sp) * (kNT * LDP);
        if (tile + 1 < ntiles) load_tile(tile + 1, Ps + ((tile + 1) & 1) * (kRows * LDP));
        const int n0 = (tile * NS + sp) * kNT;
        if (n0 < len) {   // uniform over the wave: only the last step can leave a group without rows

        // scores S^T[n][m] for the 4 blocks of 16 rows
        v4f s[QB][kNT / 16];
#pragma unroll
        for (int nb = 0; nb < kNT / 16; ++nb) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) s[qb][nb] = v4f{0.f, 0.f, 0.f, 0.f};
            const float* prow = pt + (16 * nb + i16) * LDP;
#pragma unroll
            for (int ib = 0; ib < RB; ++ib)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float a = prow[16 * ib + 4 * t + g];
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        s[qb][nb] = mfma16x16x4(a, qt[qb][ib][t], s[qb][nb]);
                }
        }
        // mask rows past the valid length (component t of block nb is row 16*nb + 4*g + t)
        if (n0 + kNT > len) {
#pragma unroll
            for (int nb = 0; nb < kNT / 16; ++nb)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (n0 + 16 * nb + 4 * g + t >= len) {
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb) s[qb][nb][t] = -INFINITY;
                    }
        }
        // online softmax per query (= per lane column), weights overwrite the scores
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float mt = -INFINITY;
#pragma unroll
            for (int nb = 0; nb < kNT / 16; ++nb)
#pragma unroll
                for (int t = 0; t < 4; ++t) mt = fmaxf(mt, s[qb][nb][t]);
            mt = wave_xor_max(mt, 16);
            mt = wave_xor_max(mt, 32);
            const float mnew = fmaxf(mrun[qb], mt);   // finite: row 0 of tile 0 is valid
            const float alpha = __builtin_amdgcn_exp2f(mrun[qb] - mnew);
            mrun[qb] = mnew;
            float lsum = 0.f;
#pragma unroll
            for (int nb = 0; nb < kNT / 16; ++nb)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float w = __builtin_amdgcn_exp2f(s[qb][nb][t] - mnew);
                    s[qb][nb][t] = w;
                    lsum += w;
                }
            lrun[qb] = lrun[qb] * alpha + lsum;
#pragma unroll
            for (int ib = 0; ib < RB; ++ib) z[qb][ib] *= alpha;
        }
        // Z^T += P^T W^T : contraction slot g of step (nb, t) is row 16*nb + 4*g + t
#pragma unroll
        for (int nb = 0; nb < kNT / 16; ++nb)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float* prow = pt + (16 * nb + 4 * g + t) * LDP;
#pragma unroll
                for (int ib = 0; ib < RB; ++ib) {
                    const float a = prow[16 * ib + rank_perm(i16)];
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
                        z[qb][ib] = mfma16x16x4(a, s[qb][nb][t], z[qb][ib]);
                }
            }
        }
        __syncthreads();
    }

    // ---- merge of the sequence shares (group 0 takes the others in order) -----------------
    if constexpr (NS > 1) {
        constexpr int kState = QB * (4 * RB + 2);   // floats per lane
        float* st = Ps;                              // [NS-1][4 waves][kState][64 lanes]
        if (sp > 0) {
            float* mine = st + ((sp - 1) * 4 + wave) * (kState * 64) + lane;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                mine[(qb * (4 * RB + 2) + 0) * 64] = mrun[qb];
                mine[(qb * (4 * RB + 2) + 1) * 64] = lrun[qb];
#pragma unroll
                for (int ib = 0; ib < RB; ++ib)
#pragma unroll
                    for (int t = 0; t < 4; ++t) mine[(qb * (4 * RB + 2) + 2 + 4 * ib + t) * 64] = z[qb][ib][t];
            }
        }
        __syncthreads();
        if (sp > 0) return;
        for (int o = 0; o < NS - 1; ++o) {
            const float* other = st + (o * 4 + wave) * (kState * 64) + lane;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const float mo = other[(qb * (4 * RB + 2) + 0) * 64];
                const float lo = other[(qb * (4 * RB + 2) + 1) * 64];
                const float mnew = fmaxf(mrun[qb], mo);
                // a share without rows has reference -inf and contributes nothing
                const float a0 = mrun[qb] > -INFINITY ? __builtin_amdgcn_exp2f(mrun[qb] - mnew) : 0.f;
                const float a1 = mo > -INFINITY ? __builtin_amdgcn_exp2f(mo - mnew) : 0.f;
                mrun[qb] = mnew;
                lrun[qb] = lrun[qb] * a0 + lo * a1;
#pragma unroll
                for (int ib = 0; ib < RB; ++ib)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        z[qb][ib][t] = z[qb][ib][t] * a0 + other[(qb * (4 * RB + 2) + 2 + 4 * ib + t) * 64] * a1;
            }
        }
    }

    // ---- epilogue: O^T = V (Z / l)^T ------------------------------------------------
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float l = lrun[qb];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const float inv = l > 0.f ? 1.f / l : 0.f;
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
                    o = mfma16x16x4(vrow[16 * ib + 4 * t + g], z[qb][ib][t], o);
            if (m < M) *reinterpret_cast<v4f*>(O + ((size_t)b * M + m) * D + 16 * cb + 4 * g) = o;
        }
    }
}

// Literal r-token form.  One wave per candidate at a time; lane k holds token k.
template <bool BF16>
__global__ __launch_bounds__(256) void attention_tokens_kernel(
    const void* __restrict__ Qv, const float* __restrict__ S, const float* __restrict__ V, int d,
    int r, int M, float scale, int softmax, float* __restrict__ O) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int LDT = d + 1;
    float* T = smem;               // [r][LDT]  T[k][j] = S[k] V[j][k]
    const int b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int e = tid; e < d * r; e += 256) {
        const int j = e / r, k = e % r;
        T[k * LDT + j] = S[(size_t)b * r + k] * V[((size_t)b * d + j) * r + k];
    }
    __syncthreads();
    const int rows_per_block = 64;
    for (int mi = wave; mi < rows_per_block; mi += 4) {
        const int m = blockIdx.x * rows_per_block + mi;
        if (m >= M) break;   // uniform over the wave
        // lane holds q[lane], q[lane+64], ... ; values are handed round with shuffles
        float qreg[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int j = lane + 64 * c;
            qreg[c] = 0.f;
            if (j < d) {
                const size_t idx = ((size_t)b * M + m) * d + j;
                qreg[c] = BF16 ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(Qv)[idx] << 16)
                               : reinterpret_cast<const float*>(Qv)[idx];
            }
        }
        float sc = 0.f;
        const float* tk = T + (lane < r ? lane : 0) * LDT;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (64 * c < d)
                for (int jj = 0; jj < 64; ++jj) sc += __shfl(qreg[c], jj) * tk[64 * c + jj];
        sc *= scale;
        float w;
        if (softmax) {
            float mx = lane < r ? sc : -INFINITY;
            for (int msk = 1; msk < 64; msk <<= 1) mx = fmaxf(mx, __shfl_xor(mx, msk));
            float ex = lane < r ? __builtin_amdgcn_exp2f((sc - mx) * kLog2e) : 0.f;
            float sum = ex;
            for (int msk = 1; msk < 64; msk <<= 1) sum += __shfl_xor(sum, msk);
            w = ex / sum;
        } else {
            w = lane < r ? sc : 0.f;
        }
        for (int j = lane; j < d; j += 64) {
            float acc = 0.f;
            for (int k = 0; k < r; ++k) acc += __shfl(w, k) * T[k * LDT + j];
            O[((size_t)b * M + m) * d + j] = acc;
        }
    }
}

}  // namespace

template <int D, int RB, int QB, int NS>
static hipError_t launch_seq_q(const void* Q, const float* V, const float* P,
                               const int32_t* lengths, int B, int N, int r, int M, float scale,
                               bool bf16, float* O, hipStream_t stream) {
    constexpr int RP = 16 * RB;
    const size_t lds = sizeof(float) * ((size_t)D * (RP + 4) + 2 * NS * kNT * (RP + 4));
    dim3 grid(ceil_div(M, 4 * QB * 16) * 8 * ceil_div(B, 8)), block(kAttnThreads * NS);
    if (bf16) {
        auto kern = attention_seq_kernel<D, RB, true, QB, NS>;
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, Q, V, P, lengths, B, N, r, M, scale, O);
    } else {
        auto kern = attention_seq_kernel<D, RB, false, QB, NS>;
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, Q, V, P, lengths, B, N, r, M, scale, O);
    }
    return hipGetLastError();
}

// A wave takes two 16-query blocks (each row of P read from LDS serves both) unless that leaves
// fewer workgroups than compute units; then one block per wave fills the GPU.  If the workgroups
// of four waves still leave the SIMDs with fewer than four waves each, the sequence is shared
// out among two or four groups of waves per workgroup (as far as the tile buffers fit LDS).
template <int D, int RB, int QB>
static hipError_t launch_seq_n(const void* Q, const float* V, const float* P,
                               const int32_t* lengths, int B, int N, int r, int M, float scale,
                               bool bf16, float* O, hipStream_t stream) {
    const long long wgs = (long long)B * ceil_div(M, 64 * QB);
    int ns = wgs >= 1024 ? 1 : (wgs >= 512 ? 2 : 4);
    // two query blocks per wave leave room for two groups only (four would hold 16 waves to 128
    // registers each, which that variant does not fit; nor does it fit 256 at d = 256, r > 48)
    constexpr int kMaxNs = QB == 1 ? 4 : ((D == 256 && RB == 4) ? 1 : 2);
    if (ns > kMaxNs) ns = kMaxNs;
    constexpr size_t row = sizeof(float) * (16 * RB + 4);
    while (ns > 1 && D * row + 2 * ns * kNT * row > 150 * 1024) ns /= 2;
    while (ns > 1 && N <= (ns / 2) * kNT) ns /= 2;   // no more groups than tiles
    if constexpr (kMaxNs >= 4) {
        if (ns == 4) return launch_seq_q<D, RB, QB, 4>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
    }
    if constexpr (kMaxNs >= 2) {
        if (ns == 2) return launch_seq_q<D, RB, QB, 2>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
    }
    return launch_seq_q<D, RB, QB, 1>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
}

template <int D, int RB>
static hipError_t launch_seq_t(const void* Q, const float* V, const float* P,
                               const int32_t* lengths, int B, int N, int r, int M, float scale,
                               bool bf16, float* O, hipStream_t stream) {
    if ((long long)B * ceil_div(M, 128) < 256)
        return launch_seq_n<D, RB, 1>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
    return launch_seq_n<D, RB, 2>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
}

template <int D>
static hipError_t launch_seq_d(const void* Q, const float* V, const float* P,
                               const int32_t* lengths, int B, int N, int r, int M, float scale,
                               bool bf16, float* O, hipStream_t stream) {
    switch ((r + 15) / 16) {
        case 1: return launch_seq_t<D, 1>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
        case 2: return launch_seq_t<D, 2>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
        case 3: return launch_seq_t<D, 3>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
        case 4: return launch_seq_t<D, 4>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_attention_seq(const void* Q, const float* V, const float* P,
                                const int32_t* lengths, int B, int N, int d, int r, int M,
                                float scale, bool bf16, float* O, hipStream_t stream) {
    switch (d) {
        case 64: return launch_seq_d<64>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
        case 128: return launch_seq_d<128>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
        case 256: return launch_seq_d<256>(Q, V, P, lengths, B, N, r, M, scale, bf16, O, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_attention_tokens(const void* Q, const float* S, const float* V, int B, int d,
                                   int r, int M, float scale, bool softmax, bool bf16, float* O,
                                   hipStream_t stream) {
    const size_t lds = sizeof(float) * ((size_t)r * (d + 1));
    dim3 grid(ceil_div(M, 64), B), block(256);
    if (bf16) {
        auto kern = attention_tokens_kernel<true>;
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, Q, S, V, d, r, M, scale, softmax ? 1 : 0, O);
    } else {
        auto kern = attention_tokens_kernel<false>;
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, Q, S, V, d, r, M, scale, softmax ? 1 : 0, O);
    }
    return hipGetLastError();
}

}  // namespace solar
