// SVD-Attention in its sequence-softmax form, O = softmax_n(scale * Qt P^T) P V^T
// (Section "SVD-Attention"; Qt = Q V, P = X V), fast path for bf16 inputs and rank <= 64
// on the 32x32x16 fp16 matrix instruction of gfx950.  The rank is padded to RP = 32 (one
// 32-rank half; what follows describes it) or RP = 64 (two halves: twice the score and Z
// products per block, which loads the matrix unit as heavily as the vector ALU's issue port).
//
// The kernel is bound by the issue port of the vector ALU, which the matrix instructions
// share.  Measured per wave instruction: an MFMA holds the port for about 8 cycles whatever
// its shape, an exponential (f32 or f16) for 8.5, a float-pair-to-fp16 pack for 7.4, a plain
// operation for 5.  Hence
//   * 32x32x16 products: one instruction covers 1024 scores where the 16x16x32 shape covers
//     256, so a block of 32 rows of P against 32 queries costs two MFMAs for the scores and
//     two for Z^T += P^T W^T;
//   * row sums of the rounded weights by one more (16x16x32) MFMA per 16 rows against ones:
//     it costs the issue port a fraction of what a chain of dependent vector adds or packed
//     dot products costs (their result latency is exposed), and the matrix pipe has room;
//   * the softmax reference is not maintained at all on the first, optimistic pass over the
//     sequence (it stays a few log2 units above the first block's maximum; a weight that
//     leaves the fp16 range turns the row sum infinite), and only a workgroup that saw that
//     happen repeats the sequence with a guarded pass whose reference moves lazily: a
//     block's scores are compared against it (a maximum over the lane's 16 scores, taken
//     while the block before is exponentiated).
//
// P and Qt are rounded to fp16 once (11-bit significands; P is first scaled by 1/S[0] when
// S[0] lies outside [1, 2^13]); the scores carry about 2^-11 relative error, inside the 2e-2
// contract for bf16 inputs.  Accumulation is in float throughout.
//
// As in the other attention kernels the products are evaluated transposed (S^T = P Qt^T,
// Z^T = P^T W^T) so that a query is a lane (lane l and l+32 share query l%32 and split the
// rows of a block): the accumulators of the score product are the B operand of the Z
// product without any data movement, because the contraction index can be enumerated in any
// order as long as both operands agree.  Register t of a 32x32 accumulator in lane l is row
// 8*(t/4) + 4*(l/32) + t%4, so contraction slot u (0..7) of lane half h is
//   * rank 16*c + 8*(u/4) + 4*h + u%4 for chunk c of the score product: the loader stores
//     rank quads 1 and 2 of every 16 ranks swapped, which makes a lane's eight ranks one
//     16-byte LDS read;
//   * row 16*c + 8*(u/4) + 4*h + u%4 of the block for chunk c of the Z product: two
//     transposing LDS reads (four rows each) out of the same row-major image.
//
// A workgroup is eight waves of 32 queries.  The sequence is walked in tiles of 128 rows
// through three LDS buffers (one being multiplied, the next complete, the third being
// converted) and, inside a tile, in blocks of 32 rows through a software pipeline: while the
// exponentials of block j run, the matrix unit computes the scores of block j+1 and adds
// block j-1 to Z.
#include <cstdlib>
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kQW = 32;              // queries per wave
constexpr int kNT = 128;             // rows of P per tile
constexpr int kNB = kNT / 32;        // blocks per tile
// RP is the padded rank (32 or 64); LDR = RP + 8 fp16 elements per row of a tile image [kNT][LDR]
constexpr float kLog2e = 1.4426950408889634f;
// a score more than kShift (in log2 units) above the reference moves the reference there, so
// no weight exceeds 2^kShift: far inside the fp16 range, and the row sums stay far inside float
#ifndef SOLAR_X32_KSHIFT
#define SOLAR_X32_KSHIFT 8.f
#endif
constexpr float kShift = SOLAR_X32_KSHIFT;
// optimistic pass: the reference stays `head` log2 units above the largest score of the first
// block, so weights stay inside the fp16 range while no score lies more than 16 + head above it.
// A weight below 2^-25 rounds to zero, so against a peak weight of 2^-head a flat tail of N rows
// can lose N * 2^(head - 25) of the softmax mass at worst; the host lowers the head room with N
// so that this stays below 2^-7: 4 up to N = 16384, 2 up to 65536, 0 up to 262144, and the
// guarded pass alone beyond that (its peak weight is at least 1).
inline float optimistic_head_room(int N) { return N <= 16384 ? 4.f : (N <= 65536 ? 2.f : 0.f); }
constexpr int kOptimisticMaxN = 262144;

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));

__device__ __forceinline__ v16f mma32(v4u a, v4u b, v16f c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c,
                                                  0, 0, 0);
}

__device__ __forceinline__ v16f mma32bf(v4u a, v4u b, v16f c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

__device__ __forceinline__ v4f mma16(v4u a, v4u b, v4f c) {
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

// transposing 64-bit LDS read of 16-bit elements: within a group of 16 lanes, lane i passes
// the address of four consecutive elements and receives element i%4 of the lanes i/4,
// 4 + i/4, 8 + i/4, 12 + i/4
__device__ __forceinline__ uint2 lds_read_tr16(const uint16_t* p) {
    typedef short v4s __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;
    const v4s v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(p));
    return __builtin_bit_cast(uint2, v);
}

// position of rank quad c4 (ranks 4*c4 .. 4*c4+3) in a row of the tile image: quads 1 and 2
// of every 16 ranks are swapped
__device__ __forceinline__ int quad_pos(int c4) { return (c4 & ~3) | ((c4 & 1) << 1) | ((c4 >> 1) & 1); }

// FUSED: Pin is the user's X (bf16, [B][N][D]) and the loader forms the rows of P = X V itself
// (the projection of Section "SVD-Attention" evaluated where it is consumed; every workgroup of
// a user repeats it); otherwise Pin is P (float, [B][N][r]).
template <int D, int RP, bool FUSED>
__global__ __launch_bounds__(kThreads) void attention_seq_x32_kernel(
    const void* __restrict__ Qv, const float* __restrict__ S, const float* __restrict__ V,
    const void* __restrict__ Pin, const int32_t* __restrict__ lengths, int B, int N, int r, int M,
    float scale, int guarded_only, float head, int longest_first, float* __restrict__ O) {
    static_assert(RP == 32 || RP == 64, "one or two 32-rank halves");
    static_assert(RP == 32 || D <= 128, "the bf16 images of V for 64 ranks of d = 256 do not fit LDS");
    constexpr int LDR = RP + 8, kBuf = kNT * LDR;
    constexpr int NC = RP / 16;   // 16-rank chunks of the score product
    constexpr int NH = RP / 32;   // 32-rank halves of Z
    extern __shared__ __attribute__((aligned(16))) float smem[];
    // V as bf16 head (truncated, so the remainder is exact) and tail, in the two orders the
    // matrix unit wants it: transposed for Qt^T = V^T Q^T (and the fused projection), and row
    // by row with the rank quads in the order of the tile images for O^T = V Z^T
    constexpr int LDVT = D + 8, LDI = RP + 8;                      // bf16 elements
    uint16_t* tiles = reinterpret_cast<uint16_t*>(smem);           // [3][kBuf]
    int* redo = reinterpret_cast<int*>(tiles + 3 * kBuf);          // set when a wave's optimistic pass overflowed
    uint16_t* vt = reinterpret_cast<uint16_t*>(redo + 4);          // [2][RP][LDVT]
    uint16_t* vimg = vt + 2 * RP * LDVT;                           // [2][D][LDI]
    // Workgroups are dealt to the 8 XCDs round-robin by linear id.  All M-tiles of a user
    // get ids that agree modulo 8, so they share one XCD and its L2 holds that user's P once.
    const int mtiles = ceil_div(M, kWaves * kQW);
    const int slot_id = blockIdx.x >> 3;
    const int place = (slot_id / mtiles) * 8 + (blockIdx.x & 7);
    if (place >= B) return;   // uniform over the workgroup
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n32 = lane & 31, h = lane >> 5;
    // When the launch has more workgroups than the GPU holds at once, the users are taken in order of
    // decreasing length (ties by index), so that the long sequences start first and the short
    // ones fill the tail: the workgroup at place k takes the user of rank k.
    int b = place;
    if (longest_first) {   // uniform over the launch
        int* lens = reinterpret_cast<int*>(tiles);
        for (int u = tid; u < B; u += kThreads) lens[u] = user_len(lengths, u, N);
        __syncthreads();
        for (int u = tid; u < B; u += kThreads) {
            const int lu = lens[u];
            int rank = 0;
            for (int j = 0; j < B; ++j) {
                const int lj = lens[j];
                rank += (lj > lu || (lj == lu && j < u)) ? 1 : 0;
            }
            if (rank == place) *redo = u;   // exactly one thread of the workgroup
        }
        __syncthreads();
        b = *redo;
        __syncthreads();
    }
    const int len = user_len(lengths, b, N);
    const int m_wave = (slot_id % mtiles) * (kWaves * kQW) + wave * kQW;
    // P is scaled into [-1, 1] by the largest singular value before it is rounded to fp16
    // when that value lies outside [1, 2^13]; inside that range fp16 holds P as it is
    float pscale = 1.f, punscale = 1.f;
    bool rescale = false;
    {
        const float s0 = S[(size_t)b * r];
        rescale = s0 > 0.f && !(s0 >= 1.f && s0 <= 8192.f);
        if (rescale) { pscale = 1.f / s0; punscale = s0; }
    }

    // The loads of the prologue are issued before anything waits: the wave's queries (HBM), then
    // this thread's share of V; the tile buffers are zeroed while they are in flight.
    constexpr int KQ = D / 16;            // 16-column steps of the query product
    const int m = m_wave + n32;
    const bool valid = m < M;
    v4u qreg[KQ];
    {
        const uint16_t* qrow = reinterpret_cast<const uint16_t*>(Qv) + ((size_t)b * M + (valid ? m : 0)) * D + 8 * h;
#pragma unroll
        for (int kk = 0; kk < KQ; ++kk) qreg[kk] = *reinterpret_cast<const v4u*>(qrow + 16 * kk);
    }
    // V by rank quads (r is a multiple of 4): quad e of the D * RP / 4 is row e / (RP/4), ranks
    // 4 * (e % (RP/4)) .. +3; consecutive threads read consecutive quads of a row
    constexpr int VQ = D * (RP / 4) / kThreads;   // quads per thread
    static_assert(VQ * kThreads == D * (RP / 4), "whole quads per thread");
    v4f vreg[VQ];
#pragma unroll
    for (int i = 0; i < VQ; ++i) {
        const int e = tid + i * kThreads, k = e / (RP / 4), c4 = e % (RP / 4);
        vreg[i] = 4 * c4 < r ? *reinterpret_cast<const v4f*>(V + ((size_t)b * D + k) * r + 4 * c4) : v4f{0.f, 0.f, 0.f, 0.f};
    }
    // zero the tile buffers once: padded rank columns stay zero for ever
    static_assert((3 * kBuf) % 8 == 0, "whole 16-byte stores");
    for (int e = tid; e < 3 * kBuf / 8; e += kThreads) reinterpret_cast<v4u*>(tiles)[e] = v4u{0u, 0u, 0u, 0u};
    if (tid == 0) *redo = 0;
#pragma unroll
    for (int i = 0; i < VQ; ++i) {
        const int e = tid + i * kThreads, k = e / (RP / 4), c4 = e % (RP / 4);
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float v = vreg[i][u];
            hi[u] = __float_as_uint(v) & 0xffff0000u;
            const float rem = v - __uint_as_float(hi[u]);
            lo[u] = (__float_as_uint(rem) + 0x7fffu + ((__float_as_uint(rem) >> 16) & 1u)) >> 16;
            vt[(4 * c4 + u) * LDVT + k] = (uint16_t)(hi[u] >> 16);
            vt[(RP + 4 * c4 + u) * LDVT + k] = (uint16_t)lo[u];
        }
        const int pos = 4 * quad_pos(c4);
        *reinterpret_cast<uint2*>(vimg + k * LDI + pos) = uint2{(hi[0] >> 16) | hi[1], (hi[2] >> 16) | hi[3]};
        *reinterpret_cast<uint2*>(vimg + (D + k) * LDI + pos) = uint2{lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16)};
    }
    __syncthreads();

    // ---- prologue: Qt^T = V^T Q^T on the 32x32x16 bf16 MFMA (head and tail of V against the
    // bf16 queries as they are: both contraction operands are 16-byte reads), scaled by
    // scale*log2(e), rounded to fp16 ----------------------------------------------------------
    v4u qB[NC];
    {
        v16f qt[NH];
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
#pragma unroll
            for (int t = 0; t < 16; ++t) qt[hh][t] = 0.f;
        const uint16_t* va = vt + n32 * LDVT + 8 * h;
#pragma unroll
        for (int kk = 0; kk < KQ; ++kk) {
            v4u w = qreg[kk];
            if (!valid) w = v4u{0u, 0u, 0u, 0u};
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                qt[hh] = mma32bf(*reinterpret_cast<const v4u*>(va + (32 * hh) * LDVT + 16 * kk), w, qt[hh]);
                qt[hh] = mma32bf(*reinterpret_cast<const v4u*>(va + (RP + 32 * hh) * LDVT + 16 * kk), w, qt[hh]);
            }
        }
        // B operand of the score product, chunk c: slot u of lane half h is register 8*(c%2) + u of
        // rank half c/2
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            float q[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                q[u] = fminf(fmaxf(qt[c / 2][8 * (c % 2) + u] * (scale * kLog2e * punscale), -6.0e4f), 6.0e4f);
            qB[c] = v4u{pack_f16(q[0], q[1]), pack_f16(q[2], q[3]), pack_f16(q[4], q[5]), pack_f16(q[6], q[7])};
        }
    }

    // ---- tile loader: float P -> fp16 image [kNT][LDR] ------------------------------------
    // A thread owns RPT consecutive rows and four consecutive ranks of a tile.  The loads carry
    // no predicate: byte offsets into the user's P advance by one tile per fetch, and for a
    // ragged last tile the rows are clamped to the last valid one (they are zeroed when that
    // tile is converted).  Rank quads at or beyond r load quad r/4-1 and are never stored.
    constexpr int kQuads = RP / 4;
    constexpr int RPT = kNT * kQuads / kThreads;   // rows per thread: 2 or 4
    static_assert((kNT / RPT) * kQuads == kThreads, "one loader task per thread");
    const int nfull = len / kNT;   // tiles whose rows are all valid
    const int last_row = max(len - 1, 0);   // clamp of the row index of loads past the valid length
    // -- P given: a thread owns RPT consecutive rows and four consecutive ranks of a tile
    const int ld_np = tid / kQuads, ld_c4 = tid % kQuads;
    const bool ld_active = 4 * ld_c4 < r;
    const int ld_dst = (RPT * ld_np) * LDR + 4 * quad_pos(ld_c4);
    const uint32_t row_bytes = FUSED ? 2u * D : 4u * (uint32_t)r;
    const uint32_t ld_col = 16u * (uint32_t)min(ld_c4, (r >> 2) - 1);
    // -- X given: wave w owns rows 16*w .. 16*w+15 of a tile; lane (row l%16, group l/16) loads
    // the quarter l/16 of its row (D/4 consecutive columns), which it supplies as contraction
    // slots of the products P^T = V^T X^T (16x16x32 bf16: eight columns per lane and step; the
    // A operand from vt enumerates the columns in the same order)
    constexpr int KS = D / 32;   // products per rank block
    const int fx_row = 16 * wave + (lane & 15), fx_g = lane >> 4;
    const char* Pbytes = reinterpret_cast<const char*>(Pin) +
                         (FUSED ? (size_t)b * N * (2u * D) + (size_t)fx_g * (D / 2) : (size_t)b * N * (4u * r));
    const uint32_t ld_off0 = FUSED ? (uint32_t)fx_row * row_bytes : (uint32_t)(RPT * ld_np) * row_bytes + ld_col;
    uint32_t ld_off = ld_off0;   // this thread's first row of the next tile to fetch
    // NST sets of staging registers: a tile is loaded NST - 1/2 loop iterations before it is
    // converted, so that the loads (L2 or HBM) have more than a tile of arithmetic to arrive;
    // three sets where the registers allow it (4 % fewer cycles than two at r <= 32)
    constexpr int NST = (FUSED || RP == 64) ? 2 : 3;
    v4f stage[NST][RPT];
    v4u xst[NST][FUSED ? KS : 1];
    auto fetch = [&](int tile, auto par_tag) __attribute__((always_inline)) {
        constexpr int par = decltype(par_tag)::value;
        if constexpr (FUSED) {
            uint32_t o0 = ld_off;
            if (__builtin_expect(tile >= nfull, 0))   // uniform: the ragged last tile
                o0 = (uint32_t)min(tile * kNT + fx_row, last_row) * row_bytes;
            const v4u* p = reinterpret_cast<const v4u*>(Pbytes + o0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) xst[par][ks] = p[ks];
        } else {
            uint32_t o[RPT];
#pragma unroll
            for (int i = 0; i < RPT; ++i) o[i] = ld_off + i * row_bytes;
            if (__builtin_expect(tile >= nfull, 0)) {   // uniform: the ragged last tile
#pragma unroll
                for (int i = 0; i < RPT; ++i)
                    o[i] = (uint32_t)min(tile * kNT + RPT * ld_np + i, last_row) * row_bytes + ld_col;
            }
#pragma unroll
            for (int i = 0; i < RPT; ++i) stage[par][i] = *reinterpret_cast<const v4f*>(Pbytes + o[i]);
        }
        ld_off += (uint32_t)kNT * row_bytes;
    };
    auto commit = [&](uint16_t* buf, int tile, auto par_tag) __attribute__((always_inline)) {
        constexpr int par = decltype(par_tag)::value;
        if constexpr (FUSED) {
            // result register t of rank block nb: rank 16*nb + 4*(l/16) + t of row l%16, i.e.
            // one rank quad of the lane's row
#pragma unroll
            for (int nb = 0; nb < RP / 16; ++nb) {
                v4f pa = v4f{0.f, 0.f, 0.f, 0.f};
                const uint16_t* va = vt + (16 * nb + (lane & 15)) * LDVT + (D / 4) * fx_g;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    pa = mfma16x16x32bf16(*reinterpret_cast<const v4u*>(va + 8 * ks), xst[par][ks], pa);
                    pa = mfma16x16x32bf16(*reinterpret_cast<const v4u*>(va + RP * LDVT + 8 * ks), xst[par][ks], pa);
                }
                if (__builtin_expect(tile >= nfull, 0)) {   // uniform
                    if (tile * kNT + fx_row >= len) pa = v4f{0.f, 0.f, 0.f, 0.f};
                }
                if (__builtin_expect(rescale, 0)) pa *= pscale;   // uniform
                const int quad = 4 * nb + fx_g;
                if (4 * quad < r)
                    *reinterpret_cast<uint2*>(buf + fx_row * LDR + 4 * quad_pos(quad)) =
                        uint2{pack_f16(pa[0], pa[1]), pack_f16(pa[2], pa[3])};
            }
        } else if (ld_active) {
            uint16_t* dst = buf + ld_dst;
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                v4f x = stage[par][i];
                if (__builtin_expect(tile >= nfull, 0)) {   // uniform
                    if (tile * kNT + RPT * ld_np + i >= len) x = v4f{0.f, 0.f, 0.f, 0.f};
                }
                if (__builtin_expect(rescale, 0)) x *= pscale;   // uniform
                *reinterpret_cast<uint2*>(dst + i * LDR) = uint2{pack_f16(x[0], x[1]), pack_f16(x[2], x[3])};
            }
        }
    };

    // ---- operands of a block ----------------------------------------------------------------
    // score product: lane (row n32 of the block, half h) reads image positions 16*c + 8*h ..+7
    const int sa_off = n32 * LDR + 8 * h;
    // Z product: lanes 16*G .. 16*G+15 receive ranks 16*(G%2) .. +15 for the rows of lane half
    // G/2; lane i of the group points at row 4*(G/2) + i/4 (+8 for the second read, +16 for
    // the second chunk), rank quad 4*(G%2) + i%4
    const int za_off = (4 * h + ((lane & 15) >> 2)) * LDR + 4 * quad_pos(4 * ((lane >> 4) & 1) + (lane & 3));
    v4u sA[2][NC];              // [block parity][rank chunk]
    v4u zA[2][NH][2];           // [block parity][rank half][row chunk]

    // ---- state --------------------------------------------------------------------------------
    v16f s[2];          // scores of two consecutive blocks, relative to mref
    v4u wp[2][2];       // packed weights [block parity][chunk]
    v16f z[NH];         // Z^T, rank 32*half + 8*(t/4) + 4*h + t%4 of query n32
    v16f cinit;         // -mref in every register: start value of the score accumulators
    v4f lacc;           // row sums of the weights: lanes 0..15 hold query `lane` in component 0 and
                        // query `lane + 16` in component 1 (rows 0 and 1 of a 16x16 product)
    float mref = 0.f;
    float smax = 0.f;   // guarded pass: largest score of the lane in the block that is exponentiated next
    // A operand of the row-sum product (16x16x32: contraction slot 8*(l/16) + e, result row l%16):
    // row 0 takes the slots of the lane groups that hold queries 0..15 (even l/16), row 1 those of
    // queries 16..31; every other row is zero
    const bool sel = ((lane & 15) == 0 && ((lane >> 4) & 1) == 0) || ((lane & 15) == 1 && ((lane >> 4) & 1) == 1);
    const uint32_t one2 = sel ? 0x3c003c00u : 0u;   // two fp16 ones
    const v4u ones = v4u{one2, one2, one2, one2};
    auto reset_state = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            cinit[t] = 0.f;
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) z[hh][t] = 0.f;
        }
        lacc = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            wp[0][c] = wp[1][c] = v4u{0u, 0u, 0u, 0u};
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) zA[0][hh][c] = zA[1][hh][c] = v4u{0u, 0u, 0u, 0u};
        }
        mref = 0.f; smax = 0.f;
        ld_off = ld_off0;
    };

    // Online softmax with a lazily updated reference: weights are exp2(s - mref) and may exceed
    // one.  The scores of a block are compared with the reference before they are
    // exponentiated; only when one of them exceeds it by more than kShift (or for the first
    // block) is the block maximum formed per query, mref moved there for the queries that need
    // it, and everything that is relative to the old reference rescaled: Z, the row sums and
    // the packed weights of the block before, whose Z product is still to be issued.
    // everything that is relative to the reference moves with it by shift (log2 units)
    auto apply_shift = [&](int cur, float shift, float alpha) __attribute__((always_inline)) {
        mref += shift;
        lacc[0] *= alpha;                                   // lanes 0..15: their own query
        lacc[1] *= __shfl(alpha, (lane & 15) + 16);         // and the query 16 lanes up
        const _Float16 ah = (_Float16)alpha;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            s[cur][t] -= shift;
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) z[hh][t] *= alpha;
            cinit[t] = -mref;
        }
#pragma unroll
        for (int c = 0; c < 2; ++c)
            wp[cur ^ 1][c] = __builtin_bit_cast(v4u, __builtin_bit_cast(v8h, wp[cur ^ 1][c]) * ah);
    };
    auto move_reference = [&](int cur, bool first, float head) __attribute__((always_inline)) {
        float v = -INFINITY;
#pragma unroll
        for (int t = 0; t < 16; ++t) v = fmaxf(v, s[cur][t]);
        v = wave_xor_max(v, 32);   // block maximum of the query, relative to mref
        const float shift = first ? v + head : (v > kShift ? v : 0.f);
        apply_shift(cur, shift, first ? 0.f : __builtin_amdgcn_exp2f(-shift));
    };
    // rows of the block past the valid length get weight zero
    auto mask_block = [&](int cur, int j) __attribute__((always_inline)) {
        if (__builtin_expect((j + 1) * 32 > len, 0)) {   // uniform, only the last block
#pragma unroll
            for (int t = 0; t < 16; ++t)
                if (j * 32 + 8 * (t / 4) + 4 * h + (t % 4) >= len) s[cur][t] = -INFINITY;
        }
    };

    // One slot of the pipeline, block j of parity cur = j % 2: E(j) on the vector ALU next to
    // S(j+1), Z(j-1) and the row sums of block j on the matrix unit, the maximum of the scores
    // of block j+1 (guarded pass), and the LDS reads for S(j+2) and Z(j).  The order of issue is
    // written out and fenced pair by pair: a pack waits for its two exponentials, so it sits
    // behind the exponentials of the group after, and the matrix instructions are spread
    // between the groups so that each finds the matrix pipe free.
    // sa_next and za_this point at the score operands of block j+2 and the Z operands of block j.
    // (Raising the wave priority around every MFMA cost 4 % of the loop's cycles for the twelve
    // extra scalar instructions per slot; the oldest-first arbitration feeds the matrix unit as well.)
#define SOLAR_FENCE __builtin_amdgcn_sched_barrier(0)
    auto slot = [&](int j, auto cur_tag, auto guard_tag, const uint16_t* sa_next, const uint16_t* za_this)
                    __attribute__((always_inline)) {
        constexpr int cur = decltype(cur_tag)::value, nxt = cur ^ 1;
        constexpr bool guarded = decltype(guard_tag)::value;
        mask_block(cur, j);
        if constexpr (guarded) {
            if (__builtin_expect(__any(smax > kShift), 0)) move_reference(cur, false, 0.f);   // uniform over the wave, rare
        }
        float w[16];
        auto E = [&](int t) __attribute__((always_inline)) { w[t] = __builtin_amdgcn_exp2f(s[cur][t]); };
        // pack weights 2*e, 2*e+1 of the block (e = 0..7)
        // (optimistic pass: to nearest, so that a weight beyond the fp16 range becomes infinite
        // and shows in the row sum)
        auto C = [&](int e) __attribute__((always_inline)) {
            wp[cur][e / 4][e % 4] = guarded ? pack_f16_rtz(w[2 * e], w[2 * e + 1]) : pack_f16(w[2 * e], w[2 * e + 1]);
        };
        // running maximum of the scores of block j+1 (registers 4*i .. 4*i+3)
        auto X = [&](int i) __attribute__((always_inline)) {
            if constexpr (guarded) smax = fmaxf(fmaxf(i == 0 ? s[nxt][0] : smax, s[nxt][4 * i + (i == 0 ? 1 : 0)]),
                         fmaxf(s[nxt][4 * i + (i == 0 ? 2 : 1)], fmaxf(s[nxt][4 * i + (i == 0 ? 3 : 2)], s[nxt][4 * i + 3])));
        };
        if constexpr (RP == 32) {
            SOLAR_FENCE;
            
            s[nxt] = mma32(sA[nxt][0], qB[0], cinit);
            
            SOLAR_FENCE;
            E(0); sA[cur][0] = *reinterpret_cast<const v4u*>(sa_next);
            SOLAR_FENCE;
            E(1); sA[cur][1] = *reinterpret_cast<const v4u*>(sa_next + 16);
            SOLAR_FENCE;
            uint2 zlo, zhi;
            E(2); zlo = lds_read_tr16(za_this);
            SOLAR_FENCE;
            E(3); zhi = lds_read_tr16(za_this + 8 * LDR);
            SOLAR_FENCE;
            
            s[nxt] = mma32(sA[nxt][1], qB[1], s[nxt]);
            
            SOLAR_FENCE;
            E(4); C(0);
            SOLAR_FENCE;
            E(5); C(1);
            SOLAR_FENCE;
            E(6);
            SOLAR_FENCE;
            E(7);
            SOLAR_FENCE;
            
            z[0] = mma32(zA[nxt][0][0], wp[nxt][0], z[0]);
            
            SOLAR_FENCE;
            zA[cur][0][0] = v4u{zlo.x, zlo.y, zhi.x, zhi.y};
            E(8); C(2);
            SOLAR_FENCE;
            E(9); C(3);
            SOLAR_FENCE;
            E(10);
            SOLAR_FENCE;
            E(11);
            SOLAR_FENCE;
            
            z[0] = mma32(zA[nxt][0][1], wp[nxt][1], z[0]);
            
            SOLAR_FENCE;
            
            lacc = mma16(ones, wp[cur][0], lacc);
            
            SOLAR_FENCE;
            E(12); zlo = lds_read_tr16(za_this + 16 * LDR);
            SOLAR_FENCE;
            E(13); zhi = lds_read_tr16(za_this + 24 * LDR);
            SOLAR_FENCE;
            E(14); C(4); X(0);
            SOLAR_FENCE;
            E(15); C(5); X(1);
            SOLAR_FENCE;
            C(6); C(7);
            zA[cur][0][1] = v4u{zlo.x, zlo.y, zhi.x, zhi.y};
            SOLAR_FENCE;
            
            lacc = mma16(ones, wp[cur][1], lacc);
            
            SOLAR_FENCE;
            X(2); X(3);
            SOLAR_FENCE;
        } else {
            // two rank halves: four score products and four Z products per block; the matrix unit
            // is then as busy as the vector ALU's issue port, so its instructions are spread evenly
#define SOLAR_MFMA(stmt) SOLAR_FENCE;  stmt;  SOLAR_FENCE
            uint2 t0, t1, t2, t3;
            SOLAR_MFMA(s[nxt] = mma32(sA[nxt][0], qB[0], cinit));
            E(0); sA[cur][0] = *reinterpret_cast<const v4u*>(sa_next);
            SOLAR_FENCE;
            E(1); sA[cur][1] = *reinterpret_cast<const v4u*>(sa_next + 16);
            SOLAR_MFMA(s[nxt] = mma32(sA[nxt][1], qB[1], s[nxt]));
            E(2); sA[cur][2] = *reinterpret_cast<const v4u*>(sa_next + 32);
            SOLAR_FENCE;
            E(3); sA[cur][3] = *reinterpret_cast<const v4u*>(sa_next + 48);
            SOLAR_MFMA(s[nxt] = mma32(sA[nxt][2], qB[2], s[nxt]));
            E(4); C(0); t0 = lds_read_tr16(za_this);
            SOLAR_FENCE;
            E(5); C(1); t1 = lds_read_tr16(za_this + 8 * LDR);
            SOLAR_MFMA(s[nxt] = mma32(sA[nxt][3], qB[3], s[nxt]));
            E(6); t2 = lds_read_tr16(za_this + 32);
            SOLAR_FENCE;
            E(7); t3 = lds_read_tr16(za_this + 32 + 8 * LDR);
            SOLAR_MFMA(z[0] = mma32(zA[nxt][0][0], wp[nxt][0], z[0]));
            zA[cur][0][0] = v4u{t0.x, t0.y, t1.x, t1.y};
            E(8); C(2);
            SOLAR_FENCE;
            E(9); C(3);
            SOLAR_MFMA(z[1] = mma32(zA[nxt][1][0], wp[nxt][0], z[1]));
            zA[cur][1][0] = v4u{t2.x, t2.y, t3.x, t3.y};
            E(10); t0 = lds_read_tr16(za_this + 16 * LDR);
            SOLAR_FENCE;
            E(11); t1 = lds_read_tr16(za_this + 24 * LDR);
            SOLAR_MFMA(z[0] = mma32(zA[nxt][0][1], wp[nxt][1], z[0]));
            E(12); t2 = lds_read_tr16(za_this + 32 + 16 * LDR);
            SOLAR_FENCE;
            E(13); t3 = lds_read_tr16(za_this + 32 + 24 * LDR);
            SOLAR_MFMA(z[1] = mma32(zA[nxt][1][1], wp[nxt][1], z[1]));
            SOLAR_MFMA(lacc = mma16(ones, wp[cur][0], lacc));
            E(14); C(4); X(0);
            SOLAR_FENCE;
            E(15); C(5); X(1);
            SOLAR_FENCE;
            C(6); C(7);
            zA[cur][0][1] = v4u{t0.x, t0.y, t1.x, t1.y};
            zA[cur][1][1] = v4u{t2.x, t2.y, t3.x, t3.y};
            SOLAR_MFMA(lacc = mma16(ones, wp[cur][1], lacc));
            X(2); X(3);
            SOLAR_FENCE;
#undef SOLAR_MFMA
        }
    };

    // ---- the sequence loop ---------------------------------------------------------------------
    // Two versions of one pass over the sequence.  The optimistic one keeps the reference where
    // the first block put it (`head` above that block's largest score) and spends nothing on the
    // scores before they are exponentiated.  It is exact as long as every weight fits fp16,
    // i.e. no score lies 16 + head log2 units above the first block's maximum; a weight
    // beyond that rounds to infinity, which the row sum keeps.  If that happened to any query
    // of the workgroup, the guarded version (block maxima before every exponentiation, lazily
    // moving reference) runs the sequence again from the start.
    const int ntiles = ceil_div(len, kNT);
    const int nblocks = ceil_div(len, 32);
    using tag0 = std::integral_constant<int, 0>;
    using tag1 = std::integral_constant<int, 1>;
    auto pass = [&](auto guard_tag) __attribute__((always_inline)) {
    constexpr bool guarded = decltype(guard_tag)::value;
    reset_state();
    if (ntiles > 0) { fetch(0, tag0{}); commit(tiles, 0, tag0{}); }
    if (ntiles > 1) { fetch(1, tag0{}); commit(tiles + kBuf, 1, tag0{}); }
    fetch(2, std::integral_constant<int, 2 % NST>{});
    if constexpr (NST == 3) fetch(3, tag0{});
    __syncthreads();
    if (nblocks > 0) {
        // S(0) and the reference of the first block; the score operands of block 1
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            sA[0][c] = *reinterpret_cast<const v4u*>(tiles + sa_off + 16 * c);
            sA[1][c] = *reinterpret_cast<const v4u*>(tiles + 32 * LDR + sa_off + 16 * c);
        }
        s[0] = mma32(sA[0][0], qB[0], cinit);
#pragma unroll
        for (int c = 1; c < NC; ++c) s[0] = mma32(sA[0][c], qB[c], s[0]);
#pragma unroll
        for (int t = 0; t < 16; ++t) s[1][t] = 0.f;
        mask_block(0, 0);
        move_reference(0, true, guarded ? 0.f : head);
    }
    // byte-free rotation of the three tile buffers: element offsets of the tile being
    // multiplied, the next one and the one being converted
    int o_cur = 0, o_nxt = kBuf, o_wr = 2 * kBuf;
    // one tile: its four slots, the loads of tile + 1 + NST into the staging set that the
    // conversion of the tile before freed and, half way, the conversion of tile + 2 (loaded
    // NST - 1 iterations ago) into the free buffer
    auto run_tile = [&](int tile, auto par_tag) __attribute__((always_inline)) {
        constexpr int par = decltype(par_tag)::value;
        // (tiles past the end are loaded from clamped rows and converted into a buffer nobody
        // reads: the loop body stays free of branches around its loads, so the wait before a
        // conversion counts the younger loads instead of draining them)
        fetch(tile + 1 + NST, std::integral_constant<int, (par + 1) % NST>{});
        const uint16_t* sa_cur = tiles + o_cur + sa_off;
        const uint16_t* sa_nxt = tiles + o_nxt + sa_off;
        const uint16_t* za_cur = tiles + o_cur + za_off;
        const int j0 = tile * kNB;
        slot(j0, tag0{}, guard_tag, sa_cur + 2 * 32 * LDR, za_cur);
        if (__builtin_expect(j0 + 1 < nblocks, 1)) slot(j0 + 1, tag1{}, guard_tag, sa_cur + 3 * 32 * LDR, za_cur + 32 * LDR);
        commit(tiles + o_wr, tile + 2, std::integral_constant<int, (par + 2) % NST>{});
        if (__builtin_expect(j0 + 2 < nblocks, 1)) slot(j0 + 2, tag0{}, guard_tag, sa_nxt, za_cur + 2 * 32 * LDR);
        if (__builtin_expect(j0 + 3 < nblocks, 1)) slot(j0 + 3, tag1{}, guard_tag, sa_nxt + 32 * LDR, za_cur + 3 * 32 * LDR);
        __syncthreads();
        const int o = o_cur; o_cur = o_nxt; o_nxt = o_wr; o_wr = o;
    };
    int tile = 0;
    for (; tile + NST - 1 < ntiles; tile += NST) {
        run_tile(tile, tag0{});
        run_tile(tile + 1, tag1{});
        if constexpr (NST == 3) run_tile(tile + 2, std::integral_constant<int, 2>{});
    }
    if (tile < ntiles) run_tile(tile, tag0{});
    if constexpr (NST == 3) { if (tile + 1 < ntiles) run_tile(tile + 1, tag1{}); }
    // Z of the last block trails the loop
    if (nblocks > 0) {
        if ((nblocks - 1) & 1) {
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                z[hh] = mma32(zA[1][hh][0], wp[1][0], z[hh]);
                z[hh] = mma32(zA[1][hh][1], wp[1][1], z[hh]);
            }
        } else {
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                z[hh] = mma32(zA[0][hh][0], wp[0][0], z[hh]);
                z[hh] = mma32(zA[0][hh][1], wp[0][1], z[hh]);
            }
        }
    }
    };
    if (__builtin_expect(!guarded_only, 1)) {
        pass(std::false_type{});
        if (!(lacc[0] < 3.0e38f) || !(lacc[1] < 3.0e38f)) *redo = 1;   // some weight left the fp16 range (or the input is not finite)
    } else if (tid == 0) {
        *redo = 1;
    }
    __syncthreads();
    if (__builtin_expect(*redo != 0, 0)) {   // uniform over the workgroup
        __syncthreads();
        pass(std::true_type{});
    }
#undef SOLAR_FENCE

    // ---- epilogue: O^T = V (Z / l)^T on the bf16 MFMA with head and tail of both operands
    // (the tail-tail term, 2^-16 of the result, is dropped); chunk c of the contraction takes the
    // ranks of registers 8*(c%2) .. +7 of rank half c/2, which the V image lists in the same order
    {
        float l;
        {
            const float l0 = __shfl(lacc[0], n32 & 15), l1 = __shfl(lacc[1], n32 & 15);
            l = n32 < 16 ? l0 : l1;
        }
        const float inv = l > 0.f ? punscale / l : 0.f;
        v4u zh[NC], zl[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            uint32_t hw[4], lw[4];
#pragma unroll
            for (int u2 = 0; u2 < 4; ++u2) {
                const float a0 = z[c / 2][8 * (c % 2) + 2 * u2] * inv, a1 = z[c / 2][8 * (c % 2) + 2 * u2 + 1] * inv;
                const uint32_t h0 = __float_as_uint(a0) & 0xffff0000u, h1 = __float_as_uint(a1) & 0xffff0000u;
                hw[u2] = (h0 >> 16) | h1;
                typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
                const v2bf t = {(__bf16)(a0 - __uint_as_float(h0)), (__bf16)(a1 - __uint_as_float(h1))};
                lw[u2] = __builtin_bit_cast(uint32_t, t);
            }
            zh[c] = v4u{hw[0], hw[1], hw[2], hw[3]};
            zl[c] = v4u{lw[0], lw[1], lw[2], lw[3]};
        }
        for (int db = 0; db < D / 32; ++db) {
            v16f o;
#pragma unroll
            for (int t = 0; t < 16; ++t) o[t] = 0.f;
            const uint16_t* vh = vimg + (32 * db + n32) * LDI + 8 * h;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const v4u ah = *reinterpret_cast<const v4u*>(vh + 16 * c);
                const v4u al = *reinterpret_cast<const v4u*>(vh + D * LDI + 16 * c);
                o = mma32bf(ah, zh[c], o);
                o = mma32bf(ah, zl[c], o);
                o = mma32bf(al, zh[c], o);
            }
            if (m < M) {
                float* orow = O + ((size_t)b * M + m) * D + 32 * db + 4 * h;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<v4f*>(orow + 8 * q) = v4f{o[4 * q], o[4 * q + 1], o[4 * q + 2], o[4 * q + 3]};
            }
        }
    }
}

template <int D, int RP, bool FUSED>
hipError_t launch_d(const void* Q, const float* S, const float* V, const void* P, const int32_t* lengths,
                    int B, int N, int r, int M, float scale, float* O, hipStream_t stream) {
    // debug switch (solar_debug_option): skip the optimistic pass
    const int guarded_only = (debug_force_guarded_pass() || N > kOptimisticMaxN) ? 1 : 0;
    const float head = optimistic_head_room(N);
    constexpr int kBuf = kNT * (RP + 8);
    const size_t lds = sizeof(uint16_t) * (3 * (size_t)kBuf + 2 * RP * (size_t)(D + 8) + 2 * D * (size_t)(RP + 8)) + 16;
    dim3 grid(ceil_div(M, kWaves * kQW) * 8 * ceil_div(B, 8)), block(kThreads);
    // ranking the users costs every workgroup B^2 / 512 comparisons per thread: worth it only when the
    // launch runs in several rounds of workgroups and the lengths can differ
    const int longest_first = lengths != nullptr && grid.x > 256 && B <= 512;
    auto kern = attention_seq_x32_kernel<D, RP, FUSED>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, lds, stream, Q, S, V, P, lengths, B, N, r, M, scale, guarded_only,
                       head, longest_first, O);
    return hipGetLastError();
}

}  // namespace

bool attention_seq_x32_supported(int d, int r) {
    return (d == 64 || d == 128 || d == 256) && r >= 4 && r <= (d == 256 ? 32 : 64) && (r % 4) == 0;
}

bool attention_seq_x32_from_x_supported(int d, int r) { return attention_seq_x32_supported(d, r); }

// Q is bf16; S must not be null.
hipError_t launch_attention_seq_x32(const void* Q, const float* S, const float* V, const float* P,
                                    const int32_t* lengths, int B, int N, int d, int r, int M, float scale,
                                    float* O, hipStream_t stream) {
    if (r <= 32) {
        switch (d) {
            case 64: return launch_d<64, 32, false>(Q, S, V, P, lengths, B, N, r, M, scale, O, stream);
            case 128: return launch_d<128, 32, false>(Q, S, V, P, lengths, B, N, r, M, scale, O, stream);
            case 256: return launch_d<256, 32, false>(Q, S, V, P, lengths, B, N, r, M, scale, O, stream);
            default: return hipErrorInvalidValue;
        }
    }
    switch (d) {
        case 64: return launch_d<64, 64, false>(Q, S, V, P, lengths, B, N, r, M, scale, O, stream);
        case 128: return launch_d<128, 64, false>(Q, S, V, P, lengths, B, N, r, M, scale, O, stream);
        default: return hipErrorInvalidValue;   // d = 256 takes ranks up to 32
    }
}

// The same with the projection P = X V formed inside the kernel: X and Q are bf16.
hipError_t launch_attention_seq_x32_from_x(const void* Q, const float* S, const float* V, const void* X,
                                           const int32_t* lengths, int B, int N, int d, int r, int M, float scale,
                                           float* O, hipStream_t stream) {
    if (r > 32) {
        switch (d) {
            case 64: return launch_d<64, 64, true>(Q, S, V, X, lengths, B, N, r, M, scale, O, stream);
            case 128: return launch_d<128, 64, true>(Q, S, V, X, lengths, B, N, r, M, scale, O, stream);
            default: return hipErrorInvalidValue;
        }
    }
    switch (d) {
        case 64: return launch_d<64, 32, true>(Q, S, V, X, lengths, B, N, r, M, scale, O, stream);
        case 128: return launch_d<128, 32, true>(Q, S, V, X, lengths, B, N, r, M, scale, O, stream);
        case 256: return launch_d<256, 32, true>(Q, S, V, X, lengths, B, N, r, M, scale, O, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace solar
