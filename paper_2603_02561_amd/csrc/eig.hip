// Top-r eigenpairs of each user's d x d Gram matrix G = X^T X, one workgroup per
// user, iterate blocks held in LDS.  S = sqrt(eigenvalues), V = eigenvectors are
// the s and R that Algorithm 1 ("Randomized SVD with Power Iteration") returns.
//
// The iteration is Algorithm 1 expressed on G: a Gaussian start block Omega
// (d x L, L = r + oversampling), power steps Omega <- X^T (X Omega) = G Omega, an
// orthonormal basis of the block, and a small decomposition of the projected
// problem.  On the first power steps only the span of the block matters, and the
// basis comes from one modified Gram-Schmidt pass.  After those, basis and small
// decomposition are done together by a one-sided (Hestenes) Jacobi method on the
// d x L block Z = G Q: rotating column pairs of Z until they are mutually orthogonal
// diagonalizes Q^T G^2 Q, which is the Rayleigh-Ritz step for G^2 on span(Q), and the
// normalized columns are the next orthonormal basis.  One-sided Jacobi is insensitive
// to the huge dynamic range of the block (G Omega is dominated by the leading
// eigenvectors) and to rank deficiency (columns that vanish are dropped).  The power
// step after a Jacobi phase yields the residuals |G q_i - theta_i q_i| of the Ritz
// pairs; the iteration ends when every wanted pair is below tol_res * theta_max, and a
// failed check doubles the number of Gram-Schmidt steps before the next Jacobi phase.
//
// The phase is bound by latency, not by throughput: a Jacobi sweep is L-1 rounds of
// L/2 independent column rotations with a workgroup barrier after each round.  The
// kernel runs eight waves (two per SIMD), gives every column pair a team of up to 16
// lanes whose partial dot products are combined with DPP lane permutations, and keeps
// every trip count a compile-time constant.
#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kEigThreads = 512;
constexpr int kEigWaves = kEigThreads / 64;
// A column of the iterate whose norm falls below this fraction of the largest column norm
// is rounding noise of the float Gram matrix (about sqrt(d) * 2^-24 relative) and is dropped.
constexpr float kDeadRel = 1.0e-5f;
// Rotations are skipped below kSkipCos.  The Jacobi phase converges quadratically: a sweep whose
// largest |cos| was c leaves about c^2 behind (L * c^2 at worst), so the phase ends after the
// first sweep that met no |cos| above kSweepDone = 5e-4, with a few 1e-6 left; the residual
// check of the following power step is what accepts the result.  (1e-3 leaves V^T V up to 1.3e-5
// off the identity at 72 columns and 3e-3 up to 4e-5; 3e-2 makes the check fail and the iteration
// longer.  In a batch some user nearly always needs the sweep that a looser limit would save
// the others, so the launch is no shorter with 1e-3.)
constexpr float kSkipCos = 1.0e-7f;
constexpr float kSweepDone = 5.0e-4f;

__host__ __device__ constexpr int pow2floor_c(int x) {
    int p = 1;
    while (2 * p <= x) p *= 2;
    return p;
}
__host__ __device__ constexpr int min_c(int a, int b) { return a < b ? a : b; }

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// Standard normal draw for start-block entry (b, j, i): counter-based, Box-Muller.
__device__ __forceinline__ float omega_entry(int b, int j, int i) {
    uint32_t c = mix32((uint32_t)b * 0x9e3779b9u + (uint32_t)j * 0x85ebca6bu + (uint32_t)i + 0x1234567u);
    uint32_t c2 = mix32(c ^ 0x68bc21ebu);
    float u1 = ((c >> 8) + 1u) * (1.0f / 16777217.0f);
    float u2 = (c2 >> 8) * (1.0f / 16777216.0f);
    return sqrtf(-2.0f * __logf(u1)) * __cosf(6.28318530718f * u2);
}

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// Sum over a team of T consecutive lanes (T a power of two, team aligned to T); every
// lane of the team receives the same bits.  Up to 16 lanes the exchange is a DPP operand
// (quad permutes, then mirror within 8 and within 16 lanes).
template <int T>
__device__ __forceinline__ float team_sum(float v) {
    if constexpr (T >= 2) v += dpp_mov<0xB1>(v);    // quad_perm [1,0,3,2]
    if constexpr (T >= 4) v += dpp_mov<0x4E>(v);    // quad_perm [2,3,0,1]
    if constexpr (T >= 8) v += dpp_mov<0x141>(v);   // row_half_mirror
    if constexpr (T >= 16) v += dpp_mov<0x140>(v);  // row_mirror
    if constexpr (T >= 32) v += __shfl_xor(v, 16);
    if constexpr (T >= 64) v += __shfl_xor(v, 32);
    return v;
}

// Z = G Q with the float 16x16x4 MFMA, block rows of 16 dealt round-robin to the
// waves.  G is symmetric, so A[i][k] = G[k][i] is read with the 16 lanes of a slot group
// on consecutive addresses.  Q and Z are stored column by column (column j at j*LD).
// Gb has row stride GS: the copy of G in LDS (row stride D + 16, which puts the two slot
// groups of a half wave on disjoint banks) or, when G does not fit there, G itself.
// With a shift t the result is (G - t I) Q: the accumulators start from -t Q.
template <int D, int LP, int GS, bool SHIFTED = false>
__device__ __forceinline__ void gemm_gq(const float* Gb, const float* Qc, float* Zc, float shift = 0.f) {
    constexpr int LD = D + 4;
    constexpr int NRB = D / 16, NCB = LP / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    // a wave takes whole block rows: the operand read from G serves all NCB column blocks, whose
    // accumulators are independent chains for the matrix unit
    for (int ib = wave; ib < NRB; ib += kEigWaves) {
        const float* ga = Gb + g * GS + 16 * ib + i16;
        const float* qb = Qc + i16 * LD + g;
        v4f acc[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            if constexpr (SHIFTED)
                acc[cb] = -shift * *reinterpret_cast<const v4f*>(&Qc[(16 * cb + i16) * LD + 16 * ib + 4 * g]);
            else
                acc[cb] = v4f{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll 8
        for (int k0 = 0; k0 < D; k0 += 4) {
            const float a = ga[k0 * GS];
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) acc[cb] = mfma16x16x4(a, qb[16 * cb * LD + k0], acc[cb]);
        }
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
            *reinterpret_cast<v4f*>(&Zc[(16 * cb + i16) * LD + 16 * ib + 4 * g]) = acc[cb];
    }
}

template <int D, int L>
struct EigCfg {
    static constexpr int LP = 16 * ((L + 15) / 16);
    static constexpr int LD = D + 4;
    // lanes per column outside the Jacobi rounds
    static constexpr int TC = min_c(min_c(64, D), pow2floor_c(kEigThreads / L));
    // G is staged in LDS when it fits beside the two iterate blocks
    static constexpr bool GLDS = D <= 128;
    static constexpr int GS = GLDS ? D + 16 : D;
    static constexpr size_t lds_floats = (size_t)2 * LP * LD + 3 * LP + 8 + (GLDS ? (size_t)D * GS : 0);
};

// One cyclic sweep of one-sided Jacobi over the L columns of Zc; returns this thread's largest
// |cos| met in the sweep.
//
// A rotation needs two columns and a round of disjoint rotations touches every column, so a
// sweep that keeps the columns in LDS between rounds moves the whole block through LDS and meets
// a workgroup barrier once per round: 39 times per sweep at 40 columns, about 640 of a round's
// 1280 cycles.  Here the columns are dealt to the waves in half-groups of G = 64 / T columns (T
// lanes per column pair) and a wave keeps two half-groups A, B in registers for G rounds:
// team i of the wave holds A[i] and, in round j, B[(i + j) mod G], which the teams pass on with
// lane permutations; after G rounds every column of A has met every column of B.  The half-groups
// meet each other in a round-robin tournament of H - 1 such super-rounds, with LDS and the
// workgroup barrier only between them, and the pairs inside a half-group are taken first, G - 1
// rounds through LDS.  The number of rotations per sweep is that of any cyclic ordering; the
// barriers drop from L - 1 to (H - 1) + (G - 1).
// most power steps that a slow convergence rate may add before the first Jacobi phase
constexpr int kExtraStepsCap = 4;
// the widest team (at most 16 lanes, a float4 per lane at least) whose waves fit the workgroup
__host__ __device__ constexpr int jacobi_team_lanes(int d, int l) {
    for (int t = 16; t > 8; t /= 2) {
        const int g = 64 / t;
        if (4 * t <= d && (l + 2 * g - 1) / (2 * g) <= kEigWaves) return t;
    }
    return 8;
}

template <int D, int L>
struct JacobiCfg {
    static constexpr int T = jacobi_team_lanes(D, L);   // lanes per column pair
    static constexpr int G = 64 / T;                    // column pairs per wave = columns per half-group
    static constexpr int NW = (L + 2 * G - 1) / (2 * G);  // waves that hold columns
    static constexpr int H = 2 * NW;                    // half-groups
    static constexpr int LPAD = H * G;                  // columns including the (zero) padding
    static constexpr int CH = D / (4 * T);              // float4 per lane and column
    static_assert(NW <= kEigWaves, "one wave per pair of half-groups");
    static_assert(LPAD <= EigCfg<D, L>::LP, "the padding columns exist in LDS");
    static_assert(LPAD / 2 * T <= kEigThreads, "one team per pair in the rounds through LDS");
    static_assert(D % (4 * T) == 0 && CH >= 1, "whole float4 per lane");
};

// The rotation that makes the columns a, c of a pair orthogonal, from their squared norms al, be
// and inner product ga; the norms follow in closed form (al' = al - t ga, be' = be + t ga with
// t the tangent).  With d = be - al and g = ga, both divided by |a||c| so that squares cannot
// overflow, the rotation has cos^2 = x = 1/2 + |d| / (2 sqrt(d^2 + 4 g^2)) and
// sin = sign(d) g / (sqrt(d^2 + 4 g^2) cos): two dependent reciprocal square roots, where the
// route over zeta = d / 2g and the tangent takes four dependent transcendental steps.  Columns
// that have collapsed to rounding noise are left alone (dropped later), and so are pairs whose
// cosine is below kSkipCos.  With BRANCHLESS the rotation is always applied and a pair that is
// left alone gets the identity: no lane branches in the chain of dependent instructions, which
// pays while a lane holds up to eight elements per column.
template <int T, int CH, bool BRANCHLESS>
__device__ __forceinline__ void rotate_columns(v4f (&a)[CH], v4f (&c)[CH], float& al, float& be, float ga,
                                               float dead2, float& offmax) {
    const float ra = __builtin_amdgcn_rsqf(al), rb = __builtin_amdgcn_rsqf(be);
    const float gn = ga * ra * rb;   // cosine of the angle between the columns
    const float dn = (be - al) * ra * rb;
    const float cosv = fabsf(gn);
    const bool live = al > dead2 && be > dead2;
    const bool rot = live && cosv > kSkipCos;
    const float ih = __builtin_amdgcn_rsqf(dn * dn + 4.f * gn * gn);
    const float x = 0.5f + 0.5f * fabsf(dn) * ih;
    const float r = __builtin_amdgcn_rsqf(x);
    float cs = x * r;
    float sn = (dn >= 0.f ? gn : -gn) * ih * r;
    float tg = sn * r * ga;
    if constexpr (BRANCHLESS) {
        offmax = live ? fmaxf(offmax, cosv) : offmax;
        cs = rot ? cs : 1.f;
        sn = rot ? sn : 0.f;
        tg = rot ? tg : 0.f;
#pragma unroll
        for (int k = 0; k < CH; ++k) {
            const v4f x4 = a[k], y4 = c[k];
            a[k] = cs * x4 - sn * y4;
            c[k] = sn * x4 + cs * y4;
        }
        al -= tg;
        be += tg;
    } else {
        if (live) offmax = fmaxf(offmax, cosv);
        if (rot) {
#pragma unroll
            for (int k = 0; k < CH; ++k) {
                const v4f x4 = a[k], y4 = c[k];
                a[k] = cs * x4 - sn * y4;
                c[k] = sn * x4 + cs * y4;
            }
            al -= tg;
            be += tg;
        }
    }
}

template <int CH>
__device__ __forceinline__ float dot_ch(const v4f (&a)[CH], const v4f (&c)[CH]) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < CH; ++k) s += a[k].x * c[k].x + a[k].y * c[k].y + a[k].z * c[k].z + a[k].w * c[k].w;
    return s;
}

// pair number k of round rho of a round-robin tournament of n players (n even): player n - 1
// stays, the others go round
__device__ __forceinline__ void tournament_pair(int n, int rho, int k, int& p, int& q) {
    p = rho + k;
    q = rho - k;
    if (p >= n - 1) p -= n - 1;
    if (q < 0) q += n - 1;
    if (k == 0) p = n - 1;
}

template <int D, int L>
__device__ __forceinline__ float jacobi_sweep(float* Zc, float dead2) {
    using J = JacobiCfg<D, L>;
    constexpr int T = J::T, G = J::G, CH = J::CH, LD = EigCfg<D, L>::LD;
    constexpr bool NB = T == 16;   // measured: teams of 16 lanes gain from it, teams of 8 lose
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int u = tid % T;
    float offmax = 0.f;
    v4f a[CH], c[CH];
    auto load = [&](v4f (&dst)[CH], int col) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < CH; ++k) dst[k] = *reinterpret_cast<const v4f*>(Zc + col * LD + 4 * u + 4 * T * k);
    };
    auto store = [&](const v4f (&src)[CH], int col) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < CH; ++k) *reinterpret_cast<v4f*>(Zc + col * LD + 4 * u + 4 * T * k) = src[k];
    };
    // the pairs inside every half-group: G - 1 rounds through LDS, one team per pair
    if constexpr (G > 1) {
        const int team = tid / T;
        const int hg = team / (G / 2), k = team % (G / 2);
#pragma unroll 1
        for (int rho = 0; rho < G - 1; ++rho) {
            if (team < J::LPAD / 2) {
                int p, q;
                tournament_pair(G, rho, k, p, q);
                load(a, hg * G + p);
                load(c, hg * G + q);
                float al = team_sum<T>(dot_ch<CH>(a, a)), be = team_sum<T>(dot_ch<CH>(c, c));
                rotate_columns<T, CH, NB>(a, c, al, be, team_sum<T>(dot_ch<CH>(a, c)), dead2, offmax);
                store(a, hg * G + p);
                store(c, hg * G + q);
            }
            __syncthreads();
        }
    }
    // the pairs between half-groups: wave w holds the half-groups of pair w of the super-round
    const int i = lane / T;
#pragma unroll 1
    for (int s = 0; s < J::H - 1; ++s) {
        if (wave < J::NW) {
            int ha, hb;
            tournament_pair(J::H, s, wave, ha, hb);
            load(a, ha * G + i);
            load(c, hb * G + i);
            // squared norms once per super-round; they follow the rotations in closed form, and
            // that of a B column travels with the column
            float al = team_sum<T>(dot_ch<CH>(a, a)), be = team_sum<T>(dot_ch<CH>(c, c));
#pragma unroll
            for (int j = 0; j < G; ++j) {
                rotate_columns<T, CH, NB>(a, c, al, be, team_sum<T>(dot_ch<CH>(a, c)), dead2, offmax);
                if (j + 1 < G) {
                    // team i takes over the B column of team i + 1
                    be = __shfl(be, (lane + T) & 63);
#pragma unroll
                    for (int k = 0; k < CH; ++k) {
                        c[k].x = __shfl(c[k].x, (lane + T) & 63);
                        c[k].y = __shfl(c[k].y, (lane + T) & 63);
                        c[k].z = __shfl(c[k].z, (lane + T) & 63);
                        c[k].w = __shfl(c[k].w, (lane + T) & 63);
                    }
                }
            }
            store(a, ha * G + i);
            store(c, hb * G + (i + G - 1) % G);
        }
        __syncthreads();
    }
    return offmax;
}

// One pass of modified Gram-Schmidt over the L columns of Zc, normalized into Qc: a cheap
// orthonormal basis of span(Z) for the early power steps, where only the span matters.  The
// columns are taken in panels of kPanel: every team of TM lanes loads the panel and
// orthogonalizes it in registers (all teams do the same arithmetic in the same order, so they
// hold the same bits), team i writes panel column i, normalized, to Qc, and each team then
// projects the panel, column after column, out of the later columns it owns.  The order of
// the projections is that of column-by-column Gram-Schmidt; a panel costs one barrier where
// that costs kPanel.  Columns that collapse below dead2 (squared norm) are dropped (zero in Qc).
// The basis is orthonormal to about 2^-24 * cond(Z), which is all a power step needs.  pivot2[j]
// receives the squared norm column j had when it was normalized (the squared diagonal of the
// triangular factor, which tends to the eigenvalues of G in decreasing order).
constexpr int kPanel = 4;

template <int CH>
__device__ __forceinline__ float dot_ch(const v4f* a, const v4f* b) {
    float g = 0.f;
#pragma unroll
    for (int k = 0; k < CH; ++k) g += a[k].x * b[k].x + a[k].y * b[k].y + a[k].z * b[k].z + a[k].w * b[k].w;
    return g;
}

template <int D, int L>
__device__ __forceinline__ void mgs_orthonormalize(float* Zc, float* Qc, float* pivot2, float dead2) {
    static_assert(L % kPanel == 0, "the block is a whole number of panels");
    constexpr int LD = D + 4;
    constexpr int TM = min_c(16, D / 4);         // lanes per column
    constexpr int CH = D / (4 * TM);
    constexpr int NTEAM = kEigThreads / TM;
    static_assert(NTEAM >= kPanel, "one team per panel column");
    const int tid = threadIdx.x;
    const int team = tid / TM, u = tid % TM;
#pragma unroll 1
    for (int p0 = 0; p0 < L; p0 += kPanel) {
        v4f a[kPanel][CH];
        float inv[kPanel], nrm[kPanel];
#pragma unroll
        for (int i = 0; i < kPanel; ++i) {
            const float* zi = Zc + (p0 + i) * LD + 4 * u;
#pragma unroll
            for (int k = 0; k < CH; ++k) a[i][k] = *reinterpret_cast<const v4f*>(zi + 4 * TM * k);
        }
#pragma unroll
        for (int i = 0; i < kPanel; ++i) {
            float g[kPanel];
#pragma unroll
            for (int k = i; k < kPanel; ++k) g[k] = dot_ch<CH>(a[i], a[k]);
#pragma unroll
            for (int k = i; k < kPanel; ++k) g[k] = team_sum<TM>(g[k]);
            nrm[i] = g[i];
            inv[i] = g[i] > dead2 ? __builtin_amdgcn_rcpf(g[i]) : 0.f;   // 1 ulp: a projection coefficient
#pragma unroll
            for (int k = i + 1; k < kPanel; ++k) {
                const float c = g[k] * inv[i];
#pragma unroll
                for (int q = 0; q < CH; ++q) a[k][q] -= c * a[i][q];
            }
        }
        // team i owns panel column i: normalized into Qc (nobody reads Qc during the pass)
        if (team < kPanel) {
#pragma unroll
            for (int i = 0; i < kPanel; ++i) {
                if (team == i) {
                    const float sc = nrm[i] > dead2 ? __builtin_amdgcn_rsqf(nrm[i]) : 0.f;
                    if (u == 0) pivot2[p0 + i] = nrm[i];   // squared diagonal of the triangular factor
                    float* qi = Qc + (p0 + i) * LD + 4 * u;
#pragma unroll
                    for (int k = 0; k < CH; ++k) *reinterpret_cast<v4f*>(qi + 4 * TM * k) = a[i][k] * sc;
                }
            }
        }
        for (int c = p0 + kPanel + team; c < L; c += NTEAM) {
            float* zc = Zc + c * LD + 4 * u;
            v4f b[CH];
#pragma unroll
            for (int k = 0; k < CH; ++k) b[k] = *reinterpret_cast<const v4f*>(zc + 4 * TM * k);
            // the panel is orthogonal already, so its four projections can all be taken from the
            // column as it stands (they differ from the one-after-another values by the panel's
            // loss of orthogonality times rounding): four independent reductions instead of a
            // chain of four
            float g[kPanel];
#pragma unroll
            for (int i = 0; i < kPanel; ++i) g[i] = dot_ch<CH>(a[i], b);
#pragma unroll
            for (int i = 0; i < kPanel; ++i) g[i] = team_sum<TM>(g[i]) * inv[i];
#pragma unroll
            for (int i = 0; i < kPanel; ++i)
#pragma unroll
                for (int k = 0; k < CH; ++k) b[k] -= g[i] * a[i][k];
#pragma unroll
            for (int k = 0; k < CH; ++k) *reinterpret_cast<v4f*>(zc + 4 * TM * k) = b[k];
        }
        __syncthreads();
    }
}

template <int D, int L>
__global__ __launch_bounds__(kEigThreads) void eig_topr_kernel(
    const float* __restrict__ G, const float* __restrict__ partials, int nsplit,
    const int32_t* __restrict__ lengths, int N, int r,
    float* __restrict__ S, float* __restrict__ V, int32_t* __restrict__ info, EigParams prm) {
    using C = EigCfg<D, L>;
    constexpr int LP = C::LP, LD = C::LD, TC = C::TC;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* Zc = smem;
    float* Qc = Zc + LP * LD;
    float* theta = Qc + LP * LD;   // [LP]
    float* resid = theta + LP;     // [LP] residuals, also column norms
    int* rankv = reinterpret_cast<int*>(resid + LP);              // [LP]
    float* Gs = resid + 2 * LP + 8;                               // [D][GS] when C::GLDS
    __shared__ int sh_bits;
    __shared__ int sh_bits2;
    __shared__ float sh_rate[2];
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const float* Gb = G + (size_t)b * D * D;

    {
        const int raw = lengths ? lengths[b] : N;
        if (raw < r || raw > N) {  // uniform over the workgroup
            for (int e = tid; e < D * r; e += kEigThreads) V[(size_t)b * D * r + e] = 0.f;
            for (int e = tid; e < r; e += kEigThreads) S[(size_t)b * r + e] = 0.f;
            if (tid == 0 && info) info[b] = -1;
            return;
        }
    }
    if (tid == 0) { sh_bits = 0; sh_bits2 = 0; }
    if constexpr (C::GLDS) {
        if (partials) {
            // G from the split-N partial blocks of the Gram kernel: per chunk and fragment pair
            // (s1 <= s2 of CPL = D/16 column fragments) a 16 x 16 block in MFMA layout, lane
            // i2 + 16*(i1/4), component i1%4, holding G[CPL*i1 + s1][CPL*i2 + s2]; pairs with
            // s1 < s2 also supply the mirror image.  Chunks are summed in a fixed order.
            constexpr int CPL = D / 16, NP = CPL * (CPL + 1) / 2;
            const float* pb = partials + (size_t)b * nsplit * (NP * 256);
            // all loads of four chunks are issued before the first is used: the blocks were
            // written by other compute units and come from beyond this XCD's L2
            constexpr int ITEMS = (NP * 64 + kEigThreads - 1) / kEigThreads;
            v4f acc[ITEMS];
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) acc[i] = v4f{0.f, 0.f, 0.f, 0.f};
            for (int sp0 = 0; sp0 < nsplit; sp0 += 4) {
                v4f part[4][ITEMS];
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int i = 0; i < ITEMS; ++i) {
                        const int e = tid + i * kEigThreads;
                        const bool on = e < NP * 64 && sp0 + q < nsplit;
                        part[q][i] = on ? *reinterpret_cast<const v4f*>(pb + (size_t)(sp0 + q) * (NP * 256) + e * 4)
                                        : v4f{0.f, 0.f, 0.f, 0.f};
                    }
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int i = 0; i < ITEMS; ++i) acc[i] += part[q][i];
            }
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {
                const int e = tid + i * kEigThreads;
                if (e < NP * 64) {
                    const int pair = e >> 6, ln = e & 63;
                    int s1 = 0, rest = pair;
                    while (rest >= CPL - s1) { rest -= CPL - s1; ++s1; }
                    const int s2 = s1 + rest;
                    const int c = CPL * (ln & 15) + s2;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const int a = CPL * (4 * (ln >> 4) + t) + s1;
                        Gs[a * C::GS + c] = acc[i][t];
                        if (s1 < s2) Gs[c * C::GS + a] = acc[i][t];
                    }
                }
            }
        } else {
            for (int e = tid; e < D * D / 4; e += kEigThreads) {
                const int i = e / (D / 4), c4 = e % (D / 4);
                *reinterpret_cast<v4f*>(Gs + i * C::GS + 4 * c4) =
                    *reinterpret_cast<const v4f*>(Gb + (size_t)i * D + 4 * c4);
            }
        }
    }
    const float* Gop = C::GLDS ? Gs : Gb;
    // start block Omega (columns >= L stay zero so that the padded GEMM columns are zero)
    for (int e = tid; e < LP * D; e += kEigThreads) {
        const int j = e / D, i = e % D;
        Qc[j * LD + i] = (j < L) ? omega_entry(b, j, i) : 0.f;
        Zc[j * LD + i] = 0.f;
    }
    __syncthreads();

    const int col = tid / TC, cu = tid % TC;
    // The iteration alternates cheap and full steps.  After a power step Z = G Q the block is
    // re-orthonormalized either by one Gram-Schmidt pass (`mgs_steps` times in a row: only the
    // span matters then) or by the Jacobi phase, which also rotates the basis to Ritz vectors;
    // the step after a Jacobi phase checks the residuals of those Ritz pairs.
    bool orth_ok = false;
    float prev_res = 3.0e38f;
    int it = 0;
    int status = 0;
    bool have_ritz = false;
    int cheap_left = prm.mgs_steps;
    int cycle = 0;
    // the cheap steps that the convergence rate adds are filtered: step j of k applies G - t_j I
    // with t_j the roots of the Chebyshev polynomial of degree k on [0, cheb_b]
    float cheb_b = 0.f;
    int cheb_k = 0, cheb_j = 0;
    for (;; ++it) {
        if (cheb_j < cheb_k) {
            const float shift = 0.5f * cheb_b * (1.f + __cosf((2 * cheb_j + 1) * 1.57079632679f / cheb_k));
            ++cheb_j;
            gemm_gq<D, LP, C::GS, true>(Gop, Qc, Zc, shift);
        } else {
            gemm_gq<D, LP, C::GS>(Gop, Qc, Zc);
        }
        __syncthreads();
        // column norms of Z (for the dead-column threshold), Rayleigh quotients and residuals
        if (col < L) {
            const float* q = Qc + col * LD;
            const float* z = Zc + col * LD;
            float th = 0.f, nn = 0.f;
            for (int i = cu; i < D; i += TC) { th += q[i] * z[i]; nn += z[i] * z[i]; }
            th = team_sum<TC>(th);
            nn = team_sum<TC>(nn);
            float rs = 0.f;
            for (int i = cu; i < D; i += TC) { const float e = z[i] - th * q[i]; rs += e * e; }
            rs = team_sum<TC>(rs);
            if (cu == 0) {
                theta[col] = th;
                resid[col] = sqrtf(rs);
                atomicMax(&sh_bits2, __float_as_int(nn));
            }
        }
        __syncthreads();
        const float dead2 = kDeadRel * kDeadRel * __int_as_float(sh_bits2);
        if (have_ritz) {
            if (tid < L) {
                const float th = theta[tid];
                int rk = 0;
                for (int k = 0; k < L; ++k) {
                    const float tk = theta[k];
                    rk += (tk > th || (tk == th && k < tid)) ? 1 : 0;
                }
                rankv[tid] = rk;
                if (rk < r) atomicMax(&sh_bits, __float_as_int(resid[tid]));
            }
            __syncthreads();
            const float maxres = __int_as_float(sh_bits);
            float thmax = 0.f;
            for (int k = 0; k < L; ++k) thmax = fmaxf(thmax, theta[k]);
            bool done = orth_ok && (maxres <= prm.tol_res * thmax);
            // stagnation at the rounding floor counts as converged
            if (orth_ok && it >= 3 && maxres > 0.5f * prev_res && maxres <= 1.0e-4f * thmax) done = true;
            prev_res = maxres;
            if (done) break;
            if (it >= prm.max_iter) { status = it; break; }
        }
        __syncthreads();
        if (tid == 0) { sh_bits = 0; sh_bits2 = 0; }
        if (cheap_left > 0) {
            --cheap_left;
            have_ritz = false;
            mgs_orthonormalize<D, L>(Zc, Qc, resid, dead2);
            if (cycle == 0 && cheap_left == 0 && it > 0) {   // the last of the initial cheap steps
                // Convergence rate seen by this pass: the smallest diagonal entry of the triangular
                // factor over the r-th largest estimates lambda_(L+1) / lambda_r.  A slowly decaying
                // spectrum (ratio above 0.3) would fail the check after the usual two steps and pay
                // a whole Jacobi phase for it, so cheap steps are added up front instead (each costs
                // a sixth to a tenth of that phase), and these k steps apply G - t_j I with the t_j
                // at the roots of the Chebyshev polynomial of degree k on [0, lambda_L]: together
                // they are the polynomial of degree k that is smallest on the unwanted part of the
                // spectrum relative to its value at lambda_r (at a ratio of 0.6, 1/44 after three
                // steps where three plain power steps give 1/4.6); the Gram-Schmidt pass between two
                // steps only changes the basis of the block, not its span.  Four filtered steps
                // leave the residuals of the first check ten times below the tolerance where five
                // plain ones left some users just above it, who then paid a second Jacobi phase.
                // (Ending the cheap steps after one when the
                // ratio is ~ 0, as for inputs of rank r, was tried: one user in eight then failed
                // the check by a small margin and took seven steps.)
                if (tid < L) {
                    const float v = resid[tid];
                    int rk = 0;
#pragma unroll 8
                    for (int k = 0; k < L; ++k) {
                        const float vk = resid[k];
                        rk += (vk > v || (vk == v && k < tid)) ? 1 : 0;
                    }
                    if (rk == r - 1) sh_rate[0] = v;
                    if (rk == L - 1) sh_rate[1] = v;
                }
                __syncthreads();
                const float vr = sh_rate[0], vmin = sh_rate[1];
                const float rho = vr > 0.f ? sqrtf(fmaxf(vmin, 0.f) / vr) : 0.f;
                if (rho > 0.3f && rho < 1.f) {
                    const int want = (int)ceilf(-11.5f / __logf(rho)) - 3;   // ln(1e-5) = -11.5
                    cheap_left = want < 0 ? 0 : (want > kExtraStepsCap ? kExtraStepsCap : want);
                    cycle = -1;   // the rate is not looked at again
                    // the interval that the filter damps ends at the estimate of lambda_L and in any
                    // case well below that of lambda_r (a root next to a wanted eigenvalue would
                    // remove that direction from the block)
                    cheb_b = fminf(sqrtf(fmaxf(vmin, 0.f)), 0.85f * sqrtf(vr));
                    cheb_k = cheap_left;
                }
            }
            continue;
        }
        // a failed check means slow convergence: spend more cheap steps before the next one
        cycle = cycle < 0 ? 1 : cycle + 1;
        cheap_left = prm.mgs_steps << (cycle < 3 ? cycle : 3);
        have_ritz = true;
        // orthogonalize the columns of Z (this also rotates them towards Ritz vectors)
        orth_ok = false;
        for (int sw = 0; sw < prm.sweeps; ++sw) {
            const float mine = jacobi_sweep<D, L>(Zc, dead2);
            const bool any = __syncthreads_or(mine > prm.tol_orth);
            if (!any) { orth_ok = true; break; }
        }
        // normalize; drop columns that are numerically zero
        if (col < L) {
            const float* z = Zc + col * LD;
            float nn = 0.f;
            for (int i = cu; i < D; i += TC) nn += z[i] * z[i];
            nn = team_sum<TC>(nn);
            if (cu == 0) resid[col] = sqrtf(nn);
        }
        __syncthreads();
        if (col < L) {
            float nmax = 0.f;
            for (int k = 0; k < L; ++k) nmax = fmaxf(nmax, resid[k]);
            const float nj = resid[col];
            const float inv = (nj > kDeadRel * nmax && nj > 0.f) ? 1.f / nj : 0.f;
            const float* z = Zc + col * LD;
            float* q = Qc + col * LD;
            for (int i = cu; i < D; i += TC) q[i] = z[i] * inv;
        }
        __syncthreads();
    }

    // outputs: columns ranked by Ritz value, sign fixed by the largest-magnitude entry
    if (col < L && rankv[col] < r) {
        const int k = rankv[col];
        const float* q = Qc + col * LD;
        float best = -1.f;
        int bi = 0;
        for (int i = cu; i < D; i += TC) {
            const float a = fabsf(q[i]);
            if (a > best) { best = a; bi = i; }
        }
        for (int m = 1; m < TC; m <<= 1) {
            const float ob = __shfl_xor(best, m);
            const int oi = __shfl_xor(bi, m);
            if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
        }
        const float sgn = (q[bi] < 0.f) ? -1.f : 1.f;
        for (int i = cu; i < D; i += TC) V[((size_t)b * D + i) * r + k] = sgn * q[i];
        if (cu == 0) S[(size_t)b * r + k] = sqrtf(fmaxf(theta[col], 0.f));
    }
    if (tid == 0 && info) info[b] = status;
}

// Last step of Algorithm 1 when it is run with passes over H: from W = H^T Y (d x r) and
// Gy = Y^T Y (r x r) of the final Y = H Omega, the QR factor R of Y is the Cholesky factor of
// Gy (Y = Q R  =>  Gy = R^T R), Q^T H = R^-T W^T, and the singular values s and right singular
// vectors of Q^T H are the column norms and normalized columns of (Q^T H)^T = W R^-1 once a
// one-sided Jacobi has made those columns mutually orthogonal.  One workgroup per user, all of
// it in LDS.  info: 0 ok, > 0 Jacobi sweeps exhausted, -1 bad length, -2 Gy is not numerically
// positive definite (Y has fewer than r independent columns).
template <int D, int L>
__global__ __launch_bounds__(kEigThreads) void rsvd_small_kernel(
    const float* __restrict__ W, const float* __restrict__ Gy, const int32_t* __restrict__ lengths, int N,
    float* __restrict__ S, float* __restrict__ V, int32_t* __restrict__ info, int max_sweeps) {
    using C = EigCfg<D, L>;
    constexpr int LP = C::LP, LD = C::LD, TC = C::TC, LR = L + 1;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* Zc = smem;                  // [LP][LD] columns of W R^-1
    float* Rm = Zc + LP * LD;          // [L][LR] Gy, then its Cholesky factor (upper triangle)
    float* nrm = Rm + L * LR;          // [LP] column norms
    int* rankv = reinterpret_cast<int*>(nrm + LP);   // [LP]
    __shared__ int sh_bad;
    __shared__ int sh_bits;
    const int tid = threadIdx.x, b = blockIdx.x;
    const int r = L;
    auto fail = [&](int code) {
        for (int e = tid; e < D * r; e += kEigThreads) V[(size_t)b * D * r + e] = 0.f;
        for (int e = tid; e < r; e += kEigThreads) S[(size_t)b * r + e] = 0.f;
        if (tid == 0 && info) info[b] = code;
    };
    {
        const int raw = lengths ? lengths[b] : N;
        if (raw < r || raw > N) { fail(-1); return; }   // uniform over the workgroup
    }
    if (tid == 0) { sh_bad = 0; sh_bits = 0; }
    for (int e = tid; e < L * L; e += kEigThreads) Rm[(e / L) * LR + e % L] = Gy[(size_t)b * L * L + e];
    for (int e = tid; e < LP * LD; e += kEigThreads) Zc[e] = 0.f;
    __syncthreads();
    // Cholesky, right-looking.  A pivot below 1e-5 of its diagonal entry counts as breakdown:
    // the results would carry a relative error of about 2^-24 / 1e-5, a percent.
    for (int k = 0; k < L; ++k) {
        const float piv = Rm[k * LR + k];
        const float d0 = Gy[(size_t)b * L * L + k * L + k];
        if (!(piv > 1.0e-5f * d0) || !(piv > 0.f)) { if (tid == 0) sh_bad = 1; }
        __syncthreads();
        if (sh_bad) break;   // uniform
        const float rkk = __builtin_amdgcn_sqrtf(piv);
        const float inv = 1.f / rkk;
        __syncthreads();
        for (int jx = k + tid; jx < L; jx += kEigThreads) Rm[k * LR + jx] = (jx == k) ? rkk : Rm[k * LR + jx] * inv;
        __syncthreads();
        const int m = L - k - 1;
        for (int e = tid; e < m * m; e += kEigThreads) {
            const int i = k + 1 + e / m, jx = k + 1 + e % m;
            if (jx >= i) Rm[i * LR + jx] -= Rm[k * LR + i] * Rm[k * LR + jx];
        }
        __syncthreads();
    }
    if (sh_bad) { fail(-2); return; }
    // rows of W R^-1 by forward substitution, one thread per row
    for (int a = tid; a < D; a += kEigThreads) {
        float x[L];
        const float* w = W + ((size_t)b * D + a) * L;
#pragma unroll
        for (int jx = 0; jx < L; ++jx) {
            float acc = w[jx];
#pragma unroll
            for (int i = 0; i < jx; ++i) acc -= x[i] * Rm[i * LR + jx];
            x[jx] = acc / Rm[jx * LR + jx];
            Zc[jx * LD + a] = x[jx];
        }
    }
    __syncthreads();
    const int col = tid / TC, cu = tid % TC;
    auto column_norms = [&]() {
        if (col < L) {
            const float* z = Zc + col * LD;
            float nn = 0.f;
            for (int i = cu; i < D; i += TC) nn += z[i] * z[i];
            nn = team_sum<TC>(nn);
            if (cu == 0) { nrm[col] = nn; atomicMax(&sh_bits, __float_as_int(nn)); }
        }
        __syncthreads();
    };
    column_norms();
    const float dead2 = kDeadRel * kDeadRel * __int_as_float(sh_bits);
    int status = max_sweeps;
    for (int sw = 0; sw < max_sweeps; ++sw) {
        const float mine = jacobi_sweep<D, L>(Zc, dead2);
        const bool any = __syncthreads_or(mine > kSweepDone);
        if (!any) { status = 0; break; }
    }
    column_norms();
    if (tid < L) {
        const float th = nrm[tid];
        int rk = 0;
        for (int k = 0; k < L; ++k) {
            const float tk = nrm[k];
            rk += (tk > th || (tk == th && k < tid)) ? 1 : 0;
        }
        rankv[tid] = rk;
    }
    __syncthreads();
    // outputs: columns ranked by norm, sign fixed by the largest-magnitude entry
    if (col < L) {
        const int k = rankv[col];
        const float nn = nrm[col];
        const float inv = nn > 0.f ? __builtin_amdgcn_rsqf(nn) : 0.f;
        const float* q = Zc + col * LD;
        float best = -1.f;
        int bi = 0;
        for (int i = cu; i < D; i += TC) {
            const float a = fabsf(q[i]);
            if (a > best) { best = a; bi = i; }
        }
        for (int m = 1; m < TC; m <<= 1) {
            const float ob = __shfl_xor(best, m);
            const int oi = __shfl_xor(bi, m);
            if (ob > best || (ob == best && oi < bi)) { best = ob; bi = oi; }
        }
        const float sgn = (q[bi] < 0.f) ? -inv : inv;
        for (int i = cu; i < D; i += TC) V[((size_t)b * D + i) * r + k] = sgn * q[i];
        if (cu == 0) S[(size_t)b * r + k] = __builtin_amdgcn_sqrtf(nn);
    }
    if (tid == 0 && info) info[b] = status;
}

// Re-orthonormalisation of the power-iteration block between two passes over H when Algorithm 1
// is run as printed: W (d x r, row-major) is replaced by an orthonormal basis of its range.
// The printed algorithm has no such step; it changes nothing in exact arithmetic (every later
// quantity depends on the block only through its range), and in float it is what keeps the
// r columns from collapsing onto the leading singular vector: without it cond(H Omega) grows by
// (s_1/s_r)^2 per power step.  Two passes of the panelled Gram-Schmidt above ("twice is enough"
// up to cond(W) of about 1e7); columns that vanish are dropped as zeros.
template <int D, int L>
__global__ __launch_bounds__(kEigThreads) void orthonormalize_block_kernel(float* __restrict__ W) {
    using C = EigCfg<D, L>;
    constexpr int LP = C::LP, LD = C::LD, TC = C::TC;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* Zc = smem;               // [LP][LD]
    float* Qc = Zc + LP * LD;       // [LP][LD]
    float* piv = Qc + LP * LD;      // [LP]
    __shared__ int sh_bits;
    const int tid = threadIdx.x, b = blockIdx.x;
    float* Wb = W + (size_t)b * D * L;
    if (tid == 0) sh_bits = 0;
    for (int e = tid; e < D * L; e += kEigThreads) Zc[(e % L) * LD + e / L] = Wb[e];
    __syncthreads();
    const int col = tid / TC, cu = tid % TC;
    for (int pass = 0; pass < 2; ++pass) {
        if (col < L) {
            const float* z = Zc + col * LD;
            float nn = 0.f;
            for (int i = cu; i < D; i += TC) nn += z[i] * z[i];
            nn = team_sum<TC>(nn);
            if (cu == 0) atomicMax(&sh_bits, __float_as_int(nn));
        }
        __syncthreads();
        const float dead2 = kDeadRel * kDeadRel * __int_as_float(sh_bits);
        __syncthreads();
        if (tid == 0) sh_bits = 0;
        mgs_orthonormalize<D, L>(Zc, Qc, piv, dead2);
        if (pass == 0) {
            for (int e = tid; e < L * LD; e += kEigThreads) Zc[e] = Qc[e];
            __syncthreads();
        }
    }
    for (int e = tid; e < D * L; e += kEigThreads) Wb[e] = Qc[(e % L) * LD + e / L];
}

template <int D, int L>
hipError_t launch_orthonormalize_t(float* W, int B, hipStream_t stream) {
    using C = EigCfg<D, L>;
    const size_t lds = sizeof(float) * ((size_t)2 * C::LP * C::LD + C::LP);
    auto kern = orthonormalize_block_kernel<D, L>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(B), dim3(kEigThreads), lds, stream, W);
    return hipGetLastError();
}

template <int D, int L>
hipError_t launch_rsvd_small_t(const float* W, const float* Gy, const int32_t* lengths, int B, int N,
                               float* S, float* V, int32_t* info, hipStream_t stream) {
    using C = EigCfg<D, L>;
    const size_t lds = sizeof(float) * ((size_t)C::LP * C::LD + (size_t)L * (L + 1) + 2 * C::LP + 8);
    auto kern = rsvd_small_kernel<D, L>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(B), dim3(kEigThreads), lds, stream, W, Gy, lengths, N, S, V, info, 30);
    return hipGetLastError();
}

template <int D, int L>
hipError_t launch_eig_t(const float* G, const float* partials, int nsplit, const int32_t* lengths, int B, int N,
                        int r, float* S, float* V, int32_t* info, const EigParams& prm, hipStream_t stream) {
    if (partials && !EigCfg<D, L>::GLDS) return hipErrorInvalidValue;
    const size_t lds = sizeof(float) * EigCfg<D, L>::lds_floats;
    auto kern = eig_topr_kernel<D, L>;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(B), dim3(kEigThreads), lds, stream, G, partials, nsplit, lengths, N, r, S, V,
                       info, prm);
    return hipGetLastError();
}

template <int D>
hipError_t launch_eig_d(const float* G, const float* partials, int nsplit, const int32_t* lengths, int B, int N,
                        int r, float* S, float* V, int32_t* info, const EigParams& prm, hipStream_t stream) {
    const int L = eig_block_columns(D, r);
#define SOLAR_EIG_CASE(LL)                                                                    \
    case LL:                                                                                  \
        if constexpr (LL <= D && (D < 256 || LL <= 40))                                       \
            return launch_eig_t<D, LL>(G, partials, nsplit, lengths, B, N, r, S, V, info, prm, stream); \
        else                                                                                  \
            return hipErrorInvalidValue;
    switch (L) {
        SOLAR_EIG_CASE(16)
        SOLAR_EIG_CASE(24)
        SOLAR_EIG_CASE(32)
        SOLAR_EIG_CASE(40)
        SOLAR_EIG_CASE(48)
        SOLAR_EIG_CASE(56)
        SOLAR_EIG_CASE(64)
        SOLAR_EIG_CASE(72)
        default: return hipErrorInvalidValue;
    }
#undef SOLAR_EIG_CASE
}

}  // namespace

EigParams eig_default_params() {
    EigParams p;
    p.tol_res = 5.0e-6f;
    p.tol_orth = kSweepDone;
    p.max_iter = 40;
    p.sweeps = 12;
    p.mgs_steps = 2;
    return p;
}

// Columns of the iterate block: r plus an oversampling of 8, rounded up to a multiple of 8.
int eig_block_columns(int d, int r) {
    int L = 8 * ((r + 8 + 7) / 8);
    if (L < 16) L = 16;
    if (L > d) L = d;
    return L;
}

size_t eig_lds_bytes(int d, int r) {
    const int L = eig_block_columns(d, r);
    const int LP = 16 * ((L + 15) / 16);
    return sizeof(float) * ((size_t)2 * LP * (d + 4) + 3 * LP + 8 + (d <= 128 ? (size_t)d * (d + 16) : 0));
}

hipError_t launch_eig(const float* G, const float* partials, int nsplit, const int32_t* lengths, int B, int N,
                      int d, int r, float* S, float* V, int32_t* info, const EigParams& prm, hipStream_t stream) {
    switch (d) {
        case 64: return launch_eig_d<64>(G, partials, nsplit, lengths, B, N, r, S, V, info, prm, stream);
        case 128: return launch_eig_d<128>(G, partials, nsplit, lengths, B, N, r, S, V, info, prm, stream);
        case 256: return launch_eig_d<256>(G, partials, nsplit, lengths, B, N, r, S, V, info, prm, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_orthonormalize_block(float* W, int B, int d, int r, hipStream_t stream) {
#define SOLAR_ORTH_CASE(DD, LL) \
    if (d == DD && r == LL) return launch_orthonormalize_t<DD, LL>(W, B, stream);
    SOLAR_ORTH_CASE(64, 16) SOLAR_ORTH_CASE(64, 32) SOLAR_ORTH_CASE(64, 48) SOLAR_ORTH_CASE(64, 64)
    SOLAR_ORTH_CASE(128, 16) SOLAR_ORTH_CASE(128, 32) SOLAR_ORTH_CASE(128, 48) SOLAR_ORTH_CASE(128, 64)
#undef SOLAR_ORTH_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_rsvd_small(const float* W, const float* Gy, const int32_t* lengths, int B, int N, int d,
                             int r, float* S, float* V, int32_t* info, hipStream_t stream) {
#define SOLAR_RSVD_CASE(DD, LL) \
    if (d == DD && r == LL) return launch_rsvd_small_t<DD, LL>(W, Gy, lengths, B, N, S, V, info, stream);
    SOLAR_RSVD_CASE(64, 16) SOLAR_RSVD_CASE(64, 32) SOLAR_RSVD_CASE(64, 48) SOLAR_RSVD_CASE(64, 64)
    SOLAR_RSVD_CASE(128, 16) SOLAR_RSVD_CASE(128, 32) SOLAR_RSVD_CASE(128, 48) SOLAR_RSVD_CASE(128, 64)
#undef SOLAR_RSVD_CASE
    return hipErrorInvalidValue;
}

}  // namespace solar
