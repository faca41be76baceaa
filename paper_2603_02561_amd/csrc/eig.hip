// Top-r eigenpairs of each user's d x d Gram matrix G = X^T X, one workgroup per
// user, iterate blocks held in LDS.  S = sqrt(eigenvalues), V = eigenvectors are
// the s and R that Algorithm 1 ("Randomized SVD with Power Iteration") returns.
//
// The iteration is Algorithm 1 expressed on G: a Gaussian start block Omega
// (d x L, L = r + oversampling), power steps Omega <- X^T (X Omega) = G Omega, an
// orthonormal basis of the block, and a small decomposition of the projected
// problem.  Basis and small decomposition are done together by a one-sided
// (Hestenes) Jacobi method on the d x L block Z = G Q: rotating column pairs of Z
// until they are mutually orthogonal diagonalizes Q^T G^2 Q, which is the
// Rayleigh-Ritz step for G^2 on span(Q), and the normalized columns are the next
// orthonormal basis.  One-sided Jacobi is insensitive to the huge dynamic range of
// the first block (G Omega is dominated by the leading eigenvectors) and to rank
// deficiency (columns that vanish are dropped).  Power steps are repeated until
// every wanted pair (theta_i, q_i) has residual |G q_i - theta_i q_i| below
// tol_res * theta_max.
#include "common.h"
#include "kernels.h"

namespace solar {

namespace {

constexpr int kEigThreads = 256;
// A column of the iterate whose norm falls below this fraction of the largest column norm
// is rounding noise of the float Gram matrix (about sqrt(d) * 2^-24 relative) and is dropped.
constexpr float kDeadRel = 1.0e-5f;

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

__device__ __forceinline__ int pow2floor(int x) {
    int p = 1;
    while (2 * p <= x) p *= 2;
    return p;
}

// Z = G Q with the float 16x16x4 MFMA.  G is symmetric, so A[i][k] = G[k][i] is read
// with the 16 lanes of a slot group on consecutive addresses.  Q and Z are stored
// column by column (column j at base + j*LD).
template <int D, int CB>
__device__ __forceinline__ void gemm_gq(const float* __restrict__ Gb, const float* Qc, float* Zc,
                                        int LD) {
    constexpr int RB = (D / 16 + 3) / 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i16 = lane & 15, g = lane >> 4;
    v4f acc[RB][CB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) acc[rb][cb] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int k0 = 0; k0 < D; k0 += 4) {
        float a[RB];
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const int ib = wave + 4 * rb;
            a[rb] = (16 * ib < D) ? Gb[(size_t)(k0 + g) * D + 16 * ib + i16] : 0.f;
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const float q = Qc[(16 * cb + i16) * LD + k0 + g];
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) acc[rb][cb] = mfma16x16x4(a[rb], q, acc[rb][cb]);
        }
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int ib = wave + 4 * rb;
        if (16 * ib < D) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
                *reinterpret_cast<v4f*>(&Zc[(16 * cb + i16) * LD + 16 * ib + 4 * g]) = acc[rb][cb];
        }
    }
}

// One cyclic sweep of one-sided Jacobi over the first L columns of Zc (L even):
// L-1 rounds of L/2 disjoint column pairs (round-robin tournament), one team of T
// lanes per pair.  Returns the largest |cos| between two columns met in the sweep.
template <int D>
__device__ float jacobi_sweep(float* Zc, int L, int LD, int T, float skip_tol, int* sh_bits,
                              int* sh_amax) {
    constexpr int CHMAX = 8;
    const int tid = threadIdx.x;
    const int team = tid / T, u = tid % T;
    const int npair = L / 2;
    const int CH = D / (4 * T);
    float offmax = 0.f;
    for (int rho = 0; rho < L - 1; ++rho) {
        if (team < npair) {
            int p, q;
            if (team == 0) { p = L - 1; q = rho; }
            else { p = (rho + team) % (L - 1); q = (rho - team + (L - 1)) % (L - 1); }
            if (p > q) { int t = p; p = q; q = t; }
            float* zp = Zc + p * LD;
            float* zq = Zc + q * LD;
            v4f a[CHMAX], c[CHMAX];
            float al = 0.f, be = 0.f, ga = 0.f;
#pragma unroll
            for (int k = 0; k < CHMAX; ++k)
                if (k < CH) {
                    a[k] = *reinterpret_cast<const v4f*>(zp + 4 * (u + T * k));
                    c[k] = *reinterpret_cast<const v4f*>(zq + 4 * (u + T * k));
                    al += a[k].x * a[k].x + a[k].y * a[k].y + a[k].z * a[k].z + a[k].w * a[k].w;
                    be += c[k].x * c[k].x + c[k].y * c[k].y + c[k].z * c[k].z + c[k].w * c[k].w;
                    ga += a[k].x * c[k].x + a[k].y * c[k].y + a[k].z * c[k].z + a[k].w * c[k].w;
                }
            for (int m = 1; m < T; m <<= 1) {
                al += __shfl_xor(al, m);
                be += __shfl_xor(be, m);
                ga += __shfl_xor(ga, m);
            }
            // Columns that have collapsed to rounding noise (squared norm below kDeadRel^2 of
            // the largest seen) are left alone: they are dropped at normalization.
            // (read once per team so that every lane of the team takes the same branch)
            const float amax = __shfl(__int_as_float(*sh_amax), (tid & 63) - u);
            if (u == 0 && fmaxf(al, be) > amax) atomicMax(sh_amax, __float_as_int(fmaxf(al, be)));
            const float dead = kDeadRel * kDeadRel * fmaxf(amax, fmaxf(al, be));
            const float den = sqrtf(al) * sqrtf(be);
            if (den > 0.f && al > dead && be > dead) {
                const float cosv = fabsf(ga) / den;
                offmax = fmaxf(offmax, cosv);
                if (cosv > skip_tol) {
                    const float zeta = (be - al) / (2.f * ga);
                    const float t = copysignf(1.f, zeta) / (fabsf(zeta) + sqrtf(1.f + zeta * zeta));
                    const float cs = 1.f / sqrtf(1.f + t * t);
                    const float sn = cs * t;
#pragma unroll
                    for (int k = 0; k < CHMAX; ++k)
                        if (k < CH) {
                            const v4f x = a[k], y = c[k];
                            *reinterpret_cast<v4f*>(zp + 4 * (u + T * k)) = cs * x - sn * y;
                            *reinterpret_cast<v4f*>(zq + 4 * (u + T * k)) = sn * x + cs * y;
                        }
                }
            }
        }
        __syncthreads();
    }
    atomicMax(sh_bits, __float_as_int(offmax));
    __syncthreads();
    const float result = __int_as_float(*sh_bits);
    __syncthreads();
    if (tid == 0) *sh_bits = 0;
    __syncthreads();
    return result;
}

template <int D, int CB>
__global__ __launch_bounds__(kEigThreads) void eig_topr_kernel(
    const float* __restrict__ G, const int32_t* __restrict__ lengths, int N, int r, int L,
    float* __restrict__ S, float* __restrict__ V, int32_t* __restrict__ info, EigParams prm) {
    constexpr int LP = 16 * CB;
    constexpr int LD = D + 4;
    extern __shared__ float smem[];
    float* Zc = smem;
    float* Qc = Zc + LP * LD;
    float* theta = Qc + LP * LD;   // [LP]
    float* resid = theta + LP;     // [LP] residuals, also column norms
    int* rankv = reinterpret_cast<int*>(resid + LP);  // [LP]
    __shared__ int sh_bits;
    __shared__ int sh_bits2;
    __shared__ int sh_amax;
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
    if (tid == 0) { sh_bits = 0; sh_bits2 = 0; sh_amax = 0; }

    // start block Omega (columns >= L stay zero so that the padded GEMM columns are zero)
    for (int e = tid; e < LP * D; e += kEigThreads) {
        const int j = e / D, i = e % D;
        Qc[j * LD + i] = (j < L) ? omega_entry(b, j, i) : 0.f;
        Zc[j * LD + i] = 0.f;
    }
    __syncthreads();

    const int TJ = min(min(64, D / 4), pow2floor(kEigThreads / (L / 2)));  // lanes per column pair
    const int TC = min(64, pow2floor(kEigThreads / L));                    // lanes per column
    const int col = tid / TC, cu = tid % TC;
    bool orth_ok = false;
    float prev_res = 3.0e38f;
    int it = 0;
    int status = 0;
    for (;; ++it) {
        gemm_gq<D, CB>(Gb, Qc, Zc, LD);
        __syncthreads();
        if (it > 0) {
            // Rayleigh quotients and residuals of the current basis
            if (col < L) {
                const float* q = Qc + col * LD;
                const float* z = Zc + col * LD;
                float th = 0.f;
                for (int i = cu; i < D; i += TC) th += q[i] * z[i];
                for (int m = 1; m < TC; m <<= 1) th += __shfl_xor(th, m);
                float rs = 0.f;
                for (int i = cu; i < D; i += TC) { const float e = z[i] - th * q[i]; rs += e * e; }
                for (int m = 1; m < TC; m <<= 1) rs += __shfl_xor(rs, m);
                if (cu == 0) { theta[col] = th; resid[col] = sqrtf(rs); }
            }
            __syncthreads();
            if (tid < L) {
                const float th = theta[tid];
                int rk = 0;
                for (int k = 0; k < L; ++k) {
                    const float tk = theta[k];
                    rk += (tk > th || (tk == th && k < tid)) ? 1 : 0;
                }
                rankv[tid] = rk;
                if (rk < r) atomicMax(&sh_bits, __float_as_int(resid[tid]));
                if (rk == 0) sh_bits2 = __float_as_int(fmaxf(th, 0.f));
            }
            __syncthreads();
            const float maxres = __int_as_float(sh_bits);
            const float thmax = __int_as_float(sh_bits2);
            __syncthreads();
            if (tid == 0) sh_bits = 0;
            __syncthreads();
            bool done = orth_ok && (maxres <= prm.tol_res * thmax);
            // stagnation at the rounding floor counts as converged
            if (orth_ok && it >= 3 && maxres > 0.5f * prev_res && maxres <= 1.0e-4f * thmax) done = true;
            prev_res = maxres;
            if (done) break;
            if (it >= prm.max_iter) { status = it; break; }
        }
        // orthogonalize the columns of Z (this also rotates them towards Ritz vectors)
        orth_ok = false;
        if (tid == 0) sh_amax = 0;
        __syncthreads();
        for (int sw = 0; sw < prm.sweeps; ++sw) {
            const float off = jacobi_sweep<D>(Zc, L, LD, TJ, 1.0e-7f, &sh_bits, &sh_amax);
            if (off <= prm.tol_orth) { orth_ok = true; break; }
        }
        // normalize; drop columns that are numerically zero
        if (col < L) {
            const float* z = Zc + col * LD;
            float nn = 0.f;
            for (int i = cu; i < D; i += TC) nn += z[i] * z[i];
            for (int m = 1; m < TC; m <<= 1) nn += __shfl_xor(nn, m);
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

}  // namespace

EigParams eig_default_params() {
    EigParams p;
    p.tol_res = 5.0e-6f;
    p.tol_orth = 2.0e-6f;
    p.max_iter = 40;
    p.sweeps = 12;
    return p;
}

int eig_block_columns(int d, int r) {
    int L = 8 * ((r + 8 + 7) / 8);
    if (L > d) L = d;
    return L;
}

size_t eig_lds_bytes(int d, int r) {
    const int L = eig_block_columns(d, r);
    const int LP = 16 * ((L + 15) / 16);
    return sizeof(float) * ((size_t)2 * LP * (d + 4) + 3 * LP);
}

template <int D, int CB>
static hipError_t launch_eig_t(const float* G, const int32_t* lengths, int B, int N, int r, int L,
                               float* S, float* V, int32_t* info, const EigParams& prm,
                               hipStream_t stream) {
    const size_t lds = sizeof(float) * ((size_t)2 * 16 * CB * (D + 4) + 3 * 16 * CB);
    auto kern = eig_topr_kernel<D, CB>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(B), dim3(kEigThreads), lds, stream, G, lengths, N, r, L, S, V,
                       info, prm);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_eig_d(const float* G, const int32_t* lengths, int B, int N, int r,
                               float* S, float* V, int32_t* info, const EigParams& prm,
                               hipStream_t stream) {
    const int L = eig_block_columns(D, r);
    const int CB = (L + 15) / 16;
    switch (CB) {
        case 1: return launch_eig_t<D, 1>(G, lengths, B, N, r, L, S, V, info, prm, stream);
        case 2: return launch_eig_t<D, 2>(G, lengths, B, N, r, L, S, V, info, prm, stream);
        case 3: return launch_eig_t<D, 3>(G, lengths, B, N, r, L, S, V, info, prm, stream);
        case 4: return launch_eig_t<D, 4>(G, lengths, B, N, r, L, S, V, info, prm, stream);
        case 5: return launch_eig_t<D, 5>(G, lengths, B, N, r, L, S, V, info, prm, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_eig(const float* G, const int32_t* lengths, int B, int N, int d, int r, float* S,
                      float* V, int32_t* info, const EigParams& prm, hipStream_t stream) {
    if (eig_lds_bytes(d, r) > 160 * 1024) return hipErrorInvalidValue;
    switch (d) {
        case 64: return launch_eig_d<64>(G, lengths, B, N, r, S, V, info, prm, stream);
        case 128: return launch_eig_d<128>(G, lengths, B, N, r, S, V, info, prm, stream);
        case 256: return launch_eig_d<256>(G, lengths, B, N, r, S, V, info, prm, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace solar
