// C ABI of the SVD-Attention library: argument validation on the host, workspace
// carving and kernel launches on the caller's stream.  See include/solar.h.
#include "../../include/solar.h"

#include <array>
#include <atomic>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

#include "kernels.h"

// Scratch of solar_svd_factorize_static: the split-N partial blocks of the Gram contraction and
// G, which the other entry point takes from the caller's workspace.  Every device the library
// runs on holds its own copy until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress; the device address it yields is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[SOLAR_STATIC_SCRATCH_BYTES];

namespace {

using namespace solar;

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

bool supported_shape(int d, int r) {
    if (d != 64 && d != 128 && d != 256) return false;
    if (r < 1 || r > d || r > 64) return false;
    if (d == 256 && r > 32) return false;
    return true;
}

struct Carve {
    float* partials;
    float* G;
    size_t total;
};

Carve carve(void* ws, int B, int N, int d) {
    Carve c;
    const size_t pbytes = align256(sizeof(float) * gram_partial_floats(B, N, d));
    const size_t gbytes = align256(sizeof(float) * (size_t)B * d * d);
    char* base = static_cast<char*>(ws);
    c.partials = reinterpret_cast<float*>(base);
    c.G = reinterpret_cast<float*>(base + pbytes);
    c.total = pbytes + gbytes;
    return c;
}

// Optional per-phase timing of solar_svd_factorize: HIP events recorded on the
// caller's stream at the phase boundaries.  Host-side bookkeeping only.
struct PhaseTimer {
    bool enabled = false;
    int calls = 0;
    std::vector<std::array<hipEvent_t, 4>> ev;   // one set per timed call, created on demand, kept
};
PhaseTimer g_timer;

void timer_mark(int call, int slot, hipStream_t st) {
    if (!g_timer.enabled) return;
    while ((int)g_timer.ev.size() <= call) {
        std::array<hipEvent_t, 4> e;
        for (int i = 0; i < 4; ++i) (void)hipEventCreate(&e[i]);
        g_timer.ev.push_back(e);
    }
    (void)hipEventRecord(g_timer.ev[call][slot], st);
}

// Debug switches (solar_debug_option); both default to off.
std::atomic<int> g_debug_eig_max_iter{0};
std::atomic<int> g_debug_force_guarded{0};

EigParams eig_params() {
    EigParams p = eig_default_params();
    const int cap = g_debug_eig_max_iter.load(std::memory_order_relaxed);
    if (cap > 0) p.max_iter = cap;
    return p;
}

// a byte offset into one user's rows must fit the 32 bits the attention kernels keep it in
// longest sequence for the attention kernel with 16-bit softmax weights: a weight below 2^-25 of the
// reference rounds to zero, and in the guarded pass the largest weight is at least 1, so N rows of
// such a tail are at most N * 2^-25 of the softmax mass (1.6 % at this length)
constexpr int kX32MaxN = 524288;

bool rows_fit_32bit(int N, size_t row_bytes) { return (size_t)N * row_bytes < ((size_t)1 << 32); }

solar_status factorize_check(const void* X, int B, int N, int d, int r, solar_dtype t, const float* S,
                             const float* V) {
    if (!X || !S || !V || B <= 0 || N <= 0 || d <= 0 || r <= 0) return SOLAR_ERR_INVALID_ARG;
    if (t != SOLAR_F32 && t != SOLAR_BF16) return SOLAR_ERR_INVALID_ARG;
    if (r > d || r > N) return SOLAR_ERR_INVALID_ARG;
    if (!supported_shape(d, r)) return SOLAR_ERR_UNSUPPORTED;
    return SOLAR_OK;
}

// The three phases of the factorization on `st`, with `ws` (validated by the caller) as the
// scratch for the split-N partial blocks and G.
solar_status factorize_enqueue(const void* X, const int32_t* lengths, int B, int N, int d, int r, solar_dtype t,
                               float* S, float* V, float* P, int32_t* info, void* ws, bool timed,
                               hipStream_t st) {
    Carve c = carve(ws, B, N, d);
    const bool bf16 = t == SOLAR_BF16;
    const int call = g_timer.calls;
    if (timed) timer_mark(call, 0, st);
    // where the eigen-iteration can sum the split-N partial blocks itself, G is never formed
    const bool fused = gram_partials_consumable(d);
    hipError_t e = launch_gram(X, lengths, B, N, d, bf16, c.partials, c.G, !fused, st);
    if (e != hipSuccess) return SOLAR_ERR_HIP;
    if (timed) timer_mark(call, 1, st);
    e = launch_eig(c.G, fused ? c.partials : nullptr, gram_nsplit(B, N), lengths, B, N, d, r, S, V, info,
                   eig_params(), st);
    if (e != hipSuccess) return SOLAR_ERR_HIP;
    if (timed) timer_mark(call, 2, st);
    if (P) {
        e = launch_project(X, lengths, V, info, B, N, d, r, bf16, P, st);
        if (e != hipSuccess) return SOLAR_ERR_HIP;
    }
    if (timed) {
        timer_mark(call, 3, st);
        if (g_timer.enabled) g_timer.calls = call + 1;
    }
    return SOLAR_OK;
}

// Device address of the built-in scratch array on the current device.  Every device holds its
// own copy of the array at its own address, so the address is looked up once per device (on the
// first call made with that device current) and kept.
hipError_t static_scratch_of_current_device(void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptr_of_device[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of_device[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p || ((uintptr_t)p & 255)) return hipErrorInvalidSymbol;
        ptr_of_device[dev] = p;
    }
    *out = ptr_of_device[dev];
    return hipSuccess;
}

}  // namespace

namespace solar {

hipError_t allow_dynamic_lds(const void* kernel, size_t bytes) {
    static std::mutex mu;
    static std::map<std::pair<const void*, int>, size_t> granted;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    size_t& have = granted[std::make_pair(kernel, dev)];
    if (bytes <= have) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) have = bytes;
    return e;
}

int debug_eig_max_iter() { return g_debug_eig_max_iter.load(std::memory_order_relaxed); }
bool debug_force_guarded_pass() { return g_debug_force_guarded.load(std::memory_order_relaxed) != 0; }

}  // namespace solar

extern "C" {

solar_status solar_debug_option(solar_debug_key key, int value) {
    switch (key) {
        case SOLAR_DEBUG_EIG_MAX_ITER:
            if (value < 0) return SOLAR_ERR_INVALID_ARG;
            g_debug_eig_max_iter.store(value, std::memory_order_relaxed);
            return SOLAR_OK;
        case SOLAR_DEBUG_FORCE_GUARDED_PASS:
            g_debug_force_guarded.store(value != 0, std::memory_order_relaxed);
            return SOLAR_OK;
        default:
            return SOLAR_ERR_INVALID_ARG;
    }
}

solar_status solar_info_status(const int32_t* info_host, int B) {
    if (!info_host || B <= 0) return SOLAR_ERR_INVALID_ARG;
    solar_status worst = SOLAR_OK;
    for (int b = 0; b < B; ++b) {
        if (info_host[b] < 0) return SOLAR_ERR_INVALID_ARG;
        if (info_host[b] > 0) worst = SOLAR_ERR_NOT_CONVERGED;
    }
    return worst;
}

const char* solar_status_string(solar_status s) {
    switch (s) {
        case SOLAR_OK: return "ok";
        case SOLAR_ERR_INVALID_ARG: return "invalid argument";
        case SOLAR_ERR_UNSUPPORTED: return "unsupported shape or type";
        case SOLAR_ERR_WORKSPACE: return "workspace too small or misaligned";
        case SOLAR_ERR_HIP: return "HIP launch error";
        case SOLAR_ERR_NOT_CONVERGED: return "eigen-iteration reached its cap for at least one user";
        case SOLAR_ERR_SCRATCH_LIMIT: return "sizes need more scratch than the built-in array of the allocation-free call holds";
        default: return "unknown status";
    }
}

size_t solar_workspace_bytes(int B, int N, int d, int r, int M, solar_dtype t) {
    (void)r; (void)M; (void)t;
    if (B <= 0 || N <= 0 || (d != 64 && d != 128 && d != 256)) return 0;
    return carve(nullptr, B, N, d).total;
}

void solar_phase_timing_begin(void) {
    g_timer.enabled = true;
    g_timer.calls = 0;
}

int solar_phase_timing_end(float* ms_sum) {
    const int n = g_timer.calls;
    float acc[3] = {0.f, 0.f, 0.f};
    for (int c = 0; c < n; ++c) {
        (void)hipEventSynchronize(g_timer.ev[c][3]);
        for (int i = 0; i < 3; ++i) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, g_timer.ev[c][i], g_timer.ev[c][i + 1]) == hipSuccess) acc[i] += ms;
        }
    }
    if (ms_sum) for (int i = 0; i < 3; ++i) ms_sum[i] = acc[i];
    g_timer.enabled = false;
    g_timer.calls = 0;
    return n;
}

solar_status solar_gram(const void* X, const int32_t* lengths, int B, int N, int d, solar_dtype t,
                        float* G, void* workspace, size_t workspace_bytes, void* stream) {
    if (!X || !G || B <= 0 || N <= 0 || d <= 0) return SOLAR_ERR_INVALID_ARG;
    if (t != SOLAR_F32 && t != SOLAR_BF16) return SOLAR_ERR_INVALID_ARG;
    if (!supported_shape(d, 1)) return SOLAR_ERR_UNSUPPORTED;
    Carve c = carve(workspace, B, N, d);
    if (!workspace || workspace_bytes < c.total || ((uintptr_t)workspace & 255)) return SOLAR_ERR_WORKSPACE;
    hipError_t e = launch_gram(X, lengths, B, N, d, t == SOLAR_BF16, c.partials, G, true, (hipStream_t)stream);
    return e == hipSuccess ? SOLAR_OK : SOLAR_ERR_HIP;
}

solar_status solar_svd_factorize(const void* X, const int32_t* lengths, int B, int N, int d, int r,
                                 solar_dtype t, float* S, float* V, float* P, int32_t* info,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    const solar_status v = factorize_check(X, B, N, d, r, t, S, V);
    if (v != SOLAR_OK) return v;
    if (!workspace || workspace_bytes < carve(nullptr, B, N, d).total || ((uintptr_t)workspace & 255))
        return SOLAR_ERR_WORKSPACE;
    return factorize_enqueue(X, lengths, B, N, d, r, t, S, V, P, info, workspace, true, (hipStream_t)stream);
}

solar_status solar_svd_factorize_static(const void* X, const int32_t* lengths, int B, int N, int d, int r,
                                        solar_dtype t, float* S, float* V, float* P, int32_t* info,
                                        void* stream) {
    const solar_status v = factorize_check(X, B, N, d, r, t, S, V);
    if (v != SOLAR_OK) return v;
    if (carve(nullptr, B, N, d).total > (size_t)SOLAR_STATIC_SCRATCH_BYTES) return SOLAR_ERR_SCRATCH_LIMIT;
    void* ws = nullptr;
    if (static_scratch_of_current_device(&ws) != hipSuccess) return SOLAR_ERR_HIP;
    // no phase timing here: its events are created on demand, which allocates
    return factorize_enqueue(X, lengths, B, N, d, r, t, S, V, P, info, ws, false, (hipStream_t)stream);
}

size_t solar_rsvd_workspace_bytes(int B, int N, int d, int r) {
    if (B <= 0 || N <= 0 || d <= 0 || r <= 0 || !rsvd_supported(d, r)) return 0;
    return align256(sizeof(float) * (size_t)B * N * r) + align256(sizeof(float) * (size_t)B * d * r) +
           align256(sizeof(float) * (size_t)B * r * r) + align256(sizeof(float) * xty_partial_floats(B, N, d, r));
}

solar_status solar_svd_factorize_rsvd(const void* X, const int32_t* lengths, int B, int N, int d, int r,
                                      solar_dtype t, const float* Omega, int n_iter, float* S, float* V,
                                      float* P, int32_t* info, void* workspace, size_t workspace_bytes,
                                      void* stream) {
    if (!X || !Omega || !S || !V || B <= 0 || N <= 0 || d <= 0 || r <= 0 || n_iter < 0) return SOLAR_ERR_INVALID_ARG;
    if (t != SOLAR_F32 && t != SOLAR_BF16) return SOLAR_ERR_INVALID_ARG;
    if (r > d || r > N) return SOLAR_ERR_INVALID_ARG;
    if (!rsvd_supported(d, r)) return SOLAR_ERR_UNSUPPORTED;
    const size_t need = solar_rsvd_workspace_bytes(B, N, d, r);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return SOLAR_ERR_WORKSPACE;
    char* base = static_cast<char*>(workspace);
    float* Y = reinterpret_cast<float*>(base);
    base += align256(sizeof(float) * (size_t)B * N * r);
    float* Wb = reinterpret_cast<float*>(base);
    base += align256(sizeof(float) * (size_t)B * d * r);
    float* Gy = reinterpret_cast<float*>(base);
    base += align256(sizeof(float) * (size_t)B * r * r);
    float* partials = reinterpret_cast<float*>(base);
    hipStream_t st = (hipStream_t)stream;
    const bool bf16 = t == SOLAR_BF16;
    hipError_t e = launch_project(X, lengths, Omega, nullptr, B, N, d, r, bf16, Y, st);
    if (e != hipSuccess) return SOLAR_ERR_HIP;
    for (int it = 0; it <= n_iter; ++it) {
        e = launch_xty(X, Y, lengths, B, N, d, r, bf16, partials, Wb, Gy, st);
        if (e != hipSuccess) return SOLAR_ERR_HIP;
        if (it == n_iter) break;
        // Omega <- H^T (H Omega), replaced by an orthonormal basis of the same range
        e = launch_orthonormalize_block(Wb, B, d, r, st);
        if (e != hipSuccess) return SOLAR_ERR_HIP;
        e = launch_project(X, lengths, Wb, nullptr, B, N, d, r, bf16, Y, st);
        if (e != hipSuccess) return SOLAR_ERR_HIP;
    }
    e = launch_rsvd_small(Wb, Gy, lengths, B, N, d, r, S, V, info, st);
    if (e != hipSuccess) return SOLAR_ERR_HIP;
    if (P) {
        e = launch_project(X, lengths, V, info, B, N, d, r, bf16, P, st);
        if (e != hipSuccess) return SOLAR_ERR_HIP;
    }
    return SOLAR_OK;
}

solar_status solar_linear_attention(const void* Q, const void* X, const int32_t* lengths, int B, int N,
                                    int d, int M, float scale, solar_dtype t, float* O, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    if (!Q || !X || !O || B <= 0 || N <= 0 || d <= 0 || M <= 0) return SOLAR_ERR_INVALID_ARG;
    if (t != SOLAR_F32 && t != SOLAR_BF16) return SOLAR_ERR_INVALID_ARG;
    if (d != 64 && d != 128 && d != 256) return SOLAR_ERR_UNSUPPORTED;
    Carve c = carve(workspace, B, N, d);
    if (!workspace || workspace_bytes < c.total || ((uintptr_t)workspace & 255)) return SOLAR_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const bool bf16 = t == SOLAR_BF16;
    hipError_t e = launch_gram(X, lengths, B, N, d, bf16, c.partials, c.G, true, st);
    if (e != hipSuccess) return SOLAR_ERR_HIP;
    e = launch_rowgemm(Q, c.G, (size_t)d * d, B, M, d, scale, bf16, false, O, st);
    return e == hipSuccess ? SOLAR_OK : SOLAR_ERR_HIP;
}

solar_status solar_apply_weights(const void* In, const float* W, int rows, int d, solar_dtype t_in,
                                 solar_dtype t_out, void* Out, void* stream) {
    if (!In || !W || !Out || rows <= 0 || d <= 0) return SOLAR_ERR_INVALID_ARG;
    if ((t_in != SOLAR_F32 && t_in != SOLAR_BF16) || (t_out != SOLAR_F32 && t_out != SOLAR_BF16))
        return SOLAR_ERR_INVALID_ARG;
    if (d != 64 && d != 128 && d != 256) return SOLAR_ERR_UNSUPPORTED;
    hipError_t e = launch_rowgemm(In, W, 0, 1, rows, d, 1.f, t_in == SOLAR_BF16, t_out == SOLAR_BF16, Out,
                                  (hipStream_t)stream);
    return e == hipSuccess ? SOLAR_OK : SOLAR_ERR_HIP;
}

solar_status solar_svd_backward(const float* S, const float* V, const float* P, const float* S_bar,
                                const float* V_bar, int B, int N, int d, int r, float gap_rel, float* dX,
                                void* workspace, size_t workspace_bytes, void* stream) {
    if (!S || !V || !P || !S_bar || !V_bar || !dX || B <= 0 || N <= 0 || d <= 0 || r <= 0 || !(gap_rel >= 0.f))
        return SOLAR_ERR_INVALID_ARG;
    if (r > d) return SOLAR_ERR_INVALID_ARG;
    if (!svd_backward_supported(d, r)) return SOLAR_ERR_UNSUPPORTED;
    const size_t need = sizeof(float) * (size_t)B * r * d;
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)) return SOLAR_ERR_WORKSPACE;
    hipError_t e = launch_svd_backward(S, V, P, S_bar, V_bar, B, N, d, r, gap_rel,
                                       static_cast<float*>(workspace), dX, (hipStream_t)stream);
    return e == hipSuccess ? SOLAR_OK : SOLAR_ERR_HIP;
}

solar_status solar_svd_attention(const void* Q, const float* S, const float* V, const float* P,
                                 const int32_t* lengths, int B, int N, int d, int r, int M,
                                 float scale, solar_attn_mode mode, solar_dtype t, float* O,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    if (!Q || !V || !O || B <= 0 || N <= 0 || d <= 0 || r <= 0 || M <= 0) return SOLAR_ERR_INVALID_ARG;
    if (t != SOLAR_F32 && t != SOLAR_BF16) return SOLAR_ERR_INVALID_ARG;
    if (r > d || r > N) return SOLAR_ERR_INVALID_ARG;
    if (!supported_shape(d, r)) return SOLAR_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const bool bf16 = t == SOLAR_BF16;
    hipError_t e;
    switch (mode) {
        case SOLAR_ATTN_SEQ_SOFTMAX:
            if (!P) return SOLAR_ERR_INVALID_ARG;
            // bf16 inputs with the factors' S at hand and r a multiple of 4 take the fp16
            // matrix-unit kernel (2e-2 contract); everything else keeps float arithmetic, and so
            // do sequences beyond kX32MaxN rows, where 16-bit weights could drop a flat tail
            // that holds more than a percent of the softmax mass
            if (bf16 && S && attention_seq_x32_supported(d, r) && rows_fit_32bit(N, 4u * (size_t)r) &&
                N <= kX32MaxN)
                e = launch_attention_seq_x32(Q, S, V, P, lengths, B, N, d, r, M, scale, O, st);
            else
                e = launch_attention_seq(Q, V, P, lengths, B, N, d, r, M, scale, bf16, O, st);
            break;
        case SOLAR_ATTN_EIGEN_SOFTMAX:
        case SOLAR_ATTN_LINEAR:
            if (!S) return SOLAR_ERR_INVALID_ARG;
            e = launch_attention_tokens(Q, S, V, B, d, r, M, scale, mode == SOLAR_ATTN_EIGEN_SOFTMAX,
                                        bf16, O, st);
            break;
        default:
            return SOLAR_ERR_INVALID_ARG;
    }
    return e == hipSuccess ? SOLAR_OK : SOLAR_ERR_HIP;
}

solar_status solar_svd_attention_from_x(const void* Q, const void* X, const float* S, const float* V,
                                        const int32_t* lengths, int B, int N, int d, int r, int M,
                                        float scale, solar_dtype t, float* O, void* workspace,
                                        size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    if (!Q || !X || !S || !V || !O || B <= 0 || N <= 0 || d <= 0 || r <= 0 || M <= 0) return SOLAR_ERR_INVALID_ARG;
    if (t != SOLAR_F32 && t != SOLAR_BF16) return SOLAR_ERR_INVALID_ARG;
    if (r > d || r > N) return SOLAR_ERR_INVALID_ARG;
    if (t != SOLAR_BF16 || !attention_seq_x32_from_x_supported(d, r)) return SOLAR_ERR_UNSUPPORTED;
    if (!rows_fit_32bit(N, 2u * (size_t)d) || N > kX32MaxN) return SOLAR_ERR_UNSUPPORTED;
    hipError_t e = launch_attention_seq_x32_from_x(Q, S, V, X, lengths, B, N, d, r, M, scale, O, (hipStream_t)stream);
    return e == hipSuccess ? SOLAR_OK : SOLAR_ERR_HIP;
}

solar_status solar_dense_attention_ref(const void* Q, const void* X, const int32_t* lengths, int B,
                                       int N, int d, int M, float scale, solar_dtype t, float* O,
                                       void* workspace, size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    if (!Q || !X || !O || B <= 0 || N <= 0 || d <= 0 || M <= 0) return SOLAR_ERR_INVALID_ARG;
    if (t != SOLAR_F32 && t != SOLAR_BF16) return SOLAR_ERR_INVALID_ARG;
    if (d > 256) return SOLAR_ERR_UNSUPPORTED;
    hipError_t e = launch_dense_ref(Q, X, lengths, B, N, d, M, scale, t == SOLAR_BF16, O, (hipStream_t)stream);
    return e == hipSuccess ? SOLAR_OK : SOLAR_ERR_HIP;
}

}  // extern "C"
