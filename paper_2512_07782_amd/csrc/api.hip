// C ABI of libgfwa (see include/gfwa.h): argument validation and dispatch.  No device memory is
// allocated here; everything is enqueued on the caller's stream.
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <atomic>
#include <mutex>

#include "../../include/gfwa.h"
#include "gfwa_internal.h"

namespace gfwa {

static thread_local char g_hip_msg[256] = "no HIP error recorded";

static int hip_status(hipError_t e) {
    if (e == hipSuccess) return GFWA_OK;
    snprintf(g_hip_msg, sizeof(g_hip_msg), "HIP error %d: %s", (int)e, hipGetErrorString(e));
    return GFWA_ERR_HIP;
}

static bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// Sizes every entry point shares.  Tile indices and per-head offsets are 32-bit in the kernels.
static int check_dims(int B, int H, int N, int d, int w, bool need_d) {
    if (B <= 0 || H <= 0 || N <= 0) return GFWA_ERR_DIM;
    if (need_d && (d <= 0 || w < 1)) return GFWA_ERR_DIM;
    const long long bh = (long long)B * H;
    if (bh > (1LL << 24) || (long long)N > (1LL << 24)) return GFWA_ERR_DIM;
    if (bh * ((N + 31) / 32) > 0x7fffffffLL) return GFWA_ERR_DIM;
    if (need_d && d != 64 && d != 128) return GFWA_ERR_UNSUPPORTED;
    return GFWA_OK;
}

// ---- optional per-kernel timing with HIP events on the caller's stream ----
namespace {
constexpr int kMaxRecords = 8192;
struct ProfRecord { int kernel; hipEvent_t start, stop; };
struct ProfState {
    std::atomic<bool> on{false};   // the only field read without the lock (every launch asks it)
    std::mutex lock;               // slot allocation, reset and read-out may come from different host threads
    int used = 0;
    int created = 0;
    ProfRecord rec[kMaxRecords];
};
ProfState g_prof;
}  // namespace

hipError_t allow_dynamic_lds(const void* kernel, size_t bytes, DeviceOnce& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (dev < 64 && (__atomic_load_n(&done.bits, __ATOMIC_ACQUIRE) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && dev < 64) __atomic_fetch_or(&done.bits, bit, __ATOMIC_RELEASE);
    return e;
}

int device_cu_count() {
    static int cached[64];  // 0: not asked yet
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (dev >= 0 && dev < 64 && (n = __atomic_load_n(&cached[dev], __ATOMIC_RELAXED)) > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
    if (dev >= 0 && dev < 64) __atomic_store_n(&cached[dev], n, __ATOMIC_RELAXED);
    return n;
}

ProfScope::ProfScope(int kernel, hipStream_t s) : slot_(-1), s_(s) {
    if (!g_prof.on.load(std::memory_order_relaxed)) return;
    std::lock_guard<std::mutex> hold(g_prof.lock);
    if (g_prof.used >= kMaxRecords) return;
    const int i = g_prof.used;
    if (i >= g_prof.created) {
        if (hipEventCreate(&g_prof.rec[i].start) != hipSuccess) return;
        if (hipEventCreate(&g_prof.rec[i].stop) != hipSuccess) return;
        g_prof.created = i + 1;
    }
    g_prof.rec[i].kernel = kernel;
    g_prof.used = i + 1;
    slot_ = i;
    (void)hipEventRecord(g_prof.rec[i].start, s_);
}
ProfScope::~ProfScope() {
    if (slot_ >= 0) (void)hipEventRecord(g_prof.rec[slot_].stop, s_);
}

}  // namespace gfwa

using namespace gfwa;

extern "C" {

int gfwa_gate_prefix(const float* alpha, float* c, int B, int H, int N, gfwa_stream_t stream) {
    if (!alpha || !c) return GFWA_ERR_NULL;
    if (int r = check_dims(B, H, N, 0, 1, false)) return r;
    if (!aligned(alpha, 4) || !aligned(c, 4)) return GFWA_ERR_ALIGN;
    return hip_status(gate_prefix(alpha, c, B * H, N, stream));
}

int gfwa_gate_activation_prefix(const float* hpre, const float* beta, float eps, float* c, int B, int H, int N,
                                gfwa_stream_t stream) {
    if (!hpre || !beta || !c) return GFWA_ERR_NULL;
    if (int r = check_dims(B, H, N, 0, 1, false)) return r;
    if (!(eps >= 0.0f)) return GFWA_ERR_DIM;
    if (!aligned(hpre, 4) || !aligned(beta, 4) || !aligned(c, 4)) return GFWA_ERR_ALIGN;
    return hip_status(gate_activation_prefix(hpre, beta, eps, c, B * H, N, stream));
}

size_t gfwa_gate_scan_workspace_bytes(int B, int H, int N) {
    if (check_dims(B, H, N, 0, 1, false) != GFWA_OK) return 0;
    return (gate_scan_workspace_bytes(B * H, N) + 255) & ~(size_t)255;
}

int gfwa_gate_prefix_stp(const float* in, const float* beta, float eps, float* c, void* workspace,
                         size_t workspace_bytes, int B, int H, int N, gfwa_stream_t stream) {
    if (!in || !c) return GFWA_ERR_NULL;
    if (int r = check_dims(B, H, N, 0, 1, false)) return r;
    if (beta && !(eps >= 0.0f)) return GFWA_ERR_DIM;
    if (!aligned(in, 4) || !aligned(c, 4) || (beta && !aligned(beta, 4))) return GFWA_ERR_ALIGN;
    if (!workspace || workspace_bytes < gfwa_gate_scan_workspace_bytes(B, H, N)) return GFWA_ERR_WORKSPACE;
    if (!aligned(workspace, 8)) return GFWA_ERR_ALIGN;
    return hip_status(gate_prefix_stp(in, beta, eps, c, (double*)workspace, B * H, N, stream));
}

int gfwa_gate_activation_backward(const float* hpre, const float* beta, float eps, const float* dalpha, float* dh,
                                  float* dbeta, int B, int H, int N, gfwa_stream_t stream) {
    if (!hpre || !beta || !dalpha || !dh || !dbeta) return GFWA_ERR_NULL;
    if (int r = check_dims(B, H, N, 0, 1, false)) return r;
    if (!(eps >= 0.0f)) return GFWA_ERR_DIM;
    if (!aligned(hpre, 4) || !aligned(beta, 4) || !aligned(dalpha, 4) || !aligned(dh, 4) || !aligned(dbeta, 4))
        return GFWA_ERR_ALIGN;
    return hip_status(gate_activation_backward(hpre, beta, eps, dalpha, dh, dbeta, (size_t)B * H * N, stream));
}

int gfwa_forward(gfwa_dtype_t dt, const void* Q, const void* K, const void* V, const float* c, void* O,
                 float* L, int B, int H, int N, int d, int w, float scale, gfwa_stream_t stream) {
    return gfwa_forward_gqa(dt, Q, K, V, c, O, L, B, H, H, N, d, w, scale, stream);
}

int gfwa_forward_gqa(gfwa_dtype_t dt, const void* Q, const void* K, const void* V, const float* c, void* O,
                     float* L, int B, int H, int Hkv, int N, int d, int w, float scale, gfwa_stream_t stream) {
    if (!Q || !K || !V || !c || !O || !L) return GFWA_ERR_NULL;
    if (int r = check_dims(B, H, N, d, w, true)) return r;
    if (Hkv <= 0 || H % Hkv != 0) return GFWA_ERR_DIM;
    if (dt != GFWA_BF16 && dt != GFWA_F32) return GFWA_ERR_UNSUPPORTED;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) || !aligned(c, 4) ||
        !aligned(L, 4))
        return GFWA_ERR_ALIGN;
    if (dt == GFWA_F32)
        return hip_status(forward_f32((const float*)Q, (const float*)K, (const float*)V, c, (float*)O, L,
                                      B, H, Hkv, N, d, w, scale, stream));
    return hip_status(forward_bf16(Q, K, V, c, O, L, B, H, Hkv, N, d, w, scale, stream));
}

size_t gfwa_backward_workspace_bytes(gfwa_dtype_t dt, int B, int H, int N, int d, int w) {
    if (check_dims(B, H, N, d, w, true) != GFWA_OK) return 0;
    if (dt != GFWA_BF16 && dt != GFWA_F32) return 0;
    // D, dc_col, dc_row: three fp32 vectors of B*H*N, each padded to 256 bytes; then the segment sums of the
    // gate-gradient scan (one fp64 per 4096 elements)
    const size_t one = (((size_t)B * H * N * sizeof(float)) + 255) & ~(size_t)255;
    return 3 * one + ((gate_scan_workspace_bytes(B * H, N) + 255) & ~(size_t)255);
}

size_t gfwa_backward_fast_workspace_bytes(gfwa_dtype_t dt, int B, int H, int N, int d, int w) {
    const size_t base = gfwa_backward_workspace_bytes(dt, B, H, N, d, w);
    if (base == 0 || dt != GFWA_BF16) return base;
    return base + backward_bf16_spill_bytes(B, H, N, d, w);
}

int gfwa_backward(gfwa_dtype_t dt, const void* Q, const void* K, const void* V, const void* O,
                  const void* dO, const float* c, const float* L, void* dQ, void* dK, void* dV,
                  float* dalpha, void* workspace, size_t workspace_bytes, int B, int H, int N, int d, int w,
                  float scale, gfwa_stream_t stream) {
    return gfwa_backward_gqa(dt, Q, K, V, O, dO, c, L, dQ, dK, dV, dalpha, workspace, workspace_bytes, B, H, H, N,
                             d, w, scale, stream);
}

int gfwa_backward_gqa(gfwa_dtype_t dt, const void* Q, const void* K, const void* V, const void* O,
                      const void* dO, const float* c, const float* L, void* dQ, void* dK, void* dV,
                      float* dalpha, void* workspace, size_t workspace_bytes, int B, int H, int Hkv, int N,
                      int d, int w, float scale, gfwa_stream_t stream) {
    if (!Q || !K || !V || !O || !dO || !c || !L || !dQ || !dK || !dV || !dalpha) return GFWA_ERR_NULL;
    if (int r = check_dims(B, H, N, d, w, true)) return r;
    if (Hkv <= 0 || H % Hkv != 0) return GFWA_ERR_DIM;
    if (dt != GFWA_BF16 && dt != GFWA_F32) return GFWA_ERR_UNSUPPORTED;
    const void* mats[] = {Q, K, V, O, dO, dQ, dK, dV};
    for (const void* p : mats)
        if (!aligned(p, 16)) return GFWA_ERR_ALIGN;
    if (!aligned(c, 4) || !aligned(L, 4) || !aligned(dalpha, 4)) return GFWA_ERR_ALIGN;
    const size_t need = gfwa_backward_workspace_bytes(dt, B, H, N, d, w);
    if (!workspace || workspace_bytes < need) return GFWA_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return GFWA_ERR_ALIGN;
    float* ws = (float*)workspace;
    if (dt == GFWA_F32)
        return hip_status(backward_f32((const float*)Q, (const float*)K, (const float*)V, (const float*)O,
                                       (const float*)dO, c, L, (float*)dQ, (float*)dK, (float*)dV, dalpha,
                                       ws, B, H, Hkv, N, d, w, scale, stream));
    const size_t fast = gfwa_backward_fast_workspace_bytes(dt, B, H, N, d, w);
    const bool spill = fast > need && workspace_bytes >= fast;
    return hip_status(
        backward_bf16(Q, K, V, O, dO, c, L, dQ, dK, dV, dalpha, ws, spill, B, H, Hkv, N, d, w, scale, stream));
}

size_t gfwa_decode_workspace_bytes(int B, int H, int T, int d, int w) {
    if (check_dims(B, H, T, d, w, true) != GFWA_OK) return 0;
    return (decode_workspace_bytes(B, H, T, d, w) + 255) & ~(size_t)255;
}

int gfwa_decode(gfwa_dtype_t dt, const void* q, const void* Kc, const void* Vc, float* c, const float* alpha_t,
                const int* pos, void* o, float* L, void* workspace, size_t workspace_bytes, int B, int H, int Hkv,
                int T, int d, int w, float scale, gfwa_stream_t stream) {
    if (!q || !Kc || !Vc || !c || !pos || !o) return GFWA_ERR_NULL;
    if (int r = check_dims(B, H, T, d, w, true)) return r;
    if (Hkv <= 0 || H % Hkv != 0) return GFWA_ERR_DIM;
    if (dt != GFWA_BF16 && dt != GFWA_F32) return GFWA_ERR_UNSUPPORTED;
    if (!aligned(q, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(o, 16) || !aligned(c, 4) ||
        !aligned(pos, 4) || (alpha_t && !aligned(alpha_t, 4)) || (L && !aligned(L, 4)))
        return GFWA_ERR_ALIGN;
    if (!workspace || workspace_bytes < gfwa_decode_workspace_bytes(B, H, T, d, w)) return GFWA_ERR_WORKSPACE;
    if (!aligned(workspace, 16)) return GFWA_ERR_ALIGN;
    return hip_status(decode(dt == GFWA_BF16, q, Kc, Vc, c, alpha_t, pos, o, L, (float*)workspace, B, H, Hkv, T, d,
                             w, scale, stream));
}

int gfwa_decode_static(gfwa_dtype_t dt, const void* q, const void* Kc, const void* Vc, float* c,
                       const float* alpha_t, const int* pos, void* o, float* L, int B, int H, int Hkv, int T, int d,
                       int w, float scale, gfwa_stream_t stream) {
    if (!q || !Kc || !Vc || !c || !pos || !o) return GFWA_ERR_NULL;
    if (int r = check_dims(B, H, T, d, w, true)) return r;
    if (Hkv <= 0 || H % Hkv != 0) return GFWA_ERR_DIM;
    if (dt != GFWA_BF16 && dt != GFWA_F32) return GFWA_ERR_UNSUPPORTED;
    if (!aligned(q, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(o, 16) || !aligned(c, 4) ||
        !aligned(pos, 4) || (alpha_t && !aligned(alpha_t, 4)) || (L && !aligned(L, 4)))
        return GFWA_ERR_ALIGN;
    if (gfwa_decode_workspace_bytes(B, H, T, d, w) > kDecodeStaticBytes) return GFWA_ERR_WORKSPACE;
    float* part = nullptr;
    if (hipError_t e = decode_static_scratch(&part)) return hip_status(e);
    return hip_status(decode(dt == GFWA_BF16, q, Kc, Vc, c, alpha_t, pos, o, L, part, B, H, Hkv, T, d, w, scale,
                             stream));
}

const char* gfwa_strerror(int code) {
    switch (code) {
        case GFWA_OK: return "ok";
        case GFWA_ERR_NULL: return "a required pointer is NULL";
        case GFWA_ERR_DIM: return "invalid size: B, H, N, d must be > 0, w >= 1, Hkv > 0 dividing H, within index range";
        case GFWA_ERR_UNSUPPORTED: return "unsupported head dimension (64 or 128) or dtype";
        case GFWA_ERR_ALIGN: return "pointer not sufficiently aligned (16 bytes matrices, 4 bytes vectors)";
        case GFWA_ERR_WORKSPACE:
            return "workspace missing or smaller than the matching gfwa_*_workspace_bytes() call asks for; for "
                   "gfwa_decode_static: the sizes need more than the library's 32 MiB of scratch";
        case GFWA_ERR_HIP: return g_hip_msg;
        default: return "unknown status code";
    }
}

int gfwa_version(void) { return 100; }

int gfwa_probe_mfma(float* sink, int iterations, int workgroups, int random_operands, double* flops,
                    gfwa_stream_t stream) {
    if (!sink) return GFWA_ERR_NULL;
    if (iterations < 1 || workgroups < 1 || workgroups > (1 << 20) || iterations > (1 << 24)) return GFWA_ERR_DIM;
    if (!aligned(sink, 4)) return GFWA_ERR_ALIGN;
    if (random_operands < 0 || random_operands > 2) return GFWA_ERR_DIM;
    return hip_status(probe_mfma(sink, iterations, workgroups, random_operands, flops, stream));
}

int gfwa_probe_copy(const void* src, void* dst, size_t bytes, gfwa_stream_t stream) {
    if (!src || !dst) return GFWA_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0) return GFWA_ERR_DIM;
    if (!aligned(src, 16) || !aligned(dst, 16)) return GFWA_ERR_ALIGN;
    return hip_status(probe_copy(src, dst, bytes, stream));
}

int gfwa_profile_enable(int on) {
    std::lock_guard<std::mutex> hold(g_prof.lock);
    g_prof.on.store(on != 0, std::memory_order_relaxed);
    if (on) g_prof.used = 0;  // records stay readable after profiling is switched off
    return GFWA_OK;
}

int gfwa_profile_read(float* total_ms, int* launches, int n) {
    if (!total_ms || !launches) return GFWA_ERR_NULL;
    if (n < kKernCount) return GFWA_ERR_DIM;
    for (int k = 0; k < n; ++k) {
        total_ms[k] = 0.f;
        launches[k] = 0;
    }
    std::lock_guard<std::mutex> hold(g_prof.lock);
    for (int i = 0; i < g_prof.used; ++i) {
        hipError_t e = hipEventSynchronize(g_prof.rec[i].stop);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, g_prof.rec[i].start, g_prof.rec[i].stop);
        if (e != hipSuccess) return hip_status(e);
        total_ms[g_prof.rec[i].kernel] += ms;
        launches[g_prof.rec[i].kernel] += 1;
    }
    return GFWA_OK;
}

const char* gfwa_profile_kernel_name(int k) {
    static const char* names[kKernCount] = {"gate_prefix_scan", "forward", "bwd_rowdot", "bwd_dkv", "bwd_dq",
                                            "gate_grad_scan", "gate_activation_prefix_scan",
                                            "gate_activation_bwd", "decode_partial", "decode_combine", "scan_segment_sum", "scan_propagate",
                                            "gate_grad_segment_sum"};
    return (k >= 0 && k < kKernCount) ? names[k] : "";
}

}  // extern "C"
