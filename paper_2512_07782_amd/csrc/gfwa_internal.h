// Host-side launch functions behind the C ABI (one per kernel family).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace gfwa {

// c = inclusive prefix sum of alpha along N, one row per (b,h).
hipError_t gate_prefix(const float* alpha, float* c, int rows, int N, hipStream_t s);
hipError_t gate_activation_prefix(const float* hpre, const float* beta, float eps, float* c, int rows, int N,
                                  hipStream_t s);
hipError_t gate_activation_backward(const float* hpre, const float* beta, float eps, const float* dalpha,
                                    float* dh, float* dbeta, size_t n, hipStream_t s);
// The same prefix (beta == nullptr: of `in` itself; else of the gate activation of (in, beta)) in two
// launches that cut every row into segments (scan-then-propagate); partial: gate_scan_workspace_bytes().
size_t gate_scan_workspace_bytes(int rows, int N);
hipError_t gate_prefix_stp(const float* in, const float* beta, float eps, float* c, double* partial, int rows,
                           int N, hipStream_t s);
// dalpha = reverse inclusive prefix sum of (col - row) along N.  partial: gate_scan_workspace_bytes(rows, N) of
// scratch (or nullptr); with it, few long rows are scanned in segments.
hipError_t gate_grad_scan(const float* dc_col, const float* dc_row, float* dalpha, double* partial, int rows, int N,
                          hipStream_t s);

// Q, O, dO, dQ: [B,H,N,d]; K, V, dK, dV: [B,Hkv,N,d] with Hkv dividing H (query head h reads head h / (H/Hkv));
// c, L, dalpha: [B,H,N].
hipError_t forward_bf16(const void* Q, const void* K, const void* V, const float* c, void* O, float* L,
                        int B, int H, int Hkv, int N, int d, int w, float scale, hipStream_t s);
hipError_t forward_f32(const float* Q, const float* K, const float* V, const float* c, float* O,
                       float* L, int B, int H, int Hkv, int N, int d, int w, float scale, hipStream_t s);

// Workspace layout of the backward: three fp32 vectors of B*H*N (each padded to 256 bytes): D, dc_col,
// dc_row; gate_scan_workspace_bytes(B*H, N) (padded to 256) of segment sums for the gate-gradient scan; with `spill` (bf16, d = 128 only) backward_bf16_spill_bytes() more for the dS blocks.
size_t backward_bf16_spill_bytes(int B, int H, int N, int d, int w);  // 0: no such variant for this shape
hipError_t backward_bf16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                         const float* c, const float* L, void* dQ, void* dK, void* dV, float* dalpha,
                         float* ws, bool spill, int B, int H, int Hkv, int N, int d, int w, float scale,
                         hipStream_t s);
hipError_t backward_f32(const float* Q, const float* K, const float* V, const float* O, const float* dO,
                        const float* c, const float* L, float* dQ, float* dK, float* dV, float* dalpha,
                        float* ws, int B, int H, int Hkv, int N, int d, int w, float scale, hipStream_t s);

// Decoding step: q, o [B,H,d]; caches Kc, Vc [B,Hkv,T,d]; c [B,H,T] (entry pos[b] written when alpha_t is
// given); pos [B] device ints; part: decode_workspace_bytes() of scratch.
size_t decode_workspace_bytes(int B, int H, int Tlen, int d, int w);
hipError_t decode(bool bf16, const void* q, const void* Kc, const void* Vc, float* c, const float* alpha_t,
                  const int* pos, void* o, float* L, float* part, int B, int H, int Hkv, int Tlen, int d, int w,
                  float scale, hipStream_t s);

// Device address, on the current device, of the library's own decode scratch of kDecodeStaticBytes
// (looked up on the first call per device, no allocation).
constexpr size_t kDecodeStaticBytes = (size_t)32 << 20;
hipError_t decode_static_scratch(float** ptr);

// Calibration kernels (probe.hip): a pure bf16 MFMA loop and a plain 16-byte copy.
hipError_t probe_mfma(float* sink, int iterations, int workgroups, int random_operands, double* flops, hipStream_t s);
hipError_t probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s);

// Kernel ids for the optional per-kernel event timing (see gfwa_profile_* in include/gfwa.h).
enum KernelId { kKernGatePrefix = 0, kKernForward, kKernRowDot, kKernDkv, kKernDq, kKernGateGrad, kKernGateActPrefix,
                kKernGateActBwd, kKernDecode, kKernDecodeCombine, kKernScanSegmentSum,
                kKernScanPropagate, kKernGateGradSegmentSum, kKernCount };

// Per-device launch set-up, done once per device and kernel (`done`: one bit per device id, owned by the caller):
// lets `kernel` use `bytes` of dynamic LDS on the current device.
struct DeviceOnce { unsigned long long bits = 0; };
hipError_t allow_dynamic_lds(const void* kernel, size_t bytes, DeviceOnce& done);
// Compute units of the current device (256 if the query fails).
int device_cu_count();

// RAII pair of HIP events around one kernel launch on stream s; a no-op unless profiling is on.
struct ProfScope {
    ProfScope(int kernel, hipStream_t s);
    ~ProfScope();
    int slot_;
    hipStream_t s_;
};


}  // namespace gfwa
