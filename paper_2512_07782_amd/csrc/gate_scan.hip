// Gate prefix scans on gfx950 (paper Sec. 3.2 definition of the cumulative gate; Alg. 1, the
// cumulative-sum / carry steps; Sec. 3.3 for the reverse scan that turns d(prefix) into d(alpha)).
//
// One workgroup of 16 waves streams one (b,h) row in chunks of 4096 elements: float4 per thread,
// in-thread prefix, wavefront scan of the thread totals by lane shuffles, the 16 wave totals
// through LDS, and a carry kept in fp64 across chunks.  Every element is read once and written
// once (8 bytes of HBM traffic per element).
#include "gfwa_device.h"
#include "gfwa_internal.h"

namespace gfwa {

constexpr int kScanThreads = 1024;
constexpr int kScanWaves = kScanThreads / 64;
constexpr int kScanChunk = kScanThreads * 4;

// Logical position p of the scan maps to memory index p (forward) or N-1-p (reverse).
// DIFF: the scanned value is a[idx] - b[idx].
template <bool REVERSE, bool DIFF>
__global__ __launch_bounds__(kScanThreads) void scan_rows_kernel(const float* __restrict__ a,
                                                                 const float* __restrict__ b,
                                                                 float* __restrict__ out, int N) {
    __shared__ float wave_tot[kScanWaves];
    const size_t row = (size_t)blockIdx.x * N;
    const float* ar = a + row;
    const float* br = DIFF ? b + row : nullptr;
    float* outr = out + row;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // float4 path only when every row starts 16-byte aligned
    const uintptr_t bits = (uintptr_t)a | (uintptr_t)out | (DIFF ? (uintptr_t)b : (uintptr_t)0);
    const bool vec = (N % 4 == 0) && ((bits & 15) == 0);

    double carry = 0.0;
    for (int base = 0; base < N; base += kScanChunk) {
        const int p0 = base + 4 * tid;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (vec && p0 + 3 < N) {
            const int idx = REVERSE ? N - 4 - p0 : p0;
            float4 x = *reinterpret_cast<const float4*>(ar + idx);
            if (DIFF) {
                const float4 y = *reinterpret_cast<const float4*>(br + idx);
                x.x -= y.x; x.y -= y.y; x.z -= y.z; x.w -= y.w;
            }
            if (REVERSE) { v[0] = x.w; v[1] = x.z; v[2] = x.y; v[3] = x.x; }
            else         { v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int p = p0 + e;
                if (p < N) {
                    const int idx = REVERSE ? N - 1 - p : p;
                    v[e] = DIFF ? ar[idx] - br[idx] : ar[idx];
                }
            }
        }
        v[1] += v[0];
        v[2] += v[1];
        v[3] += v[2];
        // inclusive scan of the per-thread totals across the wavefront
        float incl = v[3];
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const float up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        if (lane == 63) wave_tot[wv] = incl;
        __syncthreads();
        double before = carry;  // everything that precedes this wave in the row
        double all = 0.0;
#pragma unroll
        for (int k = 0; k < kScanWaves; ++k) {
            const float tk = wave_tot[k];
            if (k < wv) before += (double)tk;
            all += (double)tk;
        }
        carry += all;
        __syncthreads();
        const double excl = before + (double)(incl - v[3]);
        float r[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) r[e] = (float)(excl + (double)v[e]);
        if (vec && p0 + 3 < N) {
            const int idx = REVERSE ? N - 4 - p0 : p0;
            const float4 y = REVERSE ? make_float4(r[3], r[2], r[1], r[0]) : make_float4(r[0], r[1], r[2], r[3]);
            *reinterpret_cast<float4*>(outr + idx) = y;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int p = p0 + e;
                if (p < N) outr[REVERSE ? N - 1 - p : p] = r[e];
            }
        }
    }
}

hipError_t gate_prefix(const float* alpha, float* c, int rows, int N, hipStream_t s) {
    ProfScope prof(kKernGatePrefix, s);
    hipLaunchKernelGGL((scan_rows_kernel<false, false>), dim3(rows), dim3(kScanThreads), 0, s, alpha,
                       (const float*)nullptr, c, N);
    return hipGetLastError();
}

hipError_t gate_grad_scan(const float* dc_col, const float* dc_row, float* dalpha, int rows, int N,
                          hipStream_t s) {
    ProfScope prof(kKernGateGrad, s);
    hipLaunchKernelGGL((scan_rows_kernel<true, true>), dim3(rows), dim3(kScanThreads), 0, s, dc_col,
                       dc_row, dalpha, N);
    return hipGetLastError();
}

}  // namespace gfwa
