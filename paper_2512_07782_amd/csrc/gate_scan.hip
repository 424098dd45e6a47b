// Gate prefix scans on gfx950 (paper Sec. 3.2 definition of the cumulative gate; Alg. 1, the
// cumulative-sum / carry steps; Sec. 3.3 for the reverse scan that turns d(prefix) into d(alpha)).
//
// One workgroup of 16 waves streams one (b,h) row in chunks of 4096 elements: float4 per thread,
// in-thread prefix, wavefront scan of the thread totals by lane shuffles, the 16 wave totals
// through LDS, and a carry kept in fp64 across chunks.  Every element is read once and written
// once (8 bytes of HBM traffic per element).
//
// The same kernel also fuses the gate activation of Alg. 1 in front of the scan: with the
// pre-activation h and the amplitude beta as inputs it forms
//   alpha = softplus(beta h) / (beta + eps),  softplus(z) = nu + log(exp(z - nu) + exp(-nu)), nu = max(z, 0)
// (evaluated as nu + log1p(exp(-|z|)), the same sum; see softplus_parts)
// on the fly (12 bytes per element, no alpha or z tensor in HBM), which is the paper's one-pass
// gate preprocessing as a whole.
#include "gfwa_device.h"
#include "gfwa_internal.h"

namespace gfwa {

constexpr int kScanThreads = 1024;
constexpr int kScanWaves = kScanThreads / 64;
constexpr int kScanChunk = kScanThreads * 4;
constexpr int kScanTargetWorkgroups = 2048;  // scan-then-propagate: segments are cut until about this many exist

// Softplus of z in the overflow-safe form of Alg. 1, nu + log(exp(z - nu) + exp(-nu)) with nu = max(z, 0).
// One of the two exponentials is exp(0) = 1 and the other is e = exp(-|z|), so the logarithm is
// log(1 + e), 0 < e <= 1.  Built on the hardware exp2 / log2 / reciprocal (about 1 ulp each) so that
// the kernels stay bound by memory traffic, and arranged so that a small result keeps its
// relative accuracy:
//   e       = 2^(x log2(e)) with the rounding error of the product x log2(e) carried as a correction,
//   log1p(e) = log(u) * e / (u - 1),  u = fl(1 + e)   (= e when u rounds to 1),
// the second being the classical cure for the rounding of 1 + e.  Returns softplus(z); *e_out = e.
__device__ __forceinline__ float softplus_parts(float z, float* e_out) {
    constexpr float kLog2eHi = 1.44269502162933349609375f;  // fl(log2(e))
    constexpr float kLog2eLo = 1.92596299e-8f;              // log2(e) - kLog2eHi
    constexpr float kLn2 = 0.693147182464599609375f;
    const float x = fmaxf(-fabsf(z), -128.f);               // below -128 e is 0 in fp32 anyway
    const float t = x * kLog2eHi;
    const float t_lo = fmaf(x, kLog2eHi, -t) + x * kLog2eLo;
    const float p = __builtin_amdgcn_exp2f(t);
    const float e = fmaf(p, t_lo * kLn2, p);
    const float u = 1.0f + e;
    const float um1 = u - 1.0f;
    const float l = __builtin_amdgcn_logf(u) * kLn2;        // log(u), u in [1, 2]
    const float log1p_e = um1 == 0.f ? e : l * (e * __builtin_amdgcn_rcpf(um1));
    *e_out = e;
    return fmaxf(z, 0.f) + log1p_e;
}

// alpha of one element (Alg. 1, on-chip steps)
__device__ __forceinline__ float gate_alpha(float h, float beta, float eps) {
    float e;
    return softplus_parts(beta * h, &e) * __builtin_amdgcn_rcpf(beta + eps);
}

enum ScanInput { kScanPlain = 0, kScanDiff = 1, kScanGate = 2 };

// Logical position p of the scan maps to memory index p (forward) or N-1-p (reverse).
// MODE kScanDiff: the scanned value is a[idx] - b[idx]; kScanGate: gate_alpha(a[idx], b[idx], eps).
// With `partial` given (scan-then-propagate) a workgroup takes segment blockIdx.x % P of row blockIdx.x / P,
// seg_len logical positions long, and starts from the sum of the row's earlier segments.
template <bool REVERSE, int MODE>
__global__ __launch_bounds__(kScanThreads) void scan_rows_kernel(const float* __restrict__ a,
                                                                 const float* __restrict__ b,
                                                                 float* __restrict__ out, int N, float eps,
                                                                 const double* __restrict__ partial = nullptr,
                                                                 int seg_len = 0, int P = 1) {
    constexpr bool DIFF = MODE != kScanPlain;  // a second input row
    __shared__ float wave_tot[kScanWaves];
    __shared__ double wave_carry[kScanWaves];
    const int seg = partial != nullptr ? (int)(blockIdx.x % P) : 0;
    const size_t row = (size_t)(partial != nullptr ? blockIdx.x / P : blockIdx.x) * N;
    const int begin = partial != nullptr ? seg * seg_len : 0;
    const int end = partial != nullptr ? min(N, begin + seg_len) : N;
    const float* ar = a + row;
    const float* br = DIFF ? b + row : nullptr;
    float* outr = out + row;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    // float4 path only when every row starts 16-byte aligned
    const uintptr_t bits = (uintptr_t)a | (uintptr_t)out | (DIFF ? (uintptr_t)b : (uintptr_t)0);
    const bool vec = (N % 4 == 0) && ((bits & 15) == 0);

    double carry = 0.0;
    if (partial != nullptr && seg > 0) {  // sum of the earlier segments of this row, fp64
        const double* pr = partial + (size_t)(blockIdx.x / P) * P;
        double acc = 0.0;
        for (int q = tid; q < seg; q += kScanThreads) acc += pr[q];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
        if (lane == 0) wave_carry[wv] = acc;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kScanWaves; ++k) carry += wave_carry[k];
    }
    for (int base = begin; base < end; base += kScanChunk) {
        const int p0 = base + 4 * tid;
        float v[4] = {0.f, 0.f, 0.f, 0.f};
        if (vec && p0 + 3 < end) {
            const int idx = REVERSE ? N - 4 - p0 : p0;
            float4 x = *reinterpret_cast<const float4*>(ar + idx);
            if (MODE == kScanDiff) {
                const float4 y = *reinterpret_cast<const float4*>(br + idx);
                x.x -= y.x; x.y -= y.y; x.z -= y.z; x.w -= y.w;
            } else if (MODE == kScanGate) {
                const float4 y = *reinterpret_cast<const float4*>(br + idx);
                x.x = gate_alpha(x.x, y.x, eps); x.y = gate_alpha(x.y, y.y, eps);
                x.z = gate_alpha(x.z, y.z, eps); x.w = gate_alpha(x.w, y.w, eps);
            }
            if (REVERSE) { v[0] = x.w; v[1] = x.z; v[2] = x.y; v[3] = x.x; }
            else         { v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w; }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int p = p0 + e;
                if (p < end) {
                    const int idx = REVERSE ? N - 1 - p : p;
                    v[e] = MODE == kScanDiff ? ar[idx] - br[idx]
                         : MODE == kScanGate ? gate_alpha(ar[idx], br[idx], eps) : ar[idx];
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
        if (vec && p0 + 3 < end) {
            const int idx = REVERSE ? N - 4 - p0 : p0;
            const float4 y = REVERSE ? make_float4(r[3], r[2], r[1], r[0]) : make_float4(r[0], r[1], r[2], r[3]);
            *reinterpret_cast<float4*>(outr + idx) = y;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int p = p0 + e;
                if (p < end) outr[REVERSE ? N - 1 - p : p] = r[e];
            }
        }
    }
}

// Phase 1 of scan-then-propagate (App. "Preprocessing via Scan-Then-Propagate"): the sum of every
// segment, the activation recomputed on the fly when the input is (h, beta).  fp32 per thread over
// its few elements, fp64 across the workgroup.
template <bool REVERSE, int MODE>
__global__ __launch_bounds__(kScanThreads) void segment_sum_kernel(const float* __restrict__ a,
                                                                   const float* __restrict__ b,
                                                                   double* __restrict__ partial, int N, float eps,
                                                                   int seg_len, int P) {
    __shared__ double wave_sum[kScanWaves];
    const int seg = (int)(blockIdx.x % P);
    const size_t row = (size_t)(blockIdx.x / P) * N;
    const int begin = seg * seg_len, end = min(N, begin + seg_len);
    const float* ar = a + row;
    const float* br = MODE != kScanPlain ? b + row : nullptr;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uintptr_t bits = (uintptr_t)a | (MODE != kScanPlain ? (uintptr_t)b : (uintptr_t)0);
    const bool vec = (N % 4 == 0) && ((bits & 15) == 0);
    float acc = 0.f;
    for (int base = begin; base < end; base += kScanChunk) {  // logical positions, as in scan_rows_kernel
        const int p0 = base + 4 * tid;
        if (vec && p0 + 3 < end) {
            const int idx = REVERSE ? N - 4 - p0 : p0;
            float4 x = *reinterpret_cast<const float4*>(ar + idx);
            if (MODE == kScanGate) {
                const float4 y = *reinterpret_cast<const float4*>(br + idx);
                x.x = gate_alpha(x.x, y.x, eps); x.y = gate_alpha(x.y, y.y, eps);
                x.z = gate_alpha(x.z, y.z, eps); x.w = gate_alpha(x.w, y.w, eps);
            } else if (MODE == kScanDiff) {
                const float4 y = *reinterpret_cast<const float4*>(br + idx);
                x.x -= y.x; x.y -= y.y; x.z -= y.z; x.w -= y.w;
            }
            acc += (x.x + x.y) + (x.z + x.w);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int p = p0 + e;
                if (p < end) {
                    const int idx = REVERSE ? N - 1 - p : p;
                    acc += MODE == kScanGate ? gate_alpha(ar[idx], br[idx], eps) : MODE == kScanDiff ? ar[idx] - br[idx] : ar[idx];
                }
            }
        }
    }
    double t = (double)acc;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) t += __shfl_xor(t, d, 64);
    if (lane == 0) wave_sum[wv] = t;
    __syncthreads();
    if (tid == 0) {
        double all = 0.0;
#pragma unroll
        for (int k = 0; k < kScanWaves; ++k) all += wave_sum[k];
        partial[blockIdx.x] = all;
    }
}

hipError_t gate_prefix(const float* alpha, float* c, int rows, int N, hipStream_t s) {
    ProfScope prof(kKernGatePrefix, s);
    hipLaunchKernelGGL((scan_rows_kernel<false, kScanPlain>), dim3(rows), dim3(kScanThreads), 0, s, alpha,
                       (const float*)nullptr, c, N, 0.f);
    return hipGetLastError();
}

hipError_t gate_activation_prefix(const float* hpre, const float* beta, float eps, float* c, int rows, int N,
                                  hipStream_t s) {
    ProfScope prof(kKernGateActPrefix, s);
    hipLaunchKernelGGL((scan_rows_kernel<false, kScanGate>), dim3(rows), dim3(kScanThreads), 0, s, hpre, beta, c,
                       N, eps);
    return hipGetLastError();
}

// Scan-then-propagate for few, very long rows: P segments per row, each a workgroup of its own.
int scan_segments(int rows, int N, int* seg_len) {
    const int chunks = (N + kScanChunk - 1) / kScanChunk;
    int P = (kScanTargetWorkgroups + rows - 1) / rows;
    if (P > chunks) P = chunks;
    if (P < 1) P = 1;
    const int seg_chunks = (chunks + P - 1) / P;
    *seg_len = seg_chunks * kScanChunk;
    return (chunks + seg_chunks - 1) / seg_chunks;
}

size_t gate_scan_workspace_bytes(int rows, int N) {
    return (size_t)rows * ((N + kScanChunk - 1) / kScanChunk) * sizeof(double);  // at most one segment per chunk
}

hipError_t gate_prefix_stp(const float* in, const float* beta, float eps, float* c, double* partial, int rows,
                           int N, hipStream_t s) {
    int seg_len = 0;
    const int P = scan_segments(rows, N, &seg_len);
    const dim3 grid((unsigned)(rows * P)), block(kScanThreads);
    {
        ProfScope prof(kKernScanSegmentSum, s);
        if (beta != nullptr)
            hipLaunchKernelGGL((segment_sum_kernel<false, kScanGate>), grid, block, 0, s, in, beta, partial, N, eps, seg_len, P);
        else
            hipLaunchKernelGGL((segment_sum_kernel<false, kScanPlain>), grid, block, 0, s, in, beta, partial, N, eps, seg_len, P);
    }
    {
        ProfScope prof(kKernScanPropagate, s);
        if (beta != nullptr)
            hipLaunchKernelGGL((scan_rows_kernel<false, kScanGate>), grid, block, 0, s, in, beta, c, N, eps,
                               (const double*)partial, seg_len, P);
        else
            hipLaunchKernelGGL((scan_rows_kernel<false, kScanPlain>), grid, block, 0, s, in, beta, c, N, eps,
                               (const double*)partial, seg_len, P);
    }
    return hipGetLastError();
}

// d(alpha) -> d(h), d(beta): elementwise chain rule on the gate's definition
//   sigma = 1 / (1 + exp(-z)),  d alpha/d h = sigma beta / (beta + eps),
//   d alpha/d beta = sigma h / (beta + eps) - softplus(z) / (beta + eps)^2
__device__ __forceinline__ void gate_grad(float h, float b, float g, float eps, float& dh, float& dbeta) {
    const float z = b * h;
    float e;
    const float sp = softplus_parts(z, &e);
    const float sig = (z >= 0.f ? 1.0f : e) * __builtin_amdgcn_rcpf(1.0f + e);  // sigma(z), no overflow
    const float rbe = __builtin_amdgcn_rcpf(b + eps);
    const float gs = g * sig * rbe;
    dh = gs * b;
    dbeta = gs * h - g * sp * rbe * rbe;
}

// VEC: every pointer is 16-byte aligned, the body moves float4; the last n % 4 elements go one by one
template <bool VEC>
__global__ __launch_bounds__(256) void gate_activation_bwd_kernel(const float* __restrict__ hpre,
                                                                  const float* __restrict__ beta,
                                                                  const float* __restrict__ dalpha,
                                                                  float* __restrict__ dh,
                                                                  float* __restrict__ dbeta, size_t n, float eps) {
    const size_t tid = (size_t)blockIdx.x * 256 + threadIdx.x, nthr = (size_t)gridDim.x * 256;
    const size_t n4 = VEC ? n / 4 : 0;
    for (size_t i = tid; i < n4; i += nthr) {
        const float4 h = reinterpret_cast<const float4*>(hpre)[i];
        const float4 b = reinterpret_cast<const float4*>(beta)[i];
        const float4 g = reinterpret_cast<const float4*>(dalpha)[i];
        float4 oh, ob;
        gate_grad(h.x, b.x, g.x, eps, oh.x, ob.x);
        gate_grad(h.y, b.y, g.y, eps, oh.y, ob.y);
        gate_grad(h.z, b.z, g.z, eps, oh.z, ob.z);
        gate_grad(h.w, b.w, g.w, eps, oh.w, ob.w);
        reinterpret_cast<float4*>(dh)[i] = oh;
        reinterpret_cast<float4*>(dbeta)[i] = ob;
    }
    for (size_t i = n4 * 4 + tid; i < n; i += nthr) gate_grad(hpre[i], beta[i], dalpha[i], eps, dh[i], dbeta[i]);
}

hipError_t gate_activation_backward(const float* hpre, const float* beta, float eps, const float* dalpha,
                                    float* dh, float* dbeta, size_t n, hipStream_t s) {
    ProfScope prof(kKernGateActBwd, s);
    const bool vec = (((uintptr_t)hpre | (uintptr_t)beta | (uintptr_t)dalpha | (uintptr_t)dh | (uintptr_t)dbeta) & 15) == 0;
    const size_t want = ((vec ? n / 4 + 3 : n) + 255) / 256;
    const unsigned grid = (unsigned)(want < 8192 ? (want ? want : 1) : 8192);
    if (vec)
        hipLaunchKernelGGL(gate_activation_bwd_kernel<true>, dim3(grid), dim3(256), 0, s, hpre, beta, dalpha, dh,
                           dbeta, n, eps);
    else
        hipLaunchKernelGGL(gate_activation_bwd_kernel<false>, dim3(grid), dim3(256), 0, s, hpre, beta, dalpha, dh,
                           dbeta, n, eps);
    return hipGetLastError();
}

// Few long rows leave most of the chip idle with one workgroup per row: then the rows are cut into segments
// (scan-then-propagate, as gate_prefix_stp does for the forward prefix), which needs `partial`.
bool gate_grad_scan_wants_segments(int rows, int N) {
    return rows < device_cu_count() && N >= 2 * kScanChunk;
}

hipError_t gate_grad_scan(const float* dc_col, const float* dc_row, float* dalpha, double* partial, int rows, int N,
                          hipStream_t s) {
    if (partial != nullptr && gate_grad_scan_wants_segments(rows, N)) {
        int seg_len = 0;
        const int P = scan_segments(rows, N, &seg_len);
        const dim3 grid((unsigned)(rows * P)), block(kScanThreads);
        {
            ProfScope prof(kKernGateGradSegmentSum, s);
            hipLaunchKernelGGL((segment_sum_kernel<true, kScanDiff>), grid, block, 0, s, dc_col, dc_row, partial, N, 0.f,
                               seg_len, P);
        }
        ProfScope prof(kKernGateGrad, s);
        hipLaunchKernelGGL((scan_rows_kernel<true, kScanDiff>), grid, block, 0, s, dc_col, dc_row, dalpha, N, 0.f,
                           (const double*)partial, seg_len, P);
        return hipGetLastError();
    }
    ProfScope prof(kKernGateGrad, s);
    hipLaunchKernelGGL((scan_rows_kernel<true, kScanDiff>), dim3(rows), dim3(kScanThreads), 0, s, dc_col,
                       dc_row, dalpha, N, 0.f);
    return hipGetLastError();
}

}  // namespace gfwa
