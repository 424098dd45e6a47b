// Two measurement kernels that calibrate the rooflines the attention kernels are held against: what the
// matrix cores and the memory system of the device at hand actually sustain (not part of the method).
//   * a loop of nothing but v_mfma_f32_32x32x16_bf16 on every SIMD of the chip: the achievable bf16 MFMA rate
//     at the clock the part settles to under that load;
//   * a plain copy with 16-byte accesses: the achievable HBM rate, and the known-size reference the
//     FETCH_SIZE / WRITE_SIZE counters are scaled by.
#include "gfwa_device.h"
#include "gfwa_internal.h"
#include "tile_stage.h"

namespace gfwa {

constexpr int kProbeThreads = 512;  // 8 waves: two per SIMD
constexpr int kProbeUnroll = 16;    // MFMAs per loop iteration and wave

// RANDOM = false: one pair of operands with small constant values (few bits toggle: the rate at the highest clock
// the part reaches with busy matrix cores).  RANDOM = true: sixteen pairs of pseudo-random operands of unit variance,
// like the attention inputs, a different pair for every MFMA of the loop body (the rate at the clock the part
// sustains when the operand buses and multipliers switch as they do on real data).
template <bool RANDOM>
__global__ __launch_bounds__(kProbeThreads) void probe_mfma_kernel(float* __restrict__ sink, int iterations) {
    constexpr int NOP = RANDOM ? 4 : 1;
    f32x16 acc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;
    bf16x8 x[NOP], y[NOP];
#pragma unroll
    for (int k = 0; k < NOP; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (RANDOM) {
                // integer hash of (thread, workgroup, operand, element) -> uniform on [-sqrt 3, sqrt 3)
                unsigned u = (threadIdx.x * 8u + e) * 2654435761u + (blockIdx.x * 4u + k) * 2246822519u + 374761393u;
                u ^= u >> 15; u *= 2246822519u; u ^= u >> 13; u *= 3266489917u; u ^= u >> 16;
                unsigned t = u * 2654435761u + 0x9e3779b9u;
                t ^= t >> 15; t *= 2246822519u; t ^= t >> 13;
                x[k][e] = (bf16_t)(((float)(u >> 8) * (1.0f / 8388608.0f) - 1.0f) * 1.7320508f);
                y[k][e] = (bf16_t)(((float)(t >> 8) * (1.0f / 8388608.0f) - 1.0f) * 1.7320508f);
            } else {
                x[k][e] = (bf16_t)(0.001f * (float)((threadIdx.x + e) & 31));
                y[k][e] = (bf16_t)(0.002f * (float)((threadIdx.x + 3 * e) & 15));
            }
        }
    for (int it = 0; it < iterations; ++it)
#pragma unroll
        for (int i = 0; i < kProbeUnroll; ++i) acc[i % 4] = mfma32(x[i % NOP], y[(i / 4) % NOP], acc[i % 4]);
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[a][v];
    if (s == -1.0f) sink[0] = s;  // practically never true: keeps the loop alive without a store (sink is one float the caller owns)
}

// The MFMA loop with the companion work of the attention inner loops: per MFMA one operand fragment read from LDS
// (alternately a 16-byte read and a pair of transposing 8-byte reads, requested four MFMAs ahead), four fused
// multiply-adds and one exp2 on the vector unit; pseudo-random data everywhere.  The rate this reaches is what
// the matrix cores sustain beside the least an attention kernel has to do per MFMA, at the clock the part
// settles to under that load.
__global__ __launch_bounds__(kProbeThreads) void probe_mix_kernel(float* __restrict__ sink, int iterations) {
    __shared__ __attribute__((aligned(16))) char lds[2 * kTileRows * 256];  // two swizzled 64 x 128 bf16 tiles
    const int tid = threadIdx.x, lane = tid & 63;
    for (int i = tid; i < (int)sizeof(lds) / 4; i += kProbeThreads) {
        unsigned u = (unsigned)i * 2654435761u + 12345u;
        u ^= u >> 15; u *= 2246822519u; u ^= u >> 13; u *= 3266489917u; u ^= u >> 16;
        reinterpret_cast<unsigned*>(lds)[i] = (u & 0x807f807fu) | 0x3f003f00u | ((u >> 3) & 0x00800080u);  // two bf16 in +-[0.5, 2)
    }
    __syncthreads();
    f32x16 acc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][v] = 0.f;
    bf16x8 y[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            unsigned u = (threadIdx.x * 8u + e) * 2654435761u + (blockIdx.x * 4u + k) * 2246822519u + 374761393u;
            u ^= u >> 15; u *= 2246822519u; u ^= u >> 13; u *= 3266489917u; u ^= u >> 16;
            y[k][e] = (bf16_t)(((float)(u >> 8) * (1.0f / 8388608.0f) - 1.0f) * 1.7320508f);
        }
    float x[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) x[e] = 0.05f + 0.9f * (float)((lane * 16 + e) % 97) / 97.0f;
    auto fetch = [&](int f) __attribute__((always_inline)) -> bf16x8 {
        const char* tile = lds + ((f >> 3) & 1) * (kTileRows * 256);
        return (f & 1) ? lds_read_tr_frag<128>(tile, 16 * ((f >> 1) & 3), (f >> 1) & 3, lane)
                       : lds_read_frag<128>(tile, 32 * ((f >> 1) & 1), (f >> 1) & 7, lane);
    };
    constexpr int kAhead = 4;
    for (int it = 0; it < iterations; ++it) {
        bf16x8 fr[kProbeUnroll];
        asm volatile("" ::: "memory");  // the reads belong to this iteration
#pragma unroll
        for (int f = 0; f < kAhead; ++f) fr[f] = fetch(f);
        __builtin_amdgcn_sched_group_barrier(0x100, 3 * kAhead / 2, 0);
#pragma unroll
        for (int i = 0; i < kProbeUnroll; ++i) {
            acc[i % 4] = mfma32(fr[i], y[(i / 4) % 4], acc[i % 4]);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i + kAhead < kProbeUnroll) {
                fr[i + kAhead] = fetch(i + kAhead);
                if ((i + kAhead) & 1) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
#pragma unroll
            for (int r = 0; r < 5; ++r) {  // values stay inside (0, 1]
                const int e = (i * 5 + r) % 16;
                x[e] = r == 0 ? fast_exp2(-x[e]) : __builtin_fmaf(x[e], 0.999f, 0.0007f);
            }
            __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[a][v];
#pragma unroll
    for (int e = 0; e < 16; ++e) s += x[e];
    if (s == -1.0f) sink[0] = s;  // practically never true: keeps the loop alive without a store
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Launches the MFMA loop on `workgroups` workgroups of 8 waves; *flops receives the floating-point operations
// the launch performs (2 * 32 * 32 * 16 per MFMA).
hipError_t probe_mfma(float* sink, int iterations, int workgroups, int random_operands, double* flops, hipStream_t s) {
    if (random_operands == 2)
        hipLaunchKernelGGL(probe_mix_kernel, dim3(workgroups), dim3(kProbeThreads), 0, s, sink, iterations);
    else if (random_operands)
        hipLaunchKernelGGL(probe_mfma_kernel<true>, dim3(workgroups), dim3(kProbeThreads), 0, s, sink, iterations);
    else
        hipLaunchKernelGGL(probe_mfma_kernel<false>, dim3(workgroups), dim3(kProbeThreads), 0, s, sink, iterations);
    if (flops) *flops = 2.0 * 32 * 32 * 16 * kProbeUnroll * (double)iterations * (kProbeThreads / 64) * (double)workgroups;
    return hipGetLastError();
}

hipError_t probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    const int cus = device_cu_count();
    hipLaunchKernelGGL(probe_copy_kernel, dim3(cus * 16), dim3(256), 0, s, (const u32x4*)src, (u32x4*)dst, n16);
    return hipGetLastError();
}

}  // namespace gfwa
