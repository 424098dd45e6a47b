// Cooperative staging of a pair of 64-row bf16 tiles (K and V, or Q and dO) from global memory
// through registers into swizzled LDS, by a 256-thread workgroup.  Rows at or beyond N read as
// zero so that masked probabilities never multiply garbage.
#pragma once
#include "gfwa_device.h"

namespace gfwa {

constexpr int kThreads = 256;   // 4 waves
constexpr int kTileRows = 64;   // rows per staged LDS tile

template <int D>
struct TilePairSmem {
    alignas(16) char a[2][kTileRows * D * 2];
    alignas(16) char b[2][kTileRows * D * 2];
};

template <int D>
struct TilePairRegs {
    static constexpr int kChunksPerRow = D / 8;
    static constexpr int kPerThread = kTileRows * kChunksPerRow / kThreads;  // 4 (D=128) or 2 (D=64)
    uint4 a[kPerThread], b[kPerThread];

    __device__ __forceinline__ void load(const bf16_t* Ah, const bf16_t* Bh, int row0, int N, int tid) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int id = tid + i * kThreads;
            const int row = row0 + id / kChunksPerRow, chunk = id % kChunksPerRow;
            if (row < N) {
                const size_t off = (size_t)row * D + chunk * 8;
                a[i] = *reinterpret_cast<const uint4*>(Ah + off);
                b[i] = *reinterpret_cast<const uint4*>(Bh + off);
            } else {
                a[i] = make_uint4(0, 0, 0, 0);
                b[i] = make_uint4(0, 0, 0, 0);
            }
        }
    }
    __device__ __forceinline__ void store(TilePairSmem<D>& sm, int buf, int tid) const {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            const int id = tid + i * kThreads;
            const int row = id / kChunksPerRow, chunk = id % kChunksPerRow;
            *reinterpret_cast<uint4*>(sm.a[buf] + tile_off<D>(row, chunk)) = a[i];
            *reinterpret_cast<uint4*>(sm.b[buf] + tile_off<D>(row, chunk)) = b[i];
        }
    }
};

// f32x16 accumulator -> two bf16 B-operand fragments (k-chunks of 16 rows each), in the row order
// the accumulator already has.
__device__ __forceinline__ void acc_to_bfrag(const float (&p)[16], bf16x8 (&f)[2]) {
#pragma unroll
    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            f32x2 pr = {p[8 * c2 + e], p[8 * c2 + e + 1]};
            bf16x2 pb = __builtin_convertvector(pr, bf16x2);
            f[c2][e] = pb[0];
            f[c2][e + 1] = pb[1];
        }
}

}  // namespace gfwa
