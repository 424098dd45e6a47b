// Staging of a pair of 64-row bf16 tiles (K and V, or Q and dO) from global memory into swizzled
// LDS by a 256-thread workgroup, with direct global->LDS loads (no staging registers, no LDS
// stores).  Rows at or beyond N read row N-1: finite data that the band mask keeps out of every sum.
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

// Each of the WAVES waves of the workgroup fills 64 / WAVES consecutive rows of a tile with 1 KB
// loads; lane p of a load writes row p / chunks-per-row of its group at physical chunk
// p % chunks-per-row and therefore fetches the logical chunk the swizzle maps there (the swizzle
// is an involution).
template <int D, int WAVES = 4>
struct TilePairLoader {
    static constexpr int kRowBytes = D * 2;
    static constexpr int kRowsPerLoad = 1024 / kRowBytes;
    static constexpr int kChunksPerRow = kRowBytes / 16;
    static constexpr int kRowsPerWave = kTileRows / WAVES;
    static constexpr int kLoadsPerWave = kRowsPerWave / kRowsPerLoad;
    static constexpr int kLoadsPerTilePair = 2 * kLoadsPerWave;  // per wave
    static_assert(kLoadsPerWave >= 1, "a wave must cover at least one 1 KB load");
    unsigned off[kLoadsPerWave];
    int wv, lane;

    __device__ __forceinline__ void init(int wave, int lane_) {
        wv = wave;
        lane = lane_;
#pragma unroll
        for (int g = 0; g < kLoadsPerWave; ++g) {
            const int row = kRowsPerWave * wv + kRowsPerLoad * g + lane / kChunksPerRow;
            off[g] = (unsigned)(row * kRowBytes + swz_chunk<D>(row, lane % kChunksPerRow) * 16);
        }
    }
    // tile index j (rows 64j .. 64j+63) of the [N, D] matrices at Ah and Bh into buffer `buf`;
    // tiles below jfull = N / 64 lie wholly inside the sequence
    __device__ __forceinline__ void load(const char* Ah, const char* Bh, int j, int jfull, int N,
                                         char* a_tile, char* b_tile) const {
        char* al = a_tile + kRowsPerWave * wv * kRowBytes;
        char* bl = b_tile + kRowsPerWave * wv * kRowBytes;
        if (j < jfull) {
            const size_t toff = (size_t)j * (kTileRows * kRowBytes);
#pragma unroll
            for (int g = 0; g < kLoadsPerWave; ++g) {
                dma16(Ah + toff, off[g], al + g * 1024);
                dma16(Bh + toff, off[g], bl + g * 1024);
            }
        } else {
            int ln = lane;  // re-derived here (a rare path) instead of living in registers across the caller's loop
            GFWA_PIN(ln);
#pragma unroll
            for (int g = 0; g < kLoadsPerWave; ++g) {
                const int row = kRowsPerWave * wv + kRowsPerLoad * g + ln / kChunksPerRow;
                const int r = min(j * kTileRows + row, N - 1);
                const unsigned o =
                    (unsigned)r * (unsigned)kRowBytes + (unsigned)(swz_chunk<D>(row, ln % kChunksPerRow) * 16);
                dma16(Ah, o, al + g * 1024);
                dma16(Bh, o, bl + g * 1024);
            }
        }
    }
    // one tile only (the A side of load)
    __device__ __forceinline__ void load_one(const char* Ah, int j, int jfull, int N, char* a_tile) const {
        char* al = a_tile + kRowsPerWave * wv * kRowBytes;
        if (j < jfull) {
            const size_t toff = (size_t)j * (kTileRows * kRowBytes);
#pragma unroll
            for (int g = 0; g < kLoadsPerWave; ++g) dma16(Ah + toff, off[g], al + g * 1024);
        } else {
#pragma unroll
            for (int g = 0; g < kLoadsPerWave; ++g) {
                const int row = kRowsPerWave * wv + kRowsPerLoad * g + lane / kChunksPerRow;
                const int r = min(j * kTileRows + row, N - 1);
                dma16(Ah, (unsigned)r * (unsigned)kRowBytes + (unsigned)(swz_chunk<D>(row, lane % kChunksPerRow) * 16),
                      al + g * 1024);
            }
        }
    }
};

// Ring of RING key tiles (K rows and V rows, swizzled) with the gate values of their keys, as
// used by the kernels that stream keys past resident queries.
template <int D, int RING>
struct KvRingSmem {
    alignas(16) char k[RING][kTileRows * D * 2];
    alignas(16) char v[RING][kTileRows * D * 2];
    alignas(16) float craw[RING][kTileRows];  // c of the tile's keys as loaded
    alignas(16) float g[RING][kTileRows];     // (c - c_base) / scale
};

// Phase boundary of the two-phase kernels: all LDS traffic of this wave has completed, nothing is
// scheduled across it, and (unlike __syncthreads) outstanding global->LDS loads stay in flight.
__device__ __forceinline__ void wg_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

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

// accumulator rows 8r + 4h + 0..3  <-  vec[row0 + 8r + 4h + 0..3]   (r = 0..3)
__device__ __forceinline__ void acc_init_rows(f32x16& acc, const float* vec, int row0, int h) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const f32x4 g4 = *reinterpret_cast<const f32x4*>(vec + row0 + 8 * r + 4 * h);
        acc[4 * r] = g4[0];
        acc[4 * r + 1] = g4[1];
        acc[4 * r + 2] = g4[2];
        acc[4 * r + 3] = g4[3];
    }
}

// A 32-row block of a bf16 matrix with 32 DB columns, held as DB accumulators in which lane l owns row l % 32
// and register v of accumulator db column 32 db + 8 (v / 4) + 4 (l / 32) + v % 4, goes to global memory as whole
// 128-byte lines: straight from the registers a store instruction would touch 32 rows with 16 bytes each, and
// the memory pipeline takes such an instruction one line at a time.  The block passes through `stage`, 4 KB
// of LDS private to the wave, 64 columns at a time: 8-byte writes in accumulator order, 16-byte reads in row
// order (16-byte chunks XOR-swizzled by row pair, two-way conflicts on the writes, none on the reads).
// g0 = row 0, column 0 of the block; rows at or beyond rows_valid are not stored.  The stores are non-temporal: an
// output is written once and read by a later kernel at the earliest, and should not push K, V, Q or dO tiles that
// neighbouring workgroups are about to re-read out of the L2.
template <int DB>
__device__ __forceinline__ void store_acc_rows(const f32x16 (&acc)[DB], float f, char* stage, bf16_t* g0,
                                               int rows_valid, int lane) {
    GFWA_PIN(lane);  // the addresses below are derived here, not hoisted into registers that live across the caller's loops
    const int lk = lane & 31, h = lane >> 5;
    void* gs = uniform_ptr(g0);  // the block's first row: the same in every lane
    char* wr = stage + lk * 128 + 8 * h;
    const int wsw = (lk >> 1) & 7;
#pragma unroll
    for (int hf = 0; hf < DB / 2; ++hf) {
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x16& a = acc[2 * hf + b2];
                const f32x4 x4 = {a[4 * g] * f, a[4 * g + 1] * f, a[4 * g + 2] * f, a[4 * g + 3] * f};
                *reinterpret_cast<bf16x4*>(wr + ((4 * b2 + g) ^ wsw) * 16) = __builtin_convertvector(x4, bf16x4);
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the wave's writes are in LDS before its lanes read each other's
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = 8 * i + (lane >> 3), q = lane & 7;
            const bf16x8 v = *reinterpret_cast<const bf16x8*>(stage + r * 128 + ((q ^ ((r >> 1) & 7)) * 16));
            if (r < rows_valid) stream_store16<0>(gs, (unsigned)(r * (64 * DB) + 128 * hf + 16 * q), v);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // reads done before the next 64 columns overwrite the stage
    }
}

}  // namespace gfwa
