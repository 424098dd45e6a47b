// Device-side building blocks shared by the gfx950 kernels: vector types, the MFMA wrappers
// with their register layouts, the LDS swizzle, and cross-half wave exchanges.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gfwa {

// Grouped-query layout: query head (b, h), flat index bh = b * H + h, reads the keys and values of
// head h / G of the B x (H / G) key/value heads; returns that head's flat index.  G = 1: bh itself.
__device__ __forceinline__ int kv_head_of(int bh, int H, int G) {
    return G == 1 ? bh : (bh / H) * (H / G) + (bh % H) / G;
}

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for the -inf initial row max of Alg. 2

// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] * B[16x32].
//   A: lane l holds row (l % 32), k = 8*(l/32) + 0..7
//   B: lane l holds column (l % 32), k = 8*(l/32) + 0..7
//   D: lane l, register v holds column (l % 32), row 8*(v/4) + 4*(l/32) + (v%4)
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row index inside a 32-row accumulator block held by register v of a lane in half h.
__device__ __forceinline__ constexpr int acc_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

// max / sum across the two 32-lane halves of a wave (lane l <-> lane l^32), result in both.
__device__ __forceinline__ float xhalf_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// LDS tile of ROWS x D bf16, row pitch D*2 bytes, 16-byte chunks XOR-swizzled so that both
//  (a) ds_read_b128 of 16 consecutive rows at one logical chunk, and
//  (b) ds_read_b64_tr_b16 of 4 consecutive rows x 4 consecutive chunks
// spread over all 64 banks.
template <int D>
__device__ __forceinline__ int swz_chunk(int row, int chunk);
template <>
__device__ __forceinline__ int swz_chunk<128>(int row, int chunk) {
    return chunk ^ (((row & 3) << 2) | ((row >> 2) & 3));
}
template <>
__device__ __forceinline__ int swz_chunk<64>(int row, int chunk) {
    // two rows share a 256-byte bank line; rows r and r+2 must differ in chunk bit 2
    return chunk ^ ((((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1));
}
// byte offset of (row, 16-byte chunk) inside a tile
template <int D>
__device__ __forceinline__ int tile_off(int row, int chunk) {
    return row * (D * 2) + swz_chunk<D>(row, chunk) * 16;
}

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// A-operand fragment of the TRANSPOSE of an LDS tile T[rows][D] for one MFMA k-chunk:
// lane (col = l%32 of 32-column block cb, half h) receives T[r0 + 4h + e][col], e = 0..3, and
// T[r0 + 8 + 4h + e][col] -- the row order in which a 32x32 accumulator block hands its rows
// to the next MFMA as the B operand.
template <int D>
__device__ __forceinline__ bf16x8 lds_read_tr_frag(const char* tile, int r0, int cb, int lane) {
    const int h = lane >> 5;
    const int i16 = lane & 15;
    const int row = r0 + 4 * h + (i16 >> 2);
    const int col = 32 * cb + 16 * ((lane & 31) >> 4) + 4 * (i16 & 3);  // element column
    const int chunk = col >> 3;
    const int sub = (col & 7) * 2;
    const char* p0 = tile + tile_off<D>(row, chunk) + sub;
    const char* p1 = tile + tile_off<D>(row + 8, chunk) + sub;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p0);
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p1);
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// A- or B-operand fragment straight from an LDS tile: lane (row = r0 + l%32, half h) receives
// T[row][16*kc + 8h + 0..7].
template <int D>
__device__ __forceinline__ bf16x8 lds_read_frag(const char* tile, int r0, int kc, int lane) {
    const int row = r0 + (lane & 31);
    const int chunk = 2 * kc + (lane >> 5);
    return *reinterpret_cast<const bf16x8*>(tile + tile_off<D>(row, chunk));
}


// Direct global->LDS loads: every active lane p fetches 16 (4) bytes from  sbase + voff  and the
// data lands at lds_base + 16*p (4*p); lds_base is wave-uniform and travels in M0, which is saved
// and restored because the compiler may keep its own value there.  Issued through inline assembly
// on purpose: their completion is tracked by hand with vmcnt waits in front of the workgroup
// barrier, whereas loads the compiler knows about make it wait for all of them before every LDS
// read, which undoes any prefetch.
__device__ __forceinline__ void dma16(const void* sbase, unsigned voff, const void* lds_base) {
    const unsigned lds_addr = (unsigned)(uintptr_t)lds_base;  // LDS pointers are 32-bit offsets
    unsigned saved;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
        : "=&s"(saved)
        : "s"(lds_addr), "v"(voff), "s"(sbase)
        : "memory");
}
// the same for data that is read once (non-temporal: first in line for eviction from the caches)
__device__ __forceinline__ void dma16_stream(const void* sbase, unsigned voff, const void* lds_base) {
    const unsigned lds_addr = (unsigned)(uintptr_t)lds_base;
    unsigned saved;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3 nt\n\ts_mov_b32 m0, %0"
        : "=&s"(saved)
        : "s"(lds_addr), "v"(voff), "s"(sbase)
        : "memory");
}
__device__ __forceinline__ void dma4(const void* sbase, unsigned voff, const void* lds_base) {
    const unsigned lds_addr = (unsigned)(uintptr_t)lds_base;
    unsigned saved;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, %3\n\ts_mov_b32 m0, %0"
        : "=&s"(saved)
        : "s"(lds_addr), "v"(voff), "s"(sbase)
        : "memory");
}
// A pointer that is the same in every lane, moved into scalar registers (the first lane's value).
__device__ __forceinline__ void* uniform_ptr(void* p) {
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a), hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
    return reinterpret_cast<void*>(((uint64_t)hi << 32) | lo);
}
// One 16-byte non-temporal global store per lane to  sbase + voff + IMM, issued exactly here in program order (inline
// assembly with a memory clobber): for code that counts its outstanding vector-memory operations by hand.  sbase
// must be the same in every lane.  (Scalar base plus a 32-bit offset per lane: one address register instead of two.  In a
// loop of nothing but MFMAs and such stores this form costs the wave 30 ns per store against 150 ns for the form with
// a 64-bit address per lane; in the kernels here the two measure the same.)
template <int IMM = 0>
__device__ __forceinline__ void stream_store16(void* sbase, unsigned voff, bf16x8 v) {
    asm volatile("global_store_dwordx4 %0, %1, %2 offset:%3 nt" ::"v"(voff), "v"(v), "s"(sbase), "n"(IMM) : "memory");
}
// s_waitcnt that waits only for vmcnt <= n (gfx9 encoding: expcnt and lgkmcnt fields left at max)
constexpr int vmcnt_only(int n) { return 0x0f70 | (n & 0xf) | ((n >> 4) << 14); }

// Empty volatile asm that consumes and re-defines a register: keeps a loop-invariant value in a
// register instead of letting the compiler recompute it, and orders computations against
// scheduling fences.
#define GFWA_PIN(x) asm volatile("" : "+v"(x))

// Hardware spreads consecutive workgroup ids round-robin over the 8 XCDs (each with its own L2).
// Map the launch index so that every XCD owns one contiguous range of logical tiles.
__device__ __forceinline__ int xcd_remap(int pid, int total) {
    constexpr int kXcd = 8;
    const int base = total / kXcd, rem = total % kXcd;
    const int x = pid % kXcd, idx = pid / kXcd;
    return x * base + (x < rem ? x : rem) + idx;
}

}  // namespace gfwa
