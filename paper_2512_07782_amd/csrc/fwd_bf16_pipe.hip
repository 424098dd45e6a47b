// GatedFWA fused forward, software-pipelined kernel for d = 128 on gfx950 (paper Alg. 2).
//
// A workgroup of 4 waves owns 256 consecutive queries of one (b,h), 64 per wave.  Each wave runs
// alone on its SIMD with the full 512-register budget and owns two 32-query blocks A and B, so that
// every K and V
// fragment read from LDS feeds two MFMAs (the transposing LDS read V needs runs at a quarter of the
// plain LDS rate and would otherwise bound the loop).  K/V arrive in 32-key blocks through 4-slot
// LDS rings filled by direct global->LDS loads three iterations ahead (no staging registers, no LDS
// stores).  One loop iteration n keeps the matrix cores and the vector ALUs busy from the same wave:
//
//   region 1  MFMA  O_A += V(n)^T P_A(n);  S_A(n+1) = g(n+1) + K(n+1) Q_A^T
//             VALU  online softmax of S_B(n)   -> P_B(n)
//   region 2  MFMA  O_B += V(n)^T P_B(n);  S_B(n+1) = g(n+1) + K(n+1) Q_B^T
//             VALU  online softmax of S_A(n+1) -> P_A(n+1)
//
// On this hardware an MFMA keeps the vector ALU of its SIMD busy for half of its own duration, so
// the loop is bound by  16 cycles x #MFMA + 4 cycles x #VALU  rather than by the matrix pipe alone.
// The VALU count per 32x32 block is kept small:
//   * the gate bias rides in the MFMA accumulator: S is initialised with g_i = (c_i - c_base)/scale
//     straight from LDS, so  p = exp2(S * sl - m * sl)  is one fused multiply-add plus one exp2
//     (sl = scale * log2 e);
//   * the row sums take 8 packed dot-products (v_dot2c_f32_bf16 with a pair of ones) on the bf16
//     probabilities instead of 16 adds, so l is the sum of exactly the values that enter the PV
//     product;
//   * every LDS and global address is loop invariant: per-lane offsets are computed once, ring slots
//     are compile-time immediates (the loop is unrolled by the ring size), the global side advances
//     a scalar base;
//   * the running max is raised only when it grows by more than 2^8; O and l are rescaled only then.
// As in the plain kernel, products are formed transposed (a lane owns one query) and P stays in
// registers as the B operand of the PV product.
#include "gfwa_device.h"
#include "gfwa_internal.h"

namespace gfwa {

constexpr int kPipeWaves = 4;
constexpr int kPipeThreads = 64 * kPipeWaves;
constexpr int kKb = 32;           // keys per block
constexpr int kRing = 4;          // ring slots per operand; block b lives in slot (b - n0) % 4
constexpr int kPf = kRing - 1;    // prefetch distance in iterations
constexpr int kLoadsPerIter = 5;  // per wave: 2 K + 2 V + 1 c

template <int D>
struct PipeSmem {
    alignas(16) char k[kRing][kKb * D * 2];
    alignas(16) char v[kRing][kKb * D * 2];
    alignas(16) float craw[kRing][kKb];  // prefix c as loaded
    alignas(16) float g[2][kKb];         // (c - c_base) / scale
};

#define GFWA_FENCE() __builtin_amdgcn_sched_barrier(0)
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// Per-stream softmax state: running max m (raw units of S), nm = -m*sl, a = pending rescale factor
// of O, l = running row sum of this lane's half of the keys; mxa/mxb, d, x[], p[] are values in
// flight between the pieces below.
struct Stream {
    float m, nm, a, l;
    float mxa, mxb, d;
    float x[16], p[16];
};

// The online softmax of one 32x32 block is cut into pieces that are spread over the MFMA slots of
// a region such that no piece depends on a result produced in the same slot: with one wave per
// SIMD nothing else hides the latency of a dependent VALU chain (notably the exp2).
//   max<0..2>  row max, two independent partial maxima, then the exchange between wave halves
//   upd<0..1>  running-max update (raise m only when the block max exceeds it by more than thr)
//   X<C>       x = S*sl - m*sl                 for entries 2C, 2C+1
//   E<C>       p = exp2(x)
//   P<C>       pack to bf16 into the B-operand fragment (k-chunk C/4, entries 2(C%4), 2(C%4)+1)
//              and add the packed pair to the row sum with one dot-product against (1, 1)
template <int PART>
__device__ __forceinline__ void sm_max(Stream& st, const f32x16& s) {
    if constexpr (PART == 0) {
        st.mxa = fmaxf(fmaxf(s[0], s[1]), s[2]);
        st.mxb = fmaxf(fmaxf(s[8], s[9]), s[10]);
        st.mxa = fmaxf(fmaxf(st.mxa, s[3]), s[4]);
        st.mxb = fmaxf(fmaxf(st.mxb, s[11]), s[12]);
    } else if constexpr (PART == 1) {
        st.mxa = fmaxf(fmaxf(st.mxa, s[5]), s[6]);
        st.mxb = fmaxf(fmaxf(st.mxb, s[13]), s[14]);
        st.mxa = fmaxf(st.mxa, s[7]);
        st.mxb = fmaxf(st.mxb, s[15]);
    } else {
        st.mxa = xhalf_max(fmaxf(st.mxa, st.mxb));
    }
    GFWA_PIN(st.mxa);
    GFWA_PIN(st.mxb);
}
template <int PART>
__device__ __forceinline__ void sm_upd(Stream& st, float sl, float thr) {
    if constexpr (PART == 0) {
        const bool grow = st.mxa > st.m + thr;
        const float mnew = grow ? st.mxa : st.m;
        st.d = (st.m - mnew) * sl;
        st.m = mnew;
        st.nm = -mnew * sl;
        GFWA_PIN(st.d);
        GFWA_PIN(st.nm);
        GFWA_PIN(st.m);
    } else {
        st.a = fast_exp2(st.d);
        GFWA_PIN(st.a);
    }
}
template <int C>
__device__ __forceinline__ void sm_X(Stream& st, const f32x16& s, float sl) {
    GFWA_PIN(st.nm);
    st.x[2 * C] = fmaf(s[2 * C], sl, st.nm);
    st.x[2 * C + 1] = fmaf(s[2 * C + 1], sl, st.nm);
    GFWA_PIN(st.x[2 * C]);
    GFWA_PIN(st.x[2 * C + 1]);
}
template <int C>
__device__ __forceinline__ void sm_E(Stream& st) {
    GFWA_PIN(st.x[2 * C]);
    st.p[2 * C] = fast_exp2(st.x[2 * C]);
    st.p[2 * C + 1] = fast_exp2(st.x[2 * C + 1]);
    GFWA_PIN(st.p[2 * C]);
    GFWA_PIN(st.p[2 * C + 1]);
}
template <int C>
__device__ __forceinline__ void sm_P(Stream& st, bf16x8 (&pf)[2]) {
    GFWA_PIN(st.p[2 * C]);
    if constexpr (C == 0) st.l *= st.a;  // the pending rescale of the row sum
    f32x2 pr = {st.p[2 * C], st.p[2 * C + 1]};
    bf16x2 pb = __builtin_convertvector(pr, bf16x2);
    const bf16x2 one2 = {(bf16_t)1.0f, (bf16_t)1.0f};
    st.l = __builtin_amdgcn_fdot2_f32_bf16(pb, one2, st.l, false);
    GFWA_PIN(st.l);
    pf[C >> 2][2 * (C & 3)] = pb[0];
    pf[C >> 2][2 * (C & 3) + 1] = pb[1];
    if constexpr ((C & 3) == 3) {
        u32x4 bits = __builtin_bit_cast(u32x4, pf[C >> 2]);
        GFWA_PIN(bits);
        pf[C >> 2] = __builtin_bit_cast(bf16x8, bits);
    } else {
        unsigned bits = __builtin_bit_cast(unsigned, pb);
        GFWA_PIN(bits);
        pb = __builtin_bit_cast(bf16x2, bits);
        pf[C >> 2][2 * (C & 3)] = pb[0];
        pf[C >> 2][2 * (C & 3) + 1] = pb[1];
    }
}
// The pieces of one block in the order of the 16 slots of a region.
template <int SLOT>
__device__ __forceinline__ void sm_slot(Stream& st, const f32x16& s, bf16x8 (&pf)[2], float sl, float thr) {
    if constexpr (SLOT == 0) sm_max<0>(st, s);
    if constexpr (SLOT == 1) sm_max<1>(st, s);
    if constexpr (SLOT == 2) sm_max<2>(st, s);
    if constexpr (SLOT == 3) sm_upd<0>(st, sl, thr);
    if constexpr (SLOT == 4) { sm_upd<1>(st, sl, thr); sm_X<0>(st, s, sl); sm_X<1>(st, s, sl); }
    if constexpr (SLOT == 5) { sm_E<0>(st); sm_X<2>(st, s, sl); }
    if constexpr (SLOT >= 6 && SLOT <= 10) { sm_P<SLOT - 6>(st, pf); sm_E<SLOT - 5>(st); sm_X<SLOT - 3>(st, s, sl); }
    if constexpr (SLOT == 11) { sm_P<5>(st, pf); sm_E<6>(st); }
    if constexpr (SLOT == 12) { sm_P<6>(st, pf); sm_E<7>(st); }
    if constexpr (SLOT == 13) sm_P<7>(st, pf);
}

template <int D>
__global__ __launch_bounds__(kPipeThreads, 1) void fwd_bf16_pipe_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const float* __restrict__ c, bf16_t* __restrict__ O, float* __restrict__ L, int N, int w,
    float scale_log2, int num_qtiles, int total_tiles) {
    static_assert(D == 128, "row pitch of 256 bytes assumed");
    constexpr int BR = 64 * kPipeWaves;
    constexpr int KC = D / 16, DB = D / 32;
    constexpr int kBlockBytes = kKb * D * 2;
    __shared__ PipeSmem<D> sm;

    const int tile = xcd_remap(blockIdx.x, total_tiles);
    const int bh = tile / num_qtiles;
    const int q0 = (tile % num_qtiles) * BR;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, lq = lane & 31;
    const float sl = scale_log2;
    const float inv_scale = kLog2e / scale_log2;
    const float thr = 8.0f / scale_log2;

    const size_t head_off = (size_t)bh * N * D;
    const char* Kh = reinterpret_cast<const char*>(K + head_off);
    const char* Vh = reinterpret_cast<const char*>(V + head_off);
    const float* ch = c + (size_t)bh * N;
    const float cbase = ch[q0];

    const int qa0 = q0 + 64 * wv;  // first query of block A; block B starts 32 later
    const int tA = qa0 + lq, tB = qa0 + 32 + lq;

    // key blocks this workgroup visits: n0 .. n1 (32 keys each); blocks below nfull have all rows < N
    const int n0 = max(0, q0 - w + 1) / kKb;
    const int n1 = (min(N, q0 + BR) - 1) / kKb;
    const int nfull = N / kKb;

    // ---- loop-invariant per-lane addressing
    // global->LDS: wave wv fills rows 8wv..8wv+7 of a block with two loads (g = 0, 1) of 4 rows;
    // lane p writes row p/16 of its group at physical chunk p%16 and therefore fetches the logical
    // chunk the swizzle maps there (the swizzle is an involution).
    unsigned dma_off[2];
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        const int row = 8 * wv + 4 * g + (lane >> 4);
        dma_off[g] = (unsigned)(row * (D * 2) + swz_chunk<D>(row, lane & 15) * 16);
        GFWA_PIN(dma_off[g]);
    }
    unsigned dma_coff = (unsigned)(lane * 4);
    GFWA_PIN(dma_coff);
    // LDS fragment reads (byte offsets inside a block slot)
    unsigned k_off[KC];
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
        k_off[kc] = (unsigned)tile_off<D>(lq, 2 * kc + h);
        GFWA_PIN(k_off[kc]);
    }
    // V^T fragment i (k-chunk i/4, dd block i%4) takes two transposing reads, rows r and r+8; the
    // swizzle of row r+8 differs from that of row r by a flip of chunk bit 1 (32 bytes)
    unsigned v_off[2 * DB];
#pragma unroll
    for (int i = 0; i < 2 * DB; ++i) {
        const int i16 = lane & 15;
        const int row = 16 * (i >> 2) + 4 * h + (i16 >> 2);
        const int col = 32 * (i & 3) + 16 * ((lane & 31) >> 4) + 4 * (i16 & 3);
        v_off[i] = (unsigned)(tile_off<D>(row, col >> 3) + (col & 7) * 2);
        GFWA_PIN(v_off[i]);
    }
    unsigned g_off = (unsigned)(16 * h);
    GFWA_PIN(g_off);

    // One block load = K rows or V rows (2 loads per wave, G = 0, 1) or the 32 prefix values (lanes
    // 0..31 of every wave load the same words).  Blocks at or past nfull take the clamped path.
    auto load_kv_rows = [&](const char* base, int b, char* slot, int g) {
        char* lds = slot + (8 * wv + 4 * g) * (D * 2);
        if (b < nfull) {
            dma16(base + (size_t)b * kBlockBytes, dma_off[g], lds);
        } else {
            const int row = 8 * wv + 4 * g + (lane >> 4);
            const int key = min(b * kKb + row, N - 1);
            const unsigned off = (unsigned)key * (unsigned)(D * 2) + (unsigned)(swz_chunk<D>(row, lane & 15) * 16);
            dma16(base, off, lds);
        }
    };
    auto load_kv_block = [&](const char* base, int b, char* slot) {
        load_kv_rows(base, b, slot, 0);
        load_kv_rows(base, b, slot, 1);
    };
    auto load_c_block = [&](int b, float* slot) {
        if (lane < kKb) {
            if (b < nfull) {
                dma4(ch + (size_t)b * kKb, dma_coff, slot);
            } else {
                const int key = min(b * kKb + lane, N - 1);
                dma4(ch, (unsigned)key * 4u, slot);
            }
        }
    };

    // Ring schedule.  Block b is read from LDS in iteration b-1 (K and V fragments, g(b)) and b-2
    // (c, turned into g(b)); iteration n issues the loads of K(n+4), V(n+4) and c(n+5).
    // Here: what iterations before n0 would have issued.
#pragma unroll
    for (int i = 0; i <= kPf; ++i) {
        load_kv_block(Kh, n0 + i, sm.k[i]);
        load_kv_block(Vh, n0 + i, sm.v[i]);
        load_c_block(n0 + i, sm.craw[i]);
    }

    // Q^T fragments of both query blocks (B operands), resident
    bf16x8 qfA[KC], qfB[KC];
    {
        const bf16_t* qa = Q + head_off + (size_t)min(tA, N - 1) * D + 8 * h;
        const bf16_t* qb = Q + head_off + (size_t)min(tB, N - 1) * D + 8 * h;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            qfA[kc] = *reinterpret_cast<const bf16x8*>(qa + 16 * kc);
            qfB[kc] = *reinterpret_cast<const bf16x8*>(qb + 16 * kc);
        }
    }
    const float cqA = ch[min(tA, N - 1)] - cbase, cqB = ch[min(tB, N - 1)] - cbase;

    f32x16 oA[DB], oB[DB];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            oA[db][v] = 0.f;
            oB[db][v] = 0.f;
        }
    }

    __builtin_amdgcn_s_waitcnt(0);  // everything issued so far has landed
    __syncthreads();
    if (tid < kKb) {
        sm.g[0][tid] = (sm.craw[0][tid] - cbase) * inv_scale;
        sm.g[1][tid] = (sm.craw[1][tid] - cbase) * inv_scale;
    }
    __syncthreads();
    load_c_block(n0 + 4, sm.craw[0]);  // slot 0 is free again

    // accumulator <- gate terms of a block: rows 8g + 4h + 0..3 of the 32-key block
    auto init_gate = [&](f32x16& acc, int slot) {
        const char* gp = reinterpret_cast<const char*>(sm.g[slot]) + g_off;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 c4 = *reinterpret_cast<const f32x4*>(gp + 32 * g);
            acc[4 * g] = c4[0];
            acc[4 * g + 1] = c4[1];
            acc[4 * g + 2] = c4[2];
            acc[4 * g + 3] = c4[3];
        }
    };
    auto read_k = [&](const char* slot, int kc) { return *reinterpret_cast<const bf16x8*>(slot + k_off[kc]); };
    auto read_v = [&](const char* slot, int i) {
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(slot + v_off[i]));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(slot + ((v_off[i] ^ 32u) + 8u * (D * 2))));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto mask_block = [&](f32x16& s, int n, int t) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = n * kKb + acc_row(v, h);
            const bool keep = (i <= t) && (i > t - w);
            s[v] = keep ? s[v] : -INFINITY;
        }
    };
    auto rescale = [&](f32x16 (&o)[DB], float a) {
        if (__builtin_amdgcn_ballot_w64(a != 1.0f) != 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
                for (int db = 0; db < DB; ++db) o[db][v] *= a;
        }
    };

    f32x16 sA, sB;       // S_A(n+1) / S_B(n): produced by one region, consumed by the next
    bf16x8 pfA[2], pfB[2];
    bf16x8 kfr[KC];      // K(n+1) fragments, shared by both query blocks
    bf16x8 vfr[2 * DB];  // V(n) fragments, shared by both query blocks
    Stream stA, stB;
    stA.m = stB.m = kNegBig;
    stA.a = stB.a = 1.0f;
    stA.l = stB.l = 0.f;

    // blocks [lo, hi] lie wholly inside the window of all 32 queries of a stream that starts at q
    auto full_lo = [&](int q) { return ((q + 31 - w) >> 5) + 1; };  // smallest b with 32 b > q + 31 - w
    auto full_hi = [&](int q) { return (q >> 5) - 1; };             // largest b with 32 b + 31 <= q
    const int fA_lo = full_lo(qa0), fA_hi = full_hi(qa0);
    const int fB_lo = full_lo(qa0 + 32), fB_hi = full_hi(qa0 + 32);

    // ---- pipeline fill: S_A(n0), S_B(n0), softmax A(n0), V(n0) fragments
    init_gate(sA, 0);
    init_gate(sB, 0);
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
        const bf16x8 kf = read_k(sm.k[0], kc);
        sA = mfma32(kf, qfA[kc], sA);
        sB = mfma32(kf, qfB[kc], sB);
    }
    mask_block(sA, n0, tA);
    sm_slot<0>(stA, sA, pfA, sl, thr);
    sm_slot<1>(stA, sA, pfA, sl, thr);
    sm_slot<2>(stA, sA, pfA, sl, thr);
    sm_slot<3>(stA, sA, pfA, sl, thr);
    sm_slot<4>(stA, sA, pfA, sl, thr);
    sm_slot<5>(stA, sA, pfA, sl, thr);
    sm_slot<6>(stA, sA, pfA, sl, thr);
    sm_slot<7>(stA, sA, pfA, sl, thr);
    sm_slot<8>(stA, sA, pfA, sl, thr);
    sm_slot<9>(stA, sA, pfA, sl, thr);
    sm_slot<10>(stA, sA, pfA, sl, thr);
    sm_slot<11>(stA, sA, pfA, sl, thr);
    sm_slot<12>(stA, sA, pfA, sl, thr);
    sm_slot<13>(stA, sA, pfA, sl, thr);
    stA.a = 1.0f;  // O_A is still zero
#pragma unroll
    for (int i = 0; i < 2 * DB; ++i) vfr[i] = read_v(sm.v[0], i);

    // One iteration n, J = (n - n0) % 4.  Each region is 16 MFMA slots.
    //   region 1, slots 0-7:  O_A += V(n)^T P_A(n)               LDS: K(n+1) fragments, g(n+1) -> S_A
    //             slots 8-15: S_A(n+1) = g(n+1) + K(n+1) Q_A^T   global->LDS: this wave's share of
    //                         K(n+4), V(n+4), c(n+5), one load per slot;  VALU: softmax B(n) -> P_B(n)
    //   region 2, slots 0-7:  O_B += V(n)^T P_B(n)               LDS: g(n+1) -> S_B
    //             slots 8-15: S_B(n+1) = g(n+1) + K(n+1) Q_B^T   LDS: V(n+1) fragments, every other slot
    //                                                            VALU: softmax A(n+1) -> P_A(n+1)
    // A scheduling fence after every MFMA slot keeps this interleaving in the instruction stream.
#define GFWA_SLOT_END() GFWA_FENCE()
#define GFWA_PIPE_ITER(J)                                                                                       \
    {                                                                                                           \
        const bool loads = (n + kPf + 1 <= n1);                                                                 \
        if (loads) {                                                                                            \
            __builtin_amdgcn_s_waitcnt(vmcnt_only((kPf - 1) * kLoadsPerIter));                                  \
        } else {                                                                                                \
            __builtin_amdgcn_s_waitcnt(vmcnt_only(0));                                                          \
        }                                                                                                       \
        __syncthreads();                                                                                        \
        if (tid < kKb) sm.g[(J) & 1][tid] = (sm.craw[((J) + 2) & 3][tid] - cbase) * inv_scale;                  \
        rescale(oA, stA.a);                                                                                     \
        if (!(n >= fB_lo && n <= fB_hi)) mask_block(sB, n, tB);                                                 \
        const char* kt = sm.k[((J) + 1) & 3];                                                                   \
        const char* vn = sm.v[((J) + 1) & 3];                                                                   \
        GFWA_FENCE();                                                                                           \
        /* ---------------- region 1 ---------------- */                                                        \
        kfr[0] = read_k(kt, 0);                                                                                 \
        if (loads) load_kv_rows(Kh, n + 4, sm.k[(J)], 0);                                                       \
        oA[0] = mfma32(vfr[0], pfA[0], oA[0]);                                                                  \
        sm_slot<0>(stB, sB, pfB, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        kfr[1] = read_k(kt, 1);                                                                                 \
        if (loads) load_kv_rows(Kh, n + 4, sm.k[(J)], 1);                                                       \
        oA[1] = mfma32(vfr[1], pfA[0], oA[1]);                                                                  \
        sm_slot<1>(stB, sB, pfB, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        kfr[2] = read_k(kt, 2);                                                                                 \
        if (loads) load_kv_rows(Vh, n + 4, sm.v[(J)], 0);                                                       \
        oA[2] = mfma32(vfr[2], pfA[0], oA[2]);                                                                  \
        sm_slot<2>(stB, sB, pfB, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        kfr[3] = read_k(kt, 3);                                                                                 \
        if (loads) load_kv_rows(Vh, n + 4, sm.v[(J)], 1);                                                       \
        oA[3] = mfma32(vfr[3], pfA[0], oA[3]);                                                                  \
        sm_slot<3>(stB, sB, pfB, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        kfr[4] = read_k(kt, 4);                                                                                 \
        if (loads) load_c_block(n + 5, sm.craw[((J) + 1) & 3]);                                                 \
        oA[0] = mfma32(vfr[4], pfA[1], oA[0]);                                                                  \
        sm_slot<4>(stB, sB, pfB, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        kfr[5] = read_k(kt, 5);                                                                                 \
        oA[1] = mfma32(vfr[5], pfA[1], oA[1]);                                                                  \
        sm_slot<5>(stB, sB, pfB, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        kfr[6] = read_k(kt, 6);                                                                                 \
        oA[2] = mfma32(vfr[6], pfA[1], oA[2]);                                                                  \
        sm_slot<6>(stB, sB, pfB, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        kfr[7] = read_k(kt, 7);                                                                                 \
        init_gate(sA, ((J) + 1) & 1);                                                                           \
        oA[3] = mfma32(vfr[7], pfA[1], oA[3]);                                                                  \
        sm_slot<7>(stB, sB, pfB, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        sA = mfma32(kfr[0], qfA[0], sA);                                                                        \
        sm_slot<8>(stB, sB, pfB, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        sA = mfma32(kfr[1], qfA[1], sA);                                                                        \
        sm_slot<9>(stB, sB, pfB, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        sA = mfma32(kfr[2], qfA[2], sA);                                                                        \
        sm_slot<10>(stB, sB, pfB, sl, thr);                                                                     \
        GFWA_SLOT_END();                                                                                        \
        sA = mfma32(kfr[3], qfA[3], sA);                                                                        \
        sm_slot<11>(stB, sB, pfB, sl, thr);                                                                     \
        GFWA_SLOT_END();                                                                                        \
        sA = mfma32(kfr[4], qfA[4], sA);                                                                        \
        sm_slot<12>(stB, sB, pfB, sl, thr);                                                                     \
        GFWA_SLOT_END();                                                                                        \
        sA = mfma32(kfr[5], qfA[5], sA);                                                                        \
        sm_slot<13>(stB, sB, pfB, sl, thr);                                                                     \
        GFWA_SLOT_END();                                                                                        \
        sA = mfma32(kfr[6], qfA[6], sA);                                                                        \
        GFWA_SLOT_END();                                                                                        \
        sA = mfma32(kfr[7], qfA[7], sA);                                                                        \
        GFWA_SLOT_END();                                                                                        \
        rescale(oB, stB.a);                                                                                     \
        if (!(n + 1 >= fA_lo && n + 1 <= fA_hi)) mask_block(sA, n + 1, tA);                                     \
        GFWA_FENCE();                                                                                           \
        /* ---------------- region 2 ---------------- */                                                        \
        init_gate(sB, ((J) + 1) & 1);                                                                           \
        oB[0] = mfma32(vfr[0], pfB[0], oB[0]);                                                                  \
        sm_slot<0>(stA, sA, pfA, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        oB[1] = mfma32(vfr[1], pfB[0], oB[1]);                                                                  \
        sm_slot<1>(stA, sA, pfA, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        oB[2] = mfma32(vfr[2], pfB[0], oB[2]);                                                                  \
        sm_slot<2>(stA, sA, pfA, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        oB[3] = mfma32(vfr[3], pfB[0], oB[3]);                                                                  \
        sm_slot<3>(stA, sA, pfA, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        oB[0] = mfma32(vfr[4], pfB[1], oB[0]);                                                                  \
        vfr[0] = read_v(vn, 0);                                                                                 \
        sm_slot<4>(stA, sA, pfA, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        oB[1] = mfma32(vfr[5], pfB[1], oB[1]);                                                                  \
        sm_slot<5>(stA, sA, pfA, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        oB[2] = mfma32(vfr[6], pfB[1], oB[2]);                                                                  \
        vfr[1] = read_v(vn, 1);                                                                                 \
        sm_slot<6>(stA, sA, pfA, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        oB[3] = mfma32(vfr[7], pfB[1], oB[3]);                                                                  \
        sm_slot<7>(stA, sA, pfA, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        vfr[2] = read_v(vn, 2);                                                                                 \
        sB = mfma32(kfr[0], qfB[0], sB);                                                                        \
        sm_slot<8>(stA, sA, pfA, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        sB = mfma32(kfr[1], qfB[1], sB);                                                                        \
        sm_slot<9>(stA, sA, pfA, sl, thr);                                                                      \
        GFWA_SLOT_END();                                                                                        \
        vfr[3] = read_v(vn, 3);                                                                                 \
        sB = mfma32(kfr[2], qfB[2], sB);                                                                        \
        sm_slot<10>(stA, sA, pfA, sl, thr);                                                                     \
        GFWA_SLOT_END();                                                                                        \
        vfr[4] = read_v(vn, 4);                                                                                 \
        sB = mfma32(kfr[3], qfB[3], sB);                                                                        \
        sm_slot<11>(stA, sA, pfA, sl, thr);                                                                     \
        GFWA_SLOT_END();                                                                                        \
        vfr[5] = read_v(vn, 5);                                                                                 \
        sB = mfma32(kfr[4], qfB[4], sB);                                                                        \
        sm_slot<12>(stA, sA, pfA, sl, thr);                                                                     \
        GFWA_SLOT_END();                                                                                        \
        vfr[6] = read_v(vn, 6);                                                                                 \
        sB = mfma32(kfr[5], qfB[5], sB);                                                                        \
        sm_slot<13>(stA, sA, pfA, sl, thr);                                                                     \
        GFWA_SLOT_END();                                                                                        \
        vfr[7] = read_v(vn, 7);                                                                                 \
        sB = mfma32(kfr[6], qfB[6], sB);                                                                        \
        GFWA_SLOT_END();                                                                                        \
        sB = mfma32(kfr[7], qfB[7], sB);                                                                        \
        GFWA_SLOT_END();                                                                                        \
    }

    // The S computed for block n1+1 in the last iteration reads stale ring slots; every entry of it is
    // masked (the block lies beyond the diagonal), so softmax A(n1+1) leaves the state untouched.
    for (int nb = n0; nb <= n1; nb += 4) {
        int n = nb;
        GFWA_PIPE_ITER(0)
        n = nb + 1;
        if (n <= n1) GFWA_PIPE_ITER(1)
        n = nb + 2;
        if (n <= n1) GFWA_PIPE_ITER(2)
        n = nb + 3;
        if (n <= n1) GFWA_PIPE_ITER(3)
    }
#undef GFWA_PIPE_ITER
#undef GFWA_SLOT_END

    // ---- epilogue: O = O^T / l, L = ln2 * (m*sl + log2 l) - (c_t - c_base)
    auto finish = [&](f32x16 (&o)[DB], float lhalf, float m, float cq, int t) {
        const float lt = xhalf_sum(lhalf);  // the two halves of the wave hold complementary keys
        if (t >= N) return;
        const float inv = 1.0f / lt;
        bf16_t* orow = O + head_off + (size_t)t * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 o4 = {o[db][4 * g] * inv, o[db][4 * g + 1] * inv, o[db][4 * g + 2] * inv,
                            o[db][4 * g + 3] * inv};
                *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * g + 4 * h) = __builtin_convertvector(o4, bf16x4);
            }
        if (h == 0) L[(size_t)bh * N + t] = (m * sl + fast_log2(lt)) * kLn2 - cq;
    };
    finish(oA, stA.l, stA.m, cqA, tA);
    finish(oB, stB.l, stB.m, cqB, tB);
}

hipError_t forward_bf16_pipe(const void* Q, const void* K, const void* V, const float* c, void* O, float* L,
                             int B, int H, int N, int w, float scale, int occupancy, hipStream_t s) {
    (void)occupancy;
    constexpr int BR = 64 * kPipeWaves;
    const int num_qtiles = (N + BR - 1) / BR;
    const int total = B * H * num_qtiles;
    ProfScope prof(kKernForward, s);
    hipLaunchKernelGGL((fwd_bf16_pipe_kernel<128>), dim3(total), dim3(kPipeThreads), 0, s, (const bf16_t*)Q,
                       (const bf16_t*)K, (const bf16_t*)V, c, (bf16_t*)O, L, N, w, scale * kLog2e, num_qtiles,
                       total);
    return hipGetLastError();
}

}  // namespace gfwa
