// GatedFWA fused forward, software-pipelined kernel for d = 128 on gfx950 (paper Alg. 2).
//
// A workgroup of 4 waves owns 128 consecutive queries of one (b,h), 32 per wave.  K/V arrive in
// 32-key blocks through LDS rings filled by direct global->LDS loads kPf iterations ahead (no
// staging registers, no LDS stores).  One loop iteration n gives the matrix cores and the vector
// ALUs independent work from the same wave:
//
//     MFMA   O += V(n-1)^T P(n-1)   then   S(n+1) = g(n+1) + K(n+1) Q^T
//     VALU   online softmax of S(n) -> P(n)
//
// As in the plain kernel, products are formed transposed (a lane owns one query), P stays in
// registers as the B operand of the PV product, the running max is raised only when it grows by
// more than 2^8 and O is rescaled only then.
//
// The gate bias rides in the MFMA accumulator: S is initialised with g_i = (c_i - c_base) / scale
// straight from LDS before the K Q^T chain, so S = q.k + g_i and the probability is a single
// fused multiply-add plus exp2:  p = exp2(S * (scale*log2e) - m * (scale*log2e)).
#include "gfwa_device.h"
#include "gfwa_internal.h"

namespace gfwa {

constexpr int kPipeThreads = 256;
constexpr int kPipeWaves = 4;
constexpr int kPf = 3;            // prefetch distance in iterations
constexpr int kRing = kPf + 1;    // ring slots per operand
constexpr int kKb = 32;           // keys per block
constexpr int kLoadsPerIter = 5;  // per wave: 2 K + 2 V + 1 c

template <int D>
struct PipeSmem {
    alignas(16) char k[kRing][kKb * D * 2];
    alignas(16) char v[kRing][kKb * D * 2];
    alignas(16) float craw[kRing + 1][kKb];  // prefix c as loaded
    alignas(16) float g[2][kKb];         // (c - c_base) / scale
};

// Direct global->LDS load: every active lane p fetches `bytes` from its own global address and the
// data lands at lds_base + bytes*p (lds_base is wave-uniform and travels in M0).  Issued through
// inline assembly on purpose: the completion of these loads is tracked by hand with vmcnt waits in
// front of the workgroup barrier, whereas loads the compiler knows about would make it wait for all
// of them before every LDS read, which would undo the prefetch.
// M0 is saved and restored around the load because the compiler may keep its own value there.
__device__ __forceinline__ void dma16(const void* gptr, const void* lds_base) {
    const unsigned lds_addr = (unsigned)(uintptr_t)lds_base;  // LDS pointers are 32-bit offsets
    unsigned saved;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
        : "=&s"(saved)
        : "s"(lds_addr), "v"(gptr)
        : "memory");
}
__device__ __forceinline__ void dma4(const void* gptr, const void* lds_base) {
    const unsigned lds_addr = (unsigned)(uintptr_t)lds_base;
    unsigned saved;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, off\n\ts_mov_b32 m0, %0"
        : "=&s"(saved)
        : "s"(lds_addr), "v"(gptr)
        : "memory");
}

// The 4 waves load one 32-row block (row pitch 256 bytes) into a swizzled LDS slot, 8 rows per wave.
// Lane p of a load writes 16 bytes at slot + group*1024 + 16*p, i.e. row p/16 of the 4-row group,
// physical chunk p%16, so it fetches the logical chunk that the swizzle maps there.
template <int D>
__device__ __forceinline__ void load_block_rows(const bf16_t* __restrict__ base, int row0, int N, char* slot,
                                                int wv, int lane) {
    static_assert(D == 128, "row pitch of 256 bytes assumed");
    const int r4 = lane >> 4, pc = lane & 15;
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        const int row = 8 * wv + 4 * g + r4;
        const int lc = swz_chunk<D>(row, pc);  // the swizzle is an involution
        const int key = min(row0 + row, N - 1);
        const bf16_t* gp = base + (size_t)key * D + lc * 8;
        char* lp = slot + (8 * wv + 4 * g) * (D * 2);
        dma16(gp, lp);
    }
}

// Lanes 0..31 of every wave load the same 32 prefix values (identical bytes land on the same LDS
// words); lane p writes slot[p], so the upper half of the wave must stay out.
__device__ __forceinline__ void load_c_block(const float* __restrict__ ch, int key0, int N, float* slot, int lane) {
    const int key = min(key0 + lane, N - 1);
    if (lane < kKb) dma4(ch + key, slot);
}

// s_waitcnt that waits only for vmcnt <= n (gfx9 encoding: expcnt and lgkmcnt fields left at max)
constexpr int vmcnt_only(int n) { return 0x0f70 | (n & 0xf) | ((n >> 4) << 14); }


// The online softmax of one 32x32 block, cut into 16 pieces so that each piece can be issued in
// the shadow of one MFMA.  Pieces 0-2: row max; 3: running-max update; 4-11: p = exp2(S*sl - m*sl)
// and the row sum, two entries per piece; 12-15: pack P to bf16 as the B operand of the PV product.
struct SoftmaxState {
    float mx, nm, ls, a;
    float p[16];
};
// Empty volatile asm that consumes and re-defines a register: instruction selection keeps volatile
// asm in program order with the scheduling fences, so values routed through it are computed on
// this side of the next fence instead of drifting to their first use.
#define GFWA_PIN(x) asm volatile("" : "+v"(x))
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <int I>
__device__ __forceinline__ void softmax_piece(SoftmaxState& st, const f32x16& s, bf16x8 (&pf)[2], float sl,
                                              float thr, float& m, float& l) {
    if constexpr (I == 0) {
        st.mx = fmaxf(fmaxf(s[0], s[1]), s[2]);
        st.mx = fmaxf(fmaxf(st.mx, s[3]), s[4]);
        GFWA_PIN(st.mx);
    } else if constexpr (I == 1) {
        st.mx = fmaxf(fmaxf(st.mx, s[5]), s[6]);
        st.mx = fmaxf(fmaxf(st.mx, s[7]), s[8]);
        st.mx = fmaxf(fmaxf(st.mx, s[9]), s[10]);
        GFWA_PIN(st.mx);
    } else if constexpr (I == 2) {
        st.mx = fmaxf(fmaxf(st.mx, s[11]), s[12]);
        st.mx = fmaxf(fmaxf(st.mx, s[13]), s[14]);
        st.mx = fmaxf(st.mx, s[15]);
        GFWA_PIN(st.mx);
    } else if constexpr (I == 3) {
        const float mx = xhalf_max(st.mx);
        const bool grow = mx > m + thr;
        const float mnew = grow ? mx : m;
        st.a = fast_exp2((m - mnew) * sl);
        m = mnew;
        st.nm = -mnew * sl;
        st.ls = 0.f;
        GFWA_PIN(st.nm);
        GFWA_PIN(st.a);
        GFWA_PIN(m);
    } else if constexpr (I < 12) {
        constexpr int e = 2 * (I - 4);
        GFWA_PIN(st.nm);
        st.p[e] = fast_exp2(fmaf(s[e], sl, st.nm));
        st.p[e + 1] = fast_exp2(fmaf(s[e + 1], sl, st.nm));
        st.ls += st.p[e] + st.p[e + 1];
        GFWA_PIN(st.p[e]);
        GFWA_PIN(st.p[e + 1]);
        GFWA_PIN(st.ls);
    } else {
        constexpr int q = I - 12;  // one half fragment (4 entries) per piece
        constexpr int c2 = q >> 1, e0 = 4 * (q & 1);
        GFWA_PIN(st.p[8 * c2 + e0]);
        if constexpr (q == 0) {
            l = fmaf(l, st.a, st.ls);
            GFWA_PIN(l);
        }
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            f32x2 pr = {st.p[8 * c2 + e0 + e], st.p[8 * c2 + e0 + e + 1]};
            bf16x2 pb = __builtin_convertvector(pr, bf16x2);
            pf[c2][e0 + e] = pb[0];
            pf[c2][e0 + e + 1] = pb[1];
        }
        if constexpr ((q & 1) == 1) {
            u32x4 bits = __builtin_bit_cast(u32x4, pf[c2]);
            GFWA_PIN(bits);
            pf[c2] = __builtin_bit_cast(bf16x8, bits);
        }
    }
}

// A-operand fragment of V^T for MFMA number i (0..7) of the PV product: k-chunk i/4, dd block i%4
template <int D>
__device__ __forceinline__ bf16x8 read_v_frag(const char* vt, int i, int lane) {
    return lds_read_tr_frag<D>(vt, 16 * (i >> 2), i & 3, lane);
}

template <int D, int OCC>
__global__ __launch_bounds__(kPipeThreads, OCC) void fwd_bf16_pipe_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const float* __restrict__ c, bf16_t* __restrict__ O, float* __restrict__ L, int N, int w,
    float scale_log2, int num_qtiles, int total_tiles) {
    constexpr int BR = 32 * kPipeWaves;
    constexpr int KC = D / 16, DB = D / 32;
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
    const bf16_t* Kh = K + head_off;
    const bf16_t* Vh = V + head_off;
    const float* ch = c + (size_t)bh * N;
    const float cbase = ch[q0];

    const int qw0 = q0 + 32 * wv;  // first query of this wave
    const int t = qw0 + lq;

    // key blocks this workgroup visits: n0 .. n1 (32 keys each)
    const int n0 = max(0, q0 - w + 1) / kKb;
    const int n1 = (min(N, q0 + BR) - 1) / kKb;

    // Ring schedule.  Block b is read from LDS in iteration b-1 (K, for S(b)), b (V fragments for the
    // PV product of iteration b+1) and b-2 (c, turned into g(b)); iteration n issues the loads of
    // K(n+1+kPf), V(n+kPf) and c(n+2+kPf), all of which are first needed in iteration n+kPf.
    // Here: what iterations before n0 would have issued.
#pragma unroll
    for (int i = 0; i <= kPf + 1; ++i) {
        if (i <= kPf) load_block_rows<D>(Kh, (n0 + i) * kKb, N, sm.k[(n0 + i) % kRing], wv, lane);
        if (i <= kPf - 1) load_block_rows<D>(Vh, (n0 + i) * kKb, N, sm.v[(n0 + i) % kRing], wv, lane);
        load_c_block(ch, (n0 + i) * kKb, N, sm.craw[(n0 + i) % (kRing + 1)], lane);
    }

    // Q^T fragments (B operand), resident
    bf16x8 qf[KC];
    {
        const bf16_t* qp = Q + head_off + (size_t)min(t, N - 1) * D + 8 * h;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) qf[kc] = *reinterpret_cast<const bf16x8*>(qp + 16 * kc);
    }
    const float cq = ch[min(t, N - 1)] - cbase;

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m = kNegBig, l = 0.f;

    __builtin_amdgcn_s_waitcnt(0);  // everything issued so far has landed
    __syncthreads();
    if (tid < kKb) {
        sm.g[n0 & 1][tid] = (sm.craw[n0 % (kRing + 1)][tid] - cbase) * inv_scale;
        sm.g[(n0 + 1) & 1][tid] = (sm.craw[(n0 + 1) % (kRing + 1)][tid] - cbase) * inv_scale;
    }
    __syncthreads();

    // accumulator <- gate terms of a block: rows 8g + 4h + 0..3 of the 32-key block
    auto init_gate = [&](f32x16& acc, int slot) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 c4 = *reinterpret_cast<const f32x4*>(&sm.g[slot][8 * g + 4 * h]);
            acc[4 * g] = c4[0];
            acc[4 * g + 1] = c4[1];
            acc[4 * g + 2] = c4[2];
            acc[4 * g + 3] = c4[3];
        }
    };

    f32x16 sx, sy;     // S accumulators: one holds S(n) being consumed, the other S(n+1) being produced
    bf16x8 pf[2];      // P(n-1) as B operand, overwritten by P(n) at the end of the iteration
    bf16x8 kfr[KC];    // K(n+1) fragments, read during the PV half
    bf16x8 vfr[2 * DB];  // V(n-1) fragments, read during the previous iteration's QK half
    SoftmaxState st;
    st.a = 1.0f;

    // S(n0)
    init_gate(sx, n0 & 1);
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) sx = mfma32(lds_read_frag<D>(sm.k[n0 % kRing], 0, kc, lane), qf[kc], sx);
    pf[0] = pf[1] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 2 * DB; ++i) vfr[i] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};

    // iterations n in [nm_lo, nm_hi]: block n lies wholly inside the window of all 32 queries
    const int nm_lo = ((qw0 + 31 - w) >> 5) + 1;  // smallest n with 32 n > qw0 + 31 - w
    const int nm_hi = (qw0 >> 5) - 1;             // largest n with 32 n + 31 <= qw0

    // One iteration n.  SC holds S(n), SN receives S(n+1).
    //   half 1:  8 MFMAs  O += V(n-1)^T P(n-1)  (fragments already in vfr)
    //            LDS reads: K(n+1) fragments and g(n+1)       VALU: softmax pieces 0..7
    //   half 2:  8 MFMAs  S(n+1) = g(n+1) + K(n+1) Q^T
    //            LDS reads: V(n) fragments for the next iteration   VALU: softmax pieces 8..15
    // A scheduling fence after every MFMA keeps this interleaving in the instruction stream.
#define GFWA_PIPE_PIECE(I, SC) softmax_piece<I>(st, SC, pf, sl, thr, m, l);
#define GFWA_PIPE_ITER(SC, SN)                                                                                  \
    {                                                                                                           \
        const bool loads = (n + kPf <= n1);                                                                     \
        if (loads) {                                                                                            \
            __builtin_amdgcn_s_waitcnt(vmcnt_only((kPf - 1) * kLoadsPerIter));                                  \
        } else {                                                                                                \
            __builtin_amdgcn_s_waitcnt(vmcnt_only(0));                                                          \
        }                                                                                                       \
        __syncthreads();                                                                                        \
        if (loads) {                                                                                            \
            load_block_rows<D>(Kh, (n + 1 + kPf) * kKb, N, sm.k[(n + 1 + kPf) % kRing], wv, lane);              \
            load_block_rows<D>(Vh, (n + kPf) * kKb, N, sm.v[(n + kPf) % kRing], wv, lane);                      \
            load_c_block(ch, (n + 2 + kPf) * kKb, N, sm.craw[(n + 2 + kPf) % (kRing + 1)], lane);               \
        }                                                                                                       \
        if (tid < kKb) sm.g[n & 1][tid] = (sm.craw[(n + 2) % (kRing + 1)][tid] - cbase) * inv_scale;            \
        /* rescale of O decided by softmax(n-1) */                                                              \
        if (__builtin_amdgcn_ballot_w64(st.a != 1.0f) != 0) {                                                   \
            _Pragma("unroll") for (int db = 0; db < DB; ++db)                                                   \
                _Pragma("unroll") for (int v = 0; v < 16; ++v) o[db][v] *= st.a;                                \
        }                                                                                                       \
        if (!(n >= nm_lo && n <= nm_hi)) {                                                                      \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) {                                                    \
                const int i = n * kKb + acc_row(v, h);                                                          \
                const bool keep = (i <= t) && (i > t - w);                                                      \
                SC[v] = keep ? SC[v] : -INFINITY;                                                               \
            }                                                                                                   \
        }                                                                                                       \
        const char* kt = sm.k[(n + 1) % kRing];                                                                 \
        const char* vt = sm.v[n % kRing];                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                                      \
        /* ---- half 1 ---- */                                                                                  \
        kfr[0] = lds_read_frag<D>(kt, 0, 0, lane);                                                              \
        kfr[1] = lds_read_frag<D>(kt, 0, 1, lane);                                                              \
        o[0] = mfma32(vfr[0], pf[0], o[0]);                                                                     \
        GFWA_PIPE_PIECE(0, SC) __builtin_amdgcn_sched_barrier(0);                                               \
        kfr[2] = lds_read_frag<D>(kt, 0, 2, lane);                                                              \
        kfr[3] = lds_read_frag<D>(kt, 0, 3, lane);                                                              \
        o[1] = mfma32(vfr[1], pf[0], o[1]);                                                                     \
        GFWA_PIPE_PIECE(1, SC) __builtin_amdgcn_sched_barrier(0);                                               \
        kfr[4] = lds_read_frag<D>(kt, 0, 4, lane);                                                              \
        kfr[5] = lds_read_frag<D>(kt, 0, 5, lane);                                                              \
        o[2] = mfma32(vfr[2], pf[0], o[2]);                                                                     \
        GFWA_PIPE_PIECE(2, SC) __builtin_amdgcn_sched_barrier(0);                                               \
        kfr[6] = lds_read_frag<D>(kt, 0, 6, lane);                                                              \
        kfr[7] = lds_read_frag<D>(kt, 0, 7, lane);                                                              \
        o[3] = mfma32(vfr[3], pf[0], o[3]);                                                                     \
        GFWA_PIPE_PIECE(3, SC) __builtin_amdgcn_sched_barrier(0);                                               \
        init_gate(SN, (n + 1) & 1);                                                                             \
        o[0] = mfma32(vfr[4], pf[1], o[0]);                                                                     \
        GFWA_PIPE_PIECE(4, SC) __builtin_amdgcn_sched_barrier(0);                                               \
        o[1] = mfma32(vfr[5], pf[1], o[1]);                                                                     \
        GFWA_PIPE_PIECE(5, SC) __builtin_amdgcn_sched_barrier(0);                                               \
        o[2] = mfma32(vfr[6], pf[1], o[2]);                                                                     \
        GFWA_PIPE_PIECE(6, SC) __builtin_amdgcn_sched_barrier(0);                                               \
        o[3] = mfma32(vfr[7], pf[1], o[3]);                                                                     \
        GFWA_PIPE_PIECE(7, SC) __builtin_amdgcn_sched_barrier(0);                                               \
        /* ---- half 2 ---- */                                                                                  \
        vfr[0] = read_v_frag<D>(vt, 0, lane);                                                                   \
        SN = mfma32(kfr[0], qf[0], SN);                                                                         \
        GFWA_PIPE_PIECE(8, SC) __builtin_amdgcn_sched_barrier(0);                                               \
        vfr[1] = read_v_frag<D>(vt, 1, lane);                                                                   \
        SN = mfma32(kfr[1], qf[1], SN);                                                                         \
        GFWA_PIPE_PIECE(9, SC) __builtin_amdgcn_sched_barrier(0);                                               \
        vfr[2] = read_v_frag<D>(vt, 2, lane);                                                                   \
        SN = mfma32(kfr[2], qf[2], SN);                                                                         \
        GFWA_PIPE_PIECE(10, SC) __builtin_amdgcn_sched_barrier(0);                                              \
        vfr[3] = read_v_frag<D>(vt, 3, lane);                                                                   \
        SN = mfma32(kfr[3], qf[3], SN);                                                                         \
        GFWA_PIPE_PIECE(11, SC) __builtin_amdgcn_sched_barrier(0);                                              \
        vfr[4] = read_v_frag<D>(vt, 4, lane);                                                                   \
        SN = mfma32(kfr[4], qf[4], SN);                                                                         \
        GFWA_PIPE_PIECE(12, SC) __builtin_amdgcn_sched_barrier(0);                                              \
        vfr[5] = read_v_frag<D>(vt, 5, lane);                                                                   \
        SN = mfma32(kfr[5], qf[5], SN);                                                                         \
        GFWA_PIPE_PIECE(13, SC) __builtin_amdgcn_sched_barrier(0);                                              \
        vfr[6] = read_v_frag<D>(vt, 6, lane);                                                                   \
        SN = mfma32(kfr[6], qf[6], SN);                                                                         \
        GFWA_PIPE_PIECE(14, SC) __builtin_amdgcn_sched_barrier(0);                                              \
        vfr[7] = read_v_frag<D>(vt, 7, lane);                                                                   \
        SN = mfma32(kfr[7], qf[7], SN);                                                                         \
        GFWA_PIPE_PIECE(15, SC) __builtin_amdgcn_sched_barrier(0);                                              \
    }

    // Blocks past n1 are computed on clamped rows and never used: the loop runs an even number of
    // iterations and simply stops reading its S after block n1.
    {
        int n = n0;
        for (; n + 1 <= n1; n += 2) {
            GFWA_PIPE_ITER(sx, sy)
            ++n;
            GFWA_PIPE_ITER(sy, sx)
            --n;
        }
        if (n == n1) {
            GFWA_PIPE_ITER(sx, sy)
        }
        // drain: O += V(n1)^T P(n1)   (vfr already holds the V(n1) fragments)
        if (__builtin_amdgcn_ballot_w64(st.a != 1.0f) != 0) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][v] *= st.a;
        }
#pragma unroll
        for (int i = 0; i < 2 * DB; ++i) o[i & 3] = mfma32(vfr[i], pf[i >> 2], o[i & 3]);
    }
#undef GFWA_PIPE_ITER
#undef GFWA_PIPE_PIECE

    // ---- epilogue: O = O^T / l, L = ln2 * (m*sl + log2 l) - (c_t - c_base)
    const float lt = xhalf_sum(l);
    if (t < N) {
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
    }
}

hipError_t forward_bf16_pipe(const void* Q, const void* K, const void* V, const float* c, void* O, float* L,
                             int B, int H, int N, int w, float scale, int occupancy, hipStream_t s) {
    constexpr int BR = 32 * kPipeWaves;
    const int num_qtiles = (N + BR - 1) / BR;
    const int total = B * H * num_qtiles;
    ProfScope prof(kKernForward, s);
    if (occupancy == 2)
        hipLaunchKernelGGL((fwd_bf16_pipe_kernel<128, 2>), dim3(total), dim3(kPipeThreads), 0, s,
                           (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, c, (bf16_t*)O, L, N, w,
                           scale * kLog2e, num_qtiles, total);
    else
        hipLaunchKernelGGL((fwd_bf16_pipe_kernel<128, 1>), dim3(total), dim3(kPipeThreads), 0, s,
                           (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, c, (bf16_t*)O, L, N, w,
                           scale * kLog2e, num_qtiles, total);
    return hipGetLastError();
}

}  // namespace gfwa
