// GatedFWA decoding step on gfx950: one new query per (batch, head) against the cached keys and
// values of the last w positions (paper Sec. 1: O(wd) work per generated token with a KV cache; the
// arithmetic is row `pos` of the forward, Sec. 3.2 / Alg. 2).
//
// The step is bound by reading the window of the cache once (2 * w * d elements per key/value head),
// so the design is about memory traffic, not MFMA:
//   * rows of the cache are read with 16 lanes x 16 bytes (bf16, d = 128), four rows per wave
//     instruction, fully coalesced, every byte once;
//   * the G query heads that read the same key/value head are handled together (4, 2 or 1 per
//     workgroup), so the cache is read once per group, not once per head;
//   * the window is split into chunks (256 keys, longer when the batch alone fills the chip), one
//     workgroup each; the (reference exponent, sum, output) partials are merged across the four waves
//     through LDS and, when the window has more than one chunk, across chunks by a second small kernel.
// With `alpha_t` given the kernel also advances the gate prefix, c[pos] = c[pos-1] + alpha_t, the one
// step of the scan a decoding step needs.
#include "gfwa_device.h"
#include "gfwa_internal.h"
#include <type_traits>

namespace gfwa {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / 64;
constexpr int kDecChunk = 256;  // keys per workgroup, 64 per wave
constexpr float kDecNegBig = -1.0e30f;
constexpr int kDecTargetWorkgroups = 1024;  // workgroups wanted before chunks get longer than 256 keys

__device__ __forceinline__ void load8(const bf16_t* p, float (&x)[8]) {
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = (float)v[e];
}
__device__ __forceinline__ void load8(const float* p, float (&x)[8]) {
    const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

// Partial record of one (query head, chunk): D output columns (unnormalised), then the reference
// exponent they are scaled by (log2 domain) and the sum.
__host__ __device__ constexpr int dec_record(int D) { return D + 2; }

// Eight consecutive cache elements as they arrive from memory, converted to fp32 only when used (so
// that the loads of the next step can be in flight, in few registers, while the current one is computed).
template <typename T>
struct Raw8;
template <>
struct Raw8<bf16_t> {
    bf16x8 v;
    __device__ __forceinline__ void load(const bf16_t* p) { v = *reinterpret_cast<const bf16x8*>(p); }
    __device__ __forceinline__ void get(float (&x)[8]) const {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = (float)v[e];
    }
};
template <>
struct Raw8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float* p) {
        a = reinterpret_cast<const float4*>(p)[0];
        b = reinterpret_cast<const float4*>(p)[1];
    }
    __device__ __forceinline__ void get(float (&x)[8]) const {
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    }
};

// Cross-lane moves on the VALU (DPP), no LDS involved, inside a row of 16 lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
// lane i receives the value of the N-th lane of its own aligned group of GT (1, 2 or 4) lanes
template <int GT, int N>
__device__ __forceinline__ float group_from(float x) {
    static_assert((GT == 4 || GT == 2 || GT == 1) && N < GT, "aligned groups of 1, 2 or 4 lanes");
    if (GT == 1) return x;
    constexpr int ctrl = GT == 4 ? (N | N << 2 | N << 4 | N << 6) : (N | N << 2 | (2 + N) << 4 | (2 + N) << 6);
    return dpp_mov<ctrl>(x);
}
// sum over the LPR (16 or 8) consecutive lanes that share a cache row, result in all of them
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
    static_assert(LPR == 16 || LPR == 8, "one or two cache rows per row of 16 lanes");
    if (LPR == 16) {  // rotations inside the row of 16: 0x120 + n is row_ror:n
        x += dpp_mov<0x128>(x);
        x += dpp_mov<0x124>(x);
        x += dpp_mov<0x122>(x);
        x += dpp_mov<0x121>(x);
    } else {  // lane ^ 1, lane ^ 2 inside the quads, lane ^ 4 as half-row mirror (i ^ 7) then i ^ 3
        x += dpp_mov<(1 | 0 << 2 | 3 << 4 | 2 << 6)>(x);
        x += dpp_mov<(2 | 3 << 2 | 0 << 4 | 1 << 6)>(x);
        x += dpp_mov<(3 | 2 << 2 | 1 << 4 | 0 << 6)>(dpp_mov<0x141>(x));
    }
    return x;
}

// One workgroup: GT query heads of one key/value head, one chunk of the window (a multiple of 256
// keys, a quarter per wave).  A step covers UN rows per lane group (4 UN or 8 UN rows per wave).
//   * every lane holds its 16-byte piece of the row and forms the partial dot products of all GT heads
//     on it; a sum over the lanes of the row (DPP adds on the VALU) leaves every lane with the GT scores;
//   * all exponentials of a wave are taken against one reference exponent per head, the score of the
//     wave's newest key (the gate bias only falls with distance).  fp32 has room for scores 2^60 above
//     it; if one ever exceeds that, the wave raises the reference and rescales (rare, wave-uniform).
//     So there is no running maximum and the output accumulators need one fused multiply-add per element;
//   * the gate prefix of a row is loaded once per head (lane j loads head j % GT) and passed round the
//     group of GT lanes by DPP;
//   * the loads of the next step are issued before the current step is computed.
template <typename T, int D, int GT>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(
    const T* __restrict__ q, const T* __restrict__ Kc, const T* __restrict__ Vc, float* __restrict__ c,
    const float* __restrict__ alpha_t, const int* __restrict__ pos, float* __restrict__ part,
    T* __restrict__ o, float* __restrict__ L, int H, int G, int Tlen, int w, float scale, int S, int chunk) {
    constexpr int LPR = D / 8;     // lanes per cache row
    constexpr int RPI = 64 / LPR;  // rows per wave instruction
    constexpr int UN = 4;          // rows per lane group and step
    constexpr int STEP_ROWS = RPI * UN;
    __shared__ float sm_acc[kDecWaves][GT][D];
    __shared__ float sm_m[kDecWaves][GT], sm_l[kDecWaves][GT];

    int idx = blockIdx.x;
    const int s = idx % S;
    idx /= S;
    const int gchunks = G / GT;
    const int gc = idx % gchunks;
    const int bkv = idx / gchunks;  // flat key/value head
    const int Hkv = H / G;
    const int b = bkv / Hkv;
    const int bh0 = b * H + (bkv % Hkv) * G + gc * GT;  // first of the GT query heads of this workgroup

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = lane / LPR, j = lane % LPR;
    const int g_own = j % GT;  // the head whose gate prefix this lane loads

    const int p = min(max(pos[b], 0), Tlen - 1);  // an out-of-range position is clamped, never followed
    const int lo = max(0, p - w + 1);
    const int k_begin = lo + s * chunk;
    const int k_end = min(p, k_begin + chunk - 1);

    // gate prefix at the query position; with alpha_t it is formed here (and stored at the end)
    float ct[GT];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        const float* crow = c + (size_t)(bh0 + g) * Tlen;
        ct[g] = alpha_t != nullptr ? (p > 0 ? crow[p - 1] : 0.f) + alpha_t[bh0 + g] : crow[p];
    }
    float ct_own = ct[0];
#pragma unroll
    for (int g = 1; g < GT; ++g) ct_own = g_own == g ? ct[g] : ct_own;
    const float* c_own = c + (size_t)(bh0 + g_own) * Tlen;

    float acc[GT][8], l[GT], mref[GT];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        l[g] = 0.f;
        mref[g] = kDecNegBig;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }

    const int per_wave = chunk / kDecWaves;
    const int kw0 = k_begin + per_wave * wv;  // first key of this wave
    if (kw0 <= k_end) {                       // uniform over the wave
        const int kw_end = min(k_end, kw0 + per_wave - 1);
        const int nsteps = (kw_end - kw0) / STEP_ROWS + 1;
        // this lane's 8 columns of the GT queries, pre-multiplied by scale * log2(e)
        float qs[GT][8];
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            load8(q + (size_t)(bh0 + g) * D + 8 * j, qs[g]);
#pragma unroll
            for (int e = 0; e < 8; ++e) qs[g][e] *= scale * kLog2e;
        }
        const T* Kh = Kc + (size_t)bkv * Tlen * D + 8 * j;
        const T* Vh = Vc + (size_t)bkv * Tlen * D + 8 * j;

        // scores (log2 domain) of one row for the GT heads; cv_own: gate prefix of the row for head g_own
        auto scores = [&](const Raw8<T>& kr, float cv_own, float (&sc)[GT]) __attribute__((always_inline)) {
            float kx[8];
            kr.get(kx);
            const float bias_own = (cv_own - ct_own) * kLog2e;
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = fmaf(qs[g][e], kx[e], dot);
                sc[g] = row_sum<LPR>(dot);
            }
            sc[0] += group_from<GT, 0>(bias_own);
            if (GT >= 2) sc[GT >= 2 ? 1 : 0] += group_from<GT, (GT >= 2 ? 1 : 0)>(bias_own);
            if (GT == 4) {
                sc[GT == 4 ? 2 : 0] += group_from<GT, (GT == 4 ? 2 : 0)>(bias_own);
                sc[GT == 4 ? 3 : 0] += group_from<GT, (GT == 4 ? 3 : 0)>(bias_own);
            }
        };

        Raw8<T> kr[2][UN], vr[2][UN];
        float cvr[2][UN];
        auto issue = [&](int st, auto bufc) __attribute__((always_inline)) {
            constexpr int buf = decltype(bufc)::value;
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int kk = min(kw0 + st * STEP_ROWS + u * RPI + r, kw_end);  // past the range: its last row, masked
                kr[buf][u].load(Kh + (size_t)kk * D);
                vr[buf][u].load(Vh + (size_t)kk * D);
                cvr[buf][u] = (alpha_t != nullptr && kk == p) ? ct_own : c_own[kk];
            }
        };
        issue(0, std::integral_constant<int, 0>{});

        {  // reference exponents: the scores of the wave's newest key
            Raw8<T> k1;
            k1.load(Kh + (size_t)kw_end * D);
            scores(k1, (alpha_t != nullptr && kw_end == p) ? ct_own : c_own[kw_end], mref);
        }

        auto compute = [&](int st, auto bufc) __attribute__((always_inline)) {
            constexpr int buf = decltype(bufc)::value;
            float sc[UN][GT];
            float excess = -INFINITY;
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                scores(kr[buf][u], cvr[buf][u], sc[u]);
                const bool ok = kw0 + st * STEP_ROWS + u * RPI + r <= kw_end;
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    sc[u][g] = ok ? sc[u][g] : -INFINITY;
                    excess = fmaxf(excess, sc[u][g] - mref[g]);
                }
            }
            if (__any(excess > 60.f)) {  // a score far above the reference: raise it and rescale
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    float v = sc[0][g];
#pragma unroll
                    for (int u = 1; u < UN; ++u) v = fmaxf(v, sc[u][g]);
#pragma unroll
                    for (int off = LPR; off < 64; off <<= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
                    const float nref = fmaxf(mref[g], v);
                    const float f = fast_exp2(mref[g] - nref);
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[g][e] *= f;
                    l[g] *= f;
                    mref[g] = nref;
                }
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                float vx[8];
                vr[buf][u].get(vx);
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    const float pr = fast_exp2(sc[u][g] - mref[g]);
                    l[g] += pr;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(pr, vx[e], acc[g][e]);
                }
            }
        };
        for (int st = 0; st < nsteps; st += 2) {
            if (st + 1 < nsteps) issue(st + 1, std::integral_constant<int, 1>{});
            compute(st, std::integral_constant<int, 0>{});
            if (st + 1 < nsteps) {
                if (st + 2 < nsteps) issue(st + 2, std::integral_constant<int, 0>{});
                compute(st + 1, std::integral_constant<int, 1>{});
            }
        }
        // one reference per head in the whole wave: plain sums over the lane groups (the lanes of a
        // row all hold the same l)
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                l[g] += __shfl_xor(l[g], off, 64);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] += __shfl_xor(acc[g][e], off, 64);
            }
    }
    // across the waves through LDS
    if (r == 0) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sm_acc[wv][g][8 * j + e] = acc[g][e];
            if (j == 0) {
                sm_m[wv][g] = mref[g];
                sm_l[wv][g] = l[g];
            }
        }
    }
    if (alpha_t != nullptr && s == 0 && tid < GT) c[(size_t)(bh0 + tid) * Tlen + p] = ct_own;  // thread g: head g
    __syncthreads();
    for (int x = tid; x < GT * D; x += kDecThreads) {
        const int g = x / D, col = x % D;
        float mm = sm_m[0][g];
#pragma unroll
        for (int k = 1; k < kDecWaves; ++k) mm = fmaxf(mm, sm_m[k][g]);
        float ll = 0.f, oo = 0.f;
#pragma unroll
        for (int k = 0; k < kDecWaves; ++k) {
            const float f = fast_exp2(sm_m[k][g] - mm);
            ll = fmaf(sm_l[k][g], f, ll);
            oo = fmaf(sm_acc[k][g][col], f, oo);
        }
        if (S == 1) {  // the whole window in one chunk: this is the result, no merge kernel follows
            o[(size_t)(bh0 + g) * D + col] = (T)(oo / ll);
            if (L != nullptr && col == 0) L[bh0 + g] = (mm + log2f(ll)) * kLn2;
        } else {
            float* rec = part + ((size_t)(bh0 + g) * S + s) * dec_record(D);
            rec[col] = oo;
            if (col == 0) {
                rec[D] = mm;
                rec[D + 1] = ll;
            }
        }
    }
}

// o = sum_s acc_s 2^(m_s - M) / sum_s l_s 2^(m_s - M),  L = (M + log2 of that sum) ln 2
template <typename T, int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(const float* __restrict__ part, T* __restrict__ o,
                                                           float* __restrict__ L, int S) {
    const int bh = blockIdx.x, col = threadIdx.x;
    const float* rec = part + (size_t)bh * S * dec_record(D);
    float mm = kDecNegBig;
    for (int s = 0; s < S; ++s) mm = fmaxf(mm, rec[(size_t)s * dec_record(D) + D]);
    float ll = 0.f, oo = 0.f;
    for (int s = 0; s < S; ++s) {
        const float* rs = rec + (size_t)s * dec_record(D);
        const float f = fast_exp2(rs[D] - mm);
        ll = fmaf(rs[D + 1], f, ll);
        oo = fmaf(rs[col], f, oo);
    }
    o[(size_t)bh * D + col] = (T)(oo / ll);
    if (L != nullptr && col == 0) L[bh] = (mm + log2f(ll)) * kLn2;
}

int decode_splits(int Tlen, int w) {
    const int span = w < Tlen ? w : Tlen;
    return (span + kDecChunk - 1) / kDecChunk;
}

size_t decode_workspace_bytes(int B, int H, int Tlen, int d, int w) {
    return (size_t)B * H * decode_splits(Tlen, w) * dec_record(d) * sizeof(float);
}

template <typename T, int D>
static hipError_t launch_decode(const T* q, const T* Kc, const T* Vc, float* c, const float* alpha_t,
                                const int* pos, T* o, float* L, float* part, int B, int H, int Hkv, int Tlen,
                                int w, float scale, hipStream_t s) {
    const int G = H / Hkv;
    const int GT = G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1);
    const int items = B * Hkv * (G / GT);
    // 256-key chunks spread a small batch over the chip; with many (batch, head) items longer chunks
    // amortise a workgroup's start-up (position, gate prefix, first rows: three dependent trips to memory)
    const int span = w < Tlen ? w : Tlen;
    int S = decode_splits(Tlen, w);
    const int want = (kDecTargetWorkgroups + items - 1) / items;
    if (want < S) S = want < 1 ? 1 : want;
    const int chunk = ((span + S - 1) / S + kDecChunk - 1) / kDecChunk * kDecChunk;
    S = (span + chunk - 1) / chunk;
    const unsigned grid = (unsigned)(items * S);
    {
        ProfScope prof(kKernDecode, s);
        if (GT == 4)
            hipLaunchKernelGGL((decode_partial_kernel<T, D, 4>), dim3(grid), dim3(kDecThreads), 0, s, q, Kc, Vc, c,
                               alpha_t, pos, part, o, L, H, G, Tlen, w, scale, S, chunk);
        else if (GT == 2)
            hipLaunchKernelGGL((decode_partial_kernel<T, D, 2>), dim3(grid), dim3(kDecThreads), 0, s, q, Kc, Vc, c,
                               alpha_t, pos, part, o, L, H, G, Tlen, w, scale, S, chunk);
        else
            hipLaunchKernelGGL((decode_partial_kernel<T, D, 1>), dim3(grid), dim3(kDecThreads), 0, s, q, Kc, Vc, c,
                               alpha_t, pos, part, o, L, H, G, Tlen, w, scale, S, chunk);
    }
    if (S > 1) {
        ProfScope prof(kKernDecodeCombine, s);
        hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(B * H), dim3(D), 0, s, part, o, L, S);
    }
    return hipGetLastError();
}

// Scratch of the allocation-free entry point: one array per GPU, held from the moment the code object
// is loaded until the process ends.  The name `scratch` is only a host-side handle of the symbol; the
// address a kernel may use is asked for once per device and kept.
static __device__ __align__(256) float scratch[kDecodeStaticBytes / sizeof(float)];

hipError_t decode_static_scratch(float** ptr) {
    static float* per_device[64];  // nullptr: not asked for yet
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev)) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    float* p = __atomic_load_n(&per_device[dev], __ATOMIC_ACQUIRE);
    if (p == nullptr) {
        if (hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch))) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        __atomic_store_n(&per_device[dev], p, __ATOMIC_RELEASE);
    }
    *ptr = p;
    return hipSuccess;
}

hipError_t decode(bool bf16, const void* q, const void* Kc, const void* Vc, float* c, const float* alpha_t,
                  const int* pos, void* o, float* L, float* part, int B, int H, int Hkv, int Tlen, int d, int w,
                  float scale, hipStream_t s) {
    if (bf16) {
        if (d == 128)
            return launch_decode<bf16_t, 128>((const bf16_t*)q, (const bf16_t*)Kc, (const bf16_t*)Vc, c, alpha_t, pos,
                                              (bf16_t*)o, L, part, B, H, Hkv, Tlen, w, scale, s);
        return launch_decode<bf16_t, 64>((const bf16_t*)q, (const bf16_t*)Kc, (const bf16_t*)Vc, c, alpha_t, pos,
                                         (bf16_t*)o, L, part, B, H, Hkv, Tlen, w, scale, s);
    }
    if (d == 128)
        return launch_decode<float, 128>((const float*)q, (const float*)Kc, (const float*)Vc, c, alpha_t, pos,
                                         (float*)o, L, part, B, H, Hkv, Tlen, w, scale, s);
    return launch_decode<float, 64>((const float*)q, (const float*)Kc, (const float*)Vc, c, alpha_t, pos, (float*)o,
                                    L, part, B, H, Hkv, Tlen, w, scale, s);
}

}  // namespace gfwa
