// GatedFWA decoding step on gfx950: one new query per (batch, head) against the cached keys and
// values of the last w positions (paper Sec. 1: O(wd) work per generated token with a KV cache; the
// arithmetic is row `pos` of the forward, Sec. 3.2 / Alg. 2).
//
// The step is bound by reading the window of the cache once (2 * w * d elements per key/value head),
// so the design is about memory traffic, not MFMA:
//   * rows of the cache are read with 16 lanes x 16 bytes (bf16, d = 128), four rows per wave
//     instruction, fully coalesced; the lanes of a row share its dot product through four xor-shuffles;
//   * the G query heads that read the same key/value head are handled together (4, 2 or 1 per
//     workgroup), so the cache is read once per group, not once per head;
//   * the window is split into chunks of 256 keys, one workgroup each, so that a small batch still
//     spreads over the chip; every lane group keeps its own online-softmax state (running maximum, sum
//     and 8 output columns) and the states are merged pairwise: inside a wave by shuffles, across the
//     four waves through LDS, across chunks by a second small kernel reading (max, sum, output) partials.
// With `alpha_t` given the kernel also advances the gate prefix, c[pos] = c[pos-1] + alpha_t, the one
// step of the scan a decoding step needs.
#include "gfwa_device.h"
#include "gfwa_internal.h"

namespace gfwa {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / 64;
constexpr int kDecChunk = 256;  // keys per workgroup, 64 per wave
constexpr float kDecNegBig = -1.0e30f;

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

// Partial record of one (query head, chunk): D output columns (unnormalised), then the running
// maximum (log2 domain) and the sum.
__host__ __device__ constexpr int dec_record(int D) { return D + 2; }

template <typename T, int D, int GT>
__global__ __launch_bounds__(kDecThreads) void decode_partial_kernel(
    const T* __restrict__ q, const T* __restrict__ Kc, const T* __restrict__ Vc, float* __restrict__ c,
    const float* __restrict__ alpha_t, const int* __restrict__ pos, float* __restrict__ part, int H, int G,
    int Tlen, int w, float scale, int S) {
    constexpr int LPR = D / 8;     // lanes per cache row
    constexpr int RPI = 64 / LPR;  // rows per wave instruction
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

    const int p = min(max(pos[b], 0), Tlen - 1);  // an out-of-range position is clamped, never followed
    const int lo = max(0, p - w + 1);
    const int k_begin = lo + s * kDecChunk;
    const int k_end = min(p, k_begin + kDecChunk - 1);

    // gate prefix at the query position; with alpha_t it is formed here and stored by one thread
    float ct[GT];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        float* crow = c + (size_t)(bh0 + g) * Tlen;
        if (alpha_t != nullptr) {
            ct[g] = (p > 0 ? crow[p - 1] : 0.f) + alpha_t[bh0 + g];
            if (s == 0 && tid == 0) crow[p] = ct[g];
        } else {
            ct[g] = crow[p];
        }
    }

    float m[GT], l[GT], acc[GT][8];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        m[g] = kDecNegBig;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }

    if (k_begin <= k_end) {  // uniform over the workgroup
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
        const int kb = k_begin + 64 * wv + r;
        constexpr int UN = 4;  // rows in flight per lane group
        for (int it0 = 0; it0 < 64 / RPI; it0 += UN) {
            if (kb - r + it0 * RPI > k_end) break;  // uniform over the wave
            float kx[UN][8], vx[UN][8], cv[UN][GT];
            bool ok[UN];
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int key = kb + (it0 + u) * RPI;
                ok[u] = key <= k_end;
                const int kk = min(key, k_end);  // rows past the chunk re-read its last row and are masked
                load8(Kh + (size_t)kk * D, kx[u]);
                load8(Vh + (size_t)kk * D, vx[u]);
#pragma unroll
                for (int g = 0; g < GT; ++g)
                    cv[u][g] = (alpha_t != nullptr && kk == p) ? ct[g] : c[(size_t)(bh0 + g) * Tlen + kk];
            }
#pragma unroll
            for (int u = 0; u < UN; ++u) {
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    float dot = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) dot = fmaf(qs[g][e], kx[u][e], dot);
#pragma unroll
                    for (int off = 1; off < LPR; off <<= 1) dot += __shfl_xor(dot, off, 64);
                    const float sc = ok[u] ? fmaf(cv[u][g] - ct[g], kLog2e, dot) : -INFINITY;
                    const float mn = fmaxf(m[g], sc);
                    const float a = fast_exp2(m[g] - mn);
                    const float pr = fast_exp2(sc - mn);
                    m[g] = mn;
                    l[g] = fmaf(l[g], a, pr);
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(acc[g][e], a, pr * vx[u][e]);
                }
            }
        }
        // merge the lane groups of the wave (lanes that differ in the row index r)
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                const float mo = __shfl_xor(m[g], off, 64);
                const float lo2 = __shfl_xor(l[g], off, 64);
                const float mn = fmaxf(m[g], mo);
                const float fa = fast_exp2(m[g] - mn), fb = fast_exp2(mo - mn);
                l[g] = l[g] * fa + lo2 * fb;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float ao = __shfl_xor(acc[g][e], off, 64);
                    acc[g][e] = acc[g][e] * fa + ao * fb;
                }
                m[g] = mn;
            }
        }
    }
    // across the waves through LDS
    if (r == 0) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
#pragma unroll
            for (int e = 0; e < 8; ++e) sm_acc[wv][g][8 * j + e] = acc[g][e];
            if (j == 0) {
                sm_m[wv][g] = m[g];
                sm_l[wv][g] = l[g];
            }
        }
    }
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
        float* rec = part + ((size_t)(bh0 + g) * S + s) * dec_record(D);
        rec[col] = oo;
        if (col == 0) {
            rec[D] = mm;
            rec[D + 1] = ll;
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
    const int S = decode_splits(Tlen, w);
    const int GT = G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1);
    const unsigned grid = (unsigned)(B * Hkv * (G / GT) * S);
    {
        ProfScope prof(kKernDecode, s);
        if (GT == 4)
            hipLaunchKernelGGL((decode_partial_kernel<T, D, 4>), dim3(grid), dim3(kDecThreads), 0, s, q, Kc, Vc, c,
                               alpha_t, pos, part, H, G, Tlen, w, scale, S);
        else if (GT == 2)
            hipLaunchKernelGGL((decode_partial_kernel<T, D, 2>), dim3(grid), dim3(kDecThreads), 0, s, q, Kc, Vc, c,
                               alpha_t, pos, part, H, G, Tlen, w, scale, S);
        else
            hipLaunchKernelGGL((decode_partial_kernel<T, D, 1>), dim3(grid), dim3(kDecThreads), 0, s, q, Kc, Vc, c,
                               alpha_t, pos, part, H, G, Tlen, w, scale, S);
    }
    {
        ProfScope prof(kKernDecodeCombine, s);
        hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(B * H), dim3(D), 0, s, part, o, L, S);
    }
    return hipGetLastError();
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
