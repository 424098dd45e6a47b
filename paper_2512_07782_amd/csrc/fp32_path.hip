// fp32 storage path of GatedFWA on gfx950: forward (paper Alg. 2) and backward (Alg. 3) with all
// arithmetic in fp32 and no matrix cores.  It serves small problems that need fp32 accuracy; the
// bf16 MFMA kernels are the throughput path.  One wavefront owns one query row (forward, dQ) or
// one key row (dK/dV): lanes first split the keys (or queries) of a 64-wide chunk to form the
// logits, then split the head dimension to accumulate the output row.
#include "gfwa_device.h"
#include "gfwa_internal.h"

namespace gfwa {

constexpr int kF32Waves = 4;

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x = fmaxf(x, __shfl_xor(x, d, 64));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, 64);
    return x;
}
__device__ __forceinline__ float dot_row(const float* __restrict__ a_lds, const float* __restrict__ g, int D) {
    float acc = 0.f;
    for (int x = 0; x < D; x += 4) {
        const float4 gv = *reinterpret_cast<const float4*>(g + x);
        acc = fmaf(a_lds[x], gv.x, acc);
        acc = fmaf(a_lds[x + 1], gv.y, acc);
        acc = fmaf(a_lds[x + 2], gv.z, acc);
        acc = fmaf(a_lds[x + 3], gv.w, acc);
    }
    return acc;
}

// ---- forward: online softmax over 64-key chunks of the window of row t
__global__ __launch_bounds__(64 * kF32Waves) void fwd_f32_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ c, float* __restrict__ O, float* __restrict__ L, int N, int D, int w,
    float scale, int H, int G) {
    __shared__ float qs[kF32Waves][128];
    __shared__ float ps[kF32Waves][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int rows_per_head = (N + kF32Waves - 1) / kF32Waves;
    const int bh = blockIdx.x / rows_per_head;
    const int t = (blockIdx.x % rows_per_head) * kF32Waves + wv;
    if (t >= N) return;  // whole wave leaves; no workgroup barriers are used below
    const size_t ho = (size_t)bh * N * D;
    const size_t kvo = (size_t)kv_head_of(bh, H, G) * N * D;
    const float* Kh = K + kvo;
    const float* Vh = V + kvo;
    const float* ch = c + (size_t)bh * N;
    for (int x = lane; x < D; x += 64) qs[wv][x] = Q[ho + (size_t)t * D + x];
    const float ct = ch[t];
    const int lo = max(0, t - w + 1);
    float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
    for (int i0 = lo; i0 <= t; i0 += 64) {
        const int i = i0 + lane;
        float s = -INFINITY;
        if (i <= t) s = fmaf(scale, dot_row(qs[wv], Kh + (size_t)i * D, D), ch[i] - ct);
        const float mnew = fmaxf(m, wave_max(s));  // finite: the chunk always holds a valid key
        const float a = expf(m - mnew);
        const float p = expf(s - mnew);
        l = fmaf(l, a, wave_sum(p));
        m = mnew;
        ps[wv][lane] = p;
        o0 *= a;
        o1 *= a;
        const int n = min(64, t - i0 + 1);
        for (int j = 0; j < n; ++j) {
            const float pj = ps[wv][j];
            const float* vr = Vh + (size_t)(i0 + j) * D;
            o0 = fmaf(pj, vr[lane], o0);
            if (D > 64) o1 = fmaf(pj, vr[lane + 64], o1);
        }
    }
    float* orow = O + ho + (size_t)t * D;
    orow[lane] = o0 / l;
    if (D > 64) orow[lane + 64] = o1 / l;
    if (lane == 0) L[(size_t)bh * N + t] = m + logf(l);
}

// ---- D_t = <O_t, dO_t>
__global__ __launch_bounds__(64 * kF32Waves) void rowdot_f32_kernel(const float* __restrict__ O,
                                                                    const float* __restrict__ dO,
                                                                    float* __restrict__ Dv, long rows, int D) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const long r = (long)blockIdx.x * kF32Waves + wv;
    if (r >= rows) return;
    float acc = 0.f;
    for (int x = lane; x < D; x += 64) acc = fmaf(O[r * D + x], dO[r * D + x], acc);
    acc = wave_sum(acc);
    if (lane == 0) Dv[r] = acc;
}

// ---- dQ_t and the row sum of dS
__global__ __launch_bounds__(64 * kF32Waves) void bwd_dq_f32_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ dO, const float* __restrict__ c, const float* __restrict__ L,
    const float* __restrict__ Dv, float* __restrict__ dQ, float* __restrict__ dc_row, int N, int D,
    int w, float scale, int H, int G) {
    __shared__ float qs[kF32Waves][128];
    __shared__ float gs[kF32Waves][128];
    __shared__ float ds_s[kF32Waves][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int rows_per_head = (N + kF32Waves - 1) / kF32Waves;
    const int bh = blockIdx.x / rows_per_head;
    const int t = (blockIdx.x % rows_per_head) * kF32Waves + wv;
    if (t >= N) return;
    const size_t ho = (size_t)bh * N * D;
    const size_t kvo = (size_t)kv_head_of(bh, H, G) * N * D;
    const float* Kh = K + kvo;
    const float* Vh = V + kvo;
    const float* ch = c + (size_t)bh * N;
    for (int x = lane; x < D; x += 64) {
        qs[wv][x] = Q[ho + (size_t)t * D + x];
        gs[wv][x] = dO[ho + (size_t)t * D + x];
    }
    const float ct = ch[t], Lt = L[(size_t)bh * N + t], Dt = Dv[(size_t)bh * N + t];
    const int lo = max(0, t - w + 1);
    float rs = 0.f, g0 = 0.f, g1 = 0.f;
    for (int i0 = lo; i0 <= t; i0 += 64) {
        const int i = i0 + lane;
        float ds = 0.f;
        if (i <= t) {
            const float s = fmaf(scale, dot_row(qs[wv], Kh + (size_t)i * D, D), ch[i] - ct);
            const float p = expf(s - Lt);
            ds = p * (dot_row(gs[wv], Vh + (size_t)i * D, D) - Dt);
        }
        rs += ds;
        ds_s[wv][lane] = ds;
        const int n = min(64, t - i0 + 1);
        for (int j = 0; j < n; ++j) {
            const float dj = ds_s[wv][j];
            const float* kr = Kh + (size_t)(i0 + j) * D;
            g0 = fmaf(dj, kr[lane], g0);
            if (D > 64) g1 = fmaf(dj, kr[lane + 64], g1);
        }
    }
    rs = wave_sum(rs);
    float* out = dQ + ho + (size_t)t * D;
    out[lane] = scale * g0;
    if (D > 64) out[lane + 64] = scale * g1;
    if (lane == 0) dc_row[(size_t)bh * N + t] = rs;
}

// ---- dK_i, dV_i (summed over the G query heads that read this key/value head) and, per query
// head, the column sum of dS
__global__ __launch_bounds__(64 * kF32Waves) void bwd_dkv_f32_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ dO, const float* __restrict__ c, const float* __restrict__ L,
    const float* __restrict__ Dv, float* __restrict__ dK, float* __restrict__ dV,
    float* __restrict__ dc_col, int N, int D, int w, float scale, int H, int G) {
    __shared__ float ks[kF32Waves][128];
    __shared__ float vs[kF32Waves][128];
    __shared__ float p_s[kF32Waves][64];
    __shared__ float ds_s[kF32Waves][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int rows_per_head = (N + kF32Waves - 1) / kF32Waves;
    const int bkv = blockIdx.x / rows_per_head;  // flat key/value head
    const int i = (blockIdx.x % rows_per_head) * kF32Waves + wv;
    if (i >= N) return;
    const int Hkv = H / G;
    const int bh0 = (bkv / Hkv) * H + (bkv % Hkv) * G;  // first query head of the group
    const size_t kvo = (size_t)bkv * N * D;
    for (int x = lane; x < D; x += 64) {
        ks[wv][x] = K[kvo + (size_t)i * D + x];
        vs[wv][x] = V[kvo + (size_t)i * D + x];
    }
    const long t_hi = min((long)N - 1, (long)i + w - 1);  // key i is seen by rows i .. i+w-1
    float k0 = 0.f, k1 = 0.f, v0 = 0.f, v1 = 0.f;
    for (int g = 0; g < G; ++g) {
        const int bh = bh0 + g;
        const size_t ho = (size_t)bh * N * D;
        const float* Qh = Q + ho;
        const float* Gh = dO + ho;
        const float* ch = c + (size_t)bh * N;
        const float* Lh = L + (size_t)bh * N;
        const float* Dh = Dv + (size_t)bh * N;
        const float ci = ch[i];
        float cs = 0.f;
        for (long t0 = i; t0 <= t_hi; t0 += 64) {
            const long t = t0 + lane;
            float p = 0.f, ds = 0.f;
            if (t <= t_hi) {
                const float s = fmaf(scale, dot_row(ks[wv], Qh + (size_t)t * D, D), ci - ch[t]);
                p = expf(s - Lh[t]);
                ds = p * (dot_row(vs[wv], Gh + (size_t)t * D, D) - Dh[t]);
            }
            cs += ds;
            p_s[wv][lane] = p;
            ds_s[wv][lane] = ds;
            const int n = (int)min(64L, t_hi - t0 + 1);
            for (int j = 0; j < n; ++j) {
                const float pj = p_s[wv][j], dj = ds_s[wv][j];
                const float* gr = Gh + (size_t)(t0 + j) * D;
                const float* qr = Qh + (size_t)(t0 + j) * D;
                v0 = fmaf(pj, gr[lane], v0);
                k0 = fmaf(dj, qr[lane], k0);
                if (D > 64) {
                    v1 = fmaf(pj, gr[lane + 64], v1);
                    k1 = fmaf(dj, qr[lane + 64], k1);
                }
            }
        }
        cs = wave_sum(cs);
        if (lane == 0) dc_col[(size_t)bh * N + i] = cs;
    }
    dK[kvo + (size_t)i * D + lane] = scale * k0;
    dV[kvo + (size_t)i * D + lane] = v0;
    if (D > 64) {
        dK[kvo + (size_t)i * D + lane + 64] = scale * k1;
        dV[kvo + (size_t)i * D + lane + 64] = v1;
    }
}

hipError_t forward_f32(const float* Q, const float* K, const float* V, const float* c, float* O, float* L,
                       int B, int H, int Hkv, int N, int d, int w, float scale, hipStream_t s) {
    const int blocks = B * H * ((N + kF32Waves - 1) / kF32Waves);
    ProfScope prof(kKernForward, s);
    hipLaunchKernelGGL(fwd_f32_kernel, dim3(blocks), dim3(64 * kF32Waves), 0, s, Q, K, V, c, O, L, N, d, w, scale,
                       H, H / Hkv);
    return hipGetLastError();
}

hipError_t backward_f32(const float* Q, const float* K, const float* V, const float* O, const float* dO,
                        const float* c, const float* L, float* dQ, float* dK, float* dV, float* dalpha,
                        float* ws, int B, int H, int Hkv, int N, int d, int w, float scale, hipStream_t s) {
    const size_t rows = (size_t)B * H * N;
    float* Dv = ws;
    float* dc_col = ws + rows;
    float* dc_row = ws + 2 * rows;
    const int per_head = (N + kF32Waves - 1) / kF32Waves;
    const int blocks = B * H * per_head;
    {
        ProfScope prof(kKernRowDot, s);
        hipLaunchKernelGGL(rowdot_f32_kernel, dim3((unsigned)((rows + kF32Waves - 1) / kF32Waves)),
                           dim3(64 * kF32Waves), 0, s, O, dO, Dv, (long)rows, d);
    }
    {
        ProfScope prof(kKernDkv, s);
        hipLaunchKernelGGL(bwd_dkv_f32_kernel, dim3(B * Hkv * per_head), dim3(64 * kF32Waves), 0, s, Q, K, V, dO,
                           c, L, Dv, dK, dV, dc_col, N, d, w, scale, H, H / Hkv);
    }
    {
        ProfScope prof(kKernDq, s);
        hipLaunchKernelGGL(bwd_dq_f32_kernel, dim3(blocks), dim3(64 * kF32Waves), 0, s, Q, K, V, dO, c, L,
                           Dv, dQ, dc_row, N, d, w, scale, H, H / Hkv);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // behind the three vectors as the workspace query sizes them (each padded to 256 bytes)
    const size_t one = ((rows * sizeof(float)) + 255) & ~(size_t)255;
    return gate_grad_scan(dc_col, dc_row, dalpha, reinterpret_cast<double*>(reinterpret_cast<char*>(ws) + 3 * one), B * H, N, s);
}

}  // namespace gfwa
