// fp32 storage path of GatedFWA on gfx950: forward (paper Alg. 2) and backward (Alg. 3) with all
// arithmetic in fp32, for problems that need fp32 accuracy; the bf16 MFMA kernels are the throughput path.
// Two sets of kernels.  The matrix-core set (v_mfma_f32_32x32x2_f32, the structure of the bf16 kernels: a lane
// owns a query or a key, the second product takes the first one's accumulator registers as its operand) serves
// everything but tiny problems.  The one-wave-per-row set (plain FMA: lanes first split the keys of a 64-wide
// chunk to form the logits, then split the head dimension to accumulate the output row) has a launch's latency
// and serves those; forward_f32 / backward_f32 choose (f32_use_mfma).
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

// ==========================================================================================
// fp32 matrix-core kernels.  v_mfma_f32_32x32x2_f32: D[32x32] += A[32x2] * B[2x32], all fp32:
//   A: lane l holds row (l % 32), k = l / 32        B: lane l holds column (l % 32), k = l / 32
//   D: as the bf16 instruction: lane l, register v holds column (l % 32), row acc_row(v, l / 32)
// A contraction over the head dimension takes D / 2 of them; the half h of a wave supplies, in step
// 4 m + j, the element d = 8 m + 4 h + j of both operands, so a lane's four values of a group m are
// 16 contiguous bytes of a row.  The second product of each kernel takes an accumulator block as its B
// operand as it stands (register v of the two halves holds rows acc_row(v, 0) and acc_row(v, 1): the two
// k of one step) and gathers the matching rows of the other operand from LDS, 4 bytes per lane.
// ==========================================================================================
__device__ __forceinline__ f32x16 mfma_f32(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// LDS tile of 32 rows x D floats with a row pitch of D + 4 floats: every address is a per-lane base plus a
// compile-time offset, the 16-byte reads of 32 rows at one column and the 4-byte gathers of 32 consecutive columns
// of rows r (half 0) and r + 4 (half 1) conflict at most two ways - beside MFMAs of 64 cycles that is nothing.
template <int D>
constexpr int kF32Pitch = D + 4;
template <int D>
__device__ __forceinline__ constexpr int f32_tile_off(int row, int col) { return row * kF32Pitch<D> + col; }

constexpr int kF32Threads = 256;  // 4 waves: 32 queries (or keys) each

// One 32-row tile of a [N, D] matrix per workgroup step: 16-byte pieces, a thread takes every 256th.
template <int D>
struct F32TileRegs {
    static constexpr int kPieces = 32 * (D / 4) / kF32Threads;
    f32x4 r[kPieces];
    __device__ __forceinline__ void fetch(const float* M, int row0, int N, int tid) {  // rows past N read row N-1
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            const int q = tid + kF32Threads * i, row = q / (D / 4), cc = q % (D / 4);
            r[i] = *reinterpret_cast<const f32x4*>(M + (size_t)min(row0 + row, N - 1) * D + 4 * cc);
        }
    }
    __device__ __forceinline__ void stash(float* tile, int tid) const {
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            const int q = tid + kF32Threads * i, row = q / (D / 4), cc = q % (D / 4);
            *reinterpret_cast<f32x4*>(tile + f32_tile_off<D>(row, 4 * cc)) = r[i];
        }
    }
};

// ---- forward (Alg. 2): a workgroup owns 128 queries, a wave 32 of them, a lane one query (both halves of the
// wave hold it, with complementary keys).  S^T = K Q^T with the Q fragments in registers, the running maximum
// and sum per lane, O^T += V^T P^T with P^T taken from the S^T accumulator registers.
template <int D>
__global__ __launch_bounds__(kF32Threads, 2) void fwd_f32_mfma_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ c, float* __restrict__ O, float* __restrict__ L, int N, int w, float scale,
    int num_qtiles, int total_tiles, int H, int G) {
    constexpr int NM = D / 8, DB = D / 32;
    __shared__ __align__(16) float Ks[32 * kF32Pitch<D>];
    __shared__ __align__(16) float Vs[32 * kF32Pitch<D>];
    __shared__ float cs[32];
    const int tile = xcd_remap(blockIdx.x, total_tiles);
    const int bh = tile / num_qtiles, q0 = (tile % num_qtiles) * 128;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, lq = lane & 31;
    const int qw0 = q0 + 32 * wv, t = qw0 + lq, tc = min(t, N - 1);
    const size_t ho = (size_t)bh * N * D, kvo = (size_t)kv_head_of(bh, H, G) * N * D;
    const float *Kh = K + kvo, *Vh = V + kvo, *ch = c + (size_t)bh * N;

    float qf[D / 2];
#pragma unroll
    for (int m = 0; m < NM; ++m) {
        const f32x4 q4 = *reinterpret_cast<const f32x4*>(Q + ho + (size_t)tc * D + 8 * m + 4 * h);
#pragma unroll
        for (int j = 0; j < 4; ++j) qf[4 * m + j] = q4[j];
    }
    const float ct = ch[tc];
    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float mrun = kNegBig, lh = 0.f;  // lh: the sum over this half's keys

    const int jb_lo = max(0, q0 - w + 1) / 32, jb_hi = (min(N, q0 + 128) - 1) / 32;
    F32TileRegs<D> kreg, vreg;
    float creg = 0.f;
    auto fetch = [&](int jb) __attribute__((always_inline)) {
        kreg.fetch(Kh, 32 * jb, N, tid);
        vreg.fetch(Vh, 32 * jb, N, tid);
        if (tid < 32) creg = ch[min(32 * jb + tid, N - 1)];
    };
    fetch(jb_lo);
    for (int jb = jb_lo; jb <= jb_hi; ++jb) {
        __syncthreads();  // the previous block's readers are done
        kreg.stash(Ks, tid);
        vreg.stash(Vs, tid);
        if (tid < 32) cs[tid] = creg;
        __syncthreads();
        if (jb < jb_hi) fetch(jb + 1);
        const int kb0 = 32 * jb;
        if (!((kb0 <= qw0 + 31) && (kb0 + 31 > qw0 - w) && (qw0 < N))) continue;  // outside this wave's band
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const f32x4 k4 = *reinterpret_cast<const f32x4*>(Ks + f32_tile_off<D>(lq, 8 * m + 4 * h));
#pragma unroll
            for (int j = 0; j < 4; ++j) s = mfma_f32(k4[j], qf[4 * m + j], s);
        }
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = acc_row(v, h), i = kb0 + r;
            const float x = fmaf(scale, s[v], cs[r] - ct);
            s[v] = (i <= t && i > t - w) ? x : -INFINITY;
            mx = fmaxf(mx, s[v]);
        }
        // exp through the hardware exp2: the argument's rounding (2^-24 |x| log2 e) only matters for
        // probabilities that are themselves negligible
        const float mnew = fmaxf(mrun, xhalf_max(mx));
        const float a = fast_exp2((mrun - mnew) * kLog2e);
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            s[v] = fast_exp2((s[v] - mnew) * kLog2e);
            psum += s[v];
        }
        lh = fmaf(lh, a, psum);
        mrun = mnew;
        if (__builtin_amdgcn_ballot_w64(a != 1.0f) != 0) {  // the maximum of some row has moved (rare after the first blocks)
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][v] *= a;
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db] = mfma_f32(Vs[f32_tile_off<D>(acc_row(v, h), 32 * db + lq)], s[v], o[db]);
        }
    }
    const float l = xhalf_sum(lh);
    if (t < N) {
        float* orow = O + ho + (size_t)t * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                f32x4 out;
#pragma unroll
                for (int j = 0; j < 4; ++j) out[j] = o[db][4 * i4 + j] / l;
                *reinterpret_cast<f32x4*>(orow + 32 * db + 8 * i4 + 4 * h) = out;
            }
        if (h == 0) L[(size_t)bh * N + t] = mrun + fast_log2(l) * kLn2;
    }
}

// ---- dQ and the row sums of dS (Alg. 3, query loop): the forward's layout.  S^T = K Q^T and dP^T = V dO^T with the
// Q and dO fragments in registers, dS^T = P^T (dP^T - D) in the accumulator registers, dQ^T += K^T dS^T.
template <int D>
__global__ __launch_bounds__(kF32Threads, D == 128 ? 1 : 2) void bwd_dq_f32_mfma_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ dO, const float* __restrict__ c, const float* __restrict__ L,
    const float* __restrict__ Dv, float* __restrict__ dQ, float* __restrict__ dc_row, int N, int w, float scale,
    int num_qtiles, int total_tiles, int H, int G) {
    constexpr int NM = D / 8, DB = D / 32;
    __shared__ __align__(16) float Ks[32 * kF32Pitch<D>];
    __shared__ __align__(16) float Vs[32 * kF32Pitch<D>];
    __shared__ float cs[32];
    const int tile = xcd_remap(blockIdx.x, total_tiles);
    const int bh = tile / num_qtiles, q0 = (tile % num_qtiles) * 128;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, lq = lane & 31;
    const int qw0 = q0 + 32 * wv, t = qw0 + lq, tc = min(t, N - 1);
    const size_t ho = (size_t)bh * N * D, kvo = (size_t)kv_head_of(bh, H, G) * N * D;
    const float *Kh = K + kvo, *Vh = V + kvo, *ch = c + (size_t)bh * N;

    float qf[D / 2], gf[D / 2];
#pragma unroll
    for (int m = 0; m < NM; ++m) {
        const f32x4 q4 = *reinterpret_cast<const f32x4*>(Q + ho + (size_t)tc * D + 8 * m + 4 * h);
        const f32x4 g4 = *reinterpret_cast<const f32x4*>(dO + ho + (size_t)tc * D + 8 * m + 4 * h);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            qf[4 * m + j] = q4[j];
            gf[4 * m + j] = g4[j];
        }
    }
    const float ct = ch[tc], Lt = L[(size_t)bh * N + tc], Dt = Dv[(size_t)bh * N + tc];
    f32x16 acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
    float rs = 0.f;

    const int jb_lo = max(0, q0 - w + 1) / 32, jb_hi = (min(N, q0 + 128) - 1) / 32;
    F32TileRegs<D> kreg, vreg;
    float creg = 0.f;
    auto fetch = [&](int jb) __attribute__((always_inline)) {
        kreg.fetch(Kh, 32 * jb, N, tid);
        vreg.fetch(Vh, 32 * jb, N, tid);
        if (tid < 32) creg = ch[min(32 * jb + tid, N - 1)];
    };
    fetch(jb_lo);
    for (int jb = jb_lo; jb <= jb_hi; ++jb) {
        __syncthreads();
        kreg.stash(Ks, tid);
        vreg.stash(Vs, tid);
        if (tid < 32) cs[tid] = creg;
        __syncthreads();
        if (jb < jb_hi) fetch(jb + 1);
        const int kb0 = 32 * jb;
        if (!((kb0 <= qw0 + 31) && (kb0 + 31 > qw0 - w) && (qw0 < N))) continue;
        f32x16 s, dp;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = dp[v] = 0.f;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const f32x4 k4 = *reinterpret_cast<const f32x4*>(Ks + f32_tile_off<D>(lq, 8 * m + 4 * h));
#pragma unroll
            for (int j = 0; j < 4; ++j) s = mfma_f32(k4[j], qf[4 * m + j], s);
        }
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const f32x4 v4 = *reinterpret_cast<const f32x4*>(Vs + f32_tile_off<D>(lq, 8 * m + 4 * h));
#pragma unroll
            for (int j = 0; j < 4; ++j) dp = mfma_f32(v4[j], gf[4 * m + j], dp);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int r = acc_row(v, h), i = kb0 + r;
            const float x = fmaf(scale, s[v], cs[r] - ct);
            const float p = (i <= t && i > t - w) ? fast_exp2((x - Lt) * kLog2e) : 0.f;
            s[v] = p * (dp[v] - Dt);
            rs += s[v];
        }
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[db] = mfma_f32(Ks[f32_tile_off<D>(acc_row(v, h), 32 * db + lq)], s[v], acc[db]);
    }
    rs = xhalf_sum(rs);
    if (t < N) {
        float* out = dQ + ho + (size_t)t * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                f32x4 o4;
#pragma unroll
                for (int j = 0; j < 4; ++j) o4[j] = scale * acc[db][4 * i4 + j];
                *reinterpret_cast<f32x4*>(out + 32 * db + 8 * i4 + 4 * h) = o4;
            }
        if (h == 0) dc_row[(size_t)bh * N + t] = rs;
    }
}

// ---- dK, dV (summed over the G query heads of a group) and, per query head, the column sums of dS (Alg. 3, key
// loop): a workgroup owns 128 keys, a wave 32 of them, a lane one key; the K and V fragments are the B operands
// in registers.  S = Q K^T and dP = dO V^T with 32-query tiles of Q and dO from LDS, then dV^T += dO^T P and
// dK^T += Q^T dS with P and dS taken from the accumulator registers.
template <int D>
__global__ __launch_bounds__(kF32Threads, D == 128 ? 1 : 2) void bwd_dkv_f32_mfma_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ dO, const float* __restrict__ c, const float* __restrict__ L,
    const float* __restrict__ Dv, float* __restrict__ dK, float* __restrict__ dV, float* __restrict__ dc_col,
    int N, int w, float scale, int num_ktiles, int total_tiles, int H, int G) {
    constexpr int NM = D / 8, DB = D / 32;
    __shared__ __align__(16) float Qs[32 * kF32Pitch<D>];
    __shared__ __align__(16) float Gs[32 * kF32Pitch<D>];
    __shared__ float cqs[32], Lqs[32], Dqs[32];
    const int tile = xcd_remap(blockIdx.x, total_tiles);
    const int bkv = tile / num_ktiles, k0 = (tile % num_ktiles) * 128;  // flat key/value head, first key
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, h = lane >> 5, lk = lane & 31;
    const int kw0 = k0 + 32 * wv, i = kw0 + lk, ic = min(i, N - 1);
    const int Hkv = H / G;
    const int bh0 = (bkv / Hkv) * H + (bkv % Hkv) * G;  // first query head of the group
    const size_t kvo = (size_t)bkv * N * D;

    float kf[D / 2], vf[D / 2];
#pragma unroll
    for (int m = 0; m < NM; ++m) {
        const f32x4 k4 = *reinterpret_cast<const f32x4*>(K + kvo + (size_t)ic * D + 8 * m + 4 * h);
        const f32x4 v4 = *reinterpret_cast<const f32x4*>(V + kvo + (size_t)ic * D + 8 * m + 4 * h);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            kf[4 * m + j] = k4[j];
            vf[4 * m + j] = v4[j];
        }
    }
    f32x16 dk[DB], dv[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) dk[db][v] = dv[db][v] = 0.f;

    // query blocks that see a key of the tile: rows k0 .. k0 + 127 + w - 1
    const int qb_lo = k0 / 32;
    const int qb_hi = (int)(min((long)N - 1, (long)k0 + 127 + w - 1) / 32);
    const int nblk = qb_hi - qb_lo + 1;
    F32TileRegs<D> qreg, greg;
    float creg = 0.f, lreg = 0.f, dreg = 0.f;
    auto fetch = [&](int it) __attribute__((always_inline)) {
        const int bh = bh0 + it / nblk, qb0 = 32 * (qb_lo + it % nblk);
        const size_t ho = (size_t)bh * N * D;
        qreg.fetch(Q + ho, qb0, N, tid);
        greg.fetch(dO + ho, qb0, N, tid);
        if (tid < 32) {
            const size_t r = (size_t)bh * N + min(qb0 + tid, N - 1);
            creg = c[r];
            lreg = L[r];
            dreg = Dv[r];
        }
    };
    fetch(0);
    float colsum = 0.f, ci = 0.f;
    for (int it = 0; it < G * nblk; ++it) {
        const int g = it / nblk, b = it % nblk, qb0 = 32 * (qb_lo + b);
        const int bh = bh0 + g;
        if (b == 0) {
            colsum = 0.f;
            ci = c[(size_t)bh * N + ic];
        }
        __syncthreads();
        qreg.stash(Qs, tid);
        greg.stash(Gs, tid);
        if (tid < 32) {
            cqs[tid] = creg;
            Lqs[tid] = lreg;
            Dqs[tid] = dreg;
        }
        __syncthreads();
        if (it + 1 < G * nblk) fetch(it + 1);
        if ((qb0 + 31 >= kw0) && ((long)qb0 <= (long)kw0 + 31 + w - 1) && (kw0 < N)) {
            f32x16 s, dp;
#pragma unroll
            for (int v = 0; v < 16; ++v) s[v] = dp[v] = 0.f;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const f32x4 q4 = *reinterpret_cast<const f32x4*>(Qs + f32_tile_off<D>(lk, 8 * m + 4 * h));
#pragma unroll
                for (int j = 0; j < 4; ++j) s = mfma_f32(q4[j], kf[4 * m + j], s);
            }
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const f32x4 g4 = *reinterpret_cast<const f32x4*>(Gs + f32_tile_off<D>(lk, 8 * m + 4 * h));
#pragma unroll
                for (int j = 0; j < 4; ++j) dp = mfma_f32(g4[j], vf[4 * m + j], dp);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = acc_row(v, h), tq = qb0 + r;
                const float x = fmaf(scale, s[v], ci - cqs[r]);
                const float p = (i <= tq && i > tq - w && tq < N) ? fast_exp2((x - Lqs[r]) * kLog2e) : 0.f;
                s[v] = p * (dp[v] - Dqs[r]);
                dp[v] = p;
                colsum += s[v];
            }
#pragma unroll
            for (int db = 0; db < DB; ++db) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    dv[db] = mfma_f32(Gs[f32_tile_off<D>(acc_row(v, h), 32 * db + lk)], dp[v], dv[db]);
                    dk[db] = mfma_f32(Qs[f32_tile_off<D>(acc_row(v, h), 32 * db + lk)], s[v], dk[db]);
                }
                __builtin_amdgcn_sched_barrier(0);  // keeps the gathers of one column block from all being hoisted
            }
        }
        if (b == nblk - 1) {  // the query head is finished: its column sums
            const float cs_all = xhalf_sum(colsum);
            if (i < N && h == 0) dc_col[(size_t)bh * N + i] = cs_all;
        }
    }
    if (i < N) {
        float* ok = dK + kvo + (size_t)i * D;
        float* ov = dV + kvo + (size_t)i * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                f32x4 a, b;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    a[j] = scale * dk[db][4 * i4 + j];
                    b[j] = dv[db][4 * i4 + j];
                }
                *reinterpret_cast<f32x4*>(ok + 32 * db + 8 * i4 + 4 * h) = a;
                *reinterpret_cast<f32x4*>(ov + 32 * db + 8 * i4 + 4 * h) = b;
            }
    }
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

// Which kernels serve a problem: the matrix-core ones reach half of the fp32 MFMA peak but walk a query (key) tile's
// band one 32-row block after another, about 3 us each at d = 64; the one-wave-per-row kernels sustain 7 TFLOP/s
// whatever the shape and finish a tiny problem in one launch latency.  The crossover of the two estimates:
static bool f32_use_mfma(int B, int H, int N, int d, int w) {
    const double wc = w < N ? w : N;
    const double work = (double)B * H * N * wc * d;
    const double blocks = (wc + 128.0) / 32.0;
    return work >= blocks * (d / 64.0) * 5.0e6;
}

hipError_t forward_f32(const float* Q, const float* K, const float* V, const float* c, float* O, float* L,
                       int B, int H, int Hkv, int N, int d, int w, float scale, hipStream_t s) {
    ProfScope prof(kKernForward, s);
    if (f32_use_mfma(B, H, N, d, w)) {
        const int nq = (N + 127) / 128, total = B * H * nq;
        if (d == 128)
            hipLaunchKernelGGL((fwd_f32_mfma_kernel<128>), dim3(total), dim3(kF32Threads), 0, s, Q, K, V, c, O, L, N, w,
                               scale, nq, total, H, H / Hkv);
        else
            hipLaunchKernelGGL((fwd_f32_mfma_kernel<64>), dim3(total), dim3(kF32Threads), 0, s, Q, K, V, c, O, L, N, w,
                               scale, nq, total, H, H / Hkv);
    } else {
        const int blocks = B * H * ((N + kF32Waves - 1) / kF32Waves);
        hipLaunchKernelGGL(fwd_f32_kernel, dim3(blocks), dim3(64 * kF32Waves), 0, s, Q, K, V, c, O, L, N, d, w, scale,
                           H, H / Hkv);
    }
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
    if (f32_use_mfma(B, H, N, d, w)) {
        const int nt = (N + 127) / 128;
        {
            ProfScope prof(kKernDkv, s);
            if (d == 128)
                hipLaunchKernelGGL((bwd_dkv_f32_mfma_kernel<128>), dim3(B * Hkv * nt), dim3(kF32Threads), 0, s, Q, K, V, dO,
                                   c, L, Dv, dK, dV, dc_col, N, w, scale, nt, B * Hkv * nt, H, H / Hkv);
            else
                hipLaunchKernelGGL((bwd_dkv_f32_mfma_kernel<64>), dim3(B * Hkv * nt), dim3(kF32Threads), 0, s, Q, K, V, dO,
                                   c, L, Dv, dK, dV, dc_col, N, w, scale, nt, B * Hkv * nt, H, H / Hkv);
        }
        {
            ProfScope prof(kKernDq, s);
            if (d == 128)
                hipLaunchKernelGGL((bwd_dq_f32_mfma_kernel<128>), dim3(B * H * nt), dim3(kF32Threads), 0, s, Q, K, V, dO, c, L,
                                   Dv, dQ, dc_row, N, w, scale, nt, B * H * nt, H, H / Hkv);
            else
                hipLaunchKernelGGL((bwd_dq_f32_mfma_kernel<64>), dim3(B * H * nt), dim3(kF32Threads), 0, s, Q, K, V, dO, c, L,
                                   Dv, dQ, dc_row, N, w, scale, nt, B * H * nt, H, H / Hkv);
        }
    } else {
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
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // behind the three vectors as the workspace query sizes them (each padded to 256 bytes)
    const size_t one = ((rows * sizeof(float)) + 255) & ~(size_t)255;
    return gate_grad_scan(dc_col, dc_row, dalpha, reinterpret_cast<double*>(reinterpret_cast<char*>(ws) + 3 * one), B * H, N, s);
}

}  // namespace gfwa
