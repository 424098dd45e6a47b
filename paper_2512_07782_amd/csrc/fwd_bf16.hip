// GatedFWA fused forward for bf16 storage on gfx950 (paper Alg. 2, re-designed for CDNA4).
//
// One workgroup (4 waves, two workgroups per CU so that every SIMD always has a second wave to
// issue from) owns a tile of 128 consecutive queries of one (b,h); a wave owns 32 of them.
// Key/value tiles of 64 keys travel global -> LDS by direct loads (no staging registers, no LDS
// stores), double buffered, and only the tiles that intersect the band [q0-w+1, q0+127] are
// visited; inside a tile every wave skips the 32-key blocks that lie wholly outside the band of
// its own queries, and masks only the blocks the band edge or the diagonal cuts.
//
// The products are formed transposed so that a lane owns one query:
//   S^T[key][query]  = g[key] + K_tile (A operand, from LDS)  x  Q^T (B operand, registers)
//   O^T[dd][query]  += V_tile^T (A operand, LDS transposing read)  x  P^T (B operand = the S^T
//                      accumulator registers converted to bf16 in place)
// so the row max / row sum of the online softmax are in-lane plus one exchange between the two
// halves of the wave, the rescale factor is a per-lane scalar, and P never leaves registers.
//
// The gate bias rides in the MFMA accumulator: S is initialised with g_i = (c_i - c_base) / scale
// straight from LDS before the K Q^T chain, so S = q.k + g_i and the probability is one fused
// multiply-add plus one exp2:  p = exp2(S*sl - m*sl), sl = scale * log2(e).  The per-query term
// -(c_t - c_base) is constant along a row, cancels in the softmax, and is applied only to L.
// c_base = c at the first query of the tile keeps the fp32 differences window-local.  The row sum
// is taken over the bf16-rounded probabilities (one packed dot-product per pair), i.e. over exactly
// the values that enter the PV product.  The running max is raised only when it grows by more than
// 2^8, so most blocks need no rescale of O.
#include "gfwa_device.h"
#include "gfwa_internal.h"

namespace gfwa {

constexpr int kFwdThreads = 256;
constexpr int kBC = 64;  // keys per LDS tile

template <int D>
struct FwdSmem {
    alignas(16) char k[2][kBC * D * 2];
    alignas(16) char v[2][kBC * D * 2];
    alignas(16) float g[2][kBC];  // (c - c_base) / scale
};

template <int D>
__global__ __launch_bounds__(kFwdThreads, 2) void fwd_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const float* __restrict__ c, bf16_t* __restrict__ O, float* __restrict__ L, int N, int w,
    float scale_log2, int num_qtiles, int total_tiles) {
    constexpr int BR = 128;
    constexpr int KC = D / 16;  // MFMA k-chunks along the head dimension
    constexpr int DB = D / 32;  // 32-wide blocks of the head dimension
    constexpr int kRowBytes = D * 2;
    constexpr int kRowsPerLoad = 1024 / kRowBytes;    // rows one 1 KB global->LDS load covers
    constexpr int kChunksPerRow = kRowBytes / 16;
    constexpr int kLoadsPerWave = 16 / kRowsPerLoad;  // a wave fills 16 of the 64 rows of a tile
    __shared__ FwdSmem<D> sm;

    const int tile = xcd_remap(blockIdx.x, total_tiles);
    const int bh = tile / num_qtiles;
    const int q0 = (tile % num_qtiles) * BR;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, lq = lane & 31;
    const float sl = scale_log2;
    const float inv_scale = kLog2e / scale_log2;
    const float thr = 8.0f / scale_log2;  // growth of the running max (raw units) that forces a rescale

    const size_t head_off = (size_t)bh * N * D;
    const char* Kh = reinterpret_cast<const char*>(K + head_off);
    const char* Vh = reinterpret_cast<const char*>(V + head_off);
    const float* ch = c + (size_t)bh * N;
    const float cbase = ch[q0];

    const int qw0 = q0 + wv * 32;  // first query of this wave
    const int t = qw0 + lq;

    // Q^T fragments (B operand), resident for the whole tile loop (rows past N read row N-1)
    bf16x8 qf[KC];
    {
        const bf16_t* qp = Q + head_off + (size_t)min(t, N - 1) * D + 8 * h;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) qf[kc] = *reinterpret_cast<const bf16x8*>(qp + 16 * kc);
    }
    const float cq = ch[min(t, N - 1)] - cbase;

    // key tiles that intersect the band of this query tile (window-aware pruning of Alg. 2)
    const int k_lo = max(0, q0 - w + 1);
    const int k_hi = min(N, q0 + BR) - 1;
    const int j_lo = k_lo / kBC, j_hi = k_hi / kBC;
    const int jfull = N / kBC;  // tiles below jfull have all 64 rows inside the sequence

    // global -> LDS: wave wv fills rows 16wv..16wv+15 of a tile; lane p of a load writes row p /
    // chunks-per-row of its group at physical chunk p % chunks-per-row and therefore fetches the
    // logical chunk the swizzle maps there (the swizzle is an involution)
    unsigned dma_off[kLoadsPerWave];
#pragma unroll
    for (int g = 0; g < kLoadsPerWave; ++g) {
        const int row = 16 * wv + kRowsPerLoad * g + lane / kChunksPerRow;
        dma_off[g] = (unsigned)(row * kRowBytes + swz_chunk<D>(row, lane % kChunksPerRow) * 16);
    }
    auto load_tile = [&](int j, int buf) {
        char* kl = sm.k[buf] + 16 * wv * kRowBytes;
        char* vl = sm.v[buf] + 16 * wv * kRowBytes;
        if (j < jfull) {
            const size_t toff = (size_t)j * (kBC * kRowBytes);
#pragma unroll
            for (int g = 0; g < kLoadsPerWave; ++g) {
                dma16(Kh + toff, dma_off[g], kl + g * 1024);
                dma16(Vh + toff, dma_off[g], vl + g * 1024);
            }
        } else {  // ragged last tile: rows past N read row N-1 (finite; masked by causality)
#pragma unroll
            for (int g = 0; g < kLoadsPerWave; ++g) {
                const int row = 16 * wv + kRowsPerLoad * g + lane / kChunksPerRow;
                const int key = min(j * kBC + row, N - 1);
                const unsigned off =
                    (unsigned)key * (unsigned)kRowBytes + (unsigned)(swz_chunk<D>(row, lane % kChunksPerRow) * 16);
                dma16(Kh, off, kl + g * 1024);
                dma16(Vh, off, vl + g * 1024);
            }
        }
    };
    auto gate_of = [&](int j) {  // this thread's g value of tile j (threads 0..63)
        const int key = min(j * kBC + tid, N - 1);
        return (ch[key] - cbase) * inv_scale;
    };

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.0f;
    float m = kNegBig, l = 0.0f;

    load_tile(j_lo, 0);
    if (tid < kBC) sm.g[0][tid] = gate_of(j_lo);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    for (int j = j_lo; j <= j_hi; ++j) {
        const int buf = (j - j_lo) & 1;
        float g_next = 0.f;
        if (j < j_hi) {
            load_tile(j + 1, buf ^ 1);
            if (tid < kBC) g_next = gate_of(j + 1);
        }

        const char* kt = sm.k[buf];
        const char* vt = sm.v[buf];
#pragma unroll
        for (int sb = 0; sb < kBC / 32; ++sb) {
            const int kb0 = j * kBC + 32 * sb;
            // classify this 32-key block against the 32 queries of the wave
            const bool act = (kb0 <= qw0 + 31) && (kb0 + 31 > qw0 - w) && (qw0 < N);
            if (!act) continue;
            const bool full = (kb0 + 31 <= qw0) && (kb0 > qw0 + 31 - w);

            // ---- S^T = g + K Q^T  (accumulator rows 8r + 4h + 0..3 <- g[32 sb + 8r + 4h + 0..3])
            f32x16 s;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const f32x4 g4 = *reinterpret_cast<const f32x4*>(&sm.g[buf][32 * sb + 8 * r + 4 * h]);
                s[4 * r] = g4[0];
                s[4 * r + 1] = g4[1];
                s[4 * r + 2] = g4[2];
                s[4 * r + 3] = g4[3];
            }
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) s = mfma32(lds_read_frag<D>(kt, 32 * sb, kc, lane), qf[kc], s);

            if (!full) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = kb0 + acc_row(v, h);
                    const bool keep = (i <= t) && (i > t - w);
                    s[v] = keep ? s[v] : -INFINITY;
                }
            }
            float mx = fmaxf(fmaxf(s[0], s[1]), s[2]);
            float mx2 = fmaxf(fmaxf(s[8], s[9]), s[10]);
            mx = fmaxf(fmaxf(mx, s[3]), s[4]);
            mx2 = fmaxf(fmaxf(mx2, s[11]), s[12]);
            mx = fmaxf(fmaxf(mx, s[5]), s[6]);
            mx2 = fmaxf(fmaxf(mx2, s[13]), s[14]);
            mx = xhalf_max(fmaxf(fmaxf(mx, s[7]), fmaxf(mx2, s[15])));
            // Raise the running max only when it grows by more than 2^8: p stays <= 256, which
            // bf16 holds as well as any other magnitude, and most blocks need no rescale.
            const bool grow = mx > m + thr;
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                const float mnew = grow ? mx : m;
                const float a = fast_exp2((m - mnew) * sl);
                m = mnew;
                l *= a;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[db][v] *= a;
            }
            const float nm = -m * sl;
            bf16x8 pf[2];
            const bf16x2 one2 = {(bf16_t)1.0f, (bf16_t)1.0f};
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) {
                f32x2 pr = {fast_exp2(fmaf(s[2 * cc], sl, nm)), fast_exp2(fmaf(s[2 * cc + 1], sl, nm))};
                const bf16x2 pb = __builtin_convertvector(pr, bf16x2);
                l = __builtin_amdgcn_fdot2_f32_bf16(pb, one2, l, false);  // per-half partial row sum
                pf[cc >> 2][2 * (cc & 3)] = pb[0];
                pf[cc >> 2][2 * (cc & 3) + 1] = pb[1];
            }

            // ---- O^T += V^T P^T
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int db = 0; db < DB; ++db)
                    o[db] = mfma32(lds_read_tr_frag<D>(vt, 32 * sb + 16 * c2, db, lane), pf[c2], o[db]);
        }

        if (j < j_hi && tid < kBC) sm.g[buf ^ 1][tid] = g_next;
        __builtin_amdgcn_s_waitcnt(vmcnt_only(0));  // this wave's share of tile j+1 has landed
        __syncthreads();
    }

    // ---- epilogue: O = O^T / l, L = ln2 * (m*sl + log2 l) - (c_t - c_base)
    const float lt = xhalf_sum(l);  // the two halves of the wave hold complementary keys
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

template <int D>
static hipError_t launch_fwd(const void* Q, const void* K, const void* V, const float* c, void* O,
                             float* L, int B, int H, int N, int w, float scale, hipStream_t s) {
    constexpr int BR = 128;
    const int num_qtiles = (N + BR - 1) / BR;
    const int total = B * H * num_qtiles;
    ProfScope prof(kKernForward, s);
    hipLaunchKernelGGL((fwd_bf16_kernel<D>), dim3(total), dim3(kFwdThreads), 0, s, (const bf16_t*)Q,
                       (const bf16_t*)K, (const bf16_t*)V, c, (bf16_t*)O, L, N, w, scale * kLog2e, num_qtiles,
                       total);
    return hipGetLastError();
}

hipError_t forward_bf16(const void* Q, const void* K, const void* V, const float* c, void* O, float* L,
                        int B, int H, int N, int d, int w, float scale, hipStream_t s) {
    if (d == 128) return launch_fwd<128>(Q, K, V, c, O, L, B, H, N, w, scale, s);
    return launch_fwd<64>(Q, K, V, c, O, L, B, H, N, w, scale, s);
}

}  // namespace gfwa
