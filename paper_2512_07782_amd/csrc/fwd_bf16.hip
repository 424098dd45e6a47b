// GatedFWA fused forward for bf16 storage on gfx950 (paper Alg. 2, re-designed for CDNA4).
//
// One workgroup (4 waves) owns a tile of BR = 128*QW consecutive queries of one (b,h); wave k owns
// QW blocks of 32 queries.  Key/value tiles of BC = 64 keys are staged through LDS, double
// buffered, and only the tiles that intersect the band [q0-w+1, q0+BR-1] are visited; inside a
// tile every wave skips the 32-key blocks that lie wholly outside the band of its own queries.
//
// The products are formed transposed so that a lane owns one query:
//   S^T[key][query]  = K_tile (A operand, from LDS)  x  Q^T (B operand, registers)
//   O^T[dd][query]  += V_tile^T (A operand, LDS transposing read)  x  P^T (B operand = the S^T
//                      accumulator registers converted to bf16 in place)
// so the row max / row sum of the online softmax are in-lane plus one exchange between the two
// halves of the wave, the rescale factor is a per-lane scalar, and P never leaves registers.
//
// Logits are kept in the exp2 domain: x = (scale*log2e) * s + (c_i - c_base)*log2e.  The per-query
// term -(c_t - c_base) is constant along a row, cancels in the softmax, and is applied only to L.
// c_base = c at the first query of the tile keeps the fp32 differences small (window-local).
#include "gfwa_device.h"
#include "gfwa_internal.h"
#include "tile_stage.h"

namespace gfwa {

constexpr int kFwdThreads = kThreads;
constexpr int kBC = kTileRows;  // keys per LDS tile

template <int D>
struct FwdSmem {
    TilePairSmem<D> kv;  // a = K tile, b = V tile
    alignas(16) float ck[2][kBC];
};

template <int D, int QW>
__global__ __launch_bounds__(kFwdThreads, QW == 1 ? 2 : 1) void fwd_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const float* __restrict__ c, bf16_t* __restrict__ O, float* __restrict__ L, int N, int w,
    float scale_log2, int num_qtiles, int total_tiles) {
    constexpr int BR = 128 * QW;
    constexpr int KC = D / 16;  // MFMA k-chunks along the head dimension
    constexpr int DB = D / 32;  // 32-wide blocks of the head dimension
    __shared__ FwdSmem<D> sm;

    const int tile = xcd_remap(blockIdx.x, total_tiles);
    const int bh = tile / num_qtiles;
    const int q0 = (tile % num_qtiles) * BR;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int h = lane >> 5, lq = lane & 31;

    const size_t head_off = (size_t)bh * N * D;
    const bf16_t* Qh = Q + head_off;
    const bf16_t* Kh = K + head_off;
    const bf16_t* Vh = V + head_off;
    const float* ch = c + (size_t)bh * N;
    const float cbase = ch[q0];

    const int qw0 = q0 + wv * 32 * QW;  // first query of this wave

    // Q^T fragments (B operand), resident for the whole tile loop
    bf16x8 qf[QW][KC];
    float cq[QW];
#pragma unroll
    for (int b = 0; b < QW; ++b) {
        const int t = qw0 + 32 * b + lq;
        if (t < N) {
#pragma unroll
            for (int kc = 0; kc < KC; ++kc)
                qf[b][kc] = *reinterpret_cast<const bf16x8*>(Qh + (size_t)t * D + 16 * kc + 8 * h);
            cq[b] = ch[t] - cbase;
        } else {
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) qf[b][kc] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            cq[b] = 0.0f;
        }
    }

    f32x16 oacc[QW][DB];
    float m[QW], l[QW];
#pragma unroll
    for (int b = 0; b < QW; ++b) {
        m[b] = kNegBig;
        l[b] = 0.0f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[b][db][v] = 0.0f;
    }

    // key tiles that intersect the band of this query tile (window-aware pruning of Alg. 2)
    const int k_lo = max(0, q0 - w + 1);
    const int k_hi = min(N, q0 + BR) - 1;
    const int j_lo = k_lo / kBC, j_hi = k_hi / kBC;

    TilePairRegs<D> stage;
    float ck_stage = 0.0f;
    auto load_ck = [&](int key0) {
        if (tid < kBC) {
            const int key = key0 + tid;
            ck_stage = key < N ? (ch[key] - cbase) * kLog2e : 0.0f;
        }
    };
    stage.load(Kh, Vh, j_lo * kBC, N, tid);
    load_ck(j_lo * kBC);
    stage.store(sm.kv, 0, tid);
    if (tid < kBC) sm.ck[0][tid] = ck_stage;
    __syncthreads();

    for (int j = j_lo; j <= j_hi; ++j) {
        const int buf = (j - j_lo) & 1;
        if (j < j_hi) {
            stage.load(Kh, Vh, (j + 1) * kBC, N, tid);
            load_ck((j + 1) * kBC);
        }

        const char* kt = sm.kv.a[buf];
        const char* vt = sm.kv.b[buf];
#pragma unroll
        for (int sb = 0; sb < kBC / 32; ++sb) {
            const int kb0 = j * kBC + 32 * sb;
            // classify this 32-key block against each 32-query block of the wave
            bool act[QW], full[QW];
            bool any = false;
#pragma unroll
            for (int b = 0; b < QW; ++b) {
                const int qb0 = qw0 + 32 * b;
                act[b] = (kb0 <= qb0 + 31) && (kb0 + 31 > qb0 - w) && (qb0 < N);
                full[b] = (kb0 + 31 <= qb0) && (kb0 > qb0 + 31 - w);
                any |= act[b];
            }
            if (!any) continue;

            // ---- S^T = K Q^T
            f32x16 s[QW];
#pragma unroll
            for (int b = 0; b < QW; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) s[b][v] = 0.0f;
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) {
                const bf16x8 kf = lds_read_frag<D>(kt, 32 * sb, kc, lane);
#pragma unroll
                for (int b = 0; b < QW; ++b)
                    if (act[b]) s[b] = mfma32(kf, qf[b][kc], s[b]);
            }

            // gate bias of the 16 keys this lane sees: ck[8g + 4h + 0..3], g = 0..3
            f32x4 ckv[4];
#pragma unroll
            for (int g = 0; g < 4; ++g)
                ckv[g] = *reinterpret_cast<const f32x4*>(&sm.ck[buf][32 * sb + 8 * g + 4 * h]);

            bf16x8 pf[QW][2];
#pragma unroll
            for (int b = 0; b < QW; ++b) {
                if (!act[b]) continue;
                float x[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) x[v] = fmaf(s[b][v], scale_log2, ckv[v >> 2][v & 3]);
                if (!full[b]) {
                    const int t = qw0 + 32 * b + lq;
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int i = kb0 + acc_row(v, h);
                        const bool keep = (i <= t) && (i > t - w);
                        x[v] = keep ? x[v] : -INFINITY;
                    }
                }
                float mx = x[0];
#pragma unroll
                for (int v = 1; v < 16; ++v) mx = fmaxf(mx, x[v]);
                mx = xhalf_max(mx);
                // Raise the running max only when it grows by more than 2^8: p stays <= 256,
                // which fp32/bf16 hold exactly as well, and most blocks need no rescale.
                const bool grow = mx > m[b] + 8.0f;
                if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                    const float mnew = grow ? mx : m[b];
                    const float a = fast_exp2(m[b] - mnew);
                    m[b] = mnew;
                    l[b] *= a;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int v = 0; v < 16; ++v) oacc[b][db][v] *= a;
                }
                float ls = 0.0f;
                float p[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    p[v] = fast_exp2(x[v] - m[b]);
                    ls += p[v];
                }
                l[b] += ls;  // per-half partial sum; the halves are added once at the end
                acc_to_bfrag(p, pf[b]);
            }

            // ---- O^T += V^T P^T
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const bf16x8 vf = lds_read_tr_frag<D>(vt, 32 * sb + 16 * c2, db, lane);
#pragma unroll
                    for (int b = 0; b < QW; ++b)
                        if (act[b]) oacc[b][db] = mfma32(vf, pf[b][c2], oacc[b][db]);
                }
        }

        if (j < j_hi) {
            stage.store(sm.kv, buf ^ 1, tid);
            if (tid < kBC) sm.ck[buf ^ 1][tid] = ck_stage;
        }
        __syncthreads();
    }

    // ---- epilogue: O = O^T / l, L = ln2 * (m + log2 l) - (c_t - c_base)
#pragma unroll
    for (int b = 0; b < QW; ++b) {
        const int t = qw0 + 32 * b + lq;
        const float lt = xhalf_sum(l[b]);
        if (t >= N) continue;
        const float inv = 1.0f / lt;
        bf16_t* orow = O + head_off + (size_t)t * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 o4 = {oacc[b][db][4 * g] * inv, oacc[b][db][4 * g + 1] * inv,
                            oacc[b][db][4 * g + 2] * inv, oacc[b][db][4 * g + 3] * inv};
                bf16x4 ob = __builtin_convertvector(o4, bf16x4);
                *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * g + 4 * h) = ob;
            }
        if (h == 0) L[(size_t)bh * N + t] = (m[b] + fast_log2(lt)) * kLn2 - cq[b];
    }
}

template <int D, int QW>
static hipError_t launch_fwd(const void* Q, const void* K, const void* V, const float* c, void* O,
                             float* L, int B, int H, int N, int w, float scale, hipStream_t s) {
    constexpr int BR = 128 * QW;
    const int num_qtiles = (N + BR - 1) / BR;
    const int total = B * H * num_qtiles;
    ProfScope prof(kKernForward, s);
    hipLaunchKernelGGL((fwd_bf16_kernel<D, QW>), dim3(total), dim3(kFwdThreads), 0, s,
                       (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, c, (bf16_t*)O, L, N, w,
                       scale * kLog2e, num_qtiles, total);
    return hipGetLastError();
}

hipError_t forward_bf16(const void* Q, const void* K, const void* V, const float* c, void* O, float* L,
                        int B, int H, int N, int d, int w, float scale, int variant, hipStream_t s) {
    if (d == 128) {
        return variant == 1 ? launch_fwd<128, 2>(Q, K, V, c, O, L, B, H, N, w, scale, s)
                            : launch_fwd<128, 1>(Q, K, V, c, O, L, B, H, N, w, scale, s);
    }
    return variant == 1 ? launch_fwd<64, 2>(Q, K, V, c, O, L, B, H, N, w, scale, s)
                        : launch_fwd<64, 1>(Q, K, V, c, O, L, B, H, N, w, scale, s);
}

}  // namespace gfwa
