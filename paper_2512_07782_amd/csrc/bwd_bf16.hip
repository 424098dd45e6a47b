// GatedFWA backward for bf16 storage on gfx950 (paper App. E.2 / Alg. 3, re-designed for CDNA4).
//
// Four launches, no atomics, deterministic:
//   1. rowdot:   D_t = <O_t, dO_t>                                   (HBM-bound)
//   2. dkv:      key-stationary.  A wave works on 32 keys, whose K and V are MFMA B operands (in
//                registers at d = 64, staged in LDS at d = 128, see the two kernels), and streams
//                64-query tiles of Q and dO through LDS (direct global->LDS loads):
//                  S[q][k]   = Q (A, LDS)       x K^T (B)            P  = exp2(x - L)
//                  dP[q][k]  = dO (A, LDS)      x V^T (B)  - D       dS = P (dP - D)
//                  dV^T[dd][k] += dO^T (A, LDS transposing read) x P  (B = accumulator registers)
//                  dK^T[dd][k] += Q^T  (A, LDS transposing read) x dS (B = accumulator registers)
//                plus the column sums of dS.  A lane owns one key.
//   3. dq:       query-stationary, the forward's layout.  A lane owns one query:
//                  S^T[k][q] = K (A, LDS) x Q^T (B, regs)   dP^T[k][q] = V (A, LDS) x dO^T (B, regs) - D
//                  dQ^T[dd][q] += K^T (A, LDS transposing read) x dS^T (B = accumulator registers)
//                plus the row sums of dS.
//   3b. (d = 128, when the caller's workspace has room) dq from the dS blocks that launch 2 then stores: one
//                matrix product instead of three, see "dS spill" below
//   4. reverse scan of (column sums - row sums) -> dalpha   (gate_scan.hip)
// In both kernels the row- (dkv) or key- (dq) dependent part of the exponent rides in the MFMA
// accumulator (it is initialised from an LDS vector before the product), the lane-constant part is
// the addend of the single fused multiply-add in front of exp2; the dP accumulator starts from -D.
// The row sums are analytically zero but are kept: with D formed from the rounded O they carry
// exactly the error that would otherwise accumulate over the whole suffix in the reverse scan.
#include "gfwa_device.h"
#include "gfwa_internal.h"
#include "tile_stage.h"

namespace gfwa {

constexpr float kPosBig = 1.0e30f;

// ------------------------------------------------------------------------------------------
// 1. D_t = <O_t, dO_t>
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void rowdot_bf16_kernel(const bf16_t* __restrict__ O,
                                                          const bf16_t* __restrict__ dO,
                                                          float* __restrict__ Dv, long rows) {
    constexpr int LPR = D / 8;  // lanes per row, 16 bytes each
    const long gid = (long)blockIdx.x * 256 + threadIdx.x;
    const long r = gid / LPR;
    const int part = (int)(gid % LPR);
    float acc = 0.f;
    if (r < rows) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(O + r * D + part * 8);
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(dO + r * D + part * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf((float)a[e], (float)b[e], acc);
    }
#pragma unroll
    for (int d = LPR / 2; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if (r < rows && part == 0) Dv[r] = acc;
}

// ------------------------------------------------------------------------------------------
// 2. dK, dV, column sums: key-stationary
// ------------------------------------------------------------------------------------------
template <int D>
struct DkvSmem {
    TilePairSmem<D> qg;                    // a = Q tile, b = dO tile
    alignas(16) float nl[2][kTileRows];    // -(L_t + c_t - c_base) / scale; -big for rows >= N
    alignas(16) float dvec[2][kTileRows];  // -D_t
};

template <int D>
__global__ __launch_bounds__(kThreads, 1) void bwd_dkv_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ c, const float* __restrict__ L,
    const float* __restrict__ Dv, bf16_t* __restrict__ dK, bf16_t* __restrict__ dV,
    float* __restrict__ dc_col, int N, int w, float scale, int num_ktiles, int total_tiles, int H, int G) {
    constexpr int BK = 128;  // keys per workgroup, 32 per wave
    constexpr int KC = D / 16, DB = D / 32;
    __shared__ DkvSmem<D> sm;

    const int tile = xcd_remap(blockIdx.x, total_tiles);
    const int bkv = tile / num_ktiles;  // flat key/value head; its G query heads are visited in turn
    const int k0 = (tile % num_ktiles) * BK;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, lk = lane & 31;
    const float sl = scale * kLog2e;
    const float inv_scale = 1.0f / scale;

    const size_t head_off = (size_t)bkv * N * D;
    const int Hkv = H / G;
    const int bh0 = (bkv / Hkv) * H + (bkv % Hkv) * G;  // first query head of the group

    const int kw0 = k0 + 32 * wv;  // first key of this wave
    const int key = kw0 + lk;

    // K^T and V^T fragments (B operands: column = key, k = head dimension), resident
    bf16x8 kf[KC], vf[KC];
    {
        const size_t roff = head_off + (size_t)min(key, N - 1) * D + 8 * h;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            kf[kc] = *reinterpret_cast<const bf16x8*>(K + roff + 16 * kc);
            vf[kc] = *reinterpret_cast<const bf16x8*>(V + roff + 16 * kc);
        }
    }

    f32x16 dk_acc[DB], dv_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            dk_acc[db][v] = 0.f;
            dv_acc[db][v] = 0.f;
        }

    // queries that can see a key of this tile: k0 <= t <= min(N-1, k0+BK-1+w-1)
    const int t_hi = (int)min((long)N - 1, (long)k0 + BK - 1 + (long)w - 1);
    const int i_lo = k0 / kTileRows, i_hi = t_hi / kTileRows;
    const int ifull = N / kTileRows;

    TilePairLoader<D> loader;
    loader.init(wv, lane);
    for (int qh = 0; qh < G; ++qh) {
        const int bh = bh0 + qh;
        const size_t qhead_off = (size_t)bh * N * D;
        const char* Qh = reinterpret_cast<const char*>(Q + qhead_off);
        const char* Gh = reinterpret_cast<const char*>(dO + qhead_off);
        const float* ch = c + (size_t)bh * N;
        const float* Lh = L + (size_t)bh * N;
        const float* Dh = Dv + (size_t)bh * N;
        const float cbase = ch[k0];
        const float ckl = (ch[min(key, N - 1)] - cbase) * kLog2e;  // lane-constant part of the exponent
        float colsum = 0.f;
        // per-row vectors of query tile i, one row per thread of the first wave
        // (the loaded values are only touched in store_vec, a tile later: arithmetic on them right here
        // would make the first wave wait for them, and for the tile loads issued just before, in every tile)
        float l_stage = kPosBig, c_stage = 0.f, d_stage = 0.f;
        auto load_vec = [&](int i) {
            if (tid < kTileRows) {
                const int t = i * kTileRows + tid;
                if (t < N) {
                    l_stage = Lh[t];
                    c_stage = ch[t];
                    d_stage = Dh[t];
                } else {
                    l_stage = kPosBig;
                    c_stage = cbase;
                    d_stage = 0.f;
                }
            }
        };
        auto store_vec = [&](int buf) {
            if (tid < kTileRows) {
                sm.nl[buf][tid] = -(l_stage + (c_stage - cbase)) * inv_scale;
                sm.dvec[buf][tid] = -d_stage;
            }
        };
        loader.load(Qh, Gh, i_lo, ifull, N, sm.qg.a[0], sm.qg.b[0]);
        load_vec(i_lo);
        store_vec(0);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();

        for (int i = i_lo; i <= i_hi; ++i) {
            const int buf = (i - i_lo) & 1;
            if (i < i_hi) {  // the plain loads first: whatever wait the compiler puts in front of them must not cover the tile loads
                load_vec(i + 1);
                loader.load(Qh, Gh, i + 1, ifull, N, sm.qg.a[buf ^ 1], sm.qg.b[buf ^ 1]);
            }
            const char* qt = sm.qg.a[buf];
            const char* gt = sm.qg.b[buf];
#pragma unroll
            for (int sb = 0; sb < kTileRows / 32; ++sb) {
                const int qb0 = i * kTileRows + 32 * sb;
                const bool act = (kw0 <= qb0 + 31) && (kw0 + 31 > qb0 - w) && (kw0 < N) && (qb0 < N);
                if (!act) continue;
                const bool full = (kw0 + 31 <= qb0) && (kw0 > qb0 + 31 - w);

                // S[q][k] starts from the row term of the exponent, dP from -D_t (so that the accumulator
                // ends as dP - D, the factor of dS, without a subtraction per element).  The fragment reads
                // run kAhead products ahead of the MFMAs, in an explicit one-read-per-MFMA pipeline.
                constexpr int kAhead = D == 128 ? 4 : 2;  // what the register budget of two waves per SIMD allows
                f32x16 s, dp;
                acc_init_rows(s, sm.nl[buf], 32 * sb, h);
                acc_init_rows(dp, sm.dvec[buf], 32 * sb, h);
                {
                    bf16x8 fr[2 * KC];
                    auto fetch = [&](int f) __attribute__((always_inline)) {
                        fr[f] = lds_read_frag<D>(f < KC ? qt : gt, 32 * sb, f % KC, lane);
                    };
#pragma unroll
                    for (int f = 0; f < kAhead; ++f) fetch(f);
                    __builtin_amdgcn_sched_group_barrier(0x100, 8 + kAhead, 0);
#pragma unroll
                    for (int f = 0; f < 2 * KC; ++f) {
                        if (f < KC) s = mfma32(fr[f], kf[f], s);
                        else dp = mfma32(fr[f], vf[f - KC], dp);
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if (f + kAhead < 2 * KC) {
                            fetch(f + kAhead);
                            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        }
                    }
                }
                float p[16], ds[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) p[v] = fast_exp2(fmaf(s[v], sl, ckl));
                if (!full) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int t = qb0 + acc_row(v, h);
                        const bool keep = (key <= t) && (key > t - w);
                        p[v] = keep ? p[v] : 0.f;
                    }
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    ds[v] = p[v] * dp[v];
                    colsum += ds[v];
                }
                bf16x8 pf[2], dsf[2];
                acc_to_bfrag(p, pf);
                acc_to_bfrag(ds, dsf);
                {
                    constexpr int NB = 4 * DB;  // products: (c2, db, dV | dK)
                    bf16x8 fr[NB];
                    auto fetch = [&](int f) __attribute__((always_inline)) {
                        const int c2 = f / (2 * DB), db = (f / 2) % DB;
                        fr[f] = lds_read_tr_frag<D>((f & 1) ? qt : gt, 32 * sb + 16 * c2, db, lane);
                    };
#pragma unroll
                    for (int f = 0; f < kAhead; ++f) fetch(f);
                    __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0);
#pragma unroll
                    for (int f = 0; f < NB; ++f) {
                        const int c2 = f / (2 * DB), db = (f / 2) % DB;
                        if (f & 1) dk_acc[db] = mfma32(fr[f], dsf[c2], dk_acc[db]);
                        else dv_acc[db] = mfma32(fr[f], pf[c2], dv_acc[db]);
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if (f + kAhead < NB) {
                            fetch(f + kAhead);
                            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                        }
                    }
                }
            }
            if (i < i_hi) store_vec(buf ^ 1);
            __builtin_amdgcn_s_waitcnt(vmcnt_only(0));  // this wave's share of tile i+1 has landed
            __syncthreads();
        }

        const float cs = xhalf_sum(colsum);
        if (key < N && h == 0) dc_col[(size_t)bh * N + key] = cs;
    }  // query heads of the group

    // dK and dV as whole lines, through 4 KB per wave of the tile buffers (free since the last barrier)
    {
        char* stage = sm.qg.a[0] + 4096 * wv;
        const size_t row0 = head_off + (size_t)kw0 * D;
        store_acc_rows<DB>(dk_acc, scale, stage, dK + row0, N - kw0, lane);
        store_acc_rows<DB>(dv_acc, 1.0f, stage, dV + row0, N - kw0, lane);
    }
}

// dS spill (d = 128, optional).  With a workspace of N x (w + 32..63) bf16 per head the dK/dV kernel also
// stores the dS blocks it forms, and dQ = dS K is computed from them by a kernel that reads them back
// instead of forming S and dP a second time: 5 executed matrix products instead of 7, for
// 2 x 2 KB of memory traffic per 32 x 32 block.  Layout: block (head bh, 32-query block qb, 32-key block kb)
// lives at slot kb - qb + nslot - 1 of the nslot = (w + 30) / 32 + 1 slots of (bh, qb); a block is two
// pieces of 1 KB (query halves c2 = 0, 1 of the block); piece c2 holds, for key k of the block and
// register half h, the 16 bytes  dS[q = 16 c2 + 4 h + 0..3][k], dS[q = 16 c2 + 8 + 4 h + 0..3][k]  (exactly the
// B-operand fragment of the dK product) at 16-byte slot 32 h + k, i.e. in lane order: a store writes 1 KB
// front to back.  The reader permutes while it copies a piece into LDS (slot (2 k + h + 8 c2) mod 64 there), so
// that a transposing LDS read of 4 keys x 16 queries touches 128 contiguous bytes.
__host__ __device__ inline int ds_spill_slots(int w, int nqb) {
    const long s = ((long)w + 30) / 32 + 1;
    return (int)(s < nqb ? s : nqb);
}
constexpr int kSpillBlockBytes = 2048;

// 8-wave variant (d = 128): two waves per SIMD.  The workgroup still owns 128 keys, but two waves work
// on every key group and take one of the two 32-query blocks of every tile each, so that on every SIMD
// one wave's MFMAs run while the other does its softmax arithmetic or waits for LDS.  Two waves per
// SIMD leave 256 registers per wave: the dK, dV accumulators (128) and
// S, dP (32) stay, the K and V fragments do not - the 128 keys of K and V are staged in LDS once per
// workgroup and read as B operands like the Q and dO tiles are read as A operands.  At the end the
// two waves of a key group trade halves of their accumulators through LDS: one ends with the whole dK,
// the other with the whole dV, and each stores its matrix.
template <int D>
struct Dkv8Smem {
    union {
        DkvSmem<D> t;
        float red[4][16 * (D / 32)][64];  // exchange space of the final reduction (64 KB at d = 128), over the tile buffers
    };
    TilePairSmem<D> kv;  // a = the two 64-key tiles of K, b = of V
    float colred[4][32];
};

template <int D, bool SPILL>
__global__ __launch_bounds__(2 * kThreads, 1) void bwd_dkv8_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ c, const float* __restrict__ L,
    const float* __restrict__ Dv, bf16_t* __restrict__ dK, bf16_t* __restrict__ dV,
    float* __restrict__ dc_col, char* __restrict__ ds_ws, int N, int w, float scale, int num_ktiles,
    int total_tiles, int H, int G) {
    constexpr int BK = 128;  // keys per workgroup, 32 per wave
    constexpr int KC = D / 16, DB = D / 32;
    __shared__ Dkv8Smem<D> sm8;
    auto& sm = sm8.t;

    const int tile = xcd_remap(blockIdx.x, total_tiles);
    const int bkv = tile / num_ktiles;  // flat key/value head; its G query heads are visited in turn
    const int k0 = (tile % num_ktiles) * BK;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    // 32-key group kg and 32-query block `half` of every tile.  The two waves of a key group sit on different
    // SIMDs (wave w runs on SIMD w % 4): in the tiles at the diagonal and at the far end of the window, where only
    // some key groups have work, the active waves then spread over the SIMDs instead of pairing up on one.
    const int half = wv >> 2;
    const int kg = (wv + 2 * half) & 3;
    const int h = lane >> 5, lk = lane & 31;
    const float sl = scale * kLog2e;
    const float inv_scale = 1.0f / scale;

    const size_t head_off = (size_t)bkv * N * D;
    const int Hkv = H / G;
    const int bh0 = (bkv / Hkv) * H + (bkv % Hkv) * G;  // first query head of the group

    const int kw0 = k0 + 32 * kg;  // first key of this wave
    const int key = kw0 + lk;

    // K^T and V^T fragments (B operands: column = key, k = head dimension) come from the staged tiles
    const char* ktile = sm8.kv.a[kg >> 1];
    const char* vtile = sm8.kv.b[kg >> 1];
    const int krow0 = 32 * (kg & 1);

    f32x16 dk_acc[DB], dv_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            dk_acc[db][v] = 0.f;
            dv_acc[db][v] = 0.f;
        }

    // queries that can see a key of this tile: k0 <= t <= min(N-1, k0+BK-1+w-1)
    const int t_hi = (int)min((long)N - 1, (long)k0 + BK - 1 + (long)w - 1);
    const int i_lo = k0 / kTileRows, i_hi = t_hi / kTileRows;
    const int ifull = N / kTileRows;

    // dS spill: 32-query blocks per head, slots per query block, this lane's 16-byte slot in the two pieces
    const int nqb = (N + 31) / 32;
    const int nslot = ds_spill_slots(w, nqb);
    const int spill_lane0 = 16 * lane;  // (the second piece: + 1024, an immediate of its store)

    TilePairLoader<D, 8> loader;
    loader.init(wv, lane);
    {  // K and V of the 128 keys; the wait and barrier in front of the first query tile cover them
        const char* Kh = reinterpret_cast<const char*>(K + head_off);
        const char* Vh = reinterpret_cast<const char*>(V + head_off);
        loader.load(Kh, Vh, k0 / kTileRows, ifull, N, sm8.kv.a[0], sm8.kv.b[0]);
        loader.load(Kh, Vh, k0 / kTileRows + 1, ifull, N, sm8.kv.a[1], sm8.kv.b[1]);
    }
    for (int qh = 0; qh < G; ++qh) {
        const int bh = bh0 + qh;
        const size_t qhead_off = (size_t)bh * N * D;
        const char* Qh = reinterpret_cast<const char*>(Q + qhead_off);
        const char* Gh = reinterpret_cast<const char*>(dO + qhead_off);
        const float* ch = c + (size_t)bh * N;
        const float* Lh = L + (size_t)bh * N;
        const float* Dh = Dv + (size_t)bh * N;
        const float cbase = ch[k0];
        const float ckl = (ch[min(key, N - 1)] - cbase) * kLog2e;  // lane-constant part of the exponent
        float colsum = 0.f;
        // per-row vectors of query tile i, one row per thread of the first wave
        // (the loaded values are only touched in store_vec, a tile later: arithmetic on them right here
        // would make the first wave wait for them, and for the tile loads issued just before, in every tile)
        float l_stage = kPosBig, c_stage = 0.f, d_stage = 0.f;
        auto load_vec = [&](int i) {
            if (tid < kTileRows) {
                // (per-lane values that only rare paths need are re-derived in place, see GFWA_PIN, rather
                // than carried through the tile loop as one more induction register each)
                int tid_l = tid;
                GFWA_PIN(tid_l);
                const int t = i * kTileRows + tid_l;
                if (t < N) {
                    l_stage = Lh[t];
                    c_stage = ch[t];
                    d_stage = Dh[t];
                } else {
                    l_stage = kPosBig;
                    c_stage = cbase;
                    d_stage = 0.f;
                }
            }
        };
        auto store_vec = [&](int buf) {
            if (tid < kTileRows) {
                sm.nl[buf][tid] = -(l_stage + (c_stage - cbase)) * inv_scale;
                sm.dvec[buf][tid] = -d_stage;
            }
        };
        loader.load(Qh, Gh, i_lo, ifull, N, sm.qg.a[0], sm.qg.b[0]);
        load_vec(i_lo);
        store_vec(0);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();

        for (int i = i_lo; i <= i_hi; ++i) {
            const int buf = (i - i_lo) & 1;
            if (i < i_hi) {  // the plain loads first: whatever wait the compiler puts in front of them must not cover the tile loads
                load_vec(i + 1);
                loader.load(Qh, Gh, i + 1, ifull, N, sm.qg.a[buf ^ 1], sm.qg.b[buf ^ 1]);
            }
            const char* qt = sm.qg.a[buf];
            const char* gt = sm.qg.b[buf];
            bool stored = false, vec_done = false;
            {
                const int sb = half;
                const int qb0 = i * kTileRows + 32 * sb;
                const bool act = (kw0 <= qb0 + 31) && (kw0 + 31 > qb0 - w) && (kw0 < N) && (qb0 < N);
                stored = act;
                if (act) {
                const bool full = (kw0 + 31 <= qb0) && (kw0 > qb0 + 31 - w);

                // S[q][k] starts from the row term of the exponent, dP from -D_t (so that the accumulator
                // ends as dP - D, the factor of dS, without a subtraction per element).  The fragment reads
                // run kAhead products ahead of the MFMAs, in an explicit one-read-per-MFMA pipeline.
                constexpr int kAhead = 2;
                f32x16 s, dp;
                acc_init_rows(s, sm.nl[buf], 32 * sb, h);
                acc_init_rows(dp, sm.dvec[buf], 32 * sb, h);
                if (D != 128) {  // d = 64 runs two waves per SIMD, which hide the reads by themselves
#pragma unroll
                    for (int kc = 0; kc < KC; ++kc)
                        s = mfma32(lds_read_frag<D>(qt, 32 * sb, kc, lane), lds_read_frag<D>(ktile, krow0, kc, lane), s);
#pragma unroll
                    for (int kc = 0; kc < KC; ++kc)
                        dp = mfma32(lds_read_frag<D>(gt, 32 * sb, kc, lane), lds_read_frag<D>(vtile, krow0, kc, lane), dp);
                } else {
                    bf16x8 fr[2 * KC], fk[2 * KC];
                    auto fetch = [&](int f) __attribute__((always_inline)) {
                        fr[f] = lds_read_frag<D>(f < KC ? qt : gt, 32 * sb, f % KC, lane);
                        fk[f] = lds_read_frag<D>(f < KC ? ktile : vtile, krow0, f % KC, lane);
                    };
#pragma unroll
                    for (int f = 0; f < kAhead; ++f) fetch(f);
                    __builtin_amdgcn_sched_group_barrier(0x100, 8 + 2 * kAhead, 0);
#pragma unroll
                    for (int f = 0; f < 2 * KC; ++f) {
                        if (f < KC) s = mfma32(fr[f], fk[f], s);
                        else dp = mfma32(fr[f], fk[f], dp);
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if (f + kAhead < 2 * KC) {
                            fetch(f + kAhead);
                            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                        }
                    }
                }
                float p[16], ds[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) p[v] = fast_exp2(fmaf(s[v], sl, ckl));
                if (!full) {
                    int h_l = h;
                    GFWA_PIN(h_l);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int t = qb0 + acc_row(v, h_l);
                        const bool keep = (key <= t) && (key > t - w);
                        p[v] = keep ? p[v] : 0.f;
                    }
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    ds[v] = p[v] * dp[v];
                    if (!SPILL) colsum += ds[v];
                }
                // (the first wave hands over the row vectors of the next tile here, before the stores below:
                // the wait in front of their first use would otherwise cover the stores too)
                if (SPILL && i < i_hi) {
                    store_vec(buf ^ 1);
                    vec_done = true;
                }
                bf16x8 pf[2], dsf[2];
                acc_to_bfrag(p, pf);
                acc_to_bfrag(ds, dsf);
                if (SPILL) {
                    // the column sums take the rounded values the dQ kernel will sum along the rows, so that
                    // the two cancel exactly in the suffix sums of the gate gradient; then the block is stored
                    // (two values per instruction through the bf16 dot product with ones: a quarter of the vector
                    // instructions of convert-and-add, and in this phase no MFMA of this wave is waiting behind it)
                    const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
#pragma unroll
                    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                        for (int e = 0; e < 8; e += 2)
                            colsum = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{dsf[c2][e], dsf[c2][e + 1]}, ones, colsum, false);
                    const int qb = 2 * i + sb, kb = kw0 >> 5;
                    char* blk = ds_ws + (((size_t)bh * nqb + qb) * nslot + (kb - qb + nslot - 1)) * kSpillBlockBytes;
                    // streaming stores: the blocks are read once, by the next kernel, and must not push the
                    // Q and dO tiles the neighbouring workgroups are about to re-read out of the L2
                    // Written as instructions, not as stores the compiler may split, merge or move: the wait at the
                    // end of the tile is s_waitcnt vmcnt(2), which leaves exactly these two in flight and therefore
                    // counts on both having been issued after the tile's direct global->LDS loads and before it.
                    stream_store16<0>(uniform_ptr(blk), (unsigned)spill_lane0, dsf[0]);
                    stream_store16<1024>(uniform_ptr(blk), (unsigned)spill_lane0, dsf[1]);
                }
                if (D != 128) {
#pragma unroll
                    for (int c2 = 0; c2 < 2; ++c2)
#pragma unroll
                        for (int db = 0; db < DB; ++db) {
                            dv_acc[db] = mfma32(lds_read_tr_frag<D>(gt, 32 * sb + 16 * c2, db, lane), pf[c2], dv_acc[db]);
                            dk_acc[db] = mfma32(lds_read_tr_frag<D>(qt, 32 * sb + 16 * c2, db, lane), dsf[c2], dk_acc[db]);
                        }
                } else {
                    constexpr int NB = 4 * DB;  // products: (c2, db, dV | dK)
                    bf16x8 fr[NB];
                    auto fetch = [&](int f) __attribute__((always_inline)) {
                        const int c2 = f / (2 * DB), db = (f / 2) % DB;
                        fr[f] = lds_read_tr_frag<D>((f & 1) ? qt : gt, 32 * sb + 16 * c2, db, lane);
                    };
                    // the two stores of a spilled block go first: their latency hides behind the 16 MFMAs
                    if (SPILL) __builtin_amdgcn_sched_group_barrier(0x040, 2, 0);
#pragma unroll
                    for (int f = 0; f < kAhead; ++f) fetch(f);
                    __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0);
#pragma unroll
                    for (int f = 0; f < NB; ++f) {
                        const int c2 = f / (2 * DB), db = (f / 2) % DB;
                        if (f & 1) dk_acc[db] = mfma32(fr[f], dsf[c2], dk_acc[db]);
                        else dv_acc[db] = mfma32(fr[f], pf[c2], dv_acc[db]);
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if (f + kAhead < NB) {
                            fetch(f + kAhead);
                            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                        }
                    }
                }
                }
            }
            if (i < i_hi && !vec_done) store_vec(buf ^ 1);
            // this wave's share of tile i+1 has landed; the two stores of a spilled block were issued after
            // those loads and may stay in flight
            if (SPILL && stored) __builtin_amdgcn_s_waitcnt(vmcnt_only(2));
            else __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
            wg_barrier();  // not __syncthreads: its fence would wait for the stores as well
        }

        // column sums of the two query halves
        float cs = xhalf_sum(colsum);
        if (half == 1 && h == 0) sm8.colred[kg][lk] = cs;
        __syncthreads();
        if (half == 0 && h == 0) {
            cs += sm8.colred[kg][lk];
            if (key < N) dc_col[(size_t)bh * N + key] = cs;
        }
    }  // query heads of the group

    // The two waves of a key group hold partial dK and dV (one 32-query block of every tile each).  They trade
    // halves through LDS (the tile buffers are free now): the wave of half 0 ends up with the whole dK, the wave
    // of half 1 with the whole dV, and each stores its matrix.  Two sub-passes of two 32-column blocks each, so
    // that the eight waves' pieces fit the 64 KB; 16-byte LDS accesses, [wave][register group][lane].
    {
        f32x4* xch = reinterpret_cast<f32x4*>(&sm8.red[0][0][0]);
        constexpr int kGroups = 8;  // register groups of 4 per sub-pass and wave: 2 blocks x 16 registers
        const int ow = half == 0 ? 4 + ((kg + 2) & 3) : kg;  // the other wave of this key group
        auto put = [&](const f32x16 (&arr)[DB], int sub) __attribute__((always_inline)) {
#pragma unroll
            for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x16& a = arr[2 * sub + b2];
                    xch[(wv * kGroups + 4 * b2 + g) * 64 + lane] = f32x4{a[4 * g], a[4 * g + 1], a[4 * g + 2], a[4 * g + 3]};
                }
        };
        auto add = [&](f32x16 (&arr)[DB], int sub) __attribute__((always_inline)) {
#pragma unroll
            for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 x = xch[(ow * kGroups + 4 * b2 + g) * 64 + lane];
                    f32x16& a = arr[2 * sub + b2];
                    a[4 * g] += x[0];
                    a[4 * g + 1] += x[1];
                    a[4 * g + 2] += x[2];
                    a[4 * g + 3] += x[3];
                }
        };
#pragma unroll
        for (int sub = 0; sub < DB / 2; ++sub) {
            __syncthreads();
            if (half == 0) put(dv_acc, sub);
            else put(dk_acc, sub);
            __syncthreads();
            if (half == 0) add(dk_acc, sub);
            else add(dv_acc, sub);
        }
    }

    // Each wave stores its matrix as whole lines, through 4 KB of the K/V staging area (free since the last tile).
    {
        char* stage = sm8.kv.a[0] + 4096 * wv;
        const size_t row0 = head_off + (size_t)kw0 * D;
        if (half == 0) store_acc_rows<DB>(dk_acc, scale, stage, dK + row0, N - kw0, lane);
        else store_acc_rows<DB>(dv_acc, 1.0f, stage, dV + row0, N - kw0, lane);
    }
}

// ------------------------------------------------------------------------------------------
// 3. dQ, row sums: query-stationary
// ------------------------------------------------------------------------------------------
template <int D>
struct DqSmem {
    TilePairSmem<D> kv;                // a = K tile, b = V tile
    alignas(16) float g[2][kTileRows];  // (c - c_base) / scale
};

template <int D>
__global__ __launch_bounds__(kThreads, 2) void bwd_dq_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ c, const float* __restrict__ L,
    const float* __restrict__ Dv, bf16_t* __restrict__ dQ, float* __restrict__ dc_row, int N, int w,
    float scale, int num_qtiles, int total_tiles, int H, int G) {
    constexpr int BR = 128;
    constexpr int KC = D / 16, DB = D / 32;
    __shared__ DqSmem<D> sm;

    const int tile = xcd_remap(blockIdx.x, total_tiles);
    const int bh = tile / num_qtiles;
    const int q0 = (tile % num_qtiles) * BR;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, lq = lane & 31;
    const float sl = scale * kLog2e;
    const float inv_scale = 1.0f / scale;

    const size_t head_off = (size_t)bh * N * D;
    const size_t kv_off = (size_t)kv_head_of(bh, H, G) * N * D;
    const char* Kh = reinterpret_cast<const char*>(K + kv_off);
    const char* Vh = reinterpret_cast<const char*>(V + kv_off);
    const float* ch = c + (size_t)bh * N;
    const float cbase = ch[q0];

    const int qw0 = q0 + 32 * wv;
    const int t = qw0 + lq;

    // Q^T and dO^T fragments (B operands: column = query), resident; rows past N read row N-1 and
    // get an exponent of -big, i.e. p = 0
    bf16x8 qf[KC], gf[KC];
    {
        const size_t roff = head_off + (size_t)min(t, N - 1) * D + 8 * h;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
            qf[kc] = *reinterpret_cast<const bf16x8*>(Q + roff + 16 * kc);
            gf[kc] = *reinterpret_cast<const bf16x8*>(dO + roff + 16 * kc);
        }
    }
    float nlsub = -kPosBig, ndt = 0.f;  // lane-constant part of the exponent: -(L_t + c_t - c_base) log2 e
    if (t < N) {
        nlsub = -(L[(size_t)bh * N + t] + (ch[t] - cbase)) * kLog2e;
        ndt = -Dv[(size_t)bh * N + t];
    }

    f32x16 dq_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) dq_acc[db][v] = 0.f;
    float rowsum = 0.f;

    const int k_lo = max(0, q0 - w + 1);
    const int k_hi = min(N, q0 + BR) - 1;
    const int j_lo = k_lo / kTileRows, j_hi = k_hi / kTileRows;
    const int jfull = N / kTileRows;

    TilePairLoader<D> loader;
    loader.init(wv, lane);
    auto gate_of = [&](int j) {  // this thread's c value of tile j (threads 0..63)
        const int key = min(j * kTileRows + tid, N - 1);
        return ch[key];
    };
    loader.load(Kh, Vh, j_lo, jfull, N, sm.kv.a[0], sm.kv.b[0]);
    if (tid < kTileRows) sm.g[0][tid] = (gate_of(j_lo) - cbase) * inv_scale;
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    for (int j = j_lo; j <= j_hi; ++j) {
        const int buf = (j - j_lo) & 1;
        float g_next = 0.f;
        if (j < j_hi) {  // the plain load first: whatever wait the compiler puts in front of it must not cover the tile loads
            if (tid < kTileRows) g_next = gate_of(j + 1);
            loader.load(Kh, Vh, j + 1, jfull, N, sm.kv.a[buf ^ 1], sm.kv.b[buf ^ 1]);
        }
        const char* kt = sm.kv.a[buf];
        const char* vt = sm.kv.b[buf];
#pragma unroll
        for (int sb = 0; sb < kTileRows / 32; ++sb) {
            const int kb0 = j * kTileRows + 32 * sb;
            const bool act = (kb0 <= qw0 + 31) && (kb0 + 31 > qw0 - w) && (qw0 < N);
            if (!act) continue;
            const bool full = (kb0 + 31 <= qw0) && (kb0 > qw0 + 31 - w);

            // S^T[k][q] starts from the key term of the exponent, dP^T from -D_t (lane-constant), so that
            // the accumulator ends as dP - D.  The fragment reads run kAhead products ahead of the MFMAs.
            constexpr int kAhead = 4;
            f32x16 s, dp;
            acc_init_rows(s, sm.g[buf], 32 * sb, h);
#pragma unroll
            for (int v = 0; v < 16; ++v) dp[v] = ndt;
            {
                bf16x8 fr[2 * KC];
                auto fetch = [&](int f) __attribute__((always_inline)) {
                    fr[f] = lds_read_frag<D>(f < KC ? kt : vt, 32 * sb, f % KC, lane);
                };
#pragma unroll
                for (int f = 0; f < kAhead; ++f) fetch(f);
                __builtin_amdgcn_sched_group_barrier(0x100, 4 + kAhead, 0);
#pragma unroll
                for (int f = 0; f < 2 * KC; ++f) {
                    if (f < KC) s = mfma32(fr[f], qf[f], s);
                    else dp = mfma32(fr[f], gf[f - KC], dp);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (f + kAhead < 2 * KC) {
                        fetch(f + kAhead);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                }
            }
            float p[16], ds[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) p[v] = fast_exp2(fmaf(s[v], sl, nlsub));
            if (!full) {  // one branch per block, not one per element
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = kb0 + acc_row(v, h);
                    const bool keep = (i <= t) && (i > t - w);
                    p[v] = keep ? p[v] : 0.f;
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                ds[v] = p[v] * dp[v];
                rowsum += ds[v];
            }
            bf16x8 dsf[2];
            acc_to_bfrag(ds, dsf);
            {
                constexpr int NB = 2 * DB;
                bf16x8 fr[NB];
                auto fetch = [&](int f) __attribute__((always_inline)) {
                    fr[f] = lds_read_tr_frag<D>(kt, 32 * sb + 16 * (f / DB), f % DB, lane);
                };
#pragma unroll
                for (int f = 0; f < kAhead; ++f) fetch(f);
                __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0);
#pragma unroll
                for (int f = 0; f < NB; ++f) {
                    dq_acc[f % DB] = mfma32(fr[f], dsf[f / DB], dq_acc[f % DB]);
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (f + kAhead < NB) {
                        fetch(f + kAhead);
                        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    }
                }
            }
        }
        // (g_next is first touched here, a tile after its load was issued, so nothing waits for it earlier)
        if (j < j_hi && tid < kTileRows) sm.g[buf ^ 1][tid] = (g_next - cbase) * inv_scale;
        __builtin_amdgcn_s_waitcnt(vmcnt_only(0));  // this wave's share of tile j+1 has landed
        __syncthreads();
    }

    const float rs = xhalf_sum(rowsum);
    if (t < N && h == 0) dc_row[(size_t)bh * N + t] = rs;
    // dQ as whole lines, through 4 KB per wave of the tile buffers (free since the last barrier)
    store_acc_rows<DB>(dq_acc, scale, sm.kv.a[0] + 4096 * wv, dQ + head_off + (size_t)qw0 * D, N - qw0, lane);
}

// ------------------------------------------------------------------------------------------
// 3b. dQ and row sums from spilled dS blocks (d = 128): one matrix product, no exponentials
// ------------------------------------------------------------------------------------------
// Query-stationary like the kernel above (a lane owns one query, a wave 32 of them, K tiles of 64 keys
// stream through LDS), but S and dP are not formed again: the dS^T fragments (B operands: column =
// query, k = key) are read back from the blocks the dK/dV kernel stored.  A block travels global -> LDS
// unchanged; a transposing LDS read then hands a lane the dS of its query for four keys.
template <int D>
struct DqSpillSmem {
    alignas(16) char k[2][kTileRows * D * 2];                        // K tile
    alignas(16) char ds[2][kThreads / 64][2][kSpillBlockBytes];      // [buffer][wave][32-key block of the tile]
};

template <int D>
__global__ __launch_bounds__(kThreads, 2) void bwd_dq_spill_bf16_kernel(
    const bf16_t* __restrict__ K, const char* __restrict__ ds_ws, bf16_t* __restrict__ dQ,
    float* __restrict__ dc_row, int N, int w, float scale, int num_qtiles, int total_tiles, int H, int G) {
    constexpr int BR = 128;
    constexpr int DB = D / 32;
    extern __shared__ __align__(16) char smem_raw[];
    DqSpillSmem<D>& sm = *reinterpret_cast<DqSpillSmem<D>*>(smem_raw);

    const int tile = xcd_remap(blockIdx.x, total_tiles);
    const int bh = tile / num_qtiles;
    const int q0 = (tile % num_qtiles) * BR;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, lq = lane & 31;

    const size_t head_off = (size_t)bh * N * D;
    const char* Kh = reinterpret_cast<const char*>(K + (size_t)kv_head_of(bh, H, G) * N * D);
    const int qw0 = q0 + 32 * wv;
    const int t = qw0 + lq;
    const int nqb = (N + 31) / 32;
    const int nslot = ds_spill_slots(w, nqb);
    const int qb = qw0 >> 5;
    // slots of this wave's query block (read only for blocks inside the band, which implies qw0 < N)
    const char* blk0 = ds_ws + ((size_t)bh * nqb + qb) * nslot * kSpillBlockBytes;

    // byte offsets of this lane's transposing reads inside a block: 16-key chunk cc, read rd (keys
    // 16 cc + 4 h + 0..3, then 16 cc + 8 + 4 h + 0..3: the order in which lds_read_tr_frag hands out rows).
    // In its group of 16 lanes, lane j supplies the 8 bytes of key (j >> 2), query group (j & 3), and
    // receives query j of the group for the four keys.
    int ds_off[2][2];
    {
        const int c2 = lq >> 4, j = lane & 15, r = j >> 2, cg = j & 3;
#pragma unroll
        for (int cc = 0; cc < 2; ++cc)
#pragma unroll
            for (int rd = 0; rd < 2; ++rd) {
                const int key = 16 * cc + 8 * rd + 4 * h + r;
                ds_off[cc][rd] = 1024 * c2 + 16 * ((2 * key + (cg & 1) + 8 * c2) & 63) + 8 * (cg >> 1);
            }
    }

    // LDS slot p of piece c2 takes (key, h) with 2 key + h = (p - 8 c2) mod 64, stored at slot 32 h + key
    const unsigned gather0 = 16u * (32u * (lane & 1) + (lane >> 1));
    const unsigned gather1 = 1024u + 16u * (32u * (((lane - 8) & 63) & 1) + (((lane - 8) & 63) >> 1));

    f32x16 dq_acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) dq_acc[db][v] = 0.f;
    float rowsum = 0.f;

    const int k_lo = max(0, q0 - w + 1);
    const int k_hi = min(N, q0 + BR) - 1;
    const int j_lo = k_lo / kTileRows, j_hi = k_hi / kTileRows;
    const int jfull = N / kTileRows;
    auto in_band = [&](int kb0) { return (kb0 <= qw0 + 31) && (kb0 + 31 > qw0 - w) && (qw0 < N); };

    TilePairLoader<D> loader;
    loader.init(wv, lane);
    auto issue = [&](int j, int buf) {
        loader.load_one(Kh, j, jfull, N, sm.k[buf]);
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
            const int kb0 = j * kTileRows + 32 * sb;
            if (in_band(kb0)) {
                const char* src = blk0 + (size_t)((kb0 >> 5) - qb + nslot - 1) * kSpillBlockBytes;
                dma16_stream(src, gather0, sm.ds[buf][wv][sb]);
                dma16_stream(src, gather1, sm.ds[buf][wv][sb] + 1024);
            }
        }
    };
    issue(j_lo, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    for (int j = j_lo; j <= j_hi; ++j) {
        const int buf = (j - j_lo) & 1;
        if (j < j_hi) issue(j + 1, buf ^ 1);
        const char* kt = sm.k[buf];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
            if (!in_band(j * kTileRows + 32 * sb)) continue;
            const char* blk = sm.ds[buf][wv][sb];
            bf16x8 dsf[2];
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(blk + ds_off[cc][0]));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(blk + ds_off[cc][1]));
                typedef short s16x8 __attribute__((ext_vector_type(8)));
                const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                dsf[cc] = __builtin_bit_cast(bf16x8, both);
            }
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                for (int db = 0; db < DB; ++db)
                    dq_acc[db] = mfma32(lds_read_tr_frag<D>(kt, 32 * sb + 16 * cc, db, lane), dsf[cc], dq_acc[db]);
            // (pairs through the bf16 dot-product instruction, as the dK/dV kernel sums the same values along the columns)
            const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
#pragma unroll
                for (int e = 0; e < 8; e += 2)
                    rowsum = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{dsf[cc][e], dsf[cc][e + 1]}, ones, rowsum, false);
        }
        __builtin_amdgcn_s_waitcnt(vmcnt_only(0));  // this wave's loads of tile j+1 have landed
        __syncthreads();
    }

    const float rs = xhalf_sum(rowsum);
    if (t < N && h == 0) dc_row[(size_t)bh * N + t] = rs;
    // dQ as whole lines, through this wave's own block buffer (its last block was consumed above)
    store_acc_rows<DB>(dq_acc, scale, sm.ds[0][wv][0], dQ + head_off + (size_t)qw0 * D, N - qw0, lane);
}

size_t backward_bf16_spill_bytes(int B, int H, int N, int d, int w) {
    if (d != 128) return 0;
    const int nqb = (N + 31) / 32;
    return (size_t)B * H * nqb * ds_spill_slots(w, nqb) * kSpillBlockBytes;
}

template <int D>
static hipError_t launch_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                             const float* c, const float* L, void* dQ, void* dK, void* dV, float* dalpha,
                             float* ws, bool spill, int B, int H, int Hkv, int N, int w, float scale,
                             hipStream_t s) {
    const size_t rows = (size_t)B * H * N;
    const size_t pad = ((rows * sizeof(float) + 255) & ~(size_t)255) / sizeof(float);
    float* Dv = ws;
    float* dc_col = ws + pad;
    float* dc_row = ws + 2 * pad;
    double* scan_partial = reinterpret_cast<double*>(ws + 3 * pad);
    const size_t scan_pad = (gate_scan_workspace_bytes(B * H, N) + 255) & ~(size_t)255;
    char* ds_ws = reinterpret_cast<char*>(ws + 3 * pad) + scan_pad;  // only with `spill`
    constexpr int LPR = D / 8;
    const unsigned dot_blocks = (unsigned)((rows * LPR + 255) / 256);
    {
        ProfScope prof(kKernRowDot, s);
        hipLaunchKernelGGL((rowdot_bf16_kernel<D>), dim3(dot_blocks), dim3(256), 0, s, (const bf16_t*)O,
                           (const bf16_t*)dO, Dv, (long)rows);
    }
    const int nk = (N + 127) / 128;
    {
        ProfScope prof(kKernDkv, s);
        if constexpr (D == 128) {  // two waves per SIMD that share a key group (at d = 64 the 4-wave kernel has them already)
            if (spill)
                hipLaunchKernelGGL((bwd_dkv8_bf16_kernel<D, true>), dim3(B * Hkv * nk), dim3(2 * kThreads), 0, s,
                                   (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, c, L, Dv,
                                   (bf16_t*)dK, (bf16_t*)dV, dc_col, ds_ws, N, w, scale, nk, B * Hkv * nk, H, H / Hkv);
            else
                hipLaunchKernelGGL((bwd_dkv8_bf16_kernel<D, false>), dim3(B * Hkv * nk), dim3(2 * kThreads), 0, s,
                                   (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, c, L, Dv,
                                   (bf16_t*)dK, (bf16_t*)dV, dc_col, ds_ws, N, w, scale, nk, B * Hkv * nk, H, H / Hkv);
        } else
            hipLaunchKernelGGL((bwd_dkv_bf16_kernel<D>), dim3(B * Hkv * nk), dim3(kThreads), 0, s,
                               (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, c, L, Dv,
                               (bf16_t*)dK, (bf16_t*)dV, dc_col, N, w, scale, nk, B * Hkv * nk, H, H / Hkv);
    }
    const int nq = (N + 127) / 128;
    {
        ProfScope prof(kKernDq, s);
        bool launched = false;
        if constexpr (D == 128) {
            if (spill) {
                static DeviceOnce lds_allowed;
                if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(&bwd_dq_spill_bf16_kernel<D>),
                                                     sizeof(DqSpillSmem<D>), lds_allowed))
                    return e;
                hipLaunchKernelGGL((bwd_dq_spill_bf16_kernel<D>), dim3(B * H * nq), dim3(kThreads),
                                   sizeof(DqSpillSmem<D>), s, (const bf16_t*)K, ds_ws, (bf16_t*)dQ, dc_row, N, w,
                                   scale, nq, B * H * nq, H, H / Hkv);
                launched = true;
            }
        }
        if (!launched)
            hipLaunchKernelGGL((bwd_dq_bf16_kernel<D>), dim3(B * H * nq), dim3(kThreads), 0, s,
                               (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, c, L, Dv,
                               (bf16_t*)dQ, dc_row, N, w, scale, nq, B * H * nq, H, H / Hkv);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return gate_grad_scan(dc_col, dc_row, dalpha, scan_partial, B * H, N, s);
}

hipError_t backward_bf16(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                         const float* c, const float* L, void* dQ, void* dK, void* dV, float* dalpha,
                         float* ws, bool spill, int B, int H, int Hkv, int N, int d, int w, float scale,
                         hipStream_t s) {
    if (d == 128)
        return launch_bwd<128>(Q, K, V, O, dO, c, L, dQ, dK, dV, dalpha, ws, spill, B, H, Hkv, N, w, scale, s);
    return launch_bwd<64>(Q, K, V, O, dO, c, L, dQ, dK, dV, dalpha, ws, false, B, H, Hkv, N, w, scale, s);
}

}  // namespace gfwa
