// GatedFWA fused forward for bf16 storage on gfx950 (paper Alg. 2, re-designed for CDNA4).
//
// One workgroup of 8 waves per CU owns a tile of 256 consecutive queries of one (b,h); a wave owns
// 32 of them.  Key/value tiles of 64 keys travel global -> LDS by direct loads (no staging
// registers, no LDS stores) through a ring of kRing buffers, and only the tiles that intersect the
// band [q0-w+1, q0+255] are visited; inside a tile every wave skips the 32-key blocks that lie
// wholly outside the band of its own queries, and masks only the blocks the band edge or the
// diagonal cuts.
//
// The products are formed transposed so that a lane owns one query:
//   S^T[key][query]  = g[key] + K_tile (A operand, from LDS)  x  Q^T (B operand, registers)
//   O^T[dd][query]  += V_tile^T (A operand, LDS transposing read)  x  P^T (B operand = the S^T
//                      accumulator registers converted to bf16 in place)
// so the row max / row sum of the online softmax are in-lane plus one exchange between the two
// halves of the wave, the rescale factor is a per-lane scalar, and P never leaves registers.
//
// Two-phase schedule.  The work of a wave on key tile T (two 32-key blocks) is split into a
// matrix phase
//   M(T):  S_T = g + K_T Q^T   and   O += V_{T-1}^T P_{T-1}        (32 MFMAs at d = 128)
// and a vector phase
//   X(T):  P_T = exp2(S_T * sl - m * sl), row sums                 (no MFMA)
// The two waves that share a SIMD belong to different groups (waves 0-3 and 4-7).  There is one
// workgroup barrier per key tile; the first group takes it after X(T), the second after M(T), so
// the second group's vector phase runs next to the first group's next matrix phase: on every SIMD
// one wave issues MFMAs while the other does the softmax arithmetic, instead of all waves queueing
// for the same unit.
//
// The gate bias rides in the MFMA accumulator: S is initialised with g_i = (c_i - c_base) / scale
// straight from LDS before the K Q^T chain, so S = q.k + g_i and the probability is one fused
// multiply-add plus one exp2, sl = scale * log2(e).  The per-query term -(c_t - c_base) is
// constant along a row, cancels in the softmax, and is applied only to L.  c_base = c at the first
// query of the tile keeps the fp32 differences window-local.  The row sum is taken over the
// bf16-rounded probabilities (one packed dot-product per pair), i.e. over exactly the values that
// enter the PV product.
//
// Deferred running max.  exp2 is taken against the reference exponent m left by earlier tiles
// without first looking for the tile's own maximum; fp32 and bf16 share their exponent range, so a
// probability may grow to 2^60 with no loss of precision.  Only when a lane's tile sum exceeds that
// (always on a wave's first tile, where m is still "minus infinity") does the wave take the slow
// path: find the true maximum, raise m, rescale O and l, and redo the exponentials.  Tiles are
// visited from the diagonal backwards, where the gate bias is largest, so this is rare.
#include <cstddef>
#include <type_traits>

#include "gfwa_device.h"
#include "gfwa_internal.h"
#include "tile_stage.h"

namespace gfwa {

constexpr int kFwdWaves = 8;
constexpr int kFwdThreads = 64 * kFwdWaves;
constexpr int kFwdBR = 32 * kFwdWaves;  // queries per workgroup
constexpr int kRing = 4;                // K/V tile slots: read for PV, read for S, two in flight

template <int D>
using FwdSmem = KvRingSmem<D, kRing>;

template <int D>
__global__ __launch_bounds__(kFwdThreads, 2) void fwd_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const float* __restrict__ c, bf16_t* __restrict__ O, float* __restrict__ L, int N, int w,
    float scale_log2, int num_qtiles, int total_tiles, int H, int G) {
    constexpr int BR = kFwdBR;
    constexpr int KC = D / 16;  // MFMA k-chunks along the head dimension
    constexpr int DB = D / 32;  // 32-wide blocks of the head dimension
    using Loader = TilePairLoader<D, kFwdWaves>;
    constexpr int kBatch = Loader::kLoadsPerTilePair + 1;  // loads one wave issues per tile (K, V, c)
    extern __shared__ __align__(16) char smem_raw[];
    FwdSmem<D>& sm = *reinterpret_cast<FwdSmem<D>*>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wv >> 2;  // waves wv and wv + 4 share a SIMD and run in opposite phases
    const int h = lane >> 5, lq = lane & 31;
    const float sl = scale_log2;
    const float inv_scale = kLog2e / scale_log2;
    const int jfull = N / kTileRows;  // tiles below jfull have all 64 rows inside the sequence

    // Persistent workgroups: workgroup b takes the query tiles xcd_remap(b) + k * gridDim.x, so the
    // loads of the next tile are issued before the results of the current one are stored.
    // (the slot inside a step is rotated from step to step so that the short tiles at the ends of a
    // head do not always fall to the same workgroups)
    const int wg_slot = xcd_remap(blockIdx.x, gridDim.x);
    int wg_step = 0;
    auto tile_of = [&](int k) { return k * (int)gridDim.x + (wg_slot + 37 * k) % (int)gridDim.x; };
    int tile = tile_of(0);
    int bh, q0, qw0, t, j_lo, j_hi, ntiles;
    size_t head_off;
    const char *Kh, *Vh;
    const float* ch;
    float cbase, cq;
    bf16x8 qf[KC];  // Q^T fragments (B operand), resident for the whole tile loop
    auto set_tile = [&](int tl) __attribute__((always_inline)) {
        bh = tl / num_qtiles;
        q0 = (tl % num_qtiles) * BR;
        head_off = (size_t)bh * N * D;
        const size_t kv_off = (size_t)kv_head_of(bh, H, G) * N * D;
        Kh = reinterpret_cast<const char*>(K + kv_off);
        Vh = reinterpret_cast<const char*>(V + kv_off);
        ch = c + (size_t)bh * N;
        cbase = ch[q0];
        // the two waves of a SIMD take slabs 128 queries apart: in the first and last key tiles of the band, where
        // only the upper or the lower half of the queries has keys, every SIMD then still has one wave at work
        qw0 = q0 + 32 * (wv & 3) + 128 * grp;  // first query of this wave
        t = qw0 + lq;
        {  // rows past N read row N-1
            const bf16_t* qp = Q + head_off + (size_t)min(t, N - 1) * D + 8 * h;
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) qf[kc] = *reinterpret_cast<const bf16x8*>(qp + 16 * kc);
        }
        cq = ch[min(t, N - 1)] - cbase;
        // key tiles that intersect the band of this query tile (window-aware pruning of Alg. 2)
        const int k_lo = max(0, q0 - w + 1);
        const int k_hi = min(N, q0 + BR) - 1;
        j_lo = k_lo / kTileRows;
        j_hi = k_hi / kTileRows;
        ntiles = j_hi - j_lo + 1;
    };
    set_tile(tile);

    Loader loader;
    loader.init(wv, lane);
    // every wave issues the same kBatch loads per tile, so the vmcnt bookkeeping is uniform; the
    // 64 c values are fetched by all waves to the same place (identical data)
    // Tiles are visited from the diagonal backwards: the gate bias only falls with distance, so
    // the first blocks set the running max and later ones hardly ever force a rescale of O.
    auto issue_tile = [&](int T) {  // T = position in visiting order, tile j_hi - T
        const int j = j_hi - T, buf = T % kRing;
        dma4(ch, (unsigned)min(j * kTileRows + lane, N - 1) * 4u, sm.craw[buf]);
        loader.load(Kh, Vh, j, jfull, N, sm.k[buf], sm.v[buf]);
    };
    auto publish_gate = [&](int T) {  // wave 0: raw c it loaded itself -> accumulator initial values
        const int buf = T % kRing;
        sm.g[buf][lane] = (sm.craw[buf][lane] - cbase) * inv_scale;
    };

    f32x16 o[DB];
    float m, l;
    // first two key tiles of the current query tile in flight, everything else of the ring idle
    auto open_tile = [&]() __attribute__((always_inline)) {
        issue_tile(0);
        if (ntiles > 1) issue_tile(1);
    };
    auto start_tile = [&]() __attribute__((always_inline)) {
        // the first step multiplies pf = 0 with the last ring slot: make it finite
        for (int o16 = tid * 16; o16 < kTileRows * D * 2; o16 += kFwdThreads * 16)
            *reinterpret_cast<f32x4*>(sm.v[kRing - 1] + o16) = f32x4{0.f, 0.f, 0.f, 0.f};
        __builtin_amdgcn_s_waitcnt(0);
        if (wv == 0) {
            publish_gate(0);
            if (ntiles > 1) publish_gate(1);
        }
        wg_barrier();
    };
    open_tile();
    start_tile();

    // per-lane LDS byte offsets of the operand fragments inside ring slot 0; ring slot, 32-key
    // block and 16-row group are compile-time displacements on top (the swizzle has period 16 rows)
    typedef __attribute__((address_space(3))) const char* lds_ptr;
    lds_ptr kaddr[KC], vaddr[DB][2], gaddr;
    {
        lds_ptr base = (lds_ptr)smem_raw;
#pragma unroll
        for (int kc = 0; kc < KC; ++kc)
            kaddr[kc] = base + offsetof(FwdSmem<D>, k) + tile_off<D>(lane & 31, 2 * kc + h);
        const int i16 = lane & 15;
        const int row = 4 * h + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const int col = 32 * db + 16 * ((lane & 31) >> 4) + 4 * (i16 & 3);
            vaddr[db][0] = base + offsetof(FwdSmem<D>, v) + tile_off<D>(row, col >> 3) + (col & 7) * 2;
            vaddr[db][1] = base + offsetof(FwdSmem<D>, v) + tile_off<D>(row + 8, col >> 3) + (col & 7) * 2;
        }
        gaddr = base + offsetof(FwdSmem<D>, g) + 16 * h;
    }
    constexpr int kTileBytes = kTileRows * D * 2;
    auto read_k = [&](int kc, int disp) -> bf16x8 {
        return *reinterpret_cast<__attribute__((address_space(3))) const bf16x8*>(kaddr[kc] + disp);
    };
    auto read_vt = [&](int db, int disp) -> bf16x8 {
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vaddr[db][0] + disp));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vaddr[db][1] + disp));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto read_g = [&](f32x16& acc, int disp) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const f32x4 g4 = *reinterpret_cast<__attribute__((address_space(3))) const f32x4*>(gaddr + disp + 32 * r);
            acc[4 * r] = g4[0];
            acc[4 * r + 1] = g4[1];
            acc[4 * r + 2] = g4[2];
            acc[4 * r + 3] = g4[3];
        }
    };

    f32x16 s[2];     // S^T of the two blocks of the current tile (0: upper 32 keys, 1: lower)
    u32x4 pf[2][2];  // their probabilities as B operands (bf16 pairs)
    bool pending;    // the previous tile left a P that still has to be multiplied into O
    bool fresh;      // no tile of the current query tile has set this wave's reference exponent yet
    constexpr bool kFirstTileShortcut = D == 64;
    constexpr float kBig = 1.152921504606846976e18f;  // 2^60

    // one key tile; the ring slot is a compile-time constant so that every LDS address is a
    // loop-invariant register plus an immediate.  Block 0 is the upper half of the tile.
    auto tile_step = [&](auto buf_c, int T) {
        constexpr int buf = decltype(buf_c)::value;
        constexpr int pbuf = (buf + kRing - 1) % kRing;  // slot of the previous tile
        const int kt0 = (j_hi - T) * kTileRows;
        bool act[2], full[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int kb0 = kt0 + 32 * (1 - b);
            act[b] = (T < ntiles) && (kb0 <= qw0 + 31) && (kb0 + 31 > qw0 - w) && (qw0 < N);
            full[b] = (kb0 + 31 <= qw0) && (kb0 > qw0 + 31 - w);
        }
        const bool any_act = act[0] || act[1];
        // slot (T+2) % kRing held tile T-2, whose V was last read in M(T-1)
        const bool issue = T + 2 < ntiles;
        if (issue) issue_tile(T + 2);

        // ---------------- matrix phase M(T): one straight-line body.  A block outside the band
        // of this wave still gets its S formed (never looked at); a wave with no pending P
        // multiplies V by pf = 0.  Only a wave with neither skips the phase.
        if (any_act || pending) {
            constexpr int kAhead = 4, NS = 2 * KC, NP = 4 * DB, NF = NS + NP;
            bf16x8 fr[NF];  // fragment f: K chunk of block f / KC for f < NS, else V^T fragment
            auto fetch = [&](int f) {
                if (f < NS) {
                    fr[f] = read_k(f % KC, buf * kTileBytes + 32 * (1 - f / KC) * (D * 2));
                } else {
                    const int g = f - NS, b = g / (2 * DB), c2 = (g / DB) % 2, db = g % DB;
                    fr[f] = read_vt(db, pbuf * kTileBytes + (32 * (1 - b) + 16 * c2) * (D * 2));
                }
            };
            read_g(s[0], buf * (kTileRows * 4) + 32 * 4);
            read_g(s[1], buf * (kTileRows * 4));
#pragma unroll
            for (int f = 0; f < kAhead; ++f) fetch(f);
            __builtin_amdgcn_sched_group_barrier(0x100, 8 + kAhead, 0);
#pragma unroll
            for (int i = 0; i < NF; ++i) {
                if (i < NS) {
                    s[i / KC] = mfma32(fr[i], qf[i % KC], s[i / KC]);
                } else {
                    const int g = i - NS, b = g / (2 * DB), c2 = (g / DB) % 2, db = g % DB;
                    o[db] = mfma32(fr[i], __builtin_bit_cast(bf16x8, pf[b][c2]), o[db]);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (i + kAhead < NF) {
                    fetch(i + kAhead);
                    if (i + kAhead < NS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    else __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                }
            }
        }
        // The one workgroup barrier of this tile: the second group takes it here, between its
        // matrix and vector phase, the first group at the end of the step.  Both groups therefore
        // run M(T) in the same interval (same ring slots), but the second group's X(T) falls into
        // the next one, next to the first group's M(T+1).  Tile T+1 is first read after it.
        if (grp == 1) {
            if (issue) __builtin_amdgcn_s_waitcnt(vmcnt_only(kBatch));
            else __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
            wg_barrier();
        }

        // ---------------- vector phase X(T)
        if (any_act) {
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                if (act[b] && !full[b]) {
                    const int kb0 = kt0 + 32 * (1 - b);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int i = kb0 + acc_row(v, h);
                        const bool keep = (i <= t) && (i > t - w);
                        s[b][v] = keep ? s[b][v] : -INFINITY;
                    }
                }
            }
            float tsum = 0.f;
            auto exponentiate = [&]() __attribute__((always_inline)) {
                const float nm = -m * sl;
                float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    if (act[b]) {
#pragma unroll
                        for (int cc = 0; cc < 8; ++cc) {
                            f32x2 pr = {fast_exp2(fmaf(s[b][2 * cc], sl, nm)), fast_exp2(fmaf(s[b][2 * cc + 1], sl, nm))};
                            const bf16x2 pb = __builtin_convertvector(pr, bf16x2);
                            // plain adds: the packed dot-product instructions run on the matrix
                            // pipe and would stall behind the other wave's MFMAs
                            part[2 * b] += pr[0];
                            part[2 * b + 1] += pr[1];
                            pf[b][cc >> 2][cc & 3] = __builtin_bit_cast(unsigned, pb);
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) pf[b][0][e] = pf[b][1][e] = 0u;
                    }
                }
                tsum = (part[0] + part[1]) + (part[2] + part[3]);
            };
            // d = 64 (short bands, the first tile weighs more): a wave's first tile, whose reference exponent is
            // still the initial one, goes straight to the slow path instead of trying the fast one first
            const bool first = kFirstTileShortcut && fresh;
            if (!first) exponentiate();
            if (first || __builtin_amdgcn_ballot_w64(!(tsum <= kBig)) != 0) {
                // slow path: true maximum of the tile, common to the two halves of the wave
                float mx = -INFINITY;
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    if (act[b]) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[b][v]);
                    }
                mx = xhalf_max(mx);
                const float mnew = fmaxf(m, mx);
                const float a = fast_exp2((m - mnew) * sl);
                m = mnew;
                l *= a;
                if (!first) {  // (O is still zero on a first tile)
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int v = 0; v < 16; ++v) o[db][v] *= a;
                }
                exponentiate();
            }
            l += tsum;
            fresh = false;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) pf[0][0][e] = pf[0][1][e] = pf[1][0][e] = pf[1][1][e] = 0u;
        }
        pending = any_act;
        if (grp == 0) {
            if (issue) __builtin_amdgcn_s_waitcnt(vmcnt_only(kBatch));
            else __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
            if (wv == 0 && T + 1 < ntiles && T >= 1) publish_gate(T + 1);  // tiles 0, 1: prologue
            wg_barrier();
        }
    };
    static_assert(kRing == 4, "the tile loop is unrolled over the ring");
    for (;;) {  // query tiles of this workgroup
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.0f;
    m = kNegBig;
    l = 0.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e) pf[0][0][e] = pf[0][1][e] = pf[1][0][e] = pf[1][1][e] = 0u;
    pending = false;
    fresh = true;
    // T = ntiles is the drain step (only the PV product of the last tile)
    for (int T = 0; T <= ntiles; T += 4) {
        tile_step(std::integral_constant<int, 0>{}, T);
        if (T + 1 > ntiles) break;
        tile_step(std::integral_constant<int, 1>{}, T + 1);
        if (T + 2 > ntiles) break;
        tile_step(std::integral_constant<int, 2>{}, T + 2);
        if (T + 3 > ntiles) break;
        tile_step(std::integral_constant<int, 3>{}, T + 3);
    }

    // all LDS reads of this query tile are done (last barrier): open the next one before storing
    const int t_done = t, bh_done = bh;
    const size_t head_done = head_off;
    const float cq_done = cq;
    const bool more = tile_of(wg_step + 1) < total_tiles;
    if (more) {
        tile = tile_of(++wg_step);
        set_tile(tile);
        open_tile();
    }
    // ---- epilogue: O = O^T / l, L = ln2 * (m*sl + log2 l) - (c_t - c_base)
    const float lt = xhalf_sum(l);  // the two halves of the wave hold complementary keys
    if (t_done < N) {
        const float inv = 1.0f / lt;
        bf16_t* orow = O + head_done + (size_t)t_done * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 o4 = {o[db][4 * g] * inv, o[db][4 * g + 1] * inv, o[db][4 * g + 2] * inv,
                            o[db][4 * g + 3] * inv};
                *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * g + 4 * h) = __builtin_convertvector(o4, bf16x4);
            }
        if (h == 0) L[(size_t)bh_done * N + t_done] = (m * sl + fast_log2(lt)) * kLn2 - cq_done;
    }
    if (!more) break;
    start_tile();
    }
}

template <int D>
static hipError_t launch_fwd(const void* Q, const void* K, const void* V, const float* c, void* O,
                             float* L, int B, int H, int Hkv, int N, int w, float scale, hipStream_t s) {
    const int num_qtiles = (N + kFwdBR - 1) / kFwdBR;
    const int total = B * H * num_qtiles;
    static DeviceOnce lds_allowed;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(&fwd_bf16_kernel<D>), sizeof(FwdSmem<D>),
                                         lds_allowed))
        return e;
    const int num_cu = device_cu_count();
    const int grid = total < num_cu ? total : num_cu;  // one resident workgroup per CU
    ProfScope prof(kKernForward, s);
    hipLaunchKernelGGL((fwd_bf16_kernel<D>), dim3(grid), dim3(kFwdThreads), sizeof(FwdSmem<D>), s,
                       (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, c, (bf16_t*)O, L, N, w,
                       scale * kLog2e, num_qtiles, total, H, H / Hkv);
    return hipGetLastError();
}

hipError_t forward_bf16(const void* Q, const void* K, const void* V, const float* c, void* O, float* L,
                        int B, int H, int Hkv, int N, int d, int w, float scale, hipStream_t s) {
    if (d == 128) return launch_fwd<128>(Q, K, V, c, O, L, B, H, Hkv, N, w, scale, s);
    return launch_fwd<64>(Q, K, V, c, O, L, B, H, Hkv, N, w, scale, s);
}

}  // namespace gfwa
