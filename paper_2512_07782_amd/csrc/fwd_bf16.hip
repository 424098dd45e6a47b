// GatedFWA fused forward for bf16 storage on gfx950 (paper Alg. 2, re-designed for CDNA4).
//
// Workgroups of 4 waves, two resident per CU (two waves per SIMD, 256 registers each), persistent: a
// workgroup takes one tile of 128 consecutive queries of one (b,h) after another, and a wave owns one block of
// 32 of them.  Key/value tiles of 64 keys travel global -> LDS by direct loads (no staging registers, no LDS
// stores) through rings of two K and two V slots; only the tiles that intersect the band [q0-w+1, q0+127] are
// visited, from the diagonal backwards.  Inside a tile a wave computes only in the steps that hold blocks of its
// own band (in the others it just issues its share of the loads) and masks only the blocks the band edge or
// the diagonal cuts.
//
// The products are formed transposed so that a lane owns one query:
//   S^T[key][query]  = g[key] + K_tile (A operand, from LDS)  x  Q^T (B operand, registers)
//   O^T[dd][query]  += V_tile^T (A operand, LDS transposing read)  x  P^T (B operand = the S^T
//                      accumulator registers converted to bf16 in place)
// so the row max / row sum of the online softmax are in-lane plus one exchange between the two
// halves of the wave, the rescale factor is a per-lane scalar, and P never leaves registers.
//
// Software pipeline inside the wave.  With blocks of 32 keys numbered n in visiting order, iteration n
// issues, as one straight-line instruction stream,
//   matrix pipe:  S(n) = g + K Q^T      and      O += V^T P(n-2)          (16 MFMAs at d = 128)
//   vector unit:  P(n-1) = exp2(S(n-1) * sl - m * sl), row sums
//   LDS:          the fragments of the MFMAs four steps ahead
//   load unit:    in the first block of a tile, this wave's share of the keys of tile T+1 and of the values of
//                 tile T, in three groups between the MFMAs (both target slots are idle from the start of the step)
// Nothing in an iteration depends on anything else in it, so the MFMAs issue back to back while the
// exponentials of the previous block and the fragment reads of the next MFMAs fill the issue slots
// between them (an MFMA occupies the matrix pipe for 32 cycles; about five vector and two LDS
// instructions fit beside it).  A step is the two iterations of one key tile; one workgroup barrier per
// step hands the ring slots over.  The V tile of step T is requested in step T and first read in step
// T+1 (by the PV products, which lag two blocks), the K tile of step T+1 is requested in step T.
// When a tile is finished the first key tile of the next one is requested before O is stored, and O
// leaves as whole 128-byte lines through the idle V ring.  The next tile's queries arrive through the rings as
// well when the tile count is even (d = 128): the last step's loads, which no product reads, fetch them.
//
// The gate bias rides in the MFMA accumulator: S is initialised with g_i = (c_i - c_base) / scale
// straight from LDS before the K Q^T chain, so S = q.k + g_i and the probability is one fused
// multiply-add plus one exp2, sl = scale * log2(e).  The per-query term -(c_t - c_base) is
// constant along a row, cancels in the softmax, and is applied only to L.  c_base = c at the first
// query of the tile keeps the fp32 differences window-local.  The row sum is taken in fp32 over the
// unrounded probabilities with plain adds.
//
// Deferred running max.  exp2 is taken against the reference exponent m left by earlier blocks
// without first looking for the block's own maximum; fp32 and bf16 share their exponent range, so a
// probability may grow to 2^60 with no loss of precision.  Only when a lane's block sum exceeds that
// (always on a query block's first key block, where m is still "minus infinity") does the wave take the
// slow path: find the true maximum, raise m, rescale O and l, and redo the exponentials.  Blocks are
// visited from the diagonal backwards, where the gate bias is largest, so this is rare.
#include <cstddef>
#include <type_traits>

#include "gfwa_device.h"
#include "gfwa_internal.h"
#include "tile_stage.h"

namespace gfwa {

constexpr int kFwdWaves = 4;
constexpr int kFwdThreads = 64 * kFwdWaves;
// 32-query blocks per wave.  One: at d = 128 that is the register budget of two waves per SIMD; at d = 64 two blocks
// fit (254 registers, every K and V fragment read from LDS then feeds two MFMAs) but measured slower, 84 us against
// 74 us on the LM-scale workload: the 256-query tile staggers the waves' bands further and the waves run out of
// independent work to cover each other.
template <int D>
constexpr int kQueryBlocks = 1;
template <int D>
constexpr int kFwdBR = 32 * kQueryBlocks<D> * kFwdWaves;  // queries per workgroup
constexpr int kRing = 2;                         // K and V tile slots each: one being read, one in flight
// Resident workgroups per CU: two at d = 128 (256 registers per wave); three at d = 64, where the accumulators are
// half as large (the kernel fits 168 registers) and a workgroup's rings take 33 KB of LDS.
template <int D>
constexpr int kFwdResident = D == 64 ? 3 : 2;

template <int D>
using FwdSmem = KvRingSmem<D, kRing>;

template <int D>
__global__ __launch_bounds__(kFwdThreads, kFwdResident<D>) void fwd_bf16_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const float* __restrict__ c, bf16_t* __restrict__ O, float* __restrict__ L, int N, int w,
    float scale_log2, int num_qtiles, int total_tiles, int H, int G) {
    constexpr int kQB = kQueryBlocks<D>;
    constexpr int BR = kFwdBR<D>;
    constexpr int KC = D / 16;  // MFMA k-chunks along the head dimension
    constexpr int DB = D / 32;  // 32-wide blocks of the head dimension
    using Loader = TilePairLoader<D, kFwdWaves>;
    extern __shared__ __align__(16) char smem_raw[];
    FwdSmem<D>& sm = *reinterpret_cast<FwdSmem<D>*>(smem_raw);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, lq = lane & 31;
    const float sl = scale_log2;
    const float inv_scale = kLog2e / scale_log2;

    // Persistent workgroups: workgroup b takes the query tiles xcd_remap(b) + k * gridDim.x, so the
    // loads of the next tile are issued before the results of the current one are stored.
    // (the slot inside a round is rotated from round to round so that the short tiles at the ends of a
    // head do not always fall to the same workgroups).  A last round with fewer tiles than workgroups is
    // dealt out per XCD - every XCD an equal, contiguous share, taken by as many of its workgroups -
    // instead of filling some XCDs and leaving the others without work; total_tiles stands for "none".
    const int wg_slot = xcd_remap(blockIdx.x, gridDim.x);
    int wg_step = 0;
    auto tile_of = [&](int k) __attribute__((always_inline)) {
        constexpr int kXcd = 8;
        const int G_ = (int)gridDim.x, base = k * G_, left = total_tiles - base;
        if (left >= G_ || k == 0 || G_ % kXcd != 0) return base + (wg_slot + 37 * k) % G_;
        if (left <= 0) return total_tiles;
        const int per_xcd = G_ / kXcd, share = (left + kXcd - 1) / kXcd;
        const int x = wg_slot / per_xcd, idx = (wg_slot % per_xcd + 37 * k) % per_xcd;
        const int t = x * share + idx;
        return (idx < share && t < left) ? base + t : total_tiles;
    };
    int tile = tile_of(0);
    int bh, q0, qw0, t0, j_lo, j_hi, ntiles;
    size_t head_off;
    const char *Kh, *Vh;
    const float* ch;
    float cbase, cq[kQB];
    bf16x8 qf[kQB][KC];  // Q^T fragments (B operand), resident for the whole tile loop
    auto set_tile = [&](int tl) __attribute__((always_inline)) {
        bh = tl / num_qtiles;
        q0 = (tl % num_qtiles) * BR;
        head_off = (size_t)bh * N * D;
        const size_t kv_off = (size_t)kv_head_of(bh, H, G) * N * D;
        Kh = reinterpret_cast<const char*>(K + kv_off);
        Vh = reinterpret_cast<const char*>(V + kv_off);
        ch = c + (size_t)bh * N;
        cbase = ch[q0];
        qw0 = q0 + 32 * kQB * wv;  // first query of this wave
        t0 = qw0 + lq;             // this lane's query in block 0; block qb: t0 + 32 qb
        // key tiles that intersect the band of this query tile (window-aware pruning of Alg. 2)
        const int k_lo = max(0, q0 - w + 1);
        const int k_hi = min(N, q0 + BR) - 1;
        j_lo = k_lo / kTileRows;
        j_hi = k_hi / kTileRows;
        ntiles = j_hi - j_lo + 1;
    };
    // The queries of the next tile can travel through the rings: the last step of a tile (the drain step, T = ntiles)
    // still issues a load of K tile ntiles + 1 and of V tile ntiles, which nothing reads; when the tile count is even
    // those land in K slot 1 and V slot 0, both idle by then, and the first key tile of the next query tile goes to
    // K slot 0.  So in that step the two loads fetch the next tile's 128 queries instead (first 64 into the K slot,
    // last 64 into the V slot, swizzled like any tile), and the waves pick their Q fragments up from LDS when the tile
    // starts instead of waiting for a round trip to memory.  (d = 128 only: at d = 64 the output staging needs both
    // V slots.  Odd tile counts keep the loads from global memory.)
    constexpr bool kStageQ = D == 128 && kQB == 1;
    int stage_T = -1000;      // the step whose spare loads fetch the next tile's queries, if any
    const char* Qn = nullptr; // Q of the next tile's head
    int qn0 = 0;              // first query of the next tile
    auto plan_next = [&]() __attribute__((always_inline)) {
        const int tn = tile_of(wg_step + 1);
        const bool ok = kStageQ && tn < total_tiles && (ntiles & 1) == 0;
        stage_T = ok ? ntiles : -1000;
        qn0 = (tn % num_qtiles) * BR;
        Qn = reinterpret_cast<const char*>(Q + (size_t)(tn / num_qtiles) * N * D);
    };
    auto load_query_gates = [&]() __attribute__((always_inline)) {  // c_t - c_base of the tile set_tile has chosen (rows past N read row N-1)
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) cq[qb] = ch[min(t0 + 32 * qb, N - 1)] - cbase;
    };
    auto load_queries = [&]() __attribute__((always_inline)) {  // Q fragments of that tile, from global memory
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) {
            const int t = min(t0 + 32 * qb, N - 1);
            const bf16_t* qp = Q + head_off + (size_t)t * D + 8 * h;
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) qf[qb][kc] = *reinterpret_cast<const bf16x8*>(qp + 16 * kc);
        }
    };
    set_tile(tile);
    load_queries();
    load_query_gates();
    // ring slots that were never loaded are read by the first and last iterations of a band (as operands
    // of products with zero probabilities, or into scores that the mask overrides): make them finite once
    for (int o16 = tid * 16; o16 < (int)(offsetof(FwdSmem<D>, craw)); o16 += kFwdThreads * 16)
        *reinterpret_cast<f32x4*>(smem_raw + o16) = f32x4{0.f, 0.f, 0.f, 0.f};
    __syncthreads();

    // Tile loads, 1 KB per wave instruction (kRowsPerLoad rows of a tile): wave wv fills rows
    // kRowsPerWave wv .. of a tile with kLoadsPerWave loads.  Lane p of a load writes LDS row p / chunks-per-row
    // of its group at physical chunk p % chunks-per-row and therefore fetches the logical chunk the swizzle
    // maps there.  Rows at or beyond N read row N-1 (finite data that the band mask keeps out of every sum);
    // a tile index below 0 reads tile 0 (the loads of the two steps after a band's last tile, which nothing reads).
    constexpr int kRowsPerLoad = Loader::kRowsPerLoad, kLoadsPerWave = Loader::kLoadsPerWave;
    constexpr int kRowsPerWave = Loader::kRowsPerWave, kChunksPerRow = Loader::kChunksPerRow;
    static_assert(kRowsPerLoad == 4 || kRowsPerLoad == 8, "1 KB loads of 256- or 128-byte rows");
    // load g fetches row ld_row0 + kRowsPerLoad g of the tile; the swizzle of that row differs from load 0's only
    // in chunk bits that g alone sets (d = 128: bits 0-1 = (row >> 2) & 3 = g; d = 64: bit 0 = (row >> 3) & 1 = g & 1)
    const int ld_row0 = kRowsPerWave * wv + lane / kChunksPerRow;
    const unsigned ld_chunk0 = (unsigned)(swz_chunk<D>(ld_row0, lane % kChunksPerRow) * 16);
    // load g of tile T (position in visiting order: tile j_hi - T) of the matrix at Mh into its ring slot
    // (is_v: the V ring; the spare loads of the drain step fetch the next tile's queries, see plan_next)
    auto load_piece = [&](const char* Mh, char (&ring)[kRing][kTileRows * D * 2], int T, int g, bool is_v) __attribute__((always_inline)) {
        const bool spare = kStageQ && T == stage_T + (is_v ? 0 : 1);
        const int j = max(j_hi - T, 0);
        const int row0 = spare ? qn0 + (is_v ? kTileRows : 0) : j * kTileRows;
        const char* M = spare ? Qn : Mh;
        const int row = min(row0 + kRowsPerLoad * g + ld_row0, N - 1);
        const unsigned chunk = ld_chunk0 ^ (unsigned)((swz_chunk<D>(kRowsPerLoad * g, 0)) * 16);
        dma16(M, (unsigned)row * (unsigned)(D * 2) + chunk, ring[T % kRing] + (kRowsPerWave * wv + kRowsPerLoad * g) * (D * 2));
    };
    auto load_gate = [&](int T) __attribute__((always_inline)) {  // the 64 gate values of tile T's keys (every wave, same place)
        const int j = max(j_hi - T, 0);
        dma4(ch, (unsigned)min(j * kTileRows + lane, N - 1) * 4u, sm.craw[T % kRing]);
    };
    auto issue_k = [&](int T) __attribute__((always_inline)) {  // keys of tile T and their gate values
        load_gate(T);
#pragma unroll
        for (int g = 0; g < kLoadsPerWave; ++g) load_piece(Kh, sm.k, T, g, false);
    };
    auto issue_v = [&](int T) __attribute__((always_inline)) {
#pragma unroll
        for (int g = 0; g < kLoadsPerWave; ++g) load_piece(Vh, sm.v, T, g, true);
    };
    auto publish_gate = [&](int T) __attribute__((always_inline)) {  // wave 0: raw c it loaded itself -> accumulator initial values
        const int buf = T % kRing;
        sm.g[buf][lane] = (sm.craw[buf][lane] - cbase) * inv_scale;
    };

    f32x16 o[kQB][DB];
    float m[kQB], l[kQB];
    // the first key tile of the current query tile in flight
    auto open_tile = [&]() __attribute__((always_inline)) { issue_k(0); };
    auto start_tile = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_s_waitcnt(0);
        if (wv == 0) publish_gate(0);
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
    auto read_k = [&](int kc, int disp) __attribute__((always_inline)) -> bf16x8 {
        return *reinterpret_cast<__attribute__((address_space(3))) const bf16x8*>(kaddr[kc] + disp);
    };
    auto read_vt = [&](int db, int disp) __attribute__((always_inline)) -> bf16x8 {
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vaddr[db][0] + disp));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vaddr[db][1] + disp));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto read_g = [&](f32x16& acc, int disp) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const f32x4 g4 = *reinterpret_cast<__attribute__((address_space(3))) const f32x4*>(gaddr + disp + 32 * r);
            acc[4 * r] = g4[0];
            acc[4 * r + 1] = g4[1];
            acc[4 * r + 2] = g4[2];
            acc[4 * r + 3] = g4[3];
        }
    };

    // ---- per-wave software pipeline over 32-key blocks.  Block n = 2 T + b (b = 0: upper half of tile T):
    //   iteration n:   matrix pipe   S(n) = g + K Q^T           (K tile T)
    //                                O   += V^T P(n-2)          (V tile T-1)
    //                  vector unit   P(n-1) = exp2(S(n-1) sl - m sl), row sums
    // S(n) lives in s[b], P(n) in pf[b], each for the kQB query blocks of the wave.  A wave runs the
    // iterations n_first .. n_last + 2 of its own band [n_first, n_last]; there is one code path: outside the
    // band the initial value of S is minus infinity (the band mask is applied to the accumulator's initial value,
    // before the MFMA chain, and only on blocks that the diagonal or the window edge cuts or that lie outside),
    // so such a block's probabilities are exactly zero and its products add nothing.
    f32x16 s[2][kQB];
    u32x4 pf[2][kQB][2];
    int n_first, n_last;  // this wave's blocks (n_first > n_last: none)
    constexpr float kBig = 1.152921504606846976e18f;  // 2^60

    // two probabilities of block sb against the current reference exponent; their values are added to pa, pc
    auto expo_pair = [&](const f32x16& sb, u32x4 (&pb)[2], int cc, float nm, float& pa, float& pc)
                         __attribute__((always_inline)) {
        f32x2 pr = {fast_exp2(fmaf(sb[2 * cc], sl, nm)), fast_exp2(fmaf(sb[2 * cc + 1], sl, nm))};
        const bf16x2 pbf = __builtin_convertvector(pr, bf16x2);
        // plain adds: the packed dot-product instructions run on the matrix pipe and would queue
        // behind the MFMAs
        pa += pr[0];
        pc += pr[1];
        pb[cc >> 2][cc & 3] = __builtin_bit_cast(unsigned, pbf);
    };
    // slow path: true maximum of the block (common to the two halves of the wave), new reference,
    // rescale of O and l, exponentials once more.  Returns the block's row sum.
    auto raise_reference = [&](const f32x16& sb, u32x4 (&pb)[2], int qb) __attribute__((always_inline)) -> float {
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sb[v]);
        mx = xhalf_max(mx);
        const float mnew = fmaxf(m[qb], mx);
        const float a = fast_exp2((m[qb] - mnew) * sl);
        m[qb] = mnew;
        l[qb] *= a;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[qb][db][v] *= a;
        const float nm = -mnew * sl;
        float pa = 0.f, pc = 0.f;
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) expo_pair(sb, pb, cc, nm, pa, pc);
        return pa + pc;
    };

    // one iteration of the pipeline; ring slot and block are compile-time constants so that every LDS
    // address is a loop-invariant register plus an immediate
    auto iteration = [&](auto buf_c, auto blk_c, bool cut, int kb0, int T) __attribute__((always_inline)) {
        constexpr int buf = decltype(buf_c)::value;
        constexpr int b = decltype(blk_c)::value;
        constexpr int pbuf = (buf + kRing - 1) % kRing;  // slot of the previous tile's values
        constexpr int kdisp = buf * kTileBytes + 32 * (1 - b) * (D * 2);
        constexpr int vdisp = pbuf * kTileBytes + 32 * (1 - b) * (D * 2);
        constexpr int gdisp = buf * (kTileRows * 4) + 32 * (1 - b) * 4;
        f32x16 (&sn)[kQB] = s[b];           // S(n), written here
        f32x16 (&sx)[kQB] = s[1 - b];       // S(n-1), exponentiated here
        u32x4 (&px)[kQB][2] = pf[1 - b];    // P(n-1), written here
        u32x4 (&pp)[kQB][2] = pf[b];        // P(n-2), multiplied into O here
        constexpr int kAhead = 4, NF = 2 * KC;   // fragments per iteration, each feeding kQB MFMAs
        constexpr int kPairs = 8 * kQB;          // element pairs of the softmax, spread evenly over the NF steps
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) read_g(sn[qb], gdisp);
        if (__builtin_expect(cut, 0)) {  // the band mask, on the initial value: key i of the block for query t inside  t-w < i <= t, i >= 0
#pragma unroll
            for (int qb = 0; qb < kQB; ++qb) {
                const int t = t0 + 32 * qb;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = kb0 + acc_row(v, h);
                    sn[qb][v] = ((unsigned)i <= (unsigned)t && i > t - w) ? sn[qb][v] : -INFINITY;
                }
            }
        }
        bf16x8 fr[NF];  // fragment i: even i: V^T fragment i / 2 of the PV product, odd i: K chunk i / 2
        auto fetch = [&](int i) __attribute__((always_inline)) {
            if (i & 1) {
                fr[i] = read_k(i / 2, kdisp);
            } else {
                const int g = i / 2, c2 = g / DB, db = g % DB;
                fr[i] = read_vt(db, vdisp + 16 * c2 * (D * 2));
            }
        };
#pragma unroll
        for (int f = 0; f < kAhead; ++f) fetch(f);
        __builtin_amdgcn_sched_group_barrier(0x100, 3 * kAhead / 2, 0);
        float nm[kQB], pa[kQB], pc[kQB];
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) {
            nm[qb] = -m[qb] * sl;
            pa[qb] = pc[qb] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < NF; ++i) {
#pragma unroll
            for (int qb = 0; qb < kQB; ++qb) {
                if (i & 1) {
                    sn[qb] = mfma32(fr[i], qf[qb][i / 2], sn[qb]);
                } else {
                    const int g = i / 2, c2 = g / DB, db = g % DB;
                    o[qb][db] = mfma32(fr[i], __builtin_bit_cast(bf16x8, pp[qb][c2]), o[qb][db]);
                }
            }
            __builtin_amdgcn_sched_group_barrier(0x008, kQB, 0);
            if (i + kAhead < NF) {
                fetch(i + kAhead);
                if ((i + kAhead) & 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                else __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
            // this wave's share of the step's tile loads, spread between the MFMAs so that the load unit's
            // queue never fills: block 0 issues the keys of tile T+1 (and their gate values), block 1 the values of tile T
            if (b == 0 && (i == NF / 4 || i == NF / 2 || i == 3 * NF / 4)) {  // in groups (inline assembly the scheduler cannot move work across)
                // the keys of tile T+1, their gate values and the values of tile T, all in the first block of the step:
                // every slot they go to has been idle since the step began
                if (i == NF / 4) {
                    load_gate(T + 1);
#pragma unroll
                    for (int g = 0; g < kLoadsPerWave; ++g) load_piece(Kh, sm.k, T + 1, g, false);
                } else {
                    const int g0 = i == NF / 2 ? 0 : kLoadsPerWave / 2, g1 = i == NF / 2 ? kLoadsPerWave / 2 : kLoadsPerWave;
#pragma unroll
                    for (int g = g0; g < g1; ++g) load_piece(Vh, sm.v, T, g, true);
                }
            }
            // the softmax of block n-1: pairs [i kPairs / NF, (i + 1) kPairs / NF) in this step
#pragma unroll
            for (int pair = i * kPairs / NF; pair < (i + 1) * kPairs / NF; ++pair) {
                const int qb = pair / 8, cc = pair % 8;
                expo_pair(sx[qb], px[qb], cc, nm[qb], pa[qb], pc[qb]);
            }
            // (no scheduling groups for the vector work: left alone, the scheduler spreads it between the MFMAs)
        }
#pragma unroll
        for (int qb = 0; qb < kQB; ++qb) {
            float tsum = pa[qb] + pc[qb];
            if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(tsum <= kBig)) != 0, 0)) tsum = raise_reference(sx[qb], px[qb], qb);
            l[qb] += tsum;
        }
    };

    // one key tile: two iterations, then the one workgroup barrier of the tile.  Step T reads the keys of
    // tile T and the values of tile T-1; the keys of tile T+1 and the values of tile T are loaded meanwhile,
    // into the slots whose last readers (step T-1) the previous barrier has seen off.
    auto end_step = [&](int T) __attribute__((always_inline)) {
        __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
        if (wv == 0 && T + 1 < ntiles) publish_gate(T + 1);
        wg_barrier();
    };
    // whole block (first key kb0, number n) inside the band of all queries of the wave?  (a block outside the band,
    // at most one at either end of the steps a wave takes part in, runs fully masked)
    auto is_full = [&](int kb0, int n) __attribute__((always_inline)) { return (kb0 + 31 <= qw0) && (kb0 > qw0 + 32 * kQB - 1 - w) && (n <= n_last); };
    auto tile_step = [&](auto buf_c, int T) __attribute__((always_inline)) {
        const int kt0 = (j_hi - T) * kTileRows;
        iteration(buf_c, std::integral_constant<int, 0>{}, !is_full(kt0 + 32, 2 * T), kt0 + 32, T);
        iteration(buf_c, std::integral_constant<int, 1>{}, !is_full(kt0, 2 * T + 1), kt0, T);
        end_step(T);
    };
    // a step in which this wave has nothing to compute: only its share of the loads
    auto load_step = [&](int T) __attribute__((always_inline)) {
        issue_k(T + 1);
        issue_v(T);
        end_step(T);
    };
    static_assert(kRing == 2, "the tile loop is unrolled over the ring");
    for (;;) {  // query tiles of this workgroup
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[qb][db][v] = 0.0f;
        m[qb] = kNegBig;
        l[qb] = 0.0f;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s[b][qb][v] = -INFINITY;
#pragma unroll
            for (int e = 0; e < 4; ++e) pf[b][qb][0][e] = pf[b][qb][1][e] = 0u;
        }
    }
    {   // blocks of this wave's band, numbered in visiting order (descending keys from tile j_hi)
        const int khi = min(qw0 + 32 * kQB - 1, N - 1), klo = max(0, qw0 - w + 1);
        auto block_of = [&](int key) __attribute__((always_inline)) { return 2 * (j_hi - key / kTileRows) + 1 - (key % kTileRows) / 32; };
        n_first = block_of(khi);
        n_last = qw0 < N ? block_of(klo) : n_first - 3;
    }
    plan_next();
    // T = ntiles is the drain step (softmax of the last block, PV products of the last tile)
    {
        // steps this wave computes in: T_first .. T_last (its blocks n_first .. n_last + 2); the others only load
        const int T_first = min(n_first / 2, ntiles + 1), T_last = min((n_last + 2) / 2, ntiles);
        int T = 0;
        for (; T < T_first; ++T) load_step(T);
        if (T <= T_last && (T & 1)) {
            tile_step(std::integral_constant<int, 1>{}, T);
            ++T;
        }
        for (; T + 1 <= T_last; T += 2) {
            tile_step(std::integral_constant<int, 0>{}, T);
            tile_step(std::integral_constant<int, 1>{}, T + 1);
        }
        if (T <= T_last) {
            tile_step(std::integral_constant<int, 0>{}, T);
            ++T;
        }
        for (; T <= ntiles; ++T) load_step(T);
    }

    // all LDS reads of this query tile are done (last barrier): open the next one before storing
    const int t_done = t0, bh_done = bh;
    const size_t head_done = head_off;
    float cq_done[kQB];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) cq_done[qb] = cq[qb];
    const bool more = tile_of(wg_step + 1) < total_tiles;
    if (more) {
        tile = tile_of(++wg_step);
        set_tile(tile);
        open_tile();
        load_query_gates();  // requested now, first used when the tile ends
    }
    // ---- epilogue: O = O^T / l, L = ln2 * (m*sl + log2 l) - (c_t - c_base)
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
        const float lt = xhalf_sum(l[qb]);  // the two halves of the wave hold complementary keys
        const int t = t_done + 32 * qb;
        const float inv = 1.0f / lt;
        if (t < N && h == 0) L[(size_t)bh_done * N + t] = (m[qb] * sl + fast_log2(lt)) * kLn2 - cq_done[qb];
        // O as whole lines, through 4 KB per wave of the V ring (idle until the first step of the next tile; slot 0 may
        // hold the second half of the next tile's queries, slot 1 is free in either case)
        const int row0 = t - lq;
        store_acc_rows<DB>(o[qb], inv, sm.v[kStageQ ? 1 : 0] + 4096 * wv, O + head_done + (size_t)row0 * D, N - row0, lane);
    }
    if (!more) break;
    // the Q fragments, after the stores (they would otherwise be live beside the accumulators): from the rings if the
    // drain step has fetched them (rows 32 wv .. of the 128: waves 0, 1 from K slot 1, waves 2, 3 from V slot 0)
    if (kStageQ && stage_T >= 0) {
        const int disp = (wv < 2 ? 1 : kRing) * kTileBytes + (wv & 1) * 32 * (D * 2);
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) qf[0][kc] = read_k(kc, disp);
    } else {
        load_queries();
    }
    start_tile();
    }
}

template <int D>
static hipError_t launch_fwd(const void* Q, const void* K, const void* V, const float* c, void* O,
                             float* L, int B, int H, int Hkv, int N, int w, float scale, hipStream_t s) {
    const int num_qtiles = (N + kFwdBR<D> - 1) / kFwdBR<D>;
    const int total = B * H * num_qtiles;
    static DeviceOnce lds_allowed;
    if (hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(&fwd_bf16_kernel<D>), sizeof(FwdSmem<D>),
                                         lds_allowed))
        return e;
    const int num_cu = device_cu_count();
    const int grid = total < kFwdResident<D> * num_cu ? total : kFwdResident<D> * num_cu;  // every workgroup resident
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
