/*
 * gfwa.h -- C ABI of libgfwa: GatedFWA (memory-gated sliding-window softmax attention)
 * for AMD MI355X (gfx950).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - All data pointers are DEVICE pointers owned by the caller.  The library allocates no
 *    device memory and never frees anything (the one fixed-size array gfwa_decode_static works
 *    in is part of the library's code object).  Inputs are never written; outputs are fully
 *    overwritten (no accumulate-into semantics).
 *  - Dense row-major layouts: Q, K, V, O, dO, dQ, dK, dV are [B, H, N, d] with d fastest;
 *    alpha, c, L, dalpha are [B, H, N] with N fastest.  Matrix pointers must be 16-byte
 *    aligned, vector pointers 4-byte aligned.
 *  - `stream` is the caller's HIP stream (NULL = the default stream).  Work is enqueued and
 *    the call returns without synchronising.
 *  - Positions are 0-indexed.  Query t attends to keys i with  t - w < i <= t  and  i >= 0.
 *    w >= 1; w >= N is legal and means plain causal attention with the gate bias.
 *  - Return value: GFWA_OK or a negative gfwa_status_t.  On error nothing is launched and
 *    nothing is written.  alpha < 0 or non-finite inputs are not checked: results undefined.
 */
#ifndef GFWA_H
#define GFWA_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ihipStream_t *gfwa_stream_t;

/* Storage type of the matrices.  A plain int at the boundary (any value may arrive from a caller; the
 * entry points answer GFWA_ERR_UNSUPPORTED to those that are not listed here). */
typedef int gfwa_dtype_t;
enum {
    GFWA_BF16 = 0, /* Q,K,V,O,dO,dQ,dK,dV stored as bfloat16; products on bf16 MFMA, fp32 accumulate */
    GFWA_F32 = 1   /* stored as float; all arithmetic fp32 */
};

typedef enum {
    GFWA_OK = 0,
    GFWA_ERR_NULL = -1,        /* a required pointer is NULL */
    GFWA_ERR_DIM = -2,         /* B, H, N or d <= 0, w < 1, or B*H*N*d exceeds the index range */
    GFWA_ERR_UNSUPPORTED = -3, /* d not in {64, 128} or unknown dtype */
    GFWA_ERR_ALIGN = -4,       /* pointer alignment */
    GFWA_ERR_WORKSPACE = -5,   /* workspace NULL or smaller than the matching gfwa_*_workspace_bytes() call
                                  (backward, decode, scan-then-propagate) asks for; gfwa_decode_static:
                                  the sizes need more than the library's own scratch holds */
    GFWA_ERR_HIP = -6          /* the HIP runtime refused a launch; see gfwa_strerror */
} gfwa_status_t;

/*
 * Gate preprocessing, scan part (paper Sec. 3.2, definition of u_t; Alg. 1, the cumulative-sum
 * and carry steps; Sec. 3.3 "Gate Preprocessing via Fused Tiled Scan").
 *
 *   c[b,h,t] = sum_{q <= t} alpha[b,h,q]        (inclusive; c = -u in the paper's notation)
 *
 * alpha: [B,H,N] fp32, expected >= 0.   c: [B,H,N] fp32 out.  fp32 accumulation.
 */
int gfwa_gate_prefix(const float *alpha, float *c, int B, int H, int N, gfwa_stream_t stream);

/*
 * Gate preprocessing as a whole (paper Sec. 3.2, the equation that defines alpha from the gate
 * pre-activation h and the amplitude beta; Alg. 1 complete: activation with the overflow-safe
 * softplus, scan and carry in one pass; Sec. 3.3 "Gate Preprocessing via Fused Tiled Scan"):
 *
 *   alpha = softplus(beta * h) / (beta + eps),     c[b,h,t] = sum_{q <= t} alpha[b,h,q]
 *
 * hpre, beta: [B,H,N] fp32 (head-major, like alpha; beta > 0 expected, eps >= 0);  c: [B,H,N] fp32 out.
 * Neither alpha nor beta*h is written to memory: 12 bytes of traffic per element.
 */
int gfwa_gate_activation_prefix(const float *hpre, const float *beta, float eps, float *c, int B, int H,
                                int N, gfwa_stream_t stream);

/*
 * The same prefix by scan-then-propagate (paper App. "Preprocessing via Scan-Then-Propagate"): every row
 * is cut into segments, one launch sums the segments (recomputing the activation), a second one scans
 * each segment starting from the fp64 sum of the segments before it.  It reads the inputs twice and is
 * meant for few, very long rows, where one workgroup per row leaves the chip idle.
 * in: [B,H,N] fp32 - alpha when beta is NULL (eps ignored), else the pre-activation h with beta [B,H,N]
 * as in gfwa_gate_activation_prefix.  c: [B,H,N] fp32 out.  workspace: device scratch of at least
 * gfwa_gate_scan_workspace_bytes(B, H, N) bytes, 8-byte aligned, contents undefined before and after.
 */
size_t gfwa_gate_scan_workspace_bytes(int B, int H, int N);
int gfwa_gate_prefix_stp(const float *in, const float *beta, float eps, float *c, void *workspace,
                         size_t workspace_bytes, int B, int H, int N, gfwa_stream_t stream);

/*
 * Its derivative (chain rule on the definition in Sec. 3.2; the paper prints no listing for it):
 * from d(alpha) as gfwa_backward returns it,
 *
 *   dh    = dalpha * sigma(beta h) * beta / (beta + eps)
 *   dbeta = dalpha * (sigma(beta h) * h / (beta + eps) - softplus(beta h) / (beta + eps)^2)
 *
 * hpre, beta, dalpha: [B,H,N] fp32;  dh, dbeta: [B,H,N] fp32 out.
 */
int gfwa_gate_activation_backward(const float *hpre, const float *beta, float eps, const float *dalpha,
                                  float *dh, float *dbeta, int B, int H, int N, gfwa_stream_t stream);

/*
 * Fused forward (paper Sec. 3.2, the gated score; Alg. 2).  For every (b,h) and query t:
 *
 *   S_ti = scale * <q_t, k_i> + (c_i - c_t)     for  max(0, t-w+1) <= i <= t
 *   O_t  = sum_i softmax_i(S_ti) v_i
 *   L_t  = log sum_i exp(S_ti)                  (natural log; what Alg. 2 returns as m + log l)
 *
 * The N x N matrix is never formed; key tiles wholly outside the band are skipped.
 * `scale` multiplies q.k only (1/sqrt(d) in the paper's workloads), never the bias.
 * Q,K,V: [B,H,N,d] of dtype `dt`;  c: [B,H,N] fp32 (from gfwa_gate_prefix);
 * O: [B,H,N,d] of dtype `dt`, out;  L: [B,H,N] fp32, out.   d in {64, 128}.
 */
int gfwa_forward(gfwa_dtype_t dt, const void *Q, const void *K, const void *V, const float *c,
                 void *O, float *L, int B, int H, int N, int d, int w, float scale,
                 gfwa_stream_t stream);

/* Bytes of device scratch gfwa_backward needs at least for these sizes (0 on invalid sizes). */
size_t gfwa_backward_workspace_bytes(gfwa_dtype_t dt, int B, int H, int N, int d, int w);
/*
 * Bytes of device scratch with which gfwa_backward runs its faster variant (0 on invalid sizes; equal to
 * gfwa_backward_workspace_bytes where there is no such variant: fp32, d = 64).  The variant keeps the dS
 * blocks of App. E.2 the dK/dV pass forms (bf16, about 2 (w + 48) bytes per token and head) for the dQ pass
 * instead of forming S and dP twice; same outputs to the rounding of dS, which both passes apply anyway.
 */
size_t gfwa_backward_fast_workspace_bytes(gfwa_dtype_t dt, int B, int H, int N, int d, int w);

/*
 * Backward (paper App. E.2, Alg. 3, plus the chain-rule factor `scale` on dQ and dK and the
 * reverse scan of Sec. 3.3 "gradients into U flow through the same streamed scan").
 * With P_ti = exp(S_ti - L_t) recomputed from the saved L:
 *
 *   D_t   = <dO_t, O_t>                         dP_ti = <dO_t, v_i>
 *   dS_ti = P_ti (dP_ti - D_t)
 *   dV_i  = sum_t P_ti dO_t                     dK_i = scale * sum_t dS_ti q_t
 *   dQ_t  = scale * sum_i dS_ti k_i
 *   dc_p  = sum_t dS_tp - sum_i dS_pi           dalpha_q = sum_{p >= q} dc_p
 *
 * Inputs: Q,K,V,O,dO [B,H,N,d] of dtype `dt` (O and L as written by gfwa_forward), c, L [B,H,N] fp32.
 * Outputs: dQ,dK,dV [B,H,N,d] of dtype `dt`; dalpha [B,H,N] fp32.
 * workspace: device scratch of at least gfwa_backward_workspace_bytes(...) bytes, 16-byte
 * aligned, contents undefined before and after the call; with workspace_bytes >=
 * gfwa_backward_fast_workspace_bytes(...) the faster variant runs.
 */
int gfwa_backward(gfwa_dtype_t dt, const void *Q, const void *K, const void *V, const void *O,
                  const void *dO, const float *c, const float *L, void *dQ, void *dK, void *dV,
                  float *dalpha, void *workspace, size_t workspace_bytes, int B, int H, int N,
                  int d, int w, float scale, gfwa_stream_t stream);

/*
 * Grouped-query layout of the two calls above (the group size heads_per_gqa_group of the paper's
 * training configurations, App. "Additional Experiment Details"; the paper gives no formula for it, the
 * usual meaning is taken): K, V, dK, dV are [B,Hkv,N,d] with Hkv dividing H, query head h reads the
 * keys and values of head h / (H / Hkv), and dK, dV sum over the H / Hkv query heads that read a head.
 * Everything per query head (Q, O, dO, dQ [B,H,N,d]; c, L, dalpha [B,H,N]; the workspace size) is as
 * above; Hkv == H is exactly gfwa_forward / gfwa_backward.
 */
int gfwa_forward_gqa(gfwa_dtype_t dt, const void *Q, const void *K, const void *V, const float *c,
                     void *O, float *L, int B, int H, int Hkv, int N, int d, int w, float scale,
                     gfwa_stream_t stream);
int gfwa_backward_gqa(gfwa_dtype_t dt, const void *Q, const void *K, const void *V, const void *O,
                      const void *dO, const float *c, const float *L, void *dQ, void *dK, void *dV,
                      float *dalpha, void *workspace, size_t workspace_bytes, int B, int H, int Hkv,
                      int N, int d, int w, float scale, gfwa_stream_t stream);

/*
 * Decoding step with a key/value cache (paper Sec. 1: with a KV cache the method costs O(wd) per
 * generated token; the arithmetic is row `pos` of the forward, Sec. 3.2 / Alg. 2).  For every batch
 * entry b with current position p = pos[b] and every query head h (grouped-query layout as above):
 *
 *   S_i = scale * <q, k_i> + (c_i - c_p)        for  max(0, p-w+1) <= i <= p
 *   o   = sum_i softmax_i(S_i) v_i              L = log sum_i exp(S_i)
 *
 * q: [B,H,d] of dtype `dt`, the new token's query.  Kc, Vc: [B,Hkv,T,d] of dtype `dt`, the caches; rows
 * 0..p of entry b must hold the keys and values of positions 0..p (the caller appends row p before
 * the call); rows past p are not read.  pos: [B] int32 in device memory, 0 <= pos[b] < T (a value
 * outside is clamped into the range).  c: [B,H,T] fp32 gate prefix.  If alpha_t ([B,H] fp32, the new
 * token's gate) is not NULL the call advances the prefix itself, c[b,h,p] = c[b,h,p-1] + alpha_t[b,h]
 * (c[b,h,-1] = 0), stores it and uses it; with alpha_t == NULL, c[b,h,p] must already be there.
 * o: [B,H,d] of dtype `dt`, out.  L: [B,H] fp32 out, may be NULL.  workspace: device scratch of at least
 * gfwa_decode_workspace_bytes(...) bytes, 16-byte aligned, contents undefined before and after.
 * Only the window is read: 2 * min(w, p+1) * d cache elements per key/value head.
 */
size_t gfwa_decode_workspace_bytes(int B, int H, int T, int d, int w);
int gfwa_decode(gfwa_dtype_t dt, const void *q, const void *Kc, const void *Vc, float *c,
                const float *alpha_t, const int *pos, void *o, float *L, void *workspace,
                size_t workspace_bytes, int B, int H, int Hkv, int T, int d, int w, float scale,
                gfwa_stream_t stream);

/*
 * gfwa_decode for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * kernels as gfwa_decode, but the per-chunk partial results live in a 32 MiB array inside the
 * library's code object (one copy per GPU, held until the process ends); the call allocates and
 * frees nothing.  Sizes with gfwa_decode_workspace_bytes(B, H, T, d, w) > 33554432 are rejected with
 * GFWA_ERR_WORKSPACE and nothing is launched.  All calls on one GPU share that array: two calls that
 * may run at the same time on one GPU (different streams) race and must be serialised by the caller;
 * calls on one stream are ordered and safe.  Nothing in the array has to start at zero.
 */
int gfwa_decode_static(gfwa_dtype_t dt, const void *q, const void *Kc, const void *Vc, float *c,
                       const float *alpha_t, const int *pos, void *o, float *L, int B, int H, int Hkv,
                       int T, int d, int w, float scale, gfwa_stream_t stream);

/* Static, human-readable text for a status code (for GFWA_ERR_HIP: the last HIP error text). */
const char *gfwa_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int gfwa_version(void);

/*
 * Instrumentation (not part of the method): per-kernel timing with HIP events recorded on the
 * caller's stream around every kernel the library launches.  gfwa_profile_enable(1) clears the
 * records and starts recording (at most 8192 launches are kept), gfwa_profile_enable(0) stops.
 * gfwa_profile_read waits for the recorded events and returns, per kernel id k in [0, 13), the
 * summed duration in milliseconds and the number of launches; n must be >= 13.  Kernel ids:
 * 0 gate prefix scan, 1 forward, 2 backward row-dot (D), 3 backward dK/dV, 4 backward dQ,
 * 5 gate-gradient reverse scan, 6 gate activation + prefix scan, 7 gate activation backward,
 * 8 decoding step (per-chunk partials), 9 decoding step (merge of the chunks), 10 and 11 the two
 * launches of gfwa_gate_prefix_stp (segment sums, scan of the segments), 12 the segment sums of the
 * gate-gradient scan when the backward cuts few long rows into segments (its scan is then id 5);
 * gfwa_profile_kernel_name gives the same as text.
 * An event pair costs a few microseconds on the stream: kernels of about ten microseconds read
 * correspondingly longer than in a trace.  The three calls may come from any host thread (the records
 * are kept under a lock; the stop event of a launch is recorded by the thread that made it); a
 * launch still in progress on another thread while gfwa_profile_read runs may be read before its
 * stop event is recorded, so read after the launching threads are done.  Host memory only.
 */
int gfwa_profile_enable(int on);
int gfwa_profile_read(float *total_ms, int *launches, int n);
const char *gfwa_profile_kernel_name(int k);

/*
 * Calibration (not part of the method): what the device at hand sustains, for the rooflines the
 * attention kernels are reported against.
 * gfwa_probe_mfma runs a loop of `iterations` x 16 bf16 32x32x16 MFMAs per wave on `workgroups`
 * workgroups of 8 waves (two per SIMD; use a multiple of the number of compute units) and writes
 * the floating-point operations of the launch to *flops (host memory, may be NULL); `sink` is one
 * device float the kernel may write.  random_operands = 0: one pair of operand registers with small
 * constant values (the rate at the highest clock the part reaches with busy matrix cores);
 * 1: sixteen pairs of pseudo-random unit-variance operands, as the attention inputs are (the rate at
 * the clock the part sustains when operands switch as on real data); 2: the same with the least
 * companion work an attention inner loop has per MFMA (one operand fragment read from LDS, four
 * fused multiply-adds and one exp2 on the vector unit); other values: GFWA_ERR_DIM.  gfwa_probe_copy copies
 * `bytes` (a multiple of 16) from src to dst (device, 16-byte aligned) with plain 16-byte accesses:
 * 2 * bytes of memory traffic.  Both only enqueue; the caller times them on its stream.
 */
int gfwa_probe_mfma(float *sink, int iterations, int workgroups, int random_operands, double *flops,
                    gfwa_stream_t stream);
int gfwa_probe_copy(const void *src, void *dst, size_t bytes, gfwa_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* GFWA_H */
