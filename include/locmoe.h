/*
 * locmoe.h - C ABI of the MI355X (gfx950) forward hot path of one LocMoE mixture-of-experts
 * layer (arXiv 2401.13920, Section 3.2) on one GPU's share of the tokens:
 *
 *   GrAP gate -> top-1 route (+ auxiliary / locality terms) -> capacity-bounded stable
 *   dispatch into a node-grouped send buffer -> expert FFN (grouped GEMM) -> combine.
 *
 * Conventions
 *   - Plain C, no exceptions cross the boundary.  Every function returns an int status:
 *     LOCMOE_OK (0) or a negative LOCMOE_ERR_* code; locmoe_status_string() names it.
 *   - All arguments are validated on the host before anything is launched, so the error
 *     paths work without a GPU.
 *   - "device" pointers are HIP device memory, 16-byte aligned, rows contiguous.  The caller
 *     owns every buffer; the library allocates nothing and keeps no state between calls: every
 *     entry point is re-entrant (any number of calls may be in flight on any streams and host
 *     threads) as long as concurrent calls are given different output and workspace buffers.
 *     The one exception is locmoe_dispatch_static, which says so.
 *   - Device functions only enqueue kernels on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and return; the caller synchronises.
 *   - Notation (the paper's where it has one): T tokens, d hidden size, E experts (the
 *     paper's n), N simulated nodes, h FFN inner width, C expert capacity in rows,
 *     cnt[e] tokens whose top-1 expert is e, kept[e] = min(cnt[e], C), K = sum kept[e].
 *   - Shape limits: d % E == 0; E % N == 0 is NOT required (e2n is free-form);
 *     d % 8 == 0 and h % 8 == 0 (16-byte rows); 1 <= E <= 1024; 1 <= N <= E;
 *     T*max(d,h) element offsets must fit in 63 bits and T, E*C in 31 bits.
 */
#ifndef LOCMOE_H
#define LOCMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  LOCMOE_OK = 0,
  LOCMOE_ERR_NULL = -1,      /* a required pointer is NULL */
  LOCMOE_ERR_SHAPE = -2,     /* a size is < 1 or breaks a divisibility / range limit above */
  LOCMOE_ERR_ARG = -3,       /* bad dtype / flag / delta / capacity-factor value */
  LOCMOE_ERR_WORKSPACE = -4, /* workspace pointer NULL or smaller than locmoe_workspace_bytes */
  LOCMOE_ERR_HIP = -5        /* a HIP launch failed (hipGetLastError was not hipSuccess) */
};

enum { LOCMOE_F32 = 0, LOCMOE_BF16 = 1 };

/* Shape of one MoE layer call.  x_dtype is the storage type of x, send, out and y; expert
 * weights and the FFN intermediate are always bf16; gating values and scores are fp32. */
typedef struct locmoe_desc {
  int32_t T, d, E, N, h, C;
  int32_t x_dtype; /* LOCMOE_F32 or LOCMOE_BF16 */
  int32_t relu;    /* 1: G = ReLU(g + eps) as printed below Eq. 3; 0: G = g + eps */
  int32_t w_packed; /* 0: W_in/W_out row-major; 1: both in the layout written by locmoe_pack_weights */
  float alpha;     /* auxiliary-loss weight of Eq. 5 (the paper uses 0.01) */
  float mu;        /* locality-loss weight of Eq. 6 (left open by the paper) */
} locmoe_desc;

const char* locmoe_status_string(int status);

/* ---- host-only scalars (Section 3.2.3) ------------------------------------------------ */

/* Theorem 1: lower bound of the expert capacity, in tokens, from the cosine threshold delta of
 * Assumption 3.  form 0: 1/(E*p_delta) with Lemma 3's p_delta = 1 - I_{delta^2}(1/2,(d-1)/2);
 * form 1: the large-d form 1/(E*erfc(sqrt(y))); form 2: exp(y)/E; y = delta^2 d/(2-delta^2).
 * Host pointers.  *ec_min may be +inf.  Errors: NULL, E<1, d<2, delta outside (0,1), form. */
int locmoe_capacity_min(int32_t E, int32_t d, double delta, int32_t form, double* ec_min);

/* Lemma 3: *p = 1 - I_{delta^2}(1/2,(d-1)/2).  Host pointer.  delta in [0,1], d >= 2. */
int locmoe_p_delta(int32_t d, double delta, double* p);

/* Capacity in rows per expert: the empirical capacity of Section 3.2.3 on one device's share,
 * ceil(cf*T/E), floored by ceil of the Theorem 1 bound (form 1) and clamped to [1,T].
 * cf == 0 selects the bound alone.  Host pointer.  Errors: NULL, sizes < 1, cf < 0, delta. */
int locmoe_capacity(int32_t T, int32_t E, int32_t d, double cf, double delta, int32_t* C);

/* Bytes of device scratch that locmoe_route and locmoe_dispatch need (one buffer serves
 * both, they do not overlap in time on one stream).  0 on an invalid descriptor. */
size_t locmoe_workspace_bytes(const locmoe_desc* desc);

/* ---- device steps ---------------------------------------------------------------------- */

/* GrAP gating value (Eq. 4 and the text below Eq. 3): g[m,i] = omega_i . x_m = mean of the
 * i-th contiguous block of d/E features of token m, accumulated in fp32.  Raw value: the
 * bias and the ReLU are applied by locmoe_route.
 *   x  device [T,d] of x_dtype (read)      g  device [T,E] fp32 (written)              */
int locmoe_gate(const locmoe_desc* desc, const void* x, float* g, void* stream);

/* Top-1 routing (Eq. 2, Eq. 3) and the forward values of Eq. 5 and Eq. 6.
 *   G = g + eps (eps NULL = 0), ReLU if desc->relu; eid[m] = lowest index attaining max_i G;
 *   w[m] = softmax(G[m,:])[eid[m]]; cnt[e] = #{m: eid[m]=e}; Psum[e] = sum_m softmax(G[m,:])[e].
 *   stats[0] L_aux = alpha*E*sum f_i P_i (f = cnt/T before any capacity drop, P = Psum/T)
 *   stats[1] KL(f || D_l)   stats[2] KL(P || D_l)   stats[3] L_loc = mu*stats[1]
 *   stats[4] fraction of tokens whose expert sits on their home node
 *   stats[5] max_e cnt[e]   stats[6] number of experts with cnt = 0   stats[7] 0
 *   D_l[i] = (#tokens whose home is node(i)) / (T * #experts on node(i)): every token spread
 *   evenly over the experts of its home node.  0 ln 0 = 0; KL = +inf if D_l[i] = 0 < D_c[i].
 *   home NULL: stats[1..4] = 0.
 *   g device [T,E] fp32; eps device [E] fp32 or NULL; home device [T] i32 in [0,N) or NULL;
 *   e2n device [E] i32 in [0,N) or NULL (= e / (E/N), which then needs E % N == 0);
 *   eid device [T] i32, w device [T] fp32, cnt device [E] i32, Psum device [E] fp32,
 *   stats device [8] fp32 (all written); ws device scratch of >= locmoe_workspace_bytes.
 * Sums are formed in a fixed order (no floating-point atomics): results are deterministic. */
int locmoe_route(const locmoe_desc* desc, const float* g, const float* eps, const int32_t* home,
                 const int32_t* e2n, int32_t* eid, float* w, int32_t* cnt, float* Psum,
                 float* stats, void* ws, size_t ws_bytes, void* stream);

/* The gating value together with the block sums of squares, in the same pass over x:
 *   g as in locmoe_gate;  q[m,i] = sum over block i of x[m,j]^2, so that |x_m|^2 = sum_i q[m,i].
 *   With Eq. 4's weight (|omega_i| = sqrt(E/d)) the cosine between token m and gating weight i
 *   (delta_{i,j} of Section 3.2.3) is g[m,i] * sqrt(d/E) / |x_m|.
 *   x device [T,d] of x_dtype; g, q device [T,E] fp32 (written). */
int locmoe_gate_sq(const locmoe_desc* desc, const void* x, float* g, float* q, void* stream);

/* Angles between tokens and gating weights: the measurement of Section 4.1 ("Analysis for Expert
 * Capacity") from which the paper reads its delta.  For token m routed to expert e = eid[m]:
 *   c_self[m]  = cos(x_m, omega_e),  c_other[m] = cos(x_m, omega_{(e + shift) mod E})  (0 for a zero token);
 *   hist_self[e][b], hist_other[e][b] count the tokens routed to e by bin b = floor((c + 1)/2 * nbins),
 *   clamped to [0, nbins-1], of c_self resp. c_other;  cmin[e] = min c_self over the tokens routed to e
 *   (2.0 for an expert without tokens);  stats[0] = delta_hat = min_e cmin[e], the literal reading of the
 *   assumption in Section 3.2.3 (every routed token has delta_{i,j} >= delta); stats[1] = number of
 *   experts with tokens; stats[2..3] = 0.
 *   g, q device [T,E] fp32 from locmoe_gate_sq; eid device [T] i32 in [0,E); 1 <= nbins <= 65536;
 *   c_self, c_other device [T] fp32 or NULL; hist_self, hist_other device [E*nbins] i32; cmin device [E]
 *   fp32; stats device [4] fp32 (all written; no workspace).  Counts and minima only: independent of
 *   the order in which tokens are processed. */
int locmoe_angle_stats(const locmoe_desc* desc, const float* g, const float* q, const int32_t* eid,
                       int32_t shift, int32_t nbins, float* c_self, float* c_other, int32_t* hist_self,
                       int32_t* hist_other, float* cmin, float* stats, void* stream);

/* Capacity-bounded stable dispatch (capacity: Section 3.2.3; layout: this library's).
 *   pos[m] = #{m' < m : eid[m'] = eid[m]}; token m is kept iff pos[m] < C (first come by token
 *   index).  Experts are laid out in buffer order = sorted by (e2n[e], e); rank r holds expert
 *   buf_expert[r] in rows [seg_off[r], seg_off[r+1]), kept[e] rows in token order; node nu owns
 *   rows [node_off[nu], node_off[nu+1]).  slot[m] = seg_off[rank(eid[m])] + pos[m] or -1 when
 *   dropped; row_token[slot[m]] = m; send[slot[m],:] = x[m,:] (bit copy).  K = seg_off[E].
 *   x device [T,d]; eid device [T] i32 in [0,E); e2n as in locmoe_route;
 *   written: pos [T], slot [T], kept [E], seg_off [E+1], node_off [N+1], buf_expert [E],
 *   row_token [E*C] (first K valid), send [E*C,d] of x_dtype (first K rows valid; rows >= K
 *   are left untouched).  ws as in locmoe_route.  Integer-only and independent of any
 *   atomic arrival order: bit-identical from run to run. */
int locmoe_dispatch(const locmoe_desc* desc, const void* x, const int32_t* eid, const int32_t* e2n,
                    int32_t* pos, int32_t* slot, int32_t* kept, int32_t* seg_off, int32_t* node_off,
                    int32_t* buf_expert, int32_t* row_token, void* send, void* ws, size_t ws_bytes,
                    void* stream);

/* locmoe_dispatch for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same kernels and the same results, bit for bit, with the scratch
 * (the per-block expert counts, ceil(T/1024) * E int32) in a static device array inside the library instead of a
 * caller workspace.  Limit: ceil(T/1024) * E <= LOCMOE_DISPATCH_STATIC_MAX_COUNTS (1 MiB of counts), else
 * LOCMOE_ERR_WORKSPACE.  The call allocates nothing and frees nothing.  The array's device address is looked up
 * once per device, on the first call made with that device current (make that call outside a graph capture);
 * LOCMOE_ERR_HIP if the lookup fails.  Every call on a device uses that device's one array: calls that overlap
 * on one device (other streams, other threads) race and must not be made; calls on one stream are ordered.
 * Nothing in the array has to be zero on entry (every count is written before it is read), and its contents
 * after a call are unspecified.  All other arguments, outputs and errors as locmoe_dispatch. */
#define LOCMOE_DISPATCH_STATIC_MAX_COUNTS 262144
int locmoe_dispatch_static(const locmoe_desc* desc, const void* x, const int32_t* eid, const int32_t* e2n,
                           int32_t* pos, int32_t* slot, int32_t* kept, int32_t* seg_off, int32_t* node_off,
                           int32_t* buf_expert, int32_t* row_token, void* send, void* stream);

/* Expert FFN of Eq. 1 as a grouped GEMM over the send buffer's segments:
 *   out[r,:] = W_out[e] . GeLU(W_in[e] . send[r,:]) for r in segment of e = buf_expert[rank],
 *   GeLU(v) = v*Phi(v) (erf form), no biases.  bf16 MFMA with fp32 accumulation; the
 *   intermediate is rounded once to bf16 (H_ws), out once to x_dtype.
 *   send device [E*C,d] of x_dtype; seg_off device [E+1]; buf_expert device [E];
 *   W_in device [E,h,d] bf16 and W_out device [E,d,h] bf16, row-major in Eq. 1's orientation;
 *   H_ws device [E*C,h] bf16 scratch; out device [E*C,d] of x_dtype (rows < K written).
 *   The row count K is read on the device from seg_off: no host synchronisation. */
int locmoe_expert_ffn(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                      const int32_t* buf_expert, const void* W_in, const void* W_out, void* H_ws,
                      void* out, void* stream);

/* One-time re-tiling of the static expert weights for the direct-to-LDS grouped GEMM (not part of
 * the timed path).  Needs d % 256 == 0, h % 256 == 0 and bf16 activations (x_dtype = LOCMOE_BF16);
 * locmoe_packed_weights_bytes returns the size of EACH packed tensor (E*h*d*2 bytes), or 0 when the
 * shape cannot be packed.  Packed layout: for expert e, 256-row tile nt and 32-column step kt, a
 * 16 KiB block at ((e*NT + nt)*KT + kt)*16 KiB whose 16-byte chunk p holds row r = p/4 of the tile,
 * columns 8*c .. 8*c+7 of the step with c = (p%4) ^ ((r/2)%4) - the LDS image the kernel consumes.
 * With desc->w_packed = 1 the three expert_ffn entry points take the packed tensors in place of
 * W_in / W_out (LOCMOE_ERR_ARG if the shape or dtype cannot use them); results are the same
 * to rounding order.  W_in [E,h,d], W_out [E,d,h] device bf16 (read); packed tensors device (written).
 * Tile scheduling of the packed-weight kernels (E a multiple of 8, at most 512; one work-group per compute unit
 * walks a list of output tiles): the entry points above and below assign tiles to work-groups in a fixed
 * round-robin order and need no memory beyond their arguments; the *_ws variants further down let the
 * work-groups claim tiles from queue words in a caller workspace, which evens out ragged segments (up to 10 %
 * less time on very uneven inputs).  Results are identical bit for bit either way.
 * No entry point allocates, clears memory or waits for the device, so calls may be recorded into a HIP graph. */
size_t locmoe_packed_weights_bytes(const locmoe_desc* desc);
int locmoe_pack_weights(const locmoe_desc* desc, const void* W_in, const void* W_out, void* W_in_packed,
                        void* W_out_packed, void* stream);

/* The two linear transformations of Eq. 1 as separate launches (locmoe_expert_ffn is exactly
 * _in followed by _out on the same stream); same buffers, layouts and errors as above.
 *   _in :  H_ws[r,:] = GeLU(W_in[e] . send[r,:])  (bf16)      _out:  out[r,:] = W_out[e] . H_ws[r,:] */
int locmoe_expert_ffn_in(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                         const int32_t* buf_expert, const void* W_in, void* H_ws, void* stream);
int locmoe_expert_ffn_out(const locmoe_desc* desc, const void* H_ws, const int32_t* seg_off,
                          const int32_t* buf_expert, const void* W_out, void* out, void* stream);

/* The expert FFN entry points with dynamic tile claims (same operation, same results bit for bit, see Eq. 1 above
 * and the backward section below for _in_save and _dgrad).
 *   ws  device memory, LOCMOE_FFN_WS_BYTES bytes, 4-byte aligned: two sets of queue words (first and second GEMM
 *       of a call).  Contract: all bytes zero when the first call that uses it is enqueued (the caller clears it
 *       once, e.g. at allocation); every launch returns its set to zero when its last work-group finishes, so the
 *       same ws serves any number of later calls.  Calls that may run concurrently (different streams, overlapping
 *       graph replays) must be given different ws; calls ordered on one stream may share one.  Shapes that do
 *       not use the packed-weight kernels ignore ws.  LOCMOE_ERR_WORKSPACE if ws is NULL, misaligned or
 *       ws_bytes < LOCMOE_FFN_WS_BYTES.  A workspace whose zero contract is broken gives wrong tile assignments
 *       (rows of the output missing or written twice), never an out-of-bounds access. */
#define LOCMOE_FFN_WS_BYTES 128
int locmoe_expert_ffn_ws(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                         const int32_t* buf_expert, const void* W_in, const void* W_out, void* H_ws, void* out,
                         void* ws, size_t ws_bytes, void* stream);
int locmoe_expert_ffn_in_ws(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                            const int32_t* buf_expert, const void* W_in, void* H_ws, void* ws, size_t ws_bytes,
                            void* stream);
int locmoe_expert_ffn_out_ws(const locmoe_desc* desc, const void* H_ws, const int32_t* seg_off,
                             const int32_t* buf_expert, const void* W_out, void* out, void* ws, size_t ws_bytes,
                             void* stream);
int locmoe_expert_ffn_in_save_ws(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                                 const int32_t* buf_expert, const void* W_in, void* H_ws, void* Z, void* ws,
                                 size_t ws_bytes, void* stream);
int locmoe_expert_ffn_dgrad_ws(const locmoe_desc* desc, const void* dout, const void* Z, const int32_t* seg_off,
                               const int32_t* buf_expert, const void* W_out_t, const void* W_in_t, void* dZ,
                               void* dsend, void* ws, size_t ws_bytes, void* stream);

/* Gate-weighted combine (Eq. 1 with the top-1 score of Eq. 3):
 *   y[m,:] = w[m]*out[slot[m],:] if slot[m] >= 0 else 0; product in fp32, rounded to x_dtype.
 *   out device [E*C,d]; slot device [T]; w device [T] fp32; y device [T,d] (every row written). */
int locmoe_combine(const locmoe_desc* desc, const void* out, const int32_t* slot, const float* w,
                   void* y, void* stream);

/* ---- The routers the paper compares with (Section 2, Section 4) ------------------------------------------
 * Only the steps that differ from the LocMoE path; dispatch, expert FFN and combine are shared. */

/* The gate as a dense layer with a learned weight (Section 3.2.1: what the gate usually is, and what GrAP's fixed
 * weight of Eq. 4 replaces; the switch router's gate): g[m,i] = omega_i . x_m, fp32 accumulation, raw value.
 * Follow it with locmoe_route (home = NULL) for the top-1 choice, the score of Eq. 3 and the auxiliary loss of
 * Eq. 5.   x device [T,d] of x_dtype; Wg device [E,d] of x_dtype, row-major; g device [T,E] fp32 (written).
 * With Wg equal to Eq. 4's weight the result is locmoe_gate's up to the order of the fp32 additions. */
int locmoe_gate_dense(const locmoe_desc* desc, const void* x, const void* Wg, float* g, void* stream);

/* Hash routing (the hash router of Section 2 / Section 4: a fixed, parameter-free, near-uniform assignment that
 * reads no feature of the token).  The paper names no hash function; this library's reading:
 *   eid[m] = mix32(key[m] + seed * 0x9E3779B9 mod 2^32) mod E, mix32 = the 32-bit finalizer of MurmurHash3
 *   (xor-shift 16, * 0x85EBCA6B, xor-shift 13, * 0xC2B2AE35, xor-shift 16, modulo 2^32);
 *   w[m] = 1 (there is no gating score: the expert's output enters Eq. 1 unweighted); cnt[e] = #{m: eid[m] = e}.
 *   key device [T] i32 (the token's vocabulary id, read as unsigned) or NULL (= the token's index m);
 *   eid device [T] i32, w device [T] fp32, cnt device [E] i32 (all written).  Integer work only. */
int locmoe_route_hash(const locmoe_desc* desc, const int32_t* key, uint32_t seed, int32_t* eid, float* w,
                      int32_t* cnt, void* stream);

/* ---- Backward of the same path -------------------------------------------------------------------
 * What is differentiated is the training objective of Section 3.2.2 (the equation after Eq. 6),
 * L_task = L_cross + L_aux + L_loc, as far as it depends on this layer: L_cross arrives as dy = dL_cross/dy,
 * L_aux is Eq. 5 with f held fixed (a count has no gradient), L_loc is Eq. 6 differentiated through the mean
 * router probability P in place of the assignment distribution (mu * KL(P || D_l)).  The argmax of Eq. 2 and
 * the capacity drop carry no gradient; ReLU'(0) = 0; the GrAP weight of Eq. 4 is not trainable, so the
 * gradients are dx, dW_in and dW_out.  Order of calls: combine_bwd, the expert FFN backward, route_bwd,
 * dispatch_bwd.  Same descriptor, dtypes, stream and error behaviour as the forward entry points. */

/* Eq. 1 under top-1 (y_m = w_m out[slot_m]), backward:
 *   dout[slot[m],:] = w[m] * dy[m,:]  (rounded to x_dtype)  and  dw[m] = <dy[m,:], out[slot[m],:]>  (fp32)
 *   for a kept token; dw[m] = 0 for a dropped one, whose dy row is not read.
 *   dy device [T,d], out device [E*C,d], dout device [E*C,d] (rows [0,K) written) of x_dtype;
 *   slot device [T] i32; w, dw device [T] fp32. */
int locmoe_combine_bwd(const locmoe_desc* desc, const void* dy, const void* out, const int32_t* slot,
                       const float* w, void* dout, float* dw, void* stream);

/* Eq. 3, the ReLU below it and the two batch losses, backward.  With s = g + eps, G = ReLU(s) (or s if
 * desc->relu == 0), p = softmax(G) recomputed as the forward did:
 *   coef[i] = alpha n f_i / T  (Eq. 5, f_i = cnt[i]/T fixed)  +  mu (ln(P_i / D_l[i]) + 1) / T  (Eq. 6 through
 *             P_i = Psum[i]/T; only if home != NULL and mu != 0; D_l as in locmoe_route);
 *   dp[m,i] = [i = eid[m]] dw[m] + coef[i];   dG = p * (dp - <p, dp>);   dg[m,i] = dG[m,i] where s > 0 (ReLU).
 *   g device [T,E] fp32; eps device [E] or NULL; home device [T] or NULL; e2n device [E] or NULL (as in
 *   locmoe_route); eid device [T]; cnt device [E] i32 and Psum device [E] fp32 from locmoe_route; dw device [T];
 *   coef device [E] fp32 (written); dg device [T,E] fp32 (written).  If some D_l[i] = 0 the forward KL is
 *   infinite and the results are not finite. */
int locmoe_route_bwd(const locmoe_desc* desc, const float* g, const float* eps, const int32_t* home,
                     const int32_t* e2n, const int32_t* eid, const int32_t* cnt, const float* Psum,
                     const float* dw, float* coef, float* dg, void* stream);

/* Eq. 1's first linear map as locmoe_expert_ffn_in, and the pre-activation kept for the backward:
 *   Z[r,:] = W_in[e] . send[r,:] (bf16),  H_ws[r,:] = GeLU of the same fp32 value (bf16).
 *   Z device [E*C,h] bf16 (rows [0,K) written); everything else as locmoe_expert_ffn_in. */
int locmoe_expert_ffn_in_save(const locmoe_desc* desc, const void* send, const int32_t* seg_off,
                              const int32_t* buf_expert, const void* W_in, void* H_ws, void* Z, void* stream);

/* Transposed copies of the expert weights, which the data gradients contract with (row-major, bf16):
 *   W_in_t[e] = W_in[e]^T  [d,h],   W_out_t[e] = W_out[e]^T  [h,d].
 *   All four device [E,h*d]; not the packed layout (to use the packed kernels for the backward, pack the
 *   transposes: locmoe_pack_weights(desc, W_out_t, W_in_t, W_out_t_packed, W_in_t_packed), W_out_t having the
 *   shape of W_in and W_in_t that of W_out). */
int locmoe_transpose_weights(const locmoe_desc* desc, const void* W_in, const void* W_out, void* W_in_t,
                             void* W_out_t, void* stream);

/* The packed layout (as locmoe_pack_weights writes it) of the transposed weights, straight from the row-major
 * weights in one pass: same result as locmoe_transpose_weights followed by
 * locmoe_pack_weights(desc, W_out_t, W_in_t, W_out_t_packed, W_in_t_packed), bit for bit, without the row-major
 * transposes in between.  Same shape conditions and errors as locmoe_pack_weights. */
int locmoe_pack_weights_t(const locmoe_desc* desc, const void* W_in, const void* W_out, void* W_in_t_packed,
                          void* W_out_t_packed, void* stream);

/* Eq. 1, backward with respect to the rows (data gradients), two grouped GEMMs like the forward:
 *   dZ[r,:]    = (W_out[e]^T . dout[r,:]) * GeLU'(Z[r,:])   (bf16; GeLU'(v) = Phi(v) + v phi(v))
 *   dsend[r,:] = W_in[e]^T . dZ[r,:]                        (x_dtype)
 *   dout device [E*C,d] x_dtype (rows [0,K) read); Z device [E*C,h] bf16 from locmoe_expert_ffn_in_save;
 *   W_out_t, W_in_t: the transposed weights, row-major or packed as desc->w_packed says (see above);
 *   dZ device [E*C,h] bf16 and dsend device [E*C,d] x_dtype (rows [0,K) written). */
int locmoe_expert_ffn_dgrad(const locmoe_desc* desc, const void* dout, const void* Z, const int32_t* seg_off,
                            const int32_t* buf_expert, const void* W_out_t, const void* W_in_t, void* dZ,
                            void* dsend, void* stream);

/* Eq. 1, backward with respect to the weights, summed over each expert's rows of the send buffer:
 *   dW_in[e]  = sum_r dZ[r,:] (x) send[r,:]   [h,d],     dW_out[e] = sum_r dout[r,:] (x) H[r,:]   [d,h]
 *   (fp32 accumulation, rounded once to bf16; zeros for an expert without rows: every element is written).
 *   send, dout device [E*C,d] x_dtype; H, dZ device [E*C,h] bf16; dW_in, dW_out device [E,h*d] bf16,
 *   row-major in Eq. 1's orientation whatever desc->w_packed says. */
int locmoe_expert_ffn_wgrad(const locmoe_desc* desc, const void* send, const void* H, const void* dout,
                            const void* dZ, const int32_t* seg_off, const int32_t* buf_expert, void* dW_in,
                            void* dW_out, void* stream);

/* The dispatch permutation and Eq. 4, backward, in one pass over dx:
 *   dx[m,j] = (slot[m] >= 0 ? dsend[slot[m],j] : 0) + (E/d) * dg[m, j / (d/E)]   (fp32 sum, rounded to x_dtype)
 *   dsend device [E*C,d] and dx device [T,d] of x_dtype (every dx row written); slot device [T]; dg device [T,E]. */
int locmoe_dispatch_bwd(const locmoe_desc* desc, const void* dsend, const int32_t* slot, const float* dg,
                        void* dx, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LOCMOE_H */
