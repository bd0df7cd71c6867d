/*
 * moe_mi355x.h -- C ABI of the single-GPU hot path of a Tutel-style Mixture-of-Experts layer on AMD MI355X (gfx950).
 *
 * Path (arXiv 2206.03382, Sec. 2.1 and Fig. 2): gating function -> encode (dispatch) -> expert feed-forward layer ->
 * decode (combine).  On one GPU both all-to-alls of the paper are the identity, so the dispatch buffer
 * [E, C, M] goes straight to the local experts.
 *
 * Symbols follow the paper: T tokens per step, M model (channel) dim -- the paper's D --, H expert hidden dim,
 * E experts, top-k routing, capacity factor f, C = expert capacity (Eq. 1).
 *
 * Conventions that hold for every entry point unless it says otherwise
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, row-major, contiguous, 16-byte aligned.
 *   - The library never allocates or frees device memory; scratch comes from a caller-provided workspace.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is enqueued
 *     asynchronously on it; no call synchronises with the host.  Outputs are fully overwritten.
 *   - dtype selects the storage type of x / weights / Z / Y / out: MOE_F32 or MOE_BF16 (raw 16-bit patterns).
 *     Accumulation is always at least fp32.  M and H must be multiples of 8 elements, else MOE_UNSUPPORTED.
 *   - Return value: MOE_OK or an error code; on a validation error (codes 1-3) nothing has been launched;
 *     MOE_HIP_ERROR reports a failed launch or event call.
 *     Arguments are validated on the host (sizes >= 1, 1 <= k <= E, non-null required pointers, alignment).
 *   - Inputs are assumed finite; routing of NaN/Inf logits is undefined (but never out of bounds).
 *   - Calls that share a workspace or output buffers must be ordered by the caller (same stream or events).
 */
#ifndef MOE_MI355X_H
#define MOE_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { MOE_OK = 0, MOE_INVALID_ARG = 1, MOE_UNSUPPORTED = 2, MOE_WORKSPACE_TOO_SMALL = 3, MOE_HIP_ERROR = 4,
       MOE_SCRATCH_TOO_SMALL = 5 };
enum { MOE_F32 = 0, MOE_BF16 = 1 };
enum { MOE_ACT_RELU = 0, MOE_ACT_GELU = 1, MOE_ACT_SILU = 2 };
enum { MOE_ROUTER_LINEAR = 0, MOE_ROUTER_COSINE = 1 };

/* Number of events moe_layer_forward records when `stage_events` is given:
 * [0] start, [1] after gate logits, [2] after top-k + slot assignment, [3] after encode,
 * [4] after the first expert GEMM (+activation), [5] after the second expert GEMM, [6] after decode. */
#define MOE_NUM_STAGE_EVENTS 7

/* Human-readable name of a status code (static storage, never NULL). */
const char* moe_status_string(int status);

/* Expert capacity, Sec. 2.1 Eq. 1:  C = k * f * T / E, rounded up (the paper states no rounding), evaluated
 * left to right in double.  Host-only, pure.  Returns -1 if T < 1, E < 1, k < 1, k > E or f <= 0. */
int64_t moe_capacity(int64_t T, int64_t E, int k, double f);

/* Bytes of workspace moe_gate_topk needs (per-block per-expert arrival counters). 0 on invalid arguments. */
size_t moe_gate_workspace_bytes(int64_t T, int64_t E, int k);

/* Bytes of workspace moe_layer_forward needs: gate intermediates, the dispatch buffer [E,C,M], the hidden
 * activations [E,C,H] and the expert output [E,C,M].  0 on invalid arguments. */
size_t moe_layer_workspace_bytes(int64_t T, int64_t M, int64_t H, int64_t E, int k, int64_t C, int dtype);

/* Gating function, linear part (Sec. 2.1):  logits[t,e] = sum_m x[t,m] * Wg[m,e] + gate_bias[e].
 *   x [T,M] and Wg [M,E] in `dtype`; gate_bias [E] fp32 or NULL; logits [T,E] fp32 (output).
 * The sum is accumulated in fp64 and rounded once to fp32, so the result does not depend on summation order
 * (up to the last bit of the fp64 sum) and the routing decisions taken on it are reproducible. */
int moe_gate_logits(const void* x, const void* Wg, const float* gate_bias, int dtype,
                    int64_t T, int64_t M, int64_t E, float* logits, void* stream);

/* Bytes of workspace moe_gate_logits_cosine needs (the projection [T,D] fp32, the expert embeddings transposed in
 * fp64, their norms).  0 on invalid arguments (D <= 4096, E <= 512). */
size_t moe_cosine_gate_workspace_bytes(int64_t T, int64_t D, int64_t E);

/* Cosine router (Appendix, "A New Cosine Router", its equation):
 *   logits[t,e] = cos(W x_t, M_e) / tau = (W x_t . M_e) / (|W x_t| |M_e|) / tau;   P = softmax(logits) as usual.
 *   x [T,M] and Wp [M,D] in `dtype`: the projection W of the paper stored input-major (Wp = W^T), D = 256 there;
 *   Me [E,D] fp32: one embedding per expert;  tau: temperature, values below 0.01 act as 0.01;
 *   logits [T,E] fp32 (output), to be passed to moe_gate_topk.
 * The projection is accumulated in fp64 and rounded once to fp32 (as moe_gate_logits does), the cosine is computed
 * in fp64 and rounded once; norms are clamped below at 1e-12.  ws: moe_cosine_gate_workspace_bytes, 256-byte aligned. */
int moe_gate_logits_cosine(const void* x, const void* Wp, const float* Me, double tau, int dtype, int64_t T, int64_t M,
                           int64_t D, int64_t E, float* logits, void* ws, size_t ws_bytes, void* stream);

/* Gating function, decision part (Sec. 2.1; Sec. 4.1 "dynamic top-ANY gating": any 1 <= k <= E per call) and
 * capacity-limited slot assignment with the GShard logic the paper keeps (Sec. 2.1 "MoE Frameworks"; the
 * location scan of Appendix B).
 *   logits   [T,E] fp32 (input).
 *   idx      [T,k] int32: expert of the j-th largest logit; equal logits -> lower expert index.
 *   gate_w   [T,k] fp32: softmax over all E experts, taken at idx; if normalize != 0 divided by the sum over
 *            the token's k choices (dropped ones included).
 *   loc      [T,k] int32: 0-based arrival position at expert idx[t,j]; arrivals are ordered by (j, t):
 *            all first choices in token order, then all second choices, ...  A choice is kept iff loc < C.
 *   counts   [E] int32: arrivals per expert before truncation (max over e = minimum capacity that drops nothing,
 *            Sec. 4.1 "dynamic capacity factor").
 *   slot_src [E,C] int32 or NULL: token occupying slot (e,c), -1 if the slot is unfilled.
 *   ws / ws_bytes: workspace of at least moe_gate_workspace_bytes(T,E,k), 16-byte aligned.
 * Limits: E <= 512 and k*E <= 16384, else MOE_UNSUPPORTED.  Integer outputs are deterministic (no
 * order-dependent atomics). */
int moe_gate_topk(const float* logits, int64_t T, int64_t E, int k, int64_t C, int normalize,
                  int32_t* idx, float* gate_w, int32_t* loc, int32_t* counts, int32_t* slot_src,
                  void* ws, size_t ws_bytes, void* stream);

/* Bytes of workspace moe_gate_route needs (the arrival counters of moe_gate_topk and, for bf16 gates, the transposed
 * gate weights, their norms and one error bound per token).  0 on invalid arguments. */
size_t moe_gate_route_workspace_bytes(int64_t T, int64_t M, int64_t E, int k, int dtype);

/* The gating function from the tokens (Sec. 2.1): moe_gate_logits followed by moe_gate_topk, at memory speed.
 *   Inputs as moe_gate_logits, outputs as moe_gate_topk (logits [T,E] fp32 is an output here, required).
 * fp32 gates run exactly those two steps.  bf16 gates compute the logits on the bf16 matrix cores (exact products, fp32
 * sums of 32 terms, fp64 sums of those) with a rigorous per-token error bound B_t = 32 * 2^-23 * |x_t| * max_e |w_e|; a
 * token whose k+1 largest logits are not separated by more than 2 B_t has the logits of every expert that can still
 * reach its top k recomputed in fp64 and rounded once, and is decided on those.  So idx, loc, counts and slot_src are
 * the ones exactly rounded logits give (what moe_gate_logits + moe_gate_topk return), while `logits` holds exactly
 * rounded values where a decision needed them and values within B_t of them elsewhere (typically within 1e-6; gate_w
 * follows the stored logits).
 *   ws: moe_gate_route_workspace_bytes, 256-byte aligned; x 16-byte aligned. */
int moe_gate_route(const void* x, const void* Wg, const float* gate_bias, int dtype, int64_t T, int64_t M, int64_t E, int k,
                   int64_t C, int normalize, float* logits, int32_t* idx, float* gate_w, int32_t* loc, int32_t* counts,
                   int32_t* slot_src, void* ws, size_t ws_bytes, void* stream);

/* moe_gate_topk for callers that cannot allocate device memory or bring a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same kernels and the same outputs, with the arrival
 * counters in a device array of fixed size that the library holds on every GPU it runs on until the process ends.
 * Calls no hipMalloc, hipFree or other allocating routine.  Arguments as moe_gate_topk, without ws / ws_bytes.
 * Limit: moe_gate_workspace_bytes(T, E, k) <= moe_gate_topk_static_max_bytes() (8 MiB: k * ceil(T / 64) * E <= 2^21),
 * else MOE_SCRATCH_TOO_SMALL and nothing is launched.  Every call on one GPU shares that GPU's array: calls that
 * overlap on one GPU (different streams, or threads) race; order them on one stream or with events.  Nothing in the
 * array has to start from zero (each call writes every counter before reading it). */
size_t moe_gate_topk_static_max_bytes(void);
int moe_gate_topk_static(const float* logits, int64_t T, int64_t E, int k, int64_t C, int normalize,
                         int32_t* idx, float* gate_w, int32_t* loc, int32_t* counts, int32_t* slot_src, void* stream);

/* Bytes of workspace moe_gate_topk_bpr needs.  0 on invalid arguments. */
size_t moe_gate_bpr_workspace_bytes(int64_t T, int64_t E, int k);

/* moe_gate_topk with batch prioritized routing (named in Sec. 3.2 and in the Appendix's comparison of routing
 * algorithms): within each choice rank, tokens take their slots in order of decreasing priority instead of token
 * order, so that under a tight capacity the least confident tokens are the ones dropped.  Priority = the token's
 * largest routing probability, computed in fp64 and rounded to fp32; equal priorities -> lower token index.
 * Arguments and outputs as moe_gate_topk (loc is the arrival position in the prioritized order).
 * The order is found by a stable radix sort of the priorities' bit patterns (integer work: deterministic).
 * ws: moe_gate_bpr_workspace_bytes, 256-byte aligned. */
int moe_gate_topk_bpr(const float* logits, int64_t T, int64_t E, int k, int64_t C, int normalize, int32_t* idx, float* gate_w,
                      int32_t* loc, int32_t* counts, int32_t* slot_src, void* ws, size_t ws_bytes, void* stream);

/* Dynamic capacity factor (Sec. 4.1 "Dynamic Capacity Factor"), for capacity_setting <= 0 (a positive setting is the
 * factor f itself: use moe_capacity).  0: the smallest capacity that drops no token, i.e. the arrivals of the fullest
 * expert; negative: the same, but never above the capacity that factor -capacity_setting gives by Eq. 1.
 *   counts [E] int32 (device): un-truncated arrivals from moe_gate_topk (which may be called with slot_src = NULL and
 *          any valid C: idx, gate_w, loc and counts do not depend on C).
 *   C_out  [2] int64 (device, output): C_out[0] = capacity to use, C_out[1] = needed capacity max_e counts[e].
 * A caller composing the path from the stage entry points reads C_out back (one synchronisation), sizes the [E,C,M]
 * buffers, builds slot_src with moe_slot_sources and continues with moe_encode / moe_expert_ffn / moe_decode;
 * moe_layer_forward_dynamic runs the same flow without that synchronisation. */
int moe_dynamic_capacity(const int32_t* counts, int64_t T, int64_t E, int k, double capacity_setting, int64_t* C_out,
                         void* stream);

/* slot_src [E,C] (output) for a capacity chosen after routing (Sec. 4.1): token occupying slot (e,c), -1 if unfilled,
 * from idx, loc [T,k] of moe_gate_topk; a choice is kept iff loc < C.  E*C must be below 2^31. */
int moe_slot_sources(const int32_t* idx, const int32_t* loc, int64_t T, int64_t E, int k, int64_t C, int32_t* slot_src,
                     void* stream);

/* Fast encode (Sec. 4.2 "Fast Encode and Decode", Appendix B):  Z[e,c,:] = x[t,:] for the kept choice (t,j) with
 * idx[t,j] = e and loc[t,j] = c; unfilled slots are set to zero.  Rows are copied unscaled (bit-exact).
 *   x [T,M], Z [E,C,M] in `dtype`; idx, loc [T,k] from moe_gate_topk.
 *   slot_src [E,C] from moe_gate_topk, or NULL: with it the kernel is a single write-coalesced gather; without
 *   it Z is zero-filled and the rows are scattered from idx/loc. */
int moe_encode(const void* x, int dtype, const int32_t* idx, const int32_t* loc, const int32_t* slot_src,
               int64_t T, int64_t M, int64_t E, int k, int64_t C, void* Z, void* stream);

/* Local experts' feed-forward layer (Sec. 2.1; the per-expert [C,M] slab layout of Sec. 4.2 "Flexible All-to-All"):
 *   Y[e] = act(Z[e] * W1[e] + b1[e]) * W2[e] + b2[e]     for every expert e.
 *   Z [E,C,M], W1 [E,M,H], W2 [E,H,M], Y [E,C,M], hidden [E,C,H] (scratch) in `dtype`; b1 [E,H], b2 [E,M] in
 *   `dtype` or NULL.  bf16: products accumulate in fp32 on the matrix cores, the hidden activations are rounded to
 *   bf16 once after the activation and Y once at the end.  fp32: plain fp32 FMA accumulation.
 *   counts [E] int32 or NULL: if given, only the first min(counts[e], C) rows of each expert are computed and the
 *   remaining rows of Y and hidden are left untouched (decode never reads them); if NULL all C rows are computed.
 *   act: ReLU, GeLU (the erf form v * Phi(v); the bf16 matrix-core path evaluates Phi to within 6e-7) or SiLU. */
int moe_expert_ffn(const void* Z, const void* W1, const void* b1, const void* W2, const void* b2,
                   int act, int dtype, const int32_t* counts,
                   int64_t E, int64_t C, int64_t M, int64_t H, void* hidden, void* Y, void* stream);

/* moe_encode followed by moe_expert_ffn without materialising the dispatch buffer (not in the paper, whose [E,C,M]
 * buffer exists to feed the all-to-all; on one GPU the first expert GEMM can fetch its rows straight from the tokens):
 * row c of expert e's operand is x[slot_src[e,c], :], read by the GEMM's own global->LDS loads.
 *   x [T,M]; slot_src [E,C] from moe_gate_topk or moe_slot_sources; everything else as moe_expert_ffn.
 *   Rows of Y and hidden past min(counts[e], C) (or, with counts = NULL, rows of unfilled slots) hold unspecified
 *   values; decode never reads them.
 * bf16 only, M % 64 == 0 and H % 256 == 0 and T*M*2 < 2^32, else MOE_UNSUPPORTED (use the two calls instead). */
int moe_expert_ffn_gather(const void* x, const int32_t* slot_src, int64_t T, const void* W1, const void* b1, const void* W2,
                          const void* b2, int act, int dtype, const int32_t* counts, int64_t E, int64_t C, int64_t M,
                          int64_t H, void* hidden, void* Y, void* stream);

/* Fast decode (Sec. 4.2, Appendix B):  out[t,:] = sum over kept choices j (ascending) of
 * gate_w[t,j] * Y[idx[t,j], loc[t,j], :], accumulated in fp32 and rounded once to `dtype`.
 * A token whose choices were all dropped gets an all-zero row.  Y [E,C,M], out [T,M] in `dtype`. */
int moe_decode(const void* Y, int dtype, const int32_t* idx, const int32_t* loc, const float* gate_w,
               int64_t T, int64_t M, int64_t E, int k, int64_t C, void* out, void* stream);

/* Bytes of workspace moe_gate_backward needs (dlogits [T,E] fp32 and the per-slice partial sums of dWg and of dbias;
 * a slice is 64 tokens, or more so that there are at most 256 slices).  0 on invalid arguments. */
size_t moe_gate_backward_workspace_bytes(int64_t T, int64_t M, int64_t E, int k);

/* Backward of the gating function (Sec. 2.1 gate; Sec. 3.2: the backward pass mirrors the forward).  With
 * p = softmax(logits), g[t,j] = p[t, idx[t,j]] and gate_w = g / sum_j g (normalize != 0) or g:
 *   dlogits = the chain rule through that map applied to dgate_w [T,k] (fp32; from moe_decode_backward);
 *   dx[t,:]  = dlogits[t,:] Wg^T   (added to what dx holds if accumulate_dx != 0, e.g. moe_encode_backward's result);
 *   dWg      = x^T dlogits;   dbias = column sums of dlogits.
 * x, dx [T,M] and Wg, dWg [M,E] in `dtype`; logits [T,E] fp32 and idx [T,k] as the forward produced them; dbias [E] and
 * dlogits [T,E] fp32.  Any of dx, dWg, dbias, dlogits may be NULL.  The choice of experts and the slot assignment carry
 * no gradient.  fp32 arithmetic, fixed summation orders (within a token slice ascending, then slice by slice); for bf16
 * gates with 32 or more experts and M % 256 == 0, dx is a matrix-core product of dlogits rounded to bf16 (fp32 sums).
 * ws: moe_gate_backward_workspace_bytes, 256-byte aligned; x and dx 16-byte aligned. */
int moe_gate_backward(const void* x, const void* Wg, const float* logits, const int32_t* idx, const float* dgate_w, int normalize,
                      int dtype, int64_t T, int64_t M, int64_t E, int k, void* ws, size_t ws_bytes, void* dx, int accumulate_dx,
                      void* dWg, float* dbias, float* dlogits, void* stream);

/* moe_expert_ffn for a training step (Sec. 3.2 runs the experts' forward and backward): the same computation, which
 * also keeps the first layer's values before the activation, pre[e] = Z[e] W1[e] + b1[e] rounded to `dtype`
 * ([E,C,H], rows past an expert's fill untouched), for moe_expert_ffn_backward.  hidden and Y are bit-identical to
 * moe_expert_ffn's.  Everything else as moe_expert_ffn. */
int moe_expert_ffn_train(const void* Z, const void* W1, const void* b1, const void* W2, const void* b2, int act, int dtype,
                         const int32_t* counts, int64_t E, int64_t C, int64_t M, int64_t H, void* pre, void* hidden, void* Y,
                         void* stream);

/* Bytes of workspace moe_expert_ffn_backward needs (recomputed pre-activations, dP, one transposed weight matrix,
 * one transposed and one row-padded activation slab).  0 on invalid arguments. */
size_t moe_ffn_backward_workspace_bytes(int64_t E, int64_t C, int64_t M, int64_t H, int dtype);

/* Backward of the local experts' feed-forward layer (Sec. 3.2: in the backward pass "the computation becomes the
 * backward computation of the expert").  With Y[e] = act(Z[e] W1[e] + b1[e]) W2[e] + b2[e] and dY = dLoss/dY:
 *   dP = (dY W2^T) * act'(Z W1 + b1);  dZ = dP W1^T;  dW1 = Z^T dP;  db1 = column sums of dP;
 *   dW2 = hidden^T dY;  db2 = column sums of dY;     sums over the first min(counts[e], C) rows of each expert (all C
 *   rows if counts is NULL).
 *   Z, dY, dZ [E,C,M]; hidden [E,C,H] = act(Z W1 + b1) as moe_expert_ffn left it; W1, dW1 [E,M,H]; W2, dW2 [E,H,M];
 *   b1 [E,H] or NULL (it enters the pre-activation); db1 [E,H]; db2 [E,M]; all in `dtype`, fp32 accumulation, each
 *   output rounded once; intermediates (pre-activations, dP) are rounded to `dtype` as well.
 *   pre [E,C,H]: the pre-activations moe_expert_ffn_train kept, or NULL: then they are recomputed from Z, W1, b1
 *   (one more product; the results are bit-identical either way).
 *   Any of dZ, dW1, db1, dW2, db2 may be NULL (not computed).  Rows of dZ past an expert's fill are left untouched.
 *   ws: at least moe_ffn_backward_workspace_bytes bytes, 16-byte aligned.  ReLU'(0) = 0. */
int moe_expert_ffn_backward(const void* Z, const void* W1, const void* b1, const void* W2, const void* pre, const void* hidden,
                            const void* dY, int act, int dtype, const int32_t* counts, int64_t E, int64_t C, int64_t M, int64_t H,
                            void* ws, size_t ws_bytes, void* dZ, void* dW1, void* db1, void* dW2, void* db2, void* stream);

/* Backward of fast encode (Appendix B, the differentiable fast encode and decode operators):
 *   dx[t,:] = sum over the kept choices j of dZ[idx[t,j], loc[t,j], :]   (a token with no kept choice gets +0).
 * dZ [E,C,M], dx [T,M] (output) in `dtype`; fp32 accumulation in rank order, one rounding.  encode copies rows
 * unscaled, so it has no gate-weight gradient; idx and loc carry no gradient. */
int moe_encode_backward(const void* dZ, int dtype, const int32_t* idx, const int32_t* loc, int64_t T, int64_t M, int64_t E,
                        int k, int64_t C, void* dx, void* stream);

/* Backward of fast decode (Appendix B):
 *   dY[e,c,:]    = gate_w[t,j] * d_out[t,:] for the kept choice (t,j) with idx = e, loc = c; 0 for an unfilled slot;
 *   dgate_w[t,j] = sum_m d_out[t,m] * Y[idx[t,j], loc[t,j], m] for a kept choice; 0 for a dropped one.
 * d_out [T,M], Y and dY [E,C,M] in `dtype`; dgate_w [T,k] fp32 (fp32 accumulation, fixed summation order).
 * Either output may be NULL (then Y, or gate_w and slot_src, may be NULL too).  slot_src [E,C] as in moe_encode. */
int moe_decode_backward(const void* d_out, const void* Y, int dtype, const int32_t* idx, const int32_t* loc,
                        const float* gate_w, const int32_t* slot_src, int64_t T, int64_t M, int64_t E, int k, int64_t C,
                        void* dY, float* dgate_w, void* stream);

/* The whole path on one stream: gate (moe_gate_route) -> encode -> expert FFN (filled rows only) -> decode,
 * with C = moe_capacity(T,E,k,f).
 *   Inputs as in the entry points above.  out [T,M] (output, required).
 *   Optional outputs (each may be NULL): idx, loc [T,k] int32; gate_w [T,k] fp32; counts [E] int32; logits [T,E] fp32.
 *   ws / ws_bytes: at least moe_layer_workspace_bytes(T,M,H,E,k,C,dtype), 256-byte aligned.
 *   stage_events: NULL, or MOE_NUM_STAGE_EVENTS hipEvent_t handles recorded on `stream` at the stage boundaries
 *   listed above (for per-stage timing; the events belong to the caller). */
int moe_layer_forward(const void* x, const void* Wg, const float* gate_bias,
                      const void* W1, const void* b1, const void* W2, const void* b2,
                      int64_t T, int64_t M, int64_t H, int64_t E, int k, double f, int normalize, int act, int dtype,
                      void* out, int32_t* idx, int32_t* loc, float* gate_w, int32_t* counts, float* logits,
                      void* ws, size_t ws_bytes, void* stream, void* const* stage_events);

/* moe_layer_forward with the dispatch fused into the first expert GEMM (moe_expert_ffn_gather) where that kernel
 * supports the shape and dtype, identical to moe_layer_forward otherwise.  Same arguments, same outputs; the encode
 * stage's events [2] and [3] are then recorded back to back. */
int moe_layer_forward_fused(const void* x, const void* Wg, const float* gate_bias, const void* W1, const void* b1,
                            const void* W2, const void* b2, int64_t T, int64_t M, int64_t H, int64_t E, int k, double f,
                            int normalize, int act, int dtype, void* out, int32_t* idx, int32_t* loc, float* gate_w,
                            int32_t* counts, float* logits, void* ws, size_t ws_bytes, void* stream,
                            void* const* stage_events);

/* The whole path with the dynamic capacity factor (Sec. 4.1 "Dynamic Capacity Factor") on one stream and without any
 * host synchronisation (so the call can be captured in a HIP graph), with the routing variants as options.
 *   capacity_setting > 0: the capacity factor f itself (Eq. 1); = 0: the smallest capacity that drops no token
 *   (the arrivals of the fullest expert); < 0: the same, but never above the capacity that factor -capacity_setting gives.
 *   C_max: the capacity the caller sized the workspace for.  The capacity is chosen on the device after the arrivals are
 *   counted and is never above C_max: every internal buffer keeps its [E, C_max, ...] layout and the kernels read the
 *   chosen capacity from device memory (a choice is kept iff loc < C).  C_max = T can hold any routing; with a smaller
 *   C_max the setting 0 behaves like a negative setting whose bound is C_max.  A positive setting whose capacity
 *   exceeds C_max is MOE_INVALID_ARG.
 *   router: MOE_ROUTER_LINEAR (Wg [M,E], gate_bias [E] or NULL; Me, D, tau ignored) or MOE_ROUTER_COSINE (Appendix, the
 *   cosine router: Wg is the projection [M,D], Me [E,D] fp32, temperature tau; gate_bias must be NULL).
 *   bpr != 0: batch prioritized routing (moe_gate_topk_bpr) instead of token order.
 *   out [T,M] (required).  Optional outputs (NULL or device): idx, loc [T,k]; gate_w [T,k]; counts [E] (un-truncated
 *   arrivals); logits [T,E]; C_out [2] int64, 8-byte aligned: C_out[0] = chosen capacity, C_out[1] = needed capacity.
 *   ws: moe_layer_dynamic_workspace_bytes(T,M,H,E,k,C_max,dtype,router,D,bpr) bytes, 256-byte aligned (0 = invalid or
 *   unsupported arguments). */
size_t moe_layer_dynamic_workspace_bytes(int64_t T, int64_t M, int64_t H, int64_t E, int k, int64_t C_max, int dtype, int router,
                                         int64_t D, int bpr);
int moe_layer_forward_dynamic(const void* x, const void* Wg, const float* gate_bias, const void* W1, const void* b1,
                              const void* W2, const void* b2, int64_t T, int64_t M, int64_t H, int64_t E, int k,
                              double capacity_setting, int64_t C_max, int normalize, int act, int dtype, int router,
                              const float* Me, int64_t D, double tau, int bpr, void* out, int32_t* idx, int32_t* loc,
                              float* gate_w, int32_t* counts, float* logits, int64_t* C_out, void* ws, size_t ws_bytes,
                              void* stream);

/* One training step of the layer (Sec. 3.2: forward, then the backward pass mirrors it).  moe_layer_forward_train
 * computes what moe_layer_forward computes (`out` is bit-identical) and keeps in `state` what the backward needs:
 * logits, routing, the dispatch buffer, the first layer's values before and after the activation, the expert outputs.
 * moe_layer_backward then takes d_out = dLoss/d out [T,M] and the same x, weights and shape arguments, and writes
 *   dx [T,M] (through encode and through the gate), dWg [M,E], dgate_bias [E] fp32, dW1 [E,M,H], db1 [E,H],
 *   dW2 [E,H,M], db2 [E,M]   (any of dWg ... db2 may be NULL; dx is required),
 * running moe_decode_backward, moe_expert_ffn_backward, moe_encode_backward and moe_gate_backward on the state's
 * buffers.  The choice of experts, the slot assignment and dropped choices carry no gradient.
 * Where the matrix-core kernels take the shape (bf16, M and H multiples of 256, T * M * 2 < 2^32) the step never writes
 * the dispatch buffer: the forward's first product and the backward's dW1 = Z^T dP read the rows of Z from x through the
 * slot -> token map, as moe_layer_forward_fused does; results are bit-identical to the buffered route.
 *   state: device memory of at least moe_layer_train_state_bytes(T, M, H, E, k, moe_capacity(T, E, k, f), dtype)
 *   bytes, 256-byte aligned, owned by the caller; its layout is private; it must not change between the two calls.
 *   One state serves one step at a time: two steps that overlap on different streams need two states. */
size_t moe_layer_train_state_bytes(int64_t T, int64_t M, int64_t H, int64_t E, int k, int64_t C, int dtype);
int moe_layer_forward_train(const void* x, const void* Wg, const float* gate_bias, const void* W1, const void* b1,
                            const void* W2, const void* b2, int64_t T, int64_t M, int64_t H, int64_t E, int k, double f,
                            int normalize, int act, int dtype, void* out, void* state, size_t state_bytes, void* stream);
int moe_layer_backward(const void* x, const void* Wg, const void* W1, const void* b1, const void* W2, int64_t T, int64_t M,
                       int64_t H, int64_t E, int k, double f, int normalize, int act, int dtype, const void* d_out, void* state,
                       size_t state_bytes, void* dx, void* dWg, float* dgate_bias, void* dW1, void* db1, void* dW2, void* db2,
                       void* stream);

/* Thin wrappers over HIP events so that a caller without HIP headers can time on the library's stream.
 * moe_event_create stores a new hipEvent_t in *event; moe_event_elapsed_ms needs both events completed. */
int moe_event_create(void** event);
int moe_event_destroy(void* event);
int moe_event_record(void* event, void* stream);
int moe_event_synchronize(void* event);
int moe_event_elapsed_ms(void* start, void* stop, float* ms);

#ifdef __cplusplus
}
#endif
#endif /* MOE_MI355X_H */
