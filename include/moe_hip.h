/*
 * moe_hip.h - C ABI of the MI355X (gfx950) Mixture-of-Experts layer library.
 *
 * One GPU's MoE layer, forward and backward, as described in
 * "Scalable and Efficient MoE Training for Multitask Multilingual Models"
 * (arXiv 2109.10465): a top-1 / top-2 softmax gate with a per-expert capacity
 * and Random-Token-Selection priority (Sec. 3.1, Sec. 5.1 "MoE setting"),
 * dispatch of the flattened [T = batch*seq, d_model] token tensor into
 * fixed-shape per-expert buffers (Sec. 3.1), the per-expert two-matmul
 * feed-forward block (Sec. 4.2 "Model details", Sec. 2.3), and the gate-weighted
 * combine.  The layer arguments mirror the paper's layer statement
 * MoE(hidden_size, expert, num_experts) (Sec. 2.4) plus k and the capacity.
 *
 * Conventions, valid for every entry point unless stated otherwise
 * ---------------------------------------------------------------
 *  - Every pointer is a DEVICE pointer owned by the caller.  The library
 *    allocates nothing, keeps no state between calls and frees nothing
 *    (moe_gate_route_static, which brings its own scratch array, is the one
 *    entry point with memory of its own; see there).
 *    Scratch memory comes from the caller through (ws, ws_bytes); ask
 *    moe_workspace_bytes() for the size.  ws must be 256-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    A call enqueues its kernels on that stream and returns without
 *    synchronising.  Calls on one stream execute in order; calls that share a
 *    workspace must not overlap.
 *  - All arrays are dense and row-major with the shapes given below.
 *    Activation tensors (x, xd, h, dact, yd, y, dy, dyd, dxd, dx) and the expert
 *    weights W1, W2 have the element type shape->dtype (MOE_F32: float,
 *    MOE_BF16: bfloat16 as uint16_t bit patterns).  Gate logits, probabilities,
 *    gate weights, RTS keys, dlogits, dgate_w, Wg, dWg, dW1 and dW2 are always
 *    float; indices are int32_t.  All accumulation is in fp32.
 *  - Outputs are overwritten, never accumulated into (the one exception,
 *    dx_accum, is named so).  Results are bit-reproducible run to run: no
 *    floating-point atomics are used.
 *  - Rows s >= expert_count[e] of the per-expert buffers xd, h, dact, yd, dyd, dxd
 *    are never read by any entry point and are left unwritten.
 *  - Return value: MOE_OK (0) or a negative moe_status.  Argument errors are
 *    detected on the host before anything is enqueued, so outputs are
 *    untouched.  Non-finite logits or keys give undefined routing values but never an
 *    out-of-range index: a NaN logit counts as -inf in the top-k, and a slot that NaN
 *    keys leave unassigned is skipped by moe_dispatch.
 *  - Index tensors that an entry point takes as input (expert_idx, slot, slot_src,
 *    expert_count) must hold what a routing call wrote for the same shape:
 *    0 <= expert_idx < E, -1 <= slot < capacity, -1 <= slot_src < T*k,
 *    0 <= expert_count <= capacity.  The two dispatch calls skip an index outside
 *    its range; the other entry points form addresses from these values unchecked.
 *  - Seeded noise (gate jitter, expert dropout) comes from the counter-based
 *    generator Philox4x32 with 10 rounds (Salmon et al., SC 2011), so a caller or
 *    a checker can reproduce every draw: element i of a tensor uses output word
 *    i % 4 of the block with counter (i/4 low word, i/4 high word, stream, 0) and
 *    key (seed low word, seed high word); stream 1 = gate jitter, indexed over
 *    x[T, d_model]; stream 2 = expert dropout, indexed over h[E, C, d_ff].
 *  - Shape limits: T, d_model, d_ff, E, capacity >= 1; k in {1,2}; E >= k;
 *    E <= 256; d_model and d_ff multiples of 8; T*k and E*capacity < 2^30.
 *    The expert FFN entry points address one expert's slice of a tensor with
 *    32-bit byte offsets and also need (capacity + 512) * max(d_model, d_ff) * 4
 *    < 2^31 and d_model * d_ff * 4 < 2^31 (else MOE_ERR_SHAPE).
 *  - One GPU per call: the device that is current when an entry point is called
 *    must be the one that owns the buffers and the stream.
 */
#ifndef MOE_HIP_H
#define MOE_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum moe_dtype { MOE_F32 = 0, MOE_BF16 = 1 };
enum moe_act { MOE_RELU = 0, MOE_GELU = 1 }; /* gelu(z) = z/2 (1 + erf(z/sqrt 2)) */

enum moe_status {
    MOE_OK = 0,
    MOE_ERR_NULL = -1,      /* a required pointer is NULL */
    MOE_ERR_SHAPE = -2,     /* shape outside the limits above */
    MOE_ERR_DTYPE = -3,     /* unknown dtype or activation */
    MOE_ERR_WORKSPACE = -4, /* ws NULL, misaligned or smaller than needed */
    MOE_ERR_LAUNCH = -5     /* the HIP runtime refused a launch */
};

/* T tokens, d_model, d_ff, E experts, k experts per token, capacity = slots per
 * expert (C).  The same struct is passed to every call of one layer step. */
typedef struct {
    int32_t T, d_model, d_ff, E, k, capacity;
    int32_t dtype; /* moe_dtype */
    int32_t act;   /* moe_act   */
} moe_shape;

/* Human-readable name of a status code (static string, host). */
const char* moe_status_string(int status);

/* Slots per expert for a capacity factor: max(1, ceil(k*cf*T/E)) (Sec. 5.1:
 * capacity factor 1.0 for training, 2.0 for evaluation; Sec. 2.3: tokens per
 * expert depend on batch, experts and top-1 vs top-2).  Host function; returns
 * -1 on invalid arguments.  The capacity is an explicit input of every other
 * call, so a caller may use another rule. */
int32_t moe_capacity(int32_t T, int32_t E, int32_t k, double capacity_factor);

/* Bytes of scratch that the largest user among the entry points needs for
 * this shape (host function; 0 on an invalid shape). */
size_t moe_workspace_bytes(const moe_shape* shape);

/* Gate projection (Sec. 3.2: the gating layer is a matrix with one column per
 * expert):  logits[T,E] = x[T,d_model] * Wg[d_model,E] (+ bias[E]).
 * bias_or_null exists only to synthesise skewed routing; the paper's gate has
 * no bias. */
int moe_gate_logits(const moe_shape* shape, const void* x, const float* Wg,
                    const float* bias_or_null, float* logits, void* stream);

/* Gate projection with jitter (Sec. 5.1: jittering noise on the gating input,
 * as in the Switch Transformer):  logits = (x .* noise) * Wg (+ bias) with
 * noise[t,i] = 1 + jitter_eps * (2u - 1), u = word / 2^32 in [0,1).  Only the
 * gate sees the noise; dispatch copies x itself.  0 <= jitter_eps < 1;
 * jitter_eps = 0 is moe_gate_logits. */
int moe_gate_logits_jitter(const moe_shape* shape, const void* x, const float* Wg,
                           const float* bias_or_null, float jitter_eps, uint64_t seed,
                           float* logits, void* stream);

/* Gate + capacity assignment (Sec. 5.1 top-1 / top-2 gating; Sec. 3.1 expert
 * capacity and Random Token Selection).
 *   probs[T,E]      = softmax over experts of logits[T,E]
 *   expert_idx[T,k] = the k experts with the largest logits, best first; equal
 *                     logits -> smaller expert id
 *   gate_w[T,k]     = k=1: probs[t,e0];  k=2: probs[t,e_j]/(probs[t,e0]+probs[t,e1])
 *   Candidates (t,j) of one expert are ordered by (j ascending, rts_keys[t]
 *   descending, t ascending); the candidate of rank r gets slot r if r <
 *   capacity, else it is dropped.  rts_keys_or_null == NULL means equal keys:
 *   position priority, i.e. tokens at the end of the batch are dropped first.
 *   slot[T,k]        = slot inside expert expert_idx[t,j], or -1 if dropped
 *   expert_demand[E] = number of candidates of each expert
 *   expert_count[E]  = min(capacity, expert_demand) = rows in use
 *   slot_src[E,C]    = t*k+j of the candidate in that slot, -1 if unused
 * Needs workspace. */
int moe_gate_route(const moe_shape* shape, const float* logits, const float* rts_keys_or_null,
                   float* probs, int32_t* expert_idx, float* gate_w, int32_t* slot,
                   int32_t* expert_count, int32_t* expert_demand, int32_t* slot_src,
                   void* ws, size_t ws_bytes, void* stream);

/* Grouped token selection (Sec. 3.1: a group dimension batches consecutive
 * sentences and the selection happens inside each group; the second arm of the
 * ablation in Sec. 5.5).  As moe_gate_route, except that the T tokens form
 * n_groups groups of T/n_groups consecutive tokens and every group routes on
 * its own with capacity/n_groups slots per expert.  The rows an expert keeps
 * from group 0 come first in its buffer, then those of group 1, ... without
 * gaps: slot = (rows kept for the expert by earlier groups) + rank inside the
 * group, so expert_count[e] rows are in use as for plain routing.
 * Limits for n_groups > 1: T % n_groups == 0, (T/n_groups) % 256 == 0,
 * capacity % n_groups == 0 (else MOE_ERR_SHAPE).  n_groups == 1 is
 * moe_gate_route.  Needs workspace. */
int moe_gate_route_grouped(const moe_shape* shape, int32_t n_groups, const float* logits,
                           const float* rts_keys_or_null, float* probs, int32_t* expert_idx,
                           float* gate_w, int32_t* slot, int32_t* expert_count,
                           int32_t* expert_demand, int32_t* slot_src, void* ws, size_t ws_bytes,
                           void* stream);

/* moe_gate_route for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * inputs, outputs and results as moe_gate_route (plain routing, one group); the
 * scratch memory is a device array built into the library instead of a caller
 * workspace, so the call allocates and frees nothing.  Limits and rules:
 *  - the shape's routing scratch must fit moe_gate_route_static_max_bytes()
 *    (5 MiB; enough for T = 65536, k = 2 with any E <= 256), else
 *    MOE_ERR_WORKSPACE is returned before anything is enqueued;
 *  - every GPU has one such array and every call on that GPU uses it: calls that
 *    may overlap on one GPU (two streams, two threads) race and must be ordered
 *    by the caller; the array keeps the last call's contents and nothing in it
 *    needs clearing (each call writes all it reads);
 *  - the array occupies its 5 MiB on every GPU the library runs on until the
 *    process ends;  MOE_ERR_LAUNCH if the array's address cannot be obtained. */
size_t moe_gate_route_static_max_bytes(void);
int moe_gate_route_static(const moe_shape* shape, const float* logits, const float* rts_keys_or_null,
                          float* probs, int32_t* expert_idx, float* gate_w, int32_t* slot,
                          int32_t* expert_count, int32_t* expert_demand, int32_t* slot_src,
                          void* stream);

/* Dispatch (Sec. 3.1: fixed-shape per-expert buffers):
 *   xd[e,s,:] = x[slot_src[e,s] / k, :]  for s < expert_count[e]  (bit copies).
 * Its backward is moe_combine_fwd with gate_w_or_null == NULL. */
int moe_dispatch(const moe_shape* shape, const void* x, const int32_t* slot_src,
                 const int32_t* expert_count, void* xd, void* stream);

/* The same dispatch (Sec. 3.1), addressed from the token side: every token row
 * x[t,:] is read once and written to the slot of each of its kept choices,
 *   xd[expert_idx[t,j], slot[t,j], :] = x[t,:]   for slot[t,j] >= 0,
 * instead of once per kept choice.  Same result as moe_dispatch, bit for bit,
 * for a slot / slot_src pair that comes from one routing call. */
int moe_dispatch_tokens(const moe_shape* shape, const void* x, const int32_t* expert_idx,
                        const int32_t* slot, void* xd, void* stream);

/* Expert feed-forward block, forward (Sec. 4.2: d_model -> d_ff -> d_model;
 * Sec. 2.3: the per-expert matmuls carry the compute).  For every expert e and
 * its first n_e = expert_count[e] rows:
 *   z = xd_e * W1_e      (W1[E,d_model,d_ff])      (not stored)
 *   h = act(z)                                      -> h_saved[E,C,d_ff]
 *   act'(z)                                         -> dact_saved[E,C,d_ff]
 *   yd_e = h * W2_e      (W2[E,d_ff,d_model])      -> yd[E,C,d_model]
 * No biases.  relu'(z) = [z > 0]; gelu'(z) = Phi(z) + z phi(z).  h_saved and
 * dact_saved are kept by the caller for the backward: the activation and its
 * derivative are both evaluated here, once, while z is in registers.
 * Forward-only use (evaluation, Sec. 5.1: capacity factor 2.0): pass
 * dact_saved = NULL and the derivative is neither computed nor written;
 * h_saved is still required (it is the second matmul's input). */
int moe_expert_ffn_fwd(const moe_shape* shape, const void* xd, const int32_t* expert_count,
                       const void* W1, const void* W2, void* h_saved, void* dact_saved, void* yd,
                       void* stream);

/* Expert utilisation for pruning (Sec. 3.3: the experts with the highest
 * utilisation are kept; utilisation = number of times a token is routed to
 * the expert over a validation set):  accum[e] += counts[e] for e < E, with
 * counts = expert_demand (every routed candidate) or expert_count (kept ones)
 * of the batch just routed.  accum[E] is int64 and is owned, and zeroed before
 * the first batch, by the caller. */
int moe_utilisation_accumulate(const moe_shape* shape, const int32_t* counts, int64_t* accum,
                               void* stream);

/* Expert FFN forward with expert dropout (Sec. 5.4: expert dropout of 0.4 in
 * fine-tuning, as in the Switch Transformer: dropout on the expert's hidden
 * activation).  As moe_expert_ffn_fwd, except that element (e, s, c) of h is
 * dropped when its noise word < floor(drop_p * 2^32) and kept elements are
 * scaled by 1 / (1 - drop_p).  The same factor is folded into dact_saved, so
 * moe_expert_ffn_bwd is used unchanged.  0 <= drop_p < 1; drop_p = 0 is
 * moe_expert_ffn_fwd; dact_saved is required. */
int moe_expert_ffn_fwd_dropout(const moe_shape* shape, const void* xd, const int32_t* expert_count,
                               const void* W1, const void* W2, float drop_p, uint64_t seed,
                               void* h_saved, void* dact_saved, void* yd, void* stream);

/* Combine (the mixture itself; a token dropped by every chosen expert gets a
 * zero row and is carried by the residual connection around the layer,
 * Sec. 4.2 / Sec. 3.1):
 *   y[t,:] = sum over j with slot[t,j] >= 0 of gate_w[t,j] * yd[expert_idx[t,j], slot[t,j], :]
 * gate_w_or_null == NULL uses unit weights (that is dispatch's backward). */
int moe_combine_fwd(const moe_shape* shape, const void* yd, const int32_t* expert_idx,
                    const int32_t* slot, const float* gate_w_or_null, void* y, void* stream);

/* Combine, backward: the derivative of the gate-weighted mixture above (the
 * combine of Sec. 3.1 / Sec. 5.1) with respect to the expert outputs and the
 * gate weights.  For kept (t,j), with e = expert_idx[t,j], s = slot[t,j]:
 *   dyd[e,s,:]   = gate_w[t,j] * dy[t,:]
 *   dgate_w[t,j] = <dy[t,:], yd[e,s,:]>          (0 for a dropped choice) */
int moe_combine_bwd(const moe_shape* shape, const void* dy, const void* yd,
                    const int32_t* expert_idx, const int32_t* slot, const float* gate_w,
                    void* dyd, float* dgate_w, void* stream);

/* Expert feed-forward block, backward: the derivative of the two-matmul expert
 * of Sec. 4.2 (moe_expert_ffn_fwd) with respect to its input rows and its two
 * weight matrices; like the forward, this is where the layer's compute sits
 * (Sec. 2.3).  Per expert, over its first n_e rows:
 *   dh = dyd * W2^T,  dz = dh .* dact_saved,  dW2 = h_saved^T * dyd,
 *   dxd = dz * W1^T,  dW1 = xd^T * dz.
 * dW1[E,d_model,d_ff] and dW2[E,d_ff,d_model] are float; an expert with no
 * rows gets zero weight gradients.  Needs workspace (holds dz). */
int moe_expert_ffn_bwd(const moe_shape* shape, const void* dyd, const void* xd,
                       const void* h_saved, const void* dact_saved, const int32_t* expert_count,
                       const void* W1, const void* W2, void* dxd, float* dW1, float* dW2,
                       void* ws, size_t ws_bytes, void* stream);

/* Gate, backward: the derivative of the top-1 / top-2 gate weights of Sec. 5.1
 * (moe_gate_route) through the softmax with respect to the logits; the
 * selection and the capacity slots (Sec. 3.1) are constants.  With dg_j = dgate_w[t,j]
 * for kept choices and 0 for dropped ones,
 *   k=1: dp[t,e0] = dg_0
 *   k=2: S = p[t,e0]+p[t,e1]; dp[t,e0] = p[t,e1](dg_0-dg_1)/S^2; dp[t,e1] = p[t,e0](dg_1-dg_0)/S^2
 *   dlogits[t,e] = p[t,e] * (dp[t,e] - sum_e' p[t,e'] dp[t,e'])       -> dlogits[T,E] */
int moe_gate_bwd(const moe_shape* shape, const float* dgate_w, const float* probs,
                 const int32_t* expert_idx, const int32_t* slot, float* dlogits, void* stream);

/* Balancing auxiliary loss of the gate (Sec. 5.1, "MoE setting": an additional
 * balancing loss, multiplied by 0.01, is added to the training loss; Switch /
 * GShard form):
 *   first_frac[E] f[e] = (tokens whose first choice expert_idx[t,0] is e) / T,
 *                        counted before capacity drops
 *   mean_prob[E]  P[e] = (1/T) sum_t probs[t,e]
 *   loss[1]            = E * sum_e f[e] * P[e]         (1 for a uniform gate)
 * All three outputs are device floats.  Needs workspace. */
int moe_aux_loss(const moe_shape* shape, const float* probs, const int32_t* expert_idx,
                 float* first_frac, float* mean_prob, float* loss, void* ws, size_t ws_bytes,
                 void* stream);

/* moe_gate_bwd plus the gradient of aux_coef * loss (f held constant, it is a
 * count):  dp[t,e] gains aux_coef * E * first_frac[e] / T for EVERY token,
 * dropped or not, before the softmax backward.  aux_coef is a host value
 * (0.01 in Sec. 5.1, times any loss scale).  dlogits[T,E] is overwritten. */
int moe_gate_bwd_aux(const moe_shape* shape, const float* dgate_w, const float* probs,
                     const int32_t* expert_idx, const int32_t* slot, const float* first_frac,
                     float aux_coef, float* dlogits, void* stream);

/* Gate projection, backward: the derivative of the gating matrix product of
 * Sec. 3.2 (moe_gate_logits) with respect to the gate matrix and the tokens:
 *   dWg[d_model,E]  = x^T * dlogits                       (overwritten)
 *   dx_accum[T,d]  += dlogits * Wg^T                      (ACCUMULATED into the
 *   caller's dx, which already holds dispatch's backward; pass NULL to skip).
 * Needs workspace. */
int moe_gate_logits_bwd(const moe_shape* shape, const void* x, const float* Wg,
                        const float* dlogits, float* dWg, void* dx_accum,
                        void* ws, size_t ws_bytes, void* stream);

/* Backward of moe_gate_logits_jitter (same jitter_eps and seed as the forward):
 *   dWg = (x .* noise)^T * dlogits,   dx_accum += (dlogits * Wg^T) .* noise. */
int moe_gate_logits_bwd_jitter(const moe_shape* shape, const void* x, const float* Wg,
                               const float* dlogits, float jitter_eps, uint64_t seed, float* dWg,
                               void* dx_accum, void* ws, size_t ws_bytes, void* stream);

/* The last two steps of the layer's backward as one call: dispatch's backward
 * (moe_combine_fwd with NULL gate weights, the transpose of the dispatch of
 * Sec. 3.1) and moe_gate_logits_bwd_jitter, without the intermediate dx ever
 * being written and read back:
 *   dWg[d_model,E] = (x .* noise)^T * dlogits                           (overwritten)
 *   dx[t,:] = sum over kept choices j of dxd[expert_idx[t,j], slot[t,j], :]
 *             + ((dlogits * Wg^T) .* noise)[t,:]                        (overwritten)
 * dxd [E, capacity, d_model] and dx [T, d_model] have the activation type; the
 * sum is formed in fp32 and rounded once.  jitter_eps = 0: no noise (seed unused).
 * Needs workspace. */
int moe_dispatch_gate_logits_bwd(const moe_shape* shape, const void* x, const float* Wg,
                                 const float* dlogits, const void* dxd, const int32_t* expert_idx,
                                 const int32_t* slot, float jitter_eps, uint64_t seed, float* dWg,
                                 void* dx, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_HIP_H */
