/*
 * libsmile: forward and backward pass of one SMILE bi-level routed
 * Mixture-of-Experts layer on one AMD MI355X (gfx950), as a C-ABI library of
 * hand-written HIP kernels.
 *
 * Method: "SMILE: Scaling Mixture-of-Experts with Efficient Bi-level Routing",
 * arXiv 2212.05191.  A token is routed to one of n groups by an inter router
 * and then to one of the m experts of that group by an intra router
 * (Section 3.2.1); its output is p_i * q_j * E_{i,j}(x) (Eq. 3); the layer
 * adds a two-term load-balancing loss (Eq. 4).  On one GPU the paper's node /
 * GPU hierarchy is a logical two-level grouping: all N = n*m experts are
 * resident and the two All2All stages become one composed row permutation.
 *
 * General rules
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, dense,
 *     row-major, 16-byte aligned.  The library reads/writes it only during the
 *     call's enqueued work and never frees or keeps it.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued asynchronously on it; no call synchronises, and no
 *     call other than smile_create/smile_destroy allocates or frees memory.
 *   - Every function returns a smile_status; nothing throws or aborts.
 *     Argument checks happen on the host before anything is enqueued, so a
 *     non-OK status means no work was submitted (except SMILE_HIP_ERROR from a
 *     failed launch).
 *   - Notation: T tokens, d = d_model, F = d_ff, n = n_groups, m = m_local,
 *     N = n*m, flat expert id e = group*m + local, C = capacity (rows of each
 *     expert's buffer).  dtype is the storage type of x, router and expert
 *     weights, the expert buffers and y: 0 = fp32, 1 = bfloat16, 2 = IEEE half.
 *     Logits, probabilities, gates and the loss are always fp32; products of
 *     16-bit values accumulate in fp32 on the matrix cores.
 *   - Limits: T, d, F, n, m, C >= 1; d % 8 == 0 and F % 8 == 0 (for the 16-bit
 *     types: d % 64 == 0 and F % 64 == 0); n <= 1024, m <= 1024, N <= 4096;
 *     N*C*max(d,F) < 2^40 elements; N*C and T below 2^31 (T <= 2^30 with a
 *     group capacity).  n = 1 (or m = 1) gives the flat one-level top-1
 *     router of Section 2 (Eq. 1-2, k = 1).
 *   - Floating-point inputs must be finite; NaN/Inf give unspecified results.
 *   - Tuning switches (never needed in normal use; tests and sweeps set them): smile_create and
 *     smile_create_with_workspace read the environment variables SMILE_FFN_TILE (0-6: tile shape of
 *     the forward expert GEMMs), SMILE_TGEMM_TILE (0-3: tile shape of the gradient GEMMs),
 *     SMILE_FFN_PERSIST (0/1: plain or persistent GEMM grid) and SMILE_ROUTER_GRAD_MFMA (0: vector-ALU
 *     router-gradient kernels) ONCE and keep the values in the ctx; no other call looks at the
 *     environment.  They change which kernel variant runs, never a result beyond rounding order.
 *     The same two calls ask the runtime for the compute-unit count of the current device, which
 *     sizes the persistent GEMM grids of that ctx.
 */
#ifndef SMILE_H
#define SMILE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum smile_status {
    SMILE_OK = 0,
    SMILE_INVALID_ARG = 1,   /* NULL or misaligned pointer, NULL ctx/desc */
    SMILE_BAD_SHAPE = 2,     /* a size is out of range or violates a divisibility rule */
    SMILE_UNSUPPORTED = 3,   /* unknown dtype / activation, or a shape no kernel covers */
    SMILE_WORKSPACE = 4,     /* caller-supplied workspace too small or misaligned */
    SMILE_HIP_ERROR = 5      /* a HIP runtime call failed (allocation, launch) */
} smile_status;

enum { SMILE_DTYPE_F32 = 0, SMILE_DTYPE_BF16 = 1, SMILE_DTYPE_F16 = 2 };   /* F16: IEEE half, the paper's training precision (Section 4.1) */
enum { SMILE_ACT_RELU = 0, SMILE_ACT_GELU = 1 };   /* GELU is the exact erf form (Section 4.1) */

/* Static description of one layer; copied by smile_create. */
typedef struct smile_layer_desc {
    int32_t T;          /* tokens per call */
    int32_t d_model;
    int32_t d_ff;
    int32_t n_groups;   /* n: fan-out of the inter router (the paper's nodes) */
    int32_t m_local;    /* m: fan-out of the intra router (the paper's GPUs per node) */
    int32_t capacity;   /* C: rows per expert buffer, see smile_capacity */
    int32_t dtype;      /* SMILE_DTYPE_* */
    int32_t act;        /* SMILE_ACT_* */
    float alpha;        /* Eq. 4 coefficients */
    float beta;
    int32_t group_capacity;   /* Cg: rows of each group's first-hop buffer (Section 3.2.3); 0 = no limit */
} smile_layer_desc;

typedef struct smile_ctx smile_ctx;   /* opaque: a validated desc + device workspace */

/* Static string for a status code (never NULL). */
const char *smile_status_string(int32_t status);

/* Library version, e.g. "0.1.0". */
const char *smile_version(void);

/* Switch-style expert capacity for the "capacity factor" of Section 4.2:
 * ceil(cf * T / N), at least 1.  Host helper; returns -1 on invalid input. */
int32_t smile_capacity(int32_t T, int32_t N, double capacity_factor);

/* Host-only check of a desc against the limits above (no GPU needed). */
smile_status smile_validate_desc(const smile_layer_desc *desc);

/* Bytes of device workspace a ctx for `desc` needs (routing histograms and
 * partial sums, and the hidden activation h[N,C,F] between the two expert
 * GEMMs).  Host-only. */
smile_status smile_workspace_bytes(const smile_layer_desc *desc, size_t *bytes);

/* Create a ctx whose workspace the library allocates with hipMalloc on the
 * current device (freed by smile_destroy). */
smile_status smile_create(const smile_layer_desc *desc, smile_ctx **ctx);

/* Create a ctx on caller-owned device memory: `workspace` must be 256-byte
 * aligned, at least smile_workspace_bytes() long and must outlive the ctx.
 * Nothing is allocated on the device.  Calls on one ctx must not overlap. */
smile_status smile_create_with_workspace(const smile_layer_desc *desc, void *workspace, size_t bytes,
                                         smile_ctx **ctx);

/* Release a ctx (and its workspace if the library allocated it).  The caller
 * must have synchronised every stream that used it.  NULL is allowed. */
smile_status smile_destroy(smile_ctx *ctx);

/* Kernel timing, for benchmarks and profiles.  `events` is an array of 2*pairs hipEvent_t handles
 * (passed as void*, created by the caller with timing enabled, owned by the caller and alive until
 * detached).  While attached, every kernel that a later call on this ctx launches takes the next pair
 * (start, stop), which receives the begin and end timestamps of that kernel itself, so that
 * hipEventElapsedTime(start, stop) after synchronisation is the kernel's own duration without launch
 * gaps.  Each call starts again at pair 0; kernels beyond `pairs` (at most 32 are used) run untimed.
 * pairs = 0 detaches.  smile_kernel_timing_count: kernels that took a pair in the most recent call;
 * smile_kernel_timing_name: the kernel's name (a static string, "" out of range).  Results are
 * unchanged.  The array must not be in use by two threads at once. */
smile_status smile_kernel_timing(smile_ctx *ctx, void **events, int32_t pairs);
int32_t smile_kernel_timing_count(const smile_ctx *ctx);
const char *smile_kernel_timing_name(const smile_ctx *ctx, int32_t i);

/* Step 1 -- router logits r(x) = W_r x (Section 2, text before Eq. 1) for the
 * two tied routers of Section 3.2.1, both reading the same token vector:
 *   logits_inter[t,i] = sum_k x[t,k] * w_inter[i,k]      [T,n] fp32
 *   logits_intra[t,j] = sum_k x[t,k] * w_intra[j,k]      [T,m] fp32
 * x[T,d], w_inter[n,d], w_intra[m,d] in the ctx dtype; products accumulate in fp32. */
smile_status smile_gate_logits(smile_ctx *ctx, const void *x, const void *w_inter, const void *w_intra,
                               float *logits_inter, float *logits_intra, void *stream);

/* Steps 2-3 -- bi-level top-1 routing with capacity (Section 3.2.1; Eq. 1
 * read as a softmax; Section 3.2.2 for the statistics; Section 4.2 capacity).
 *   a[t,:] = logits_inter[t,:] + bias_inter            (one fp32 add, bias may be NULL)
 *   group_idx[t] = lowest index of max a[t,:];  p = softmax(a[t,:]);  p_top[t] = p[group_idx[t]]
 *   c[t,:] = logits_intra[t,:] + bias_intra[group_idx[t],:]   (bias_intra[n,m] may be NULL)
 *   local_idx[t] = lowest index of max c[t,:];  q = softmax(c[t,:]);  q_top[t] = q[local_idx[t]]
 *   gate[t] = p_top[t] * q_top[t]                      (Eq. 3)
 *   pos_in_group[t] = number of earlier tokens with the same group       (stage-1 position)
 *   rank = number of earlier tokens with the same (group, local)          (stage-2 position)
 *   slot[t] = rank if rank < C, else -1 (token dropped)
 *   With desc.group_capacity = Cg > 0 the first hop of Section 3.2.3 has a buffer of Cg rows per
 *   group as well: a token with pos_in_group[t] >= Cg is dropped there (slot -1) and is not counted
 *   in `rank` of later tokens; kept_count[e] is then min(tokens of e that passed the first hop, C).
 *   The counts and sums below ignore both kinds of drops.
 *   group_count[n], local_count[m] (summed over all groups), expert_count[N]: top-1 counts of all T
 *   tokens, before drops;  kept_count[e] = min(expert_count[e], C);
 *   p_sum[i] = sum_t p[t,i];  q_sum[j] = sum_t q[t,j]    (fp32)
 * Integer outputs are exact and independent of launch geometry; float sums are
 * accumulated in a fixed order, so repeated calls give identical bits. */
smile_status smile_route_bilevel(smile_ctx *ctx, const float *logits_inter, const float *logits_intra,
                                 const float *bias_inter, const float *bias_intra,
                                 int32_t *group_idx, int32_t *local_idx, int32_t *pos_in_group, int32_t *slot,
                                 float *gate, float *p_top, float *q_top,
                                 int32_t *group_count, int32_t *local_count, int32_t *expert_count,
                                 int32_t *kept_count, float *p_sum, float *q_sum, void *stream);

/* smile_route_bilevel for callers that cannot allocate device memory or create a ctx: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels, same arguments
 * and bit-identical results; instead of a ctx it takes the layer description, and its scratch memory
 * (per-block histograms, partial probability sums, block-local ranks: about 4*(T/256)*(N+2n+2m) +
 * 8*T bytes) is a fixed array of SMILE_STATIC_SCRATCH_BYTES inside the library's device image, which
 * every GPU the library runs on holds until the process ends.  Returns SMILE_WORKSPACE when the shape
 * needs more than that (T = 65536 with 256 experts needs 0.9 MB) and enqueues nothing then.  It calls
 * no hipMalloc / hipFree and nothing that allocates; the first call on a device looks up the array's
 * address (make that call outside a graph capture).  All calls on one GPU share the array: calls that
 * overlap there (other streams, other threads) race, calls in stream order do not, and no call
 * depends on what an earlier one left in it. */
#define SMILE_STATIC_SCRATCH_BYTES (4u << 20)
smile_status smile_route_bilevel_static(const smile_layer_desc *desc, const float *logits_inter,
                                        const float *logits_intra, const float *bias_inter,
                                        const float *bias_intra, int32_t *group_idx, int32_t *local_idx,
                                        int32_t *pos_in_group, int32_t *slot, float *gate, float *p_top,
                                        float *q_top, int32_t *group_count, int32_t *local_count,
                                        int32_t *expert_count, int32_t *kept_count, float *p_sum, float *q_sum,
                                        void *stream);

/* Step 3 -- dispatch: xe[e, slot[t], :] = x[t, :] for every kept token, e =
 * group_idx[t]*m + local_idx[t] (the two routing hops of Section 3.2.1 composed
 * into one row move).  xe[N,C,d] in the ctx dtype; rows at or beyond
 * kept_count[e] are not written. */
smile_status smile_dispatch(smile_ctx *ctx, const void *x, const int32_t *group_idx, const int32_t *local_idx,
                            const int32_t *slot, void *xe, void *stream);

/* The same move as the two hops of Section 3.2.3, with the first-hop buffer materialised (what the
 * inter-node All2All delivers): xg[n, group_rows, d] in the ctx dtype.
 *   hop 1: xg[group_idx[t], pos_in_group[t], :] = x[t, :]        for pos_in_group[t] < group_rows
 *   hop 2: xe[e, slot[t], :] = xg[group_idx[t], pos_in_group[t], :]   for slot[t] >= 0
 * group_rows >= 1; with a group capacity it is normally desc.group_capacity, without one any value
 * not below the largest group_count.  hop 2 requires pos_in_group[t] < group_rows for every kept
 * token (true for the outputs of smile_route_bilevel under the rule above) and does not check it on
 * the device beyond skipping such tokens.  Rows that receive nothing are not written. */
smile_status smile_dispatch_hop1(smile_ctx *ctx, const void *x, const int32_t *group_idx,
                                 const int32_t *pos_in_group, int32_t group_rows, void *xg, void *stream);
smile_status smile_dispatch_hop2(smile_ctx *ctx, const void *xg, const int32_t *group_idx,
                                 const int32_t *local_idx, const int32_t *pos_in_group, const int32_t *slot,
                                 int32_t group_rows, void *xe, void *stream);

/* Step 3 -- expert FFN E_e of Eq. 3 (Section 4.1: hidden -> intermediate ->
 * hidden with the activation of the ctx) on rows r < kept_count[e]:
 *   h  = act(xe[e,r,:] . w1[e]^T + b1[e])     w1[N,F,d]  (out-features x in-features), b1[N,F] or NULL
 *   ye[e,r,:] = h . w2[e]^T + b2[e]           w2[N,d,F],                              b2[N,d] or NULL
 * Weights and biases in the ctx dtype; accumulation in fp32; h is rounded to
 * the ctx dtype between the two products.  kept_count is read on the device
 * (no host sync); rows at or beyond kept_count[e] of ye are not written. */
smile_status smile_expert_ffn(smile_ctx *ctx, const void *xe, const int32_t *kept_count,
                              const void *w1, const void *b1, const void *w2, const void *b2,
                              void *ye, void *stream);

/* The two halves of smile_expert_ffn as separate calls (same kernels, same results), for callers
 * that want to time or interleave them: _up computes h = act(xe . w1^T + b1) into the ctx
 * workspace, _down computes ye = h . w2^T + b2 from it.  _down must follow an _up on the same ctx
 * and stream with the same kept_count. */
smile_status smile_expert_ffn_up(smile_ctx *ctx, const void *xe, const int32_t *kept_count,
                                 const void *w1, const void *b1, void *stream);
smile_status smile_expert_ffn_down(smile_ctx *ctx, const int32_t *kept_count, const void *w2, const void *b2,
                                   void *ye, void *stream);

/* smile_expert_ffn_up with kernel timing, for benchmarks: `start_event` and `stop_event` are
 * hipEvent_t handles (passed as void*, created by the caller with timing enabled, both non-NULL).
 * They receive the begin and end timestamps of the up-projection kernel itself, so that
 * hipEventElapsedTime(start, stop) after synchronisation is the kernel's own duration without
 * launch gaps.  Same work and results as smile_expert_ffn_up. */
smile_status smile_expert_ffn_up_timed(smile_ctx *ctx, const void *xe, const int32_t *kept_count,
                                       const void *w1, const void *b1, void *start_event, void *stop_event,
                                       void *stream);

/* Step 4 -- combine (Eq. 3): y[t,:] = gate[t] * ye[e, slot[t], :] for kept
 * tokens, 0 for dropped ones; product in fp32, rounded once to the ctx dtype. */
smile_status smile_combine(smile_ctx *ctx, const void *ye, const int32_t *group_idx, const int32_t *local_idx,
                           const int32_t *slot, const float *gate, void *y, void *stream);

/* Step 4 -- additive load-balancing loss (Eq. 4), from the statistics of
 * smile_route_bilevel:
 *   out3[0] = n * sum_i (group_count[i]/T) * (p_sum[i]/T)
 *   out3[1] = m * sum_j (local_count[j]/T) * (q_sum[j]/T)
 *   out3[2] = alpha*out3[0] + beta*out3[1]
 * out3: 3 fp32 values on the device. */
smile_status smile_aux_loss(smile_ctx *ctx, const int32_t *group_count, const int32_t *local_count,
                            const float *p_sum, const float *q_sum, float *out3, void *stream);

/* All tensors of one forward pass, for smile_layer_forward. */
typedef struct smile_layer_io {
    /* inputs */
    const void *x, *w_inter, *w_intra, *w1, *b1, *w2, *b2;
    const float *bias_inter, *bias_intra;
    /* intermediates and outputs (all caller-allocated) */
    float *logits_inter, *logits_intra;
    int32_t *group_idx, *local_idx, *pos_in_group, *slot;
    float *gate, *p_top, *q_top;
    int32_t *group_count, *local_count, *expert_count, *kept_count;
    float *p_sum, *q_sum;
    void *xe, *ye;   /* expert buffers [N,C,d]: both given, or both NULL (see smile_layer_forward) */
    void *y;
    float *loss3;
    /* optional: hipEvent_t pair (both or neither) receiving the begin / end timestamps of the
     * up-projection kernel, as in smile_expert_ffn_up_timed; NULL = no timing */
    void *prof_up_start, *prof_up_stop;
    /* optional (both or neither), for a backward pass that does not recompute them: the hidden
     * activation h = act(pre) and the pre-activation pre = xe . w1^T + b1, [N,C,F] in the ctx dtype,
     * rows below kept_count[e] only.  When given, h lives there instead of in the ctx workspace. */
    void *h_save, *pre_save;
} smile_layer_io;

/* The whole forward pass in one call: enqueues the six steps above in order on
 * `stream` (gate logits, route, dispatch, expert FFN, combine, loss).  Same checks
 * and bit-identical results as calling them one by one, with fewer launches:
 *   - io->xe and io->ye given: the expert buffers are materialised as by
 *     smile_dispatch / smile_expert_ffn; the last routing step and the loss run
 *     inside the dispatch kernel and the down-projection also writes y (6 launches
 *     instead of 9);
 *   - io->xe == io->ye == NULL: the permutations are fused into the expert GEMMs --
 *     the up-projection gathers its rows from x through a slot -> token map and the
 *     down-projection returns gate-weighted rows straight to y; rows of dropped
 *     tokens are zeroed by the routing (6 launches, 5 for batches of at most
 *     16384 tokens; no [N,C,d] traffic). */
smile_status smile_layer_forward(smile_ctx *ctx, const smile_layer_io *io, void *stream);

/* ---------------------------------------------------------------------------
 * Backward pass.  The paper trains the layer (Section 4.1) and prints no gradient formulas; these
 * entry points compute the derivative of the forward map defined above (Eq. 3 for y, Eq. 4 for the
 * loss) by the chain rule, for
 *     L = sum_{t,k} dy[t,k] * y[t,k] + dloss * (alpha*inter + beta*intra),
 * with the discrete decisions (top-1 indices, slots, drops) and the fractions f of Eq. 4 held
 * constant, as for the Switch loss of Section 2.  Gradient tensors stored in the ctx dtype (dye,
 * dxe, dx, dw1, dw2) are rounded once from fp32; dgate, dlp, dlq, dw_inter, dw_intra are fp32.
 * Experts with bias vectors are not covered (there is no b1 / b2 argument and no gradient for them).
 * The steps mirror the forward ones in reverse order; the tensors "saved from the forward pass" are
 * the outputs of the forward entry points for the same inputs.
 * ------------------------------------------------------------------------- */

/* Bytes of device scratch memory smile_expert_ffn_backward, smile_gate_weights_backward and
 * smile_layer_backward need: the recomputed h and pre, the gradient at the pre-activation (3 N*C*F
 * elements), partial sums of the router-weight gradient, and for fp32 also transposed copies of the
 * GEMM operands (about 2 N*C*F + 2 N*C*d + N*d*F more).  Host-only.  The memory is the caller's,
 * 256-byte aligned, and only used during the call's enqueued work. */
smile_status smile_backward_workspace_bytes(const smile_layer_desc *desc, size_t *bytes);

/* Eq. 3 backwards: for a kept token dye[e, slot[t], :] = gate[t] * dy[t, :] and
 * dgate[t] = sum_k dy[t,k] * ye[e, slot[t], k]; a dropped token gives dgate[t] = 0.
 * dy[T,d], ye[N,C,d], dye[N,C,d] in the ctx dtype; rows of dye no token owns are not written. */
smile_status smile_combine_backward(smile_ctx *ctx, const void *dy, const void *ye, const int32_t *group_idx,
                                    const int32_t *local_idx, const int32_t *slot, const float *gate,
                                    void *dye, float *dgate, void *stream);

/* The two routers backwards (Eq. 1 softmax, Eq. 3 gate, Eq. 4 loss).  With p, q the softmax rows of
 * token t (biases as in smile_route_bilevel), g = group_idx[t], l = local_idx[t]:
 *   u_i = dloss*alpha*n*group_count[i]/T^2 + [i == g] * dgate[t] * q[l],   dlp[t,k] = p_k (u_k - sum_i u_i p_i)
 *   v_j = dloss*beta *m*local_count[j]/T^2 + [j == l] * dgate[t] * p[g],   dlq[t,k] = q_k (v_k - sum_j v_j q_j)
 * dlp[T,n], dlq[T,m] fp32: the gradients with respect to the router logits. */
smile_status smile_route_backward(smile_ctx *ctx, const float *logits_inter, const float *logits_intra,
                                  const float *bias_inter, const float *bias_intra,
                                  const int32_t *group_idx, const int32_t *local_idx, const float *dgate,
                                  const int32_t *group_count, const int32_t *local_count, float dloss,
                                  float *dlp, float *dlq, void *stream);

/* Expert FFN backwards (E_e of Eq. 3, Section 4.1, no bias vectors), rows r < kept_count[e]:
 *   pre = xe[e] . w1[e]^T, h = act(pre)     (both rounded to the ctx dtype; taken from h / pre, the
 *                                            buffers smile_layer_forward saved, or recomputed here
 *                                            when both are NULL)
 *   dpre = (dye[e] . w2[e]) * act'(pre)
 *   dxe[e] = dpre . w1[e]                                              [N,C,d]
 *   dw2[e][c,f] = sum_r dye[e,r,c] * h[r,f]                            [N,d,F]
 *   dw1[e][f,k] = sum_r dpre[r,f] * xe[e,r,k]                          [N,F,d]
 * Rows of dxe at or beyond kept_count[e] are not written; an expert without rows gets zero
 * weight gradients. */
smile_status smile_expert_ffn_backward(smile_ctx *ctx, const void *xe, const int32_t *kept_count,
                                       const void *w1, const void *w2, const void *dye,
                                       const void *h, const void *pre,
                                       void *dxe, void *dw1, void *dw2,
                                       void *workspace, size_t workspace_bytes, void *stream);

/* Dispatch and router logits backwards: dx[t,:] = dxe[e, slot[t], :] (zero for a dropped token)
 *   + sum_i dlp[t,i] * w_inter[i,:] + sum_j dlq[t,j] * w_intra[j,:], rounded once.  dx[T,d]. */
smile_status smile_dispatch_backward(smile_ctx *ctx, const void *dxe, const int32_t *group_idx,
                                     const int32_t *local_idx, const int32_t *slot, const float *dlp,
                                     const float *dlq, const void *w_inter, const void *w_intra, void *dx,
                                     void *stream);

/* Router weights backwards: dw_inter[i,:] = sum_t dlp[t,i] * x[t,:], dw_intra[j,:] = sum_t dlq[t,j] * x[t,:]
 * (fp32 [n,d] and [m,d]); summed in a fixed order, so repeated calls give identical bits. */
smile_status smile_gate_weights_backward(smile_ctx *ctx, const void *x, const float *dlp, const float *dlq,
                                         float *dw_inter, float *dw_intra,
                                         void *workspace, size_t workspace_bytes, void *stream);

/* All tensors of one backward pass, for smile_layer_backward. */
typedef struct smile_backward_io {
    /* inputs of the forward pass */
    const void *x, *w_inter, *w_intra, *w1, *w2;
    const float *bias_inter, *bias_intra;            /* may be NULL */
    /* saved from the forward pass */
    const float *logits_inter, *logits_intra;
    const int32_t *group_idx, *local_idx, *slot;
    const float *gate;
    const int32_t *group_count, *local_count, *kept_count;
    const void *xe, *ye;
    const void *h, *pre;                             /* h_save / pre_save of the forward pass, or both NULL */
    /* upstream gradient of y */
    const void *dy;
    /* intermediates (caller-allocated): dye[N,C,d], dgate[T], dlp[T,n], dlq[T,m], dxe[N,C,d] */
    void *dye;
    float *dgate, *dlp, *dlq;
    void *dxe;
    /* results */
    void *dx;
    float *dw_inter, *dw_intra;
    void *dw1, *dw2;
} smile_backward_io;

/* The five backward steps in one call, in the order combine, route, expert FFN, dispatch, router
 * weights; same results as calling them one by one.  dloss is the upstream gradient of the
 * scalar loss of Eq. 4 (out3[2] of smile_aux_loss). */
smile_status smile_layer_backward(smile_ctx *ctx, const smile_backward_io *io, float dloss,
                                  void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SMILE_H */
