/*
 * CPU oracle for one SMILE bi-level routed MoE layer: forward pass and, at the
 * end of the file, its derivative (backward pass).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, written-from-the-
 * paper definition of what the layer computes.  It exists so that the GPU
 * library can be checked against it; nothing in the product path may call it.
 * It shares no code, header, table or helper with the GPU library.
 *
 * Source: "SMILE: Scaling Mixture-of-Experts with Efficient Bi-level Routing"
 * (arXiv 2212.05191).  Each function names the passage it follows.
 *
 * Conventions
 *   - All tensors are dense, row-major, host memory.  Activations and weights
 *     come in as float (their values already rounded to the storage type of
 *     the configuration); every sum is accumulated in double.
 *   - T tokens, d = d_model, F = d_ff, n groups (the paper's nodes), m experts
 *     per group (the paper's GPUs per node), N = n*m experts, flat expert id
 *     e = i*m + j for expert j of group i (Section 3.2.1, E_{i,j}).
 *   - C = capacity = rows of each expert's buffer.
 *   - dtype 0: storage is fp32; dtype 1: storage is bfloat16, dtype 2: IEEE
 *     half precision (the precision the paper trains in, Section 4.1), so values
 *     that the layer stores (hidden activation h, expert output, layer output)
 *     are rounded to that type (nearest, ties to even) where they would be stored.
 *
 * Readings of points the paper leaves open:
 *   - Eq. 1 is read as a softmax, as the sentence introducing it says.
 *   - One inter router W_p[n,d] and ONE intra router W_q[m,d] shared by all
 *     groups ("tied parameters", router size O(m+n), Section 3.2.1).
 *   - Optional additive routing biases are added to the logits in fp32 (one
 *     IEEE add) and the top-1 decision is the lowest index attaining the
 *     maximum biased logit, compared in fp32.
 *   - Capacity is per expert; tokens claim slots in token order; a token whose
 *     expert is full is dropped and its output row is zero.
 *   - f in Eq. 4 counts the argmax decisions of all T tokens (before drops).
 *
 * Pins: see tests/test_oracle_*.py (brute force, n=1 == flat top-1 router,
 * infinite capacity, load <= capacity, dispatch/combine identity, uniform
 * router loss == 1 per term, dense-FFN cross-check against numpy/scipy).
 * Parity unpinned: whether the capacity / drop-priority rule equals that of
 * the authors' unreleased code (the paper only names a "capacity factor").
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* number of threads the loops below will use */
int smile_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Switch-style expert capacity named by Section 4.2 ("capacity factor"):
 * C = ceil(cf * T / N), at least 1. */
int32_t smile_oracle_capacity(int32_t T, int32_t N, double cf)
{
    double c = ceil(cf * (double)T / (double)N);
    if (c < 1.0) c = 1.0;
    return (int32_t)c;
}

/* value -> nearest bfloat16 (ties to even), returned as double.  bfloat16 is
 * the upper 16 bits of an IEEE fp32: 8 exponent bits, 7 stored mantissa bits. */
static double round_bf16(double v)
{
    if (v == 0.0 || !isfinite(v)) return v;
    int ex;
    (void)frexp(v, &ex);          /* |v| = f * 2^ex, f in [0.5, 1) */
    int e = ex - 1;               /* |v| in [2^e, 2^(e+1)) */
    if (e < -126) e = -126;       /* subnormal range of the format */
    double ulp = ldexp(1.0, e - 7);
    double q = nearbyint(v / ulp); /* default rounding mode: nearest even */
    return q * ulp;
}

/* nearest binary16 value (IEEE half: 11 significant bits, exponents -14..15, subnormals below 2^-14,
 * ties to even, overflow to infinity) */
static double round_f16(double v)
{
    if (v == 0.0 || !isfinite(v)) return v;
    int ex;
    (void)frexp(v, &ex);
    int e = ex - 1;               /* |v| in [2^e, 2^(e+1)) */
    if (e < -14) e = -14;
    double ulp = ldexp(1.0, e - 10);
    double q = nearbyint(v / ulp) * ulp;
    if (fabs(q) > 65504.0) return v > 0 ? INFINITY : -INFINITY;
    return q;
}

static double store_round(double v, int dtype)
{
    if (dtype == 1) return round_bf16(v);
    if (dtype == 2) return round_f16(v);
    return (double)(float)v;
}

/* Router logits r(x) = W_r x (Section 2, before Eq. 1), once for the inter
 * router W_p[n,d] and once for the intra router W_q[m,d]; both read the same
 * token vector (Eq. 3).  Output rounded once to fp32. */
void smile_oracle_gate_logits(const float *x, const float *w_inter, const float *w_intra,
                              int32_t T, int32_t d, int32_t n, int32_t m,
                              float *logits_inter, float *logits_intra)
{
#pragma omp parallel for schedule(static)
    for (int32_t t = 0; t < T; ++t) {
        const float *xt = x + (size_t)t * d;
        for (int32_t i = 0; i < n; ++i) {
            double s = 0.0;
            for (int32_t k = 0; k < d; ++k) s += (double)xt[k] * (double)w_inter[(size_t)i * d + k];
            logits_inter[(size_t)t * n + i] = (float)s;
        }
        for (int32_t j = 0; j < m; ++j) {
            double s = 0.0;
            for (int32_t k = 0; k < d; ++k) s += (double)xt[k] * (double)w_intra[(size_t)j * d + k];
            logits_intra[(size_t)t * m + j] = (float)s;
        }
    }
}

/* softmax of a[0..len) (Eq. 1 read as a softmax), max-subtracted, in double;
 * returns the lowest index of the maximum of a (compared as fp32). */
static int32_t softmax_top1(const float *a, int32_t len, double *prob)
{
    int32_t arg = 0;
    for (int32_t i = 1; i < len; ++i)
        if (a[i] > a[arg]) arg = i;
    double mx = (double)a[arg], z = 0.0;
    for (int32_t i = 0; i < len; ++i) { prob[i] = exp((double)a[i] - mx); z += prob[i]; }
    for (int32_t i = 0; i < len; ++i) prob[i] /= z;
    return arg;
}

/* Bi-level top-1 routing with per-expert capacity.
 *
 * Section 3.2.1: a token is first routed to a group by the inter router and
 * then to a local expert of that group by the intra router; Eq. 3: its output
 * is weighted by p_i * q_j, the two top-1 probabilities.  Section 3.2.2:
 * f counts argmax decisions, P and Q average the probabilities; the sums of
 * probabilities and the counts are returned here and turned into the loss by
 * smile_oracle_aux_loss.  Capacity (Section 4.2): tokens are visited in
 * increasing token index; each takes the next free slot of its expert and is
 * dropped (slot = -1) once C slots are taken.  pos_in_group is the token's
 * rank among the tokens of its group (the first-stage position).
 *
 * Optional group-level capacity Cg (Cg <= 0: none): the first hop of
 * Section 3.2.3 (the inter-node All2All) also has a buffer of fixed size per
 * group.  A token whose pos_in_group is >= Cg is dropped at that hop: it never
 * reaches the second hop, so it takes no expert slot and does not push later
 * tokens of its expert out.  The statistics of Section 3.2.2 (counts, sums)
 * are those of the router and ignore both kinds of drops.
 *
 * bias_inter[n] and bias_intra[n,m] may be NULL.
 */
void smile_oracle_route(const float *logits_inter, const float *logits_intra,
                        const float *bias_inter, const float *bias_intra,
                        int32_t T, int32_t n, int32_t m, int32_t C, int32_t Cg,
                        int32_t *group_idx, int32_t *local_idx, int32_t *pos_in_group, int32_t *slot,
                        double *gate, double *p_top, double *q_top,
                        int32_t *group_count, int32_t *local_count, int32_t *expert_count,
                        int32_t *kept_count, double *p_sum, double *q_sum)
{
    const int32_t N = n * m;
    int32_t *arrived = (int32_t *)calloc((size_t)N, sizeof(int32_t));   /* tokens that reached expert e */
    float *a = (float *)malloc(sizeof(float) * (size_t)(n > m ? n : m));
    double *pr = (double *)malloc(sizeof(double) * (size_t)(n > m ? n : m));
    for (int32_t i = 0; i < n; ++i) { group_count[i] = 0; p_sum[i] = 0.0; }
    for (int32_t j = 0; j < m; ++j) { local_count[j] = 0; q_sum[j] = 0.0; }
    for (int32_t e = 0; e < N; ++e) { expert_count[e] = 0; kept_count[e] = 0; }

    for (int32_t t = 0; t < T; ++t) {
        /* level 1: group */
        for (int32_t i = 0; i < n; ++i) {
            float v = logits_inter[(size_t)t * n + i];
            if (bias_inter) v = v + bias_inter[i];
            a[i] = v;
        }
        int32_t g = softmax_top1(a, n, pr);
        for (int32_t i = 0; i < n; ++i) p_sum[i] += pr[i];
        double pt = pr[g];
        /* level 2: local expert inside the chosen group */
        for (int32_t j = 0; j < m; ++j) {
            float v = logits_intra[(size_t)t * m + j];
            if (bias_intra) v = v + bias_intra[(size_t)g * m + j];
            a[j] = v;
        }
        int32_t l = softmax_top1(a, m, pr);
        for (int32_t j = 0; j < m; ++j) q_sum[j] += pr[j];
        double qt = pr[l];

        group_idx[t] = g;
        local_idx[t] = l;
        p_top[t] = pt;
        q_top[t] = qt;
        gate[t] = pt * qt;

        /* slots in token order */
        int32_t e = g * m + l;
        int32_t pos1 = group_count[g];
        pos_in_group[t] = pos1;
        group_count[g] += 1;
        local_count[l] += 1;
        expert_count[e] += 1;
        if (Cg > 0 && pos1 >= Cg) { slot[t] = -1; continue; }   /* dropped at the first hop */
        int32_t s = arrived[e];
        arrived[e] += 1;
        if (s < C) { slot[t] = s; kept_count[e] += 1; }
        else slot[t] = -1;
    }
    free(a);
    free(pr);
    free(arrived);
}

/* The same slot assignment done literally in two stages, as the two
 * consecutive All2Alls of Section 3.2.3 would move the tokens: stage 1 buckets
 * the tokens by group keeping token order; stage 2 walks each group's bucket
 * in that order and buckets by local expert, dropping what exceeds C.
 * Used to check that the composed single move equals the two-stage one. */
void smile_oracle_slots_two_stage(const int32_t *group_idx, const int32_t *local_idx,
                                  int32_t T, int32_t n, int32_t m, int32_t C, int32_t Cg,
                                  int32_t *pos_in_group, int32_t *slot)
{
    int32_t *bucket = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    int32_t *fill = (int32_t *)malloc(sizeof(int32_t) * (size_t)m);
    for (int32_t i = 0; i < n; ++i) {
        int32_t len = 0;
        for (int32_t t = 0; t < T; ++t)          /* stage 1 */
            if (group_idx[t] == i) { pos_in_group[t] = len; bucket[len++] = t; }
        if (Cg > 0 && len > Cg) {                 /* the group's buffer holds Cg tokens: the rest is dropped */
            for (int32_t r = Cg; r < len; ++r) slot[bucket[r]] = -1;
            len = Cg;
        }
        for (int32_t j = 0; j < m; ++j) fill[j] = 0;
        for (int32_t r = 0; r < len; ++r) {       /* stage 2 */
            int32_t t = bucket[r], j = local_idx[t];
            slot[t] = fill[j] < C ? fill[j] : -1;
            fill[j] += 1;
        }
    }
    free(bucket);
    free(fill);
}

/* Dispatch: the kept token t becomes row slot[t] of the buffer of expert
 * e = group_idx[t]*m + local_idx[t] (Section 3.2.1, first paragraph).
 * xe[N,C,d]; rows that receive no token are left as the caller set them. */
void smile_oracle_dispatch(const float *x, const int32_t *group_idx, const int32_t *local_idx,
                           const int32_t *slot, int32_t T, int32_t d, int32_t m, int32_t C, float *xe)
{
    for (int32_t t = 0; t < T; ++t) {
        if (slot[t] < 0) continue;
        size_t row = ((size_t)(group_idx[t] * m + local_idx[t]) * C + (size_t)slot[t]);
        memcpy(xe + row * d, x + (size_t)t * d, sizeof(float) * (size_t)d);
    }
}

/* The same move done in two hops (Section 3.2.3).  Hop 1: token t goes to row
 * pos_in_group[t] of the buffer of its group, xg[n,Cg,d], unless that row does
 * not exist (pos_in_group[t] >= Cg).  Hop 2: a kept token goes from there to
 * row slot[t] of its expert's buffer.  Rows that receive nothing keep the
 * caller's values. */
void smile_oracle_dispatch_stage1(const float *x, const int32_t *group_idx, const int32_t *pos_in_group,
                                  int32_t T, int32_t d, int32_t Cg, float *xg)
{
    for (int32_t t = 0; t < T; ++t) {
        if (pos_in_group[t] >= Cg) continue;
        memcpy(xg + ((size_t)group_idx[t] * Cg + (size_t)pos_in_group[t]) * d, x + (size_t)t * d,
               sizeof(float) * (size_t)d);
    }
}

void smile_oracle_dispatch_stage2(const float *xg, const int32_t *group_idx, const int32_t *local_idx,
                                  const int32_t *pos_in_group, const int32_t *slot,
                                  int32_t T, int32_t d, int32_t m, int32_t C, int32_t Cg, float *xe)
{
    for (int32_t t = 0; t < T; ++t) {
        if (slot[t] < 0) continue;
        size_t row = ((size_t)(group_idx[t] * m + local_idx[t]) * C + (size_t)slot[t]);
        memcpy(xe + row * d, xg + ((size_t)group_idx[t] * Cg + (size_t)pos_in_group[t]) * d,
               sizeof(float) * (size_t)d);
    }
}

static double act_fn(double v, int act)
{
    if (act == 0) return v > 0.0 ? v : 0.0;            /* ReLU */
    return 0.5 * v * (1.0 + erf(v / sqrt(2.0)));        /* exact GELU (Section 4.1) */
}

/* Expert FFN E_e (Eq. 3; Section 4.1: a Transformer feed-forward block,
 * hidden -> intermediate -> hidden with GELU):
 *   h  = act(xe[e,r,:] . w1[e]^T + b1[e])      w1[N,F,d]  (out x in)
 *   ye = h . w2[e]^T + b2[e]                   w2[N,d,F]
 * for rows r < kept_count[e]; other rows of ye are left untouched.
 * h and ye are rounded to the storage type where the layer stores them.
 * b1[N,F], b2[N,d] may be NULL.  act: 0 ReLU, 1 GELU. */
void smile_oracle_expert_ffn(const float *xe, const int32_t *kept_count,
                             const float *w1, const float *b1, const float *w2, const float *b2,
                             int32_t N, int32_t C, int32_t d, int32_t F, int32_t act, int32_t dtype,
                             float *ye)
{
    for (int32_t e = 0; e < N; ++e) {
        const float *W1 = w1 + (size_t)e * F * d;
        const float *W2 = w2 + (size_t)e * d * F;
        int32_t rows = kept_count[e];
#pragma omp parallel
        {
            double *h = (double *)malloc(sizeof(double) * (size_t)F);
#pragma omp for schedule(static)
            for (int32_t r = 0; r < rows; ++r) {
                const float *xr = xe + ((size_t)e * C + r) * d;
                for (int32_t f = 0; f < F; ++f) {
                    double s = 0.0;
                    for (int32_t k = 0; k < d; ++k) s += (double)xr[k] * (double)W1[(size_t)f * d + k];
                    if (b1) s += (double)b1[(size_t)e * F + f];
                    h[f] = store_round(act_fn(s, act), dtype);
                }
                float *yr = ye + ((size_t)e * C + r) * d;
                for (int32_t c = 0; c < d; ++c) {
                    double s = 0.0;
                    for (int32_t f = 0; f < F; ++f) s += h[f] * (double)W2[(size_t)c * F + f];
                    if (b2) s += (double)b2[(size_t)e * d + c];
                    yr[c] = (float)store_round(s, dtype);
                }
            }
            free(h);
        }
    }
}

/* Combine (Eq. 3): y[t,:] = p_i q_j E_{i,j}(x_t) for kept tokens, zero for
 * dropped ones; the product is rounded once to the storage type. */
void smile_oracle_combine(const float *ye, const int32_t *group_idx, const int32_t *local_idx,
                          const int32_t *slot, const double *gate,
                          int32_t T, int32_t d, int32_t m, int32_t C, int32_t dtype, float *y)
{
    for (int32_t t = 0; t < T; ++t) {
        float *yt = y + (size_t)t * d;
        if (slot[t] < 0) { for (int32_t c = 0; c < d; ++c) yt[c] = 0.0f; continue; }
        size_t row = ((size_t)(group_idx[t] * m + local_idx[t]) * C + (size_t)slot[t]);
        for (int32_t c = 0; c < d; ++c)
            yt[c] = (float)store_round(gate[t] * (double)ye[row * d + c], dtype);
    }
}

/* Additive load-balancing loss (Eq. 4):
 *   inter = n * sum_i f_i P_i,  intra = m * sum_j f_j Q_j,
 *   f = count / T,  P = p_sum / T,  Q = q_sum / T,
 *   out = { inter, intra, alpha*inter + beta*intra }. */
void smile_oracle_aux_loss(const int32_t *group_count, const int32_t *local_count,
                           const double *p_sum, const double *q_sum,
                           int32_t T, int32_t n, int32_t m, double alpha, double beta, double *out3)
{
    double inter = 0.0, intra = 0.0;
    for (int32_t i = 0; i < n; ++i) inter += ((double)group_count[i] / T) * (p_sum[i] / T);
    for (int32_t j = 0; j < m; ++j) intra += ((double)local_count[j] / T) * (q_sum[j] / T);
    inter *= (double)n;
    intra *= (double)m;
    out3[0] = inter;
    out3[1] = intra;
    out3[2] = alpha * inter + beta * intra;
}

/* ===========================================================================
 * Backward pass: the derivative of the forward map above.
 *
 * The paper trains the layer (Section 4.1) but prints no gradient formulas, so
 * the definition is the chain rule applied to Eq. 3 and Eq. 4:
 *     L = sum_{t,k} dy[t,k] * y[t,k]  +  dloss * (alpha*inter + beta*intra)
 * with the discrete decisions (top-1 indices, slots, drops) and the fractions
 * f of Eq. 4 held constant, as for the Switch loss the paper builds on
 * (Section 2).  The functions take the steps of the forward pass in reverse.
 * Values that the layer would store in its storage type are rounded there
 * (dye, the gradient at the pre-activation, dxe, dx, the expert weight
 * gradients); every sum is accumulated in double.
 * =========================================================================== */

/* Eq. 3 backwards: y[t] = gate_t * ye[row(t)] for a kept token, so
 *   dye[row(t), :] = gate_t * dy[t, :]      (rounded to the storage type)
 *   dgate[t]       = sum_k dy[t,k] * ye[row(t),k]
 * and a dropped token (y[t] = 0) sends nothing back: dgate[t] = 0.  Rows of
 * dye that no token owns keep the caller's values. */
void smile_oracle_combine_backward(const float *dy, const float *ye, const int32_t *group_idx,
                                   const int32_t *local_idx, const int32_t *slot, const double *gate,
                                   int32_t T, int32_t d, int32_t m, int32_t C, int32_t dtype,
                                   float *dye, double *dgate)
{
    for (int32_t t = 0; t < T; ++t) {
        dgate[t] = 0.0;
        if (slot[t] < 0) continue;
        size_t row = ((size_t)(group_idx[t] * m + local_idx[t]) * C + (size_t)slot[t]);
        double s = 0.0;
        for (int32_t k = 0; k < d; ++k) {
            s += (double)dy[(size_t)t * d + k] * (double)ye[row * d + k];
            dye[row * d + k] = (float)store_round(gate[t] * (double)dy[(size_t)t * d + k], dtype);
        }
        dgate[t] = s;
    }
}

/* softmax of a biased logit row into prob[len] (same arithmetic as the forward pass) */
static void softmax_row(const float *row, const float *bias, int32_t len, float *a, double *prob)
{
    for (int32_t i = 0; i < len; ++i) a[i] = bias ? row[i] + bias[i] : row[i];
    (void)softmax_top1(a, len, prob);
}

/* Routers backwards.  With p = softmax(a), q = softmax(c) (Eq. 1), gate = p_g * q_l (Eq. 3) and
 * Eq. 4's P_i = (1/T) sum_t p[t,i], Q_j likewise, the derivative of L with respect to the
 * probabilities of token t is
 *   u_i = dloss*alpha*n*f_i/T + [i == g_t] * dgate[t] * q[l_t]
 *   v_j = dloss*beta *m*f_j/T + [j == l_t] * dgate[t] * p[g_t]
 * and the softmax Jacobian gives the derivative with respect to the logits:
 *   dlp[t,k] = p_k * (u_k - sum_i u_i p_i),   dlq[t,k] = q_k * (v_k - sum_j v_j q_j). */
void smile_oracle_route_backward(const float *logits_inter, const float *logits_intra,
                                 const float *bias_inter, const float *bias_intra,
                                 const int32_t *group_idx, const int32_t *local_idx, const double *dgate,
                                 const int32_t *group_count, const int32_t *local_count,
                                 int32_t T, int32_t n, int32_t m, double alpha, double beta, double dloss,
                                 double *dlp, double *dlq)
{
    int32_t len = n > m ? n : m;
    float *a = (float *)malloc(sizeof(float) * (size_t)len);
    double *p = (double *)malloc(sizeof(double) * (size_t)n);
    double *q = (double *)malloc(sizeof(double) * (size_t)m);
    double *u = (double *)malloc(sizeof(double) * (size_t)len);
    for (int32_t t = 0; t < T; ++t) {
        int32_t g = group_idx[t], l = local_idx[t];
        softmax_row(logits_inter + (size_t)t * n, bias_inter, n, a, p);
        softmax_row(logits_intra + (size_t)t * m, bias_intra ? bias_intra + (size_t)g * m : NULL, m, a, q);
        double dot = 0.0;
        for (int32_t i = 0; i < n; ++i) {
            u[i] = dloss * alpha * (double)n * ((double)group_count[i] / T) / T;
            if (i == g) u[i] += dgate[t] * q[l];
            dot += u[i] * p[i];
        }
        for (int32_t i = 0; i < n; ++i) dlp[(size_t)t * n + i] = p[i] * (u[i] - dot);
        dot = 0.0;
        for (int32_t j = 0; j < m; ++j) {
            u[j] = dloss * beta * (double)m * ((double)local_count[j] / T) / T;
            if (j == l) u[j] += dgate[t] * p[g];
            dot += u[j] * q[j];
        }
        for (int32_t j = 0; j < m; ++j) dlq[(size_t)t * m + j] = q[j] * (u[j] - dot);
    }
    free(a); free(p); free(q); free(u);
}

static double act_grad(double v, int act)
{
    if (act == 0) return v > 0.0 ? 1.0 : 0.0;
    /* d/dv [v Phi(v)] = Phi(v) + v phi(v) */
    return 0.5 * (1.0 + erf(v / sqrt(2.0))) + v * exp(-0.5 * v * v) / sqrt(2.0 * 3.14159265358979323846);
}

/* Expert FFN backwards (the E_{i,j} of Eq. 3, Section 4.1), for the rows r < kept[e] of every expert:
 *   pre = xe . W1^T,  h = act(pre)         (recomputed; pre and h rounded to the storage type)
 *   dh   = dye . W2                         [rows, F]
 *   dpre = dh * act'(pre)                   (rounded to the storage type)
 *   dxe  = dpre . W1                        [rows, d]   (rounded)
 *   dW2[c,f] = sum_r dye[r,c] * h[r,f],   dW1[f,k] = sum_r dpre[r,f] * xe[r,k]   (rounded)
 * Rows of dxe at or beyond kept[e] keep the caller's values; an expert without tokens gets zero
 * weight gradients. */
void smile_oracle_expert_ffn_backward(const float *xe, const int32_t *kept_count, const float *w1,
                                      const float *w2, const float *dye,
                                      int32_t N, int32_t C, int32_t d, int32_t F, int32_t act, int32_t dtype,
                                      float *dxe, float *dw1, float *dw2)
{
    for (int32_t e = 0; e < N; ++e) {
        const float *W1 = w1 + (size_t)e * F * d;
        const float *W2 = w2 + (size_t)e * d * F;
        const int32_t rows = kept_count[e];
        double *h = (double *)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * F);
        double *dpre = (double *)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * F);
#pragma omp parallel for schedule(static)
        for (int32_t r = 0; r < rows; ++r) {
            const float *xr = xe + ((size_t)e * C + r) * d;
            const float *gr = dye + ((size_t)e * C + r) * d;
            for (int32_t f = 0; f < F; ++f) {
                double s = 0.0;
                for (int32_t k = 0; k < d; ++k) s += (double)xr[k] * (double)W1[(size_t)f * d + k];
                h[(size_t)r * F + f] = store_round(act_fn(s, act), dtype);
                double pre = store_round(s, dtype);
                double dh = 0.0;
                for (int32_t c = 0; c < d; ++c) dh += (double)gr[c] * (double)W2[(size_t)c * F + f];
                dpre[(size_t)r * F + f] = store_round(dh * act_grad(pre, act), dtype);
            }
            float *dxr = dxe + ((size_t)e * C + r) * d;
            for (int32_t k = 0; k < d; ++k) {
                double s = 0.0;
                for (int32_t f = 0; f < F; ++f) s += dpre[(size_t)r * F + f] * (double)W1[(size_t)f * d + k];
                dxr[k] = (float)store_round(s, dtype);
            }
        }
#pragma omp parallel for schedule(static)
        for (int32_t f = 0; f < F; ++f) {
            for (int32_t k = 0; k < d; ++k) {
                double s = 0.0;
                for (int32_t r = 0; r < rows; ++r) s += dpre[(size_t)r * F + f] * (double)xe[((size_t)e * C + r) * d + k];
                dw1[((size_t)e * F + f) * d + k] = (float)store_round(s, dtype);
            }
        }
#pragma omp parallel for schedule(static)
        for (int32_t c = 0; c < d; ++c) {
            for (int32_t f = 0; f < F; ++f) {
                double s = 0.0;
                for (int32_t r = 0; r < rows; ++r) s += (double)dye[((size_t)e * C + r) * d + c] * h[(size_t)r * F + f];
                dw2[((size_t)e * d + c) * F + f] = (float)store_round(s, dtype);
            }
        }
        free(h);
        free(dpre);
    }
}

/* Dispatch and router logits backwards: a token's input reached the output through its expert
 * (xe[row(t)] = x[t], kept tokens only) and through the two routers (logits = W x):
 *   dx[t,:] = dxe[row(t),:] (0 if dropped) + sum_i dlp[t,i] W_p[i,:] + sum_j dlq[t,j] W_q[j,:]
 * rounded once to the storage type. */
void smile_oracle_dispatch_backward(const float *dxe, const int32_t *group_idx, const int32_t *local_idx,
                                    const int32_t *slot, const double *dlp, const double *dlq,
                                    const float *w_inter, const float *w_intra,
                                    int32_t T, int32_t d, int32_t n, int32_t m, int32_t C, int32_t dtype, float *dx)
{
#pragma omp parallel for schedule(static)
    for (int32_t t = 0; t < T; ++t) {
        for (int32_t k = 0; k < d; ++k) {
            double s = 0.0;
            if (slot[t] >= 0)
                s = (double)dxe[(((size_t)(group_idx[t] * m + local_idx[t]) * C + (size_t)slot[t])) * d + k];
            for (int32_t i = 0; i < n; ++i) s += dlp[(size_t)t * n + i] * (double)w_inter[(size_t)i * d + k];
            for (int32_t j = 0; j < m; ++j) s += dlq[(size_t)t * m + j] * (double)w_intra[(size_t)j * d + k];
            dx[(size_t)t * d + k] = (float)store_round(s, dtype);
        }
    }
}

/* Router weights backwards (logits = W x): dW_p[i,:] = sum_t dlp[t,i] x[t,:], dW_q[j,:] likewise. */
void smile_oracle_gate_weights_backward(const float *x, const double *dlp, const double *dlq,
                                        int32_t T, int32_t d, int32_t n, int32_t m,
                                        double *dw_inter, double *dw_intra)
{
    for (int32_t i = 0; i < n; ++i)
        for (int32_t k = 0; k < d; ++k) {
            double s = 0.0;
            for (int32_t t = 0; t < T; ++t) s += dlp[(size_t)t * n + i] * (double)x[(size_t)t * d + k];
            dw_inter[(size_t)i * d + k] = s;
        }
    for (int32_t j = 0; j < m; ++j)
        for (int32_t k = 0; k < d; ++k) {
            double s = 0.0;
            for (int32_t t = 0; t < T; ++t) s += dlq[(size_t)t * m + j] * (double)x[(size_t)t * d + k];
            dw_intra[(size_t)j * d + k] = s;
        }
}
