// C-ABI entry points of libsmile: argument validation, ctx / workspace management and
// dispatch to the kernel launchers.  All checks run on the host before anything is enqueued.
#include <cmath>
#include <cstdlib>
#include <new>

#include "smile_internal.hpp"

namespace smile {

thread_local KernelTimer *tls_kernel_timer = nullptr;

// Installs the ctx's kernel timer (if events are attached) for the duration of one library call on this thread.
// A call made from inside another library call (smile_expert_ffn calls its two halves) leaves the outer one's
// state alone.
struct TimerScope {
    bool mine = false;
    explicit TimerScope(smile_ctx *c)
    {
        if (c && c->timer.pairs > 0 && !tls_kernel_timer) {
            c->timer.used = 0;
            tls_kernel_timer = &c->timer;
            mine = true;
        }
    }
    ~TimerScope()
    {
        if (mine) tls_kernel_timer = nullptr;
    }
};

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

Layout workspace_layout(const smile_layer_desc &d)
{
    Layout L{};
    const size_t B = ((size_t)d.T + kRouteBlock - 1) / kRouteBlock;
    const size_t N = (size_t)d.n_groups * d.m_local;
    const size_t esz = elem_size(d.dtype);
    size_t off = 0;
    L.route_blocks = (int32_t)B;
    L.off_block_expert_hist = off; off = align_up(off + B * N * sizeof(int32_t), 256);
    L.off_block_group_hist = off;  off = align_up(off + B * (d.n_groups + d.m_local) * sizeof(int32_t), 256);
    L.off_block_p_sum = off;       off = align_up(off + B * d.n_groups * sizeof(float), 256);
    L.off_block_q_sum = off;       off = align_up(off + B * d.m_local * sizeof(float), 256);
    L.off_rank_in_block = off;     off = align_up(off + (size_t)d.T * sizeof(int32_t), 256);
    L.off_pos_in_block = off;      off = align_up(off + (size_t)d.T * sizeof(int32_t), 256);
    L.off_slot_token = off;        off = align_up(off + N * (size_t)d.capacity * sizeof(int32_t), 256);
    L.off_hidden = off;            off = align_up(off + N * (size_t)d.capacity * d.d_ff * esz, 256);
    L.total = off;
    return L;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// required pointer: non-NULL and 16-byte aligned
static bool bad(const void *p) { return p == nullptr || !aligned16(p); }
// optional pointer: NULL or 16-byte aligned
static bool bad_opt(const void *p) { return p != nullptr && !aligned16(p); }

static smile_status from_hip(hipError_t e)
{
    if (e == hipSuccess) return SMILE_OK;
    (void)hipGetLastError();   // do not leave a sticky launch error behind for the caller's next call
    return SMILE_HIP_ERROR;
}

}  // namespace smile

using namespace smile;

extern "C" {

const char *smile_status_string(int32_t status)
{
    switch (status) {
    case SMILE_OK: return "ok";
    case SMILE_INVALID_ARG: return "invalid argument (NULL or misaligned pointer)";
    case SMILE_BAD_SHAPE: return "bad shape (size out of range or not divisible as required)";
    case SMILE_UNSUPPORTED: return "unsupported dtype, activation or shape";
    case SMILE_WORKSPACE: return "workspace too small or misaligned";
    case SMILE_HIP_ERROR: return "HIP runtime error";
    default: return "unknown status";
    }
}

const char *smile_version(void) { return "0.1.0"; }

int32_t smile_capacity(int32_t T, int32_t N, double capacity_factor)
{
    if (T < 1 || N < 1 || !(capacity_factor > 0.0) || !std::isfinite(capacity_factor)) return -1;
    double c = std::ceil(capacity_factor * (double)T / (double)N);
    if (c < 1.0) c = 1.0;
    if (c > 2147483647.0) return -1;
    return (int32_t)c;
}

smile_status smile_validate_desc(const smile_layer_desc *desc)
{
    if (!desc) return SMILE_INVALID_ARG;
    const smile_layer_desc &d = *desc;
    if (d.dtype != SMILE_DTYPE_F32 && d.dtype != SMILE_DTYPE_BF16 && d.dtype != SMILE_DTYPE_F16) return SMILE_UNSUPPORTED;
    if (d.act != SMILE_ACT_RELU && d.act != SMILE_ACT_GELU) return SMILE_UNSUPPORTED;
    if (d.T < 1 || d.d_model < 1 || d.d_ff < 1 || d.n_groups < 1 || d.m_local < 1 || d.capacity < 1)
        return SMILE_BAD_SHAPE;
    if (d.n_groups > 1024 || d.m_local > 1024) return SMILE_BAD_SHAPE;
    const int64_t N = (int64_t)d.n_groups * d.m_local;
    if (N > 4096) return SMILE_BAD_SHAPE;
    if (d.d_model % 8 || d.d_ff % 8) return SMILE_BAD_SHAPE;
    if (is_half(d.dtype) && (d.d_model % 64 || d.d_ff % 64)) return SMILE_BAD_SHAPE;
    if (N * d.capacity >= (int64_t)1 << 31) return SMILE_BAD_SHAPE;
    const int64_t widest = d.d_model > d.d_ff ? d.d_model : d.d_ff;
    if ((double)N * d.capacity * (double)widest >= 1099511627776.0) return SMILE_BAD_SHAPE;
    if (!std::isfinite(d.alpha) || !std::isfinite(d.beta)) return SMILE_BAD_SHAPE;
    if (d.group_capacity < 0 || (d.group_capacity > 0 && (d.T > (1 << 30) || d.capacity >= (1 << 30))))
        return SMILE_BAD_SHAPE;
    return SMILE_OK;
}

smile_status smile_workspace_bytes(const smile_layer_desc *desc, size_t *bytes)
{
    if (!bytes) return SMILE_INVALID_ARG;
    smile_status st = smile_validate_desc(desc);
    if (st != SMILE_OK) return st;
    *bytes = workspace_layout(*desc).total;
    return SMILE_OK;
}

// An integer tuning switch from the environment: its value when set to a number in [lo, hi], else -1.
static int env_switch(const char *name, int lo, int hi)
{
    const char *v = std::getenv(name);
    if (!v || !*v) return -1;
    char *end = nullptr;
    const long t = std::strtol(v, &end, 10);
    return (end && *end == '\0' && t >= lo && t <= hi) ? (int)t : -1;
}

// The tuning state of a new ctx: the SMILE_* switches as the environment holds them now, and the compute-unit
// count of the current device (256 when no device answers, e.g. in host-only tests).
static Tuning read_tuning()
{
    Tuning t;
    t.ffn_tile = env_switch("SMILE_FFN_TILE", 0, 6);
    t.tgemm_tile = env_switch("SMILE_TGEMM_TILE", 0, 3);
    t.persist = env_switch("SMILE_FFN_PERSIST", 0, 1);
    t.router_grad_mfma = env_switch("SMILE_ROUTER_GRAD_MFMA", 0, 1);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
        t.cus = cus;
    else
        (void)hipGetLastError();
    return t;
}

static smile_status make_ctx(const smile_layer_desc *desc, void *workspace, size_t bytes, bool owns, smile_ctx **out)
{
    smile_ctx *c = new (std::nothrow) smile_ctx;
    if (!c) return SMILE_HIP_ERROR;
    const Layout L = workspace_layout(*desc);
    char *b = static_cast<char *>(workspace);
    static_cast<smile_layer_desc &>(c->desc) = *desc;
    c->desc.tune = read_tuning();
    c->base = workspace;
    c->bytes = bytes;
    c->owns = owns;
    c->ws.block_expert_hist = reinterpret_cast<int32_t *>(b + L.off_block_expert_hist);
    c->ws.block_group_hist = reinterpret_cast<int32_t *>(b + L.off_block_group_hist);
    c->ws.block_p_sum = reinterpret_cast<float *>(b + L.off_block_p_sum);
    c->ws.block_q_sum = reinterpret_cast<float *>(b + L.off_block_q_sum);
    c->ws.rank_in_block = reinterpret_cast<int32_t *>(b + L.off_rank_in_block);
    c->ws.pos_in_block = reinterpret_cast<int32_t *>(b + L.off_pos_in_block);
    c->ws.slot_token = reinterpret_cast<int32_t *>(b + L.off_slot_token);
    c->ws.hidden = b + L.off_hidden;
    *out = c;
    return SMILE_OK;
}

smile_status smile_create(const smile_layer_desc *desc, smile_ctx **ctx)
{
    if (!ctx) return SMILE_INVALID_ARG;
    *ctx = nullptr;
    smile_status st = smile_validate_desc(desc);
    if (st != SMILE_OK) return st;
    const Layout L = workspace_layout(*desc);
    void *p = nullptr;
    if (hipMalloc(&p, L.total) != hipSuccess) { (void)hipGetLastError(); return SMILE_HIP_ERROR; }
    st = make_ctx(desc, p, L.total, true, ctx);
    if (st != SMILE_OK) (void)hipFree(p);
    return st;
}

smile_status smile_create_with_workspace(const smile_layer_desc *desc, void *workspace, size_t bytes, smile_ctx **ctx)
{
    if (!ctx) return SMILE_INVALID_ARG;
    *ctx = nullptr;
    smile_status st = smile_validate_desc(desc);
    if (st != SMILE_OK) return st;
    if (!workspace) return SMILE_INVALID_ARG;
    const Layout L = workspace_layout(*desc);
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || bytes < L.total) return SMILE_WORKSPACE;
    return make_ctx(desc, workspace, bytes, false, ctx);
}

smile_status smile_destroy(smile_ctx *ctx)
{
    if (!ctx) return SMILE_OK;
    smile_status st = SMILE_OK;
    if (ctx->owns && ctx->base && hipFree(ctx->base) != hipSuccess) { (void)hipGetLastError(); st = SMILE_HIP_ERROR; }
    delete ctx;
    return st;
}

smile_status smile_kernel_timing(smile_ctx *ctx, void **events, int32_t pairs)
{
    if (!ctx || pairs < 0 || (pairs > 0 && !events)) return SMILE_INVALID_ARG;
    if (pairs > kMaxTimedKernels) pairs = kMaxTimedKernels;
    for (int32_t i = 0; i < 2 * pairs; ++i)
        if (!events[i]) return SMILE_INVALID_ARG;
    ctx->timer.events = pairs ? reinterpret_cast<hipEvent_t *>(events) : nullptr;
    ctx->timer.pairs = pairs;
    ctx->timer.used = 0;
    return SMILE_OK;
}

int32_t smile_kernel_timing_count(const smile_ctx *ctx) { return ctx ? ctx->timer.used : 0; }

const char *smile_kernel_timing_name(const smile_ctx *ctx, int32_t i)
{
    return (ctx && i >= 0 && i < ctx->timer.used && ctx->timer.names[i]) ? ctx->timer.names[i] : "";
}

smile_status smile_gate_logits(smile_ctx *ctx, const void *x, const void *w_inter, const void *w_intra,
                               float *logits_inter, float *logits_intra, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(x) || bad(w_inter) || bad(w_intra) || bad(logits_inter) || bad(logits_intra))
        return SMILE_INVALID_ARG;
    return from_hip(launch_gate_logits(ctx->desc, x, w_inter, w_intra, logits_inter, logits_intra,
                                       static_cast<hipStream_t>(stream)));
}

smile_status smile_route_bilevel(smile_ctx *ctx, const float *logits_inter, const float *logits_intra,
                                 const float *bias_inter, const float *bias_intra,
                                 int32_t *group_idx, int32_t *local_idx, int32_t *pos_in_group, int32_t *slot,
                                 float *gate, float *p_top, float *q_top,
                                 int32_t *group_count, int32_t *local_count, int32_t *expert_count,
                                 int32_t *kept_count, float *p_sum, float *q_sum, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(logits_inter) || bad(logits_intra) || bad_opt(bias_inter) || bad_opt(bias_intra) ||
        bad(group_idx) || bad(local_idx) || bad(pos_in_group) || bad(slot) || bad(gate) || bad(p_top) ||
        bad(q_top) || bad(group_count) || bad(local_count) || bad(expert_count) || bad(kept_count) ||
        bad(p_sum) || bad(q_sum))
        return SMILE_INVALID_ARG;
    return from_hip(launch_route(ctx->desc, ctx->ws, logits_inter, logits_intra, bias_inter, bias_intra,
                                 group_idx, local_idx, pos_in_group, slot, gate, p_top, q_top, group_count,
                                 local_count, expert_count, kept_count, p_sum, q_sum,
                                 static_cast<hipStream_t>(stream)));
}

smile_status smile_dispatch(smile_ctx *ctx, const void *x, const int32_t *group_idx, const int32_t *local_idx,
                            const int32_t *slot, void *xe, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(x) || bad(group_idx) || bad(local_idx) || bad(slot) || bad(xe)) return SMILE_INVALID_ARG;
    return from_hip(launch_dispatch(ctx->desc, x, group_idx, local_idx, slot, xe, static_cast<hipStream_t>(stream)));
}

smile_status smile_dispatch_hop1(smile_ctx *ctx, const void *x, const int32_t *group_idx,
                                 const int32_t *pos_in_group, int32_t group_rows, void *xg, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(x) || bad(group_idx) || bad(pos_in_group) || bad(xg)) return SMILE_INVALID_ARG;
    if (group_rows < 1 || (int64_t)group_rows * ctx->desc.n_groups >= (int64_t)1 << 31) return SMILE_BAD_SHAPE;
    return from_hip(launch_dispatch_hop1(ctx->desc, x, group_idx, pos_in_group, group_rows, xg,
                                         static_cast<hipStream_t>(stream)));
}

smile_status smile_dispatch_hop2(smile_ctx *ctx, const void *xg, const int32_t *group_idx,
                                 const int32_t *local_idx, const int32_t *pos_in_group, const int32_t *slot,
                                 int32_t group_rows, void *xe, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(xg) || bad(group_idx) || bad(local_idx) || bad(pos_in_group) || bad(slot) || bad(xe))
        return SMILE_INVALID_ARG;
    if (group_rows < 1 || (int64_t)group_rows * ctx->desc.n_groups >= (int64_t)1 << 31) return SMILE_BAD_SHAPE;
    return from_hip(launch_dispatch_hop2(ctx->desc, xg, group_idx, local_idx, pos_in_group, slot, group_rows, xe,
                                         static_cast<hipStream_t>(stream)));
}

smile_status smile_expert_ffn_up(smile_ctx *ctx, const void *xe, const int32_t *kept_count,
                                 const void *w1, const void *b1, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(xe) || bad(kept_count) || bad(w1) || bad_opt(b1)) return SMILE_INVALID_ARG;
    return from_hip(launch_expert_ffn_up(ctx->desc, ctx->ws, xe, kept_count, w1, b1, static_cast<hipStream_t>(stream)));
}

smile_status smile_expert_ffn_up_timed(smile_ctx *ctx, const void *xe, const int32_t *kept_count,
                                       const void *w1, const void *b1, void *start_event, void *stop_event,
                                       void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(xe) || bad(kept_count) || bad(w1) || bad_opt(b1) || !start_event || !stop_event)
        return SMILE_INVALID_ARG;
    return from_hip(launch_expert_ffn_up(ctx->desc, ctx->ws, xe, kept_count, w1, b1, static_cast<hipStream_t>(stream),
                                         static_cast<hipEvent_t>(start_event), static_cast<hipEvent_t>(stop_event)));
}

smile_status smile_expert_ffn_down(smile_ctx *ctx, const int32_t *kept_count, const void *w2, const void *b2,
                                   void *ye, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(kept_count) || bad(w2) || bad_opt(b2) || bad(ye)) return SMILE_INVALID_ARG;
    return from_hip(launch_expert_ffn_down(ctx->desc, ctx->ws, kept_count, w2, b2, ye, static_cast<hipStream_t>(stream)));
}

smile_status smile_expert_ffn(smile_ctx *ctx, const void *xe, const int32_t *kept_count,
                              const void *w1, const void *b1, const void *w2, const void *b2,
                              void *ye, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(xe) || bad(kept_count) || bad(w1) || bad_opt(b1) || bad(w2) || bad_opt(b2) || bad(ye))
        return SMILE_INVALID_ARG;
    smile_status st = smile_expert_ffn_up(ctx, xe, kept_count, w1, b1, stream);
    if (st != SMILE_OK) return st;
    return smile_expert_ffn_down(ctx, kept_count, w2, b2, ye, stream);
}

smile_status smile_combine(smile_ctx *ctx, const void *ye, const int32_t *group_idx, const int32_t *local_idx,
                           const int32_t *slot, const float *gate, void *y, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(ye) || bad(group_idx) || bad(local_idx) || bad(slot) || bad(gate) || bad(y))
        return SMILE_INVALID_ARG;
    return from_hip(launch_combine(ctx->desc, ye, group_idx, local_idx, slot, gate, y,
                                   static_cast<hipStream_t>(stream)));
}

smile_status smile_aux_loss(smile_ctx *ctx, const int32_t *group_count, const int32_t *local_count,
                            const float *p_sum, const float *q_sum, float *out3, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(group_count) || bad(local_count) || bad(p_sum) || bad(q_sum) || bad(out3))
        return SMILE_INVALID_ARG;
    return from_hip(launch_aux_loss(ctx->desc, group_count, local_count, p_sum, q_sum, out3,
                                    static_cast<hipStream_t>(stream)));
}

smile_status smile_layer_forward(smile_ctx *ctx, const smile_layer_io *io, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || !io) return SMILE_INVALID_ARG;
    // check every pointer first so that a bad argument of a late step leaves nothing enqueued
    if (bad(io->x) || bad(io->w_inter) || bad(io->w_intra) || bad(io->w1) || bad_opt(io->b1) || bad(io->w2) ||
        bad_opt(io->b2) || bad_opt(io->bias_inter) || bad_opt(io->bias_intra) || bad(io->logits_inter) ||
        bad(io->logits_intra) || bad(io->group_idx) || bad(io->local_idx) || bad(io->pos_in_group) ||
        bad(io->slot) || bad(io->gate) || bad(io->p_top) || bad(io->q_top) || bad(io->group_count) ||
        bad(io->local_count) || bad(io->expert_count) || bad(io->kept_count) || bad(io->p_sum) ||
        bad(io->q_sum) || bad_opt(io->xe) || bad_opt(io->ye) || bad(io->y) || bad(io->loss3))
        return SMILE_INVALID_ARG;
    if ((io->xe == nullptr) != (io->ye == nullptr)) return SMILE_INVALID_ARG;
    if ((io->prof_up_start == nullptr) != (io->prof_up_stop == nullptr)) return SMILE_INVALID_ARG;
    if (bad_opt(io->h_save) || bad_opt(io->pre_save) || (io->h_save == nullptr) != (io->pre_save == nullptr))
        return SMILE_INVALID_ARG;
    // Same kernels as the step-by-step calls with fewer launches.  With expert buffers (xe, ye given):
    // the last routing step and the loss run inside the dispatch kernel, and the down-projection also
    // returns the gate-weighted rows to y (no combine launch).  Without them (both NULL):
    // nothing is materialised -- a per-token kernel finishes the routing, builds the slot -> token map
    // and zeroes the rows of dropped tokens; the up GEMM gathers its rows from x through that map and
    // the down GEMM returns gate-weighted rows straight to y.
    const LayerDesc &d = ctx->desc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool fused = io->xe == nullptr;
    const LossArgs loss{io->group_count, io->local_count, io->p_sum, io->q_sum, io->loss3};
    // small batches: the fused path's last routing kernel scans the few per-block histograms itself
    const int route_blocks = (d.T + kRouteBlock - 1) / kRouteBlock;
    const bool scan_in_finalize = fused && d.group_capacity == 0 && route_blocks <= kScanInFinalizeBlocks;
    hipError_t err = launch_gate_logits(d, io->x, io->w_inter, io->w_intra, io->logits_inter, io->logits_intra, s);
    if (err == hipSuccess)
        err = launch_route(d, ctx->ws, io->logits_inter, io->logits_intra, io->bias_inter, io->bias_intra,
                           io->group_idx, io->local_idx, io->pos_in_group, io->slot, io->gate, io->p_top, io->q_top,
                           io->group_count, io->local_count, io->expert_count, io->kept_count, io->p_sum, io->q_sum,
                           s, /*finalize=*/false, /*scan=*/!scan_in_finalize);
    if (fused) {
        if (err == hipSuccess && scan_in_finalize)
            err = launch_finalize_map_scan(d, ctx->ws, io->group_idx, io->local_idx, io->pos_in_group, io->slot, io->y,
                                           io->group_count, io->local_count, io->expert_count, io->kept_count,
                                           io->p_sum, io->q_sum, io->loss3, s);
        else if (err == hipSuccess)
            err = launch_finalize_map(d, ctx->ws, io->group_idx, io->local_idx, io->pos_in_group, io->slot, io->y,
                                      loss, s);
        if (err == hipSuccess)
            err = launch_expert_ffn_up(d, ctx->ws, nullptr, io->kept_count, io->w1, io->b1, s,
                                       static_cast<hipEvent_t>(io->prof_up_start),
                                       static_cast<hipEvent_t>(io->prof_up_stop), io->x, io->h_save, io->pre_save);
        if (err == hipSuccess)
            err = launch_expert_ffn_down(d, ctx->ws, io->kept_count, io->w2, io->b2, nullptr, s, io->y, io->gate,
                                         io->h_save);
        return from_hip(err);
    }
    if (err == hipSuccess)
        err = launch_dispatch_finalize(d, ctx->ws, io->x, io->group_idx, io->local_idx, io->pos_in_group, io->slot,
                                       io->xe, io->y, loss, s);
    if (err == hipSuccess)
        err = launch_expert_ffn_up(d, ctx->ws, io->xe, io->kept_count, io->w1, io->b1, s,
                                   static_cast<hipEvent_t>(io->prof_up_start), static_cast<hipEvent_t>(io->prof_up_stop),
                                   nullptr, io->h_save, io->pre_save);
    // the down-projection writes ye and, through the slot -> token map, the gate-weighted rows of y
    if (err == hipSuccess)
        err = launch_expert_ffn_down(d, ctx->ws, io->kept_count, io->w2, io->b2, io->ye, s, io->y, io->gate,
                                     io->h_save);
    return from_hip(err);
}

smile_status smile_backward_workspace_bytes(const smile_layer_desc *desc, size_t *bytes)
{
    if (!bytes) return SMILE_INVALID_ARG;
    smile_status st = smile_validate_desc(desc);
    if (st != SMILE_OK) return st;
    *bytes = backward_workspace_layout(*desc).total;
    return SMILE_OK;
}

static smile_status check_backward_workspace(const smile_ctx *ctx, const void *workspace, size_t bytes)
{
    if (!workspace) return SMILE_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || bytes < backward_workspace_layout(ctx->desc).total)
        return SMILE_WORKSPACE;
    return SMILE_OK;
}

smile_status smile_combine_backward(smile_ctx *ctx, const void *dy, const void *ye, const int32_t *group_idx,
                                    const int32_t *local_idx, const int32_t *slot, const float *gate,
                                    void *dye, float *dgate, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(dy) || bad(ye) || bad(group_idx) || bad(local_idx) || bad(slot) || bad(gate) || bad(dye) ||
        bad(dgate))
        return SMILE_INVALID_ARG;
    return from_hip(launch_combine_backward(ctx->desc, dy, ye, group_idx, local_idx, slot, gate, dye, dgate,
                                            static_cast<hipStream_t>(stream)));
}

smile_status smile_route_backward(smile_ctx *ctx, const float *logits_inter, const float *logits_intra,
                                  const float *bias_inter, const float *bias_intra,
                                  const int32_t *group_idx, const int32_t *local_idx, const float *dgate,
                                  const int32_t *group_count, const int32_t *local_count, float dloss,
                                  float *dlp, float *dlq, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(logits_inter) || bad(logits_intra) || bad_opt(bias_inter) || bad_opt(bias_intra) ||
        bad(group_idx) || bad(local_idx) || bad(dgate) || bad(group_count) || bad(local_count) || bad(dlp) || bad(dlq))
        return SMILE_INVALID_ARG;
    if (!std::isfinite(dloss)) return SMILE_BAD_SHAPE;
    return from_hip(launch_route_backward(ctx->desc, logits_inter, logits_intra, bias_inter, bias_intra, group_idx,
                                          local_idx, dgate, group_count, local_count, dloss, dlp, dlq,
                                          static_cast<hipStream_t>(stream)));
}

smile_status smile_expert_ffn_backward(smile_ctx *ctx, const void *xe, const int32_t *kept_count,
                                       const void *w1, const void *w2, const void *dye,
                                       const void *h, const void *pre,
                                       void *dxe, void *dw1, void *dw2,
                                       void *workspace, size_t workspace_bytes, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(xe) || bad(kept_count) || bad(w1) || bad(w2) || bad(dye) || bad(dxe) || bad(dw1) || bad(dw2) ||
        bad_opt(h) || bad_opt(pre) || (h == nullptr) != (pre == nullptr))
        return SMILE_INVALID_ARG;
    const smile_status st = check_backward_workspace(ctx, workspace, workspace_bytes);
    if (st != SMILE_OK) return st;
    return from_hip(launch_expert_ffn_backward(ctx->desc, workspace, xe, kept_count, w1, w2, dye, h, pre, dxe, dw1,
                                               dw2, static_cast<hipStream_t>(stream)));
}

smile_status smile_dispatch_backward(smile_ctx *ctx, const void *dxe, const int32_t *group_idx,
                                     const int32_t *local_idx, const int32_t *slot, const float *dlp,
                                     const float *dlq, const void *w_inter, const void *w_intra, void *dx,
                                     void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(dxe) || bad(group_idx) || bad(local_idx) || bad(slot) || bad(dlp) || bad(dlq) || bad(w_inter) ||
        bad(w_intra) || bad(dx))
        return SMILE_INVALID_ARG;
    return from_hip(launch_dispatch_backward(ctx->desc, dxe, group_idx, local_idx, slot, dlp, dlq, w_inter, w_intra,
                                             dx, static_cast<hipStream_t>(stream)));
}

smile_status smile_gate_weights_backward(smile_ctx *ctx, const void *x, const float *dlp, const float *dlq,
                                         float *dw_inter, float *dw_intra,
                                         void *workspace, size_t workspace_bytes, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || bad(x) || bad(dlp) || bad(dlq) || bad(dw_inter) || bad(dw_intra)) return SMILE_INVALID_ARG;
    const smile_status st = check_backward_workspace(ctx, workspace, workspace_bytes);
    if (st != SMILE_OK) return st;
    return from_hip(launch_gate_weights_backward(ctx->desc, workspace, x, dlp, dlq, dw_inter, dw_intra,
                                                 static_cast<hipStream_t>(stream)));
}

smile_status smile_layer_backward(smile_ctx *ctx, const smile_backward_io *io, float dloss,
                                  void *workspace, size_t workspace_bytes, void *stream)
{
    TimerScope timing(ctx);
    if (!ctx || !io) return SMILE_INVALID_ARG;
    if (bad(io->x) || bad(io->w_inter) || bad(io->w_intra) || bad(io->w1) || bad(io->w2) || bad_opt(io->bias_inter) ||
        bad_opt(io->bias_intra) || bad(io->logits_inter) || bad(io->logits_intra) || bad(io->group_idx) ||
        bad(io->local_idx) || bad(io->slot) || bad(io->gate) || bad(io->group_count) || bad(io->local_count) ||
        bad(io->kept_count) || bad(io->xe) || bad(io->ye) || bad(io->dy) || bad(io->dye) || bad(io->dgate) ||
        bad(io->dlp) || bad(io->dlq) || bad(io->dxe) || bad(io->dx) || bad(io->dw_inter) || bad(io->dw_intra) ||
        bad(io->dw1) || bad(io->dw2) || bad_opt(io->h) || bad_opt(io->pre) || (io->h == nullptr) != (io->pre == nullptr))
        return SMILE_INVALID_ARG;
    if (!std::isfinite(dloss)) return SMILE_BAD_SHAPE;
    const smile_status st = check_backward_workspace(ctx, workspace, workspace_bytes);
    if (st != SMILE_OK) return st;
    const LayerDesc &d = ctx->desc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t err = launch_combine_backward(d, io->dy, io->ye, io->group_idx, io->local_idx, io->slot, io->gate,
                                             io->dye, io->dgate, s);
    if (err == hipSuccess)
        err = launch_route_backward(d, io->logits_inter, io->logits_intra, io->bias_inter, io->bias_intra,
                                    io->group_idx, io->local_idx, io->dgate, io->group_count, io->local_count, dloss,
                                    io->dlp, io->dlq, s);
    if (err == hipSuccess)
        err = launch_expert_ffn_backward(d, workspace, io->xe, io->kept_count, io->w1, io->w2, io->dye, io->h, io->pre,
                                         io->dxe, io->dw1, io->dw2, s);
    if (err == hipSuccess)
        err = launch_dispatch_backward(d, io->dxe, io->group_idx, io->local_idx, io->slot, io->dlp, io->dlq,
                                       io->w_inter, io->w_intra, io->dx, s);
    if (err == hipSuccess)
        err = launch_gate_weights_backward(d, workspace, io->x, io->dlp, io->dlq, io->dw_inter, io->dw_intra, s);
    return from_hip(err);
}

}  // extern "C"
