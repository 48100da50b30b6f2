// Dispatch and combine: the token <-> expert-buffer row permutation (Section 3.2.1; on one GPU the
// paper's inter- and intra-node hops are composed into a single row move) and the gate-weighted
// return (Eq. 3).  Both are pure HBM streaming: a row is d*elem bytes (1.5-2 KiB for the bf16
// configurations), moved as 16-byte pieces; 8-32 consecutive lanes own a row, so every access is a
// run of full cache lines, the routing indices are read once per row, and up to kPieces loads are
// in flight per lane.
#include "smile_internal.hpp"

namespace smile {

namespace {

constexpr int kThreads = 256;
constexpr int kPieces = 4;

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

// Row mapping shared by the kernels below: LPR consecutive lanes own one token row and walk its ppr
// 16-byte pieces LPR at a time (so every access of those lanes is one contiguous run), kThreads / LPR
// rows per workgroup.  The routing indices are read once per row, not once per piece.
template <int LPR>
struct RowLanes {
    static constexpr int kRowsPerBlock = kThreads / LPR;
    int t, sub;
    __device__ __forceinline__ RowLanes() : t(blockIdx.x * kRowsPerBlock + threadIdx.x / LPR), sub(threadIdx.x % LPR) {}
};

// Copy (or gate-scale) one row, up to kPieces loads in flight per lane.  F maps a loaded piece to the stored one.
template <int LPR, typename F>
__device__ __forceinline__ void move_row(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int ppr, int sub, F f)
{
    for (int c0 = sub; c0 < ppr; c0 += LPR * kPieces) {
        u32x4 v[kPieces];
#pragma unroll
        for (int i = 0; i < kPieces; ++i)
            if (c0 + i * LPR < ppr) v[i] = src[c0 + i * LPR];
#pragma unroll
        for (int i = 0; i < kPieces; ++i)
            if (c0 + i * LPR < ppr) dst[c0 + i * LPR] = f(v[i]);
    }
}

// xe[(g*m+l)*C + slot] <- x[t] for kept tokens.  ppr = 16-byte pieces per row.
template <int LPR>
__global__ __launch_bounds__(kThreads) void dispatch_kernel(
    const u32x4 *__restrict__ x, const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx,
    const int32_t *__restrict__ slot, u32x4 *__restrict__ xe, int T, int ppr, int m, int C)
{
    const RowLanes<LPR> rl;
    if (rl.t >= T) return;
    const int sl = slot[rl.t];
    if (sl < 0) return;
    const size_t row = (size_t)(group_idx[rl.t] * m + local_idx[rl.t]) * C + sl;
    move_row<LPR>(x + (size_t)rl.t * ppr, xe + row * ppr, ppr, rl.sub, [](u32x4 v) { return v; });
}

// First hop alone: xg[g*rows + pos_in_group] <- x[t] while the group's buffer has a row for it.
template <int LPR>
__global__ __launch_bounds__(kThreads) void dispatch_hop1_kernel(
    const u32x4 *__restrict__ x, const int32_t *__restrict__ group_idx, const int32_t *__restrict__ pos_in_group,
    u32x4 *__restrict__ xg, int T, int ppr, int rows)
{
    const RowLanes<LPR> rl;
    if (rl.t >= T) return;
    const int pos = pos_in_group[rl.t];
    if (pos < 0 || pos >= rows) return;
    const size_t row = (size_t)group_idx[rl.t] * rows + pos;
    move_row<LPR>(x + (size_t)rl.t * ppr, xg + row * ppr, ppr, rl.sub, [](u32x4 v) { return v; });
}

// Second hop alone: xe[(g*m+l)*C + slot] <- xg[g*rows + pos_in_group] for kept tokens.
template <int LPR>
__global__ __launch_bounds__(kThreads) void dispatch_hop2_kernel(
    const u32x4 *__restrict__ xg, const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx,
    const int32_t *__restrict__ pos_in_group, const int32_t *__restrict__ slot, u32x4 *__restrict__ xe,
    int T, int ppr, int m, int C, int rows)
{
    const RowLanes<LPR> rl;
    if (rl.t >= T) return;
    const int sl = slot[rl.t], pos = pos_in_group[rl.t];
    if (sl < 0 || sl >= C || pos < 0 || pos >= rows) return;
    const int g = group_idx[rl.t];
    const size_t src = (size_t)g * rows + pos, dst = (size_t)(g * m + local_idx[rl.t]) * C + sl;
    move_row<LPR>(xg + src * ppr, xe + dst * ppr, ppr, rl.sub, [](u32x4 v) { return v; });
}

// Dispatch fused with the last routing step (the chained forward pass): every thread derives the
// token's final slot from the workspace (block offset of its expert + rank inside the block,
// dropped at or beyond C); the thread moving piece 0 of a token also writes slot / pos_in_group and
// the slot -> token map; the output rows of dropped tokens are zeroed here (the down-projection
// returns the gate-weighted rows of the kept ones, so no combine kernel follows).
template <int LPR>
__global__ __launch_bounds__(kThreads) void dispatch_finalize_kernel(
    const u32x4 *__restrict__ x, const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx,
    const int32_t *__restrict__ block_expert_off, const int32_t *__restrict__ block_group_off,
    const int32_t *__restrict__ rank_in_block, const int32_t *__restrict__ pos_in_block,
    int32_t *__restrict__ pos_in_group, int32_t *__restrict__ slot, u32x4 *__restrict__ xe,
    int32_t *__restrict__ slot_token, u32x4 *__restrict__ y,
    int T, int ppr, int n, int m, int C, LossArgs loss, float alpha, float beta)
{
    // Eq. 4 from the (complete) routing statistics, by the first wave of the last workgroup
    if (loss.out3 && blockIdx.x == gridDim.x - 1 && threadIdx.x < 64)
        aux_loss_wave(loss.group_count, loss.local_count, loss.p_sum, loss.q_sum, T, n, m, alpha, beta, loss.out3);
    const RowLanes<LPR> rl;
    if (rl.t >= T) return;
    const int t = rl.t, b = t / kRouteBlock;
    const int g = group_idx[t], e = g * m + local_idx[t];
    const int rank = block_expert_off[(size_t)b * n * m + e] + rank_in_block[t];
    const int sl = rank < C ? rank : -1;
    if (rl.sub == 0) {
        slot[t] = sl;
        pos_in_group[t] = block_group_off[(size_t)b * n + g] + pos_in_block[t];
        if (sl >= 0) slot_token[(size_t)e * C + sl] = t;   // for the down-projection's gate-weighted return
    }
    if (sl < 0) {   // a dropped token's output row is zero (Eq. 3 gives it no expert output)
        u32x4 *row = y + (size_t)t * ppr;
        for (int c = rl.sub; c < ppr; c += LPR) row[c] = u32x4{0u, 0u, 0u, 0u};
        return;
    }
    move_row<LPR>(x + (size_t)t * ppr, xe + ((size_t)e * C + sl) * ppr, ppr, rl.sub, [](u32x4 v) { return v; });
}

// Last routing step of the fully fused forward pass (no xe / ye buffers): one thread per token, one
// workgroup per routing block.  Final slot and stage-1 position as in the routing finalize kernel;
// kept tokens enter the slot -> token map that the expert GEMMs gather and scatter through; the
// output rows of dropped tokens are zeroed here, a wave at a time (Eq. 3 gives them no expert output).
__global__ __launch_bounds__(kRouteBlock) void finalize_map_kernel(
    const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx,
    const int32_t *__restrict__ block_expert_off, const int32_t *__restrict__ block_group_off,
    const int32_t *__restrict__ rank_in_block, const int32_t *__restrict__ pos_in_block,
    int32_t *__restrict__ pos_in_group, int32_t *__restrict__ slot, int32_t *__restrict__ slot_token,
    u32x4 *__restrict__ y, int T, int ppr, int n, int m, int C, LossArgs loss, float alpha, float beta)
{
    if (loss.out3 && blockIdx.x == gridDim.x - 1 && threadIdx.x < 64)
        aux_loss_wave(loss.group_count, loss.local_count, loss.p_sum, loss.q_sum, T, n, m, alpha, beta, loss.out3);
    const int b = blockIdx.x;
    const int t = b * kRouteBlock + threadIdx.x;
    const bool valid = t < T;
    bool dropped = false;
    if (valid) {
        const int g = group_idx[t], e = g * m + local_idx[t];
        const int rank = block_expert_off[(size_t)b * n * m + e] + rank_in_block[t];
        const int sl = rank < C ? rank : -1;
        slot[t] = sl;
        pos_in_group[t] = block_group_off[(size_t)b * n + g] + pos_in_block[t];
        if (sl >= 0) slot_token[(size_t)e * C + sl] = t;
        dropped = sl < 0;
    }
    unsigned long long mask = __ballot(dropped);
    const int lane = threadIdx.x & 63, t0 = t - lane;
    while (mask) {
        const int src = __ffsll((long long)mask) - 1;
        u32x4 *row = y + (size_t)(t0 + src) * ppr;
        for (int p = lane; p < ppr; p += 64) row[p] = u32x4{0u, 0u, 0u, 0u};
        mask &= mask - 1;
    }
}

// DT: storage type of the piece (SMILE_DTYPE_*)
// finalize_map for small batches (at most 64 routing blocks), with the scan of the per-block histograms
// folded in (no scan kernel ran).  One wave per histogram column, one lane per earlier block: block b gets its
// exclusive offsets as a masked wave sum.  The totals are spread over two otherwise idle ends of the grid: the
// last block writes the expert counts (its offsets + its own row), block 0 the group / local counts, the
// probability sums (same summation order as the scan kernel: identical bits) and the loss.
// Dynamic LDS: [N + n] offsets, then [n] + [m] counts and [n] + [m] sums.
__global__ __launch_bounds__(kRouteBlock) void finalize_map_scan_kernel(
    const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx,
    const int32_t *__restrict__ block_expert_hist, const int32_t *__restrict__ block_group_hist,
    const float *__restrict__ block_p_sum, const float *__restrict__ block_q_sum,
    const int32_t *__restrict__ rank_in_block, const int32_t *__restrict__ pos_in_block,
    int32_t *__restrict__ pos_in_group, int32_t *__restrict__ slot, int32_t *__restrict__ slot_token,
    u32x4 *__restrict__ y, int T, int ppr, int n, int m, int C,
    int32_t *__restrict__ group_count, int32_t *__restrict__ local_count, int32_t *__restrict__ expert_count,
    int32_t *__restrict__ kept_count, float *__restrict__ p_sum, float *__restrict__ q_sum,
    float *__restrict__ loss3, float alpha, float beta)
{
    extern __shared__ int32_t lds_i[];
    const int N = n * m, B = gridDim.x, b = blockIdx.x, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    constexpr int kWaves = kRouteBlock / 64;
    int32_t *eoff = lds_i, *goff = lds_i + N;
    // lane = earlier block (B <= 64); two columns per iteration so that their loads overlap
    for (int c = wave; c < N + n; c += 2 * kWaves) {
        const int c2 = c + kWaves;
        int v0 = 0, v1 = 0;
        if (lane < b) {
            v0 = c < N ? block_expert_hist[(size_t)lane * N + c] : block_group_hist[(size_t)lane * n + (c - N)];
            if (c2 < N + n)
                v1 = c2 < N ? block_expert_hist[(size_t)lane * N + c2] : block_group_hist[(size_t)lane * n + (c2 - N)];
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            v0 += __shfl_xor(v0, off, 64);
            v1 += __shfl_xor(v1, off, 64);
        }
        if (lane == 0) {
            lds_i[c] = v0;
            if (c2 < N + n) lds_i[c2] = v1;
        }
    }
    __syncthreads();

    const int t = b * kRouteBlock + tid;
    bool dropped = false;
    if (t < T) {
        const int g = group_idx[t], e = g * m + local_idx[t];
        const int rank = eoff[e] + rank_in_block[t];
        const int sl = rank < C ? rank : -1;
        slot[t] = sl;
        pos_in_group[t] = goff[g] + pos_in_block[t];
        if (sl >= 0) slot_token[(size_t)e * C + sl] = t;
        dropped = sl < 0;
    }
    unsigned long long mask = __ballot(dropped);
    const int t0 = t - lane;
    while (mask) {
        const int src = __ffsll((long long)mask) - 1;
        u32x4 *row = y + (size_t)(t0 + src) * ppr;
        for (int p = lane; p < ppr; p += 64) row[p] = u32x4{0u, 0u, 0u, 0u};
        mask &= mask - 1;
    }

    if (b == B - 1) {   // expert totals = offsets of the last block + its own histogram row
        for (int e = tid; e < N; e += kRouteBlock) {
            const int total = eoff[e] + block_expert_hist[(size_t)b * N + e];
            expert_count[e] = total;
            kept_count[e] = min(total, C);
        }
    }
    if (b != 0) return;

    // ---- block 0: one wave per column of [n group counts | m local counts | n p sums | m q sums], then the loss
    int32_t *cnt_g = lds_i + N + n, *cnt_l = cnt_g + n;
    float *sum_p = reinterpret_cast<float *>(cnt_l + m), *sum_q = sum_p + n;
    for (int c = wave; c < 2 * (n + m); c += kWaves) {
        if (c < n + m) {
            const int32_t *col = c < n ? block_group_hist + c : block_group_hist + (size_t)B * n + (c - n);
            const int stride = c < n ? n : m;
            int sum = lane < B ? col[(size_t)lane * stride] : 0;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
            if (lane == 0) {
                if (c < n) { cnt_g[c] = sum; group_count[c] = sum; }
                else { cnt_l[c - n] = sum; local_count[c - n] = sum; }
            }
        } else if (c < 2 * n + m) {
            const float v = wave_sum_column(block_p_sum, B, n, c - n - m);
            if (lane == 0) { sum_p[c - n - m] = v; p_sum[c - n - m] = v; }
        } else {
            const float v = wave_sum_column(block_q_sum, B, m, c - 2 * n - m);
            if (lane == 0) { sum_q[c - 2 * n - m] = v; q_sum[c - 2 * n - m] = v; }
        }
    }
    __syncthreads();
    if (loss3 && tid < 64) aux_loss_wave(cnt_g, cnt_l, sum_p, sum_q, T, n, m, alpha, beta, loss3);
}

template <int DT>
__device__ __forceinline__ u32x4 scale_piece(u32x4 v, float gt)
{
    u32x4 r;
    if constexpr (DT == SMILE_DTYPE_BF16) {
#pragma unroll
        for (int k = 0; k < 4; ++k) r[k] = Half<__bf16>::pack(Half<__bf16>::lo(v[k]) * gt, Half<__bf16>::hi(v[k]) * gt);
    } else if constexpr (DT == SMILE_DTYPE_F16) {
#pragma unroll
        for (int k = 0; k < 4; ++k) r[k] = Half<_Float16>::pack(Half<_Float16>::lo(v[k]) * gt, Half<_Float16>::hi(v[k]) * gt);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) r[k] = __float_as_uint(__uint_as_float(v[k]) * gt);
    }
    return r;
}

// y[t] <- gate[t] * ye[(g*m+l)*C + slot] for kept tokens, 0 for dropped ones.
template <int DT, int LPR>
__global__ __launch_bounds__(kThreads) void combine_kernel(
    const u32x4 *__restrict__ ye, const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx,
    const int32_t *__restrict__ slot, const float *__restrict__ gate, u32x4 *__restrict__ y,
    int T, int ppr, int m, int C)
{
    const RowLanes<LPR> rl;
    if (rl.t >= T) return;
    const int sl = slot[rl.t];
    u32x4 *dst = y + (size_t)rl.t * ppr;
    if (sl < 0) {
        for (int c = rl.sub; c < ppr; c += LPR) dst[c] = u32x4{0u, 0u, 0u, 0u};
        return;
    }
    const float gt = gate[rl.t];
    const size_t row = (size_t)(group_idx[rl.t] * m + local_idx[rl.t]) * C + sl;
    move_row<LPR>(ye + row * ppr, dst, ppr, rl.sub, [gt](u32x4 v) { return scale_piece<DT>(v, gt); });
}

// lanes per row: the largest power of two <= min(ppr, 64), at least 8 (ppr >= 8 for every accepted shape... d >= 64 bf16, d >= 32 fp32)
int lanes_per_row(int ppr)
{
    int l = 8;
    while (l * 2 <= ppr && l < 32) l *= 2;
    return l;
}

}  // namespace

#define SMILE_LPR_SWITCH(lpr, CALL)          \
    switch (lpr) {                           \
    case 8: { constexpr int L = 8; CALL; } break;   \
    case 16: { constexpr int L = 16; CALL; } break; \
    default: { constexpr int L = 32; CALL; } break; \
    }

hipError_t launch_dispatch(const smile_layer_desc &d, const void *x, const int32_t *group_idx,
                           const int32_t *local_idx, const int32_t *slot, void *xe, hipStream_t s)
{
    const int ppr = d.d_model * elem_size(d.dtype) / 16;
    const int lpr = lanes_per_row(ppr);
    const dim3 grid((d.T + kThreads / lpr - 1) / (kThreads / lpr)), block(kThreads);
    SMILE_LPR_SWITCH(lpr, SMILE_LAUNCH(dispatch_kernel<L>, grid, block, 0, s, static_cast<const u32x4 *>(x),
                                             group_idx, local_idx, slot, static_cast<u32x4 *>(xe), d.T, ppr, d.m_local,
                                             d.capacity));
    return hipGetLastError();
}

hipError_t launch_dispatch_hop1(const smile_layer_desc &d, const void *x, const int32_t *group_idx,
                                const int32_t *pos_in_group, int group_rows, void *xg, hipStream_t s)
{
    const int ppr = d.d_model * elem_size(d.dtype) / 16;
    const int lpr = lanes_per_row(ppr);
    const dim3 grid((d.T + kThreads / lpr - 1) / (kThreads / lpr)), block(kThreads);
    SMILE_LPR_SWITCH(lpr, SMILE_LAUNCH(dispatch_hop1_kernel<L>, grid, block, 0, s, static_cast<const u32x4 *>(x),
                                             group_idx, pos_in_group, static_cast<u32x4 *>(xg), d.T, ppr, group_rows));
    return hipGetLastError();
}

hipError_t launch_dispatch_hop2(const smile_layer_desc &d, const void *xg, const int32_t *group_idx,
                                const int32_t *local_idx, const int32_t *pos_in_group, const int32_t *slot,
                                int group_rows, void *xe, hipStream_t s)
{
    const int ppr = d.d_model * elem_size(d.dtype) / 16;
    const int lpr = lanes_per_row(ppr);
    const dim3 grid((d.T + kThreads / lpr - 1) / (kThreads / lpr)), block(kThreads);
    SMILE_LPR_SWITCH(lpr, SMILE_LAUNCH(dispatch_hop2_kernel<L>, grid, block, 0, s,
                                             static_cast<const u32x4 *>(xg), group_idx, local_idx, pos_in_group, slot,
                                             static_cast<u32x4 *>(xe), d.T, ppr, d.m_local, d.capacity, group_rows));
    return hipGetLastError();
}

hipError_t launch_dispatch_finalize(const smile_layer_desc &d, const Workspace &ws, const void *x,
                                    const int32_t *group_idx, const int32_t *local_idx, int32_t *pos_in_group,
                                    int32_t *slot, void *xe, void *y, const LossArgs &loss, hipStream_t s)
{
    const int ppr = d.d_model * elem_size(d.dtype) / 16;
    const int lpr = lanes_per_row(ppr);
    const dim3 grid((d.T + kThreads / lpr - 1) / (kThreads / lpr)), block(kThreads);
    SMILE_LPR_SWITCH(lpr, SMILE_LAUNCH(dispatch_finalize_kernel<L>, grid, block, 0, s,
                                             static_cast<const u32x4 *>(x), group_idx, local_idx, ws.block_expert_hist,
                                             ws.block_group_hist, ws.rank_in_block, ws.pos_in_block, pos_in_group, slot,
                                             static_cast<u32x4 *>(xe), ws.slot_token, static_cast<u32x4 *>(y), d.T, ppr,
                                             d.n_groups, d.m_local, d.capacity, loss, d.alpha, d.beta));
    return hipGetLastError();
}

hipError_t launch_finalize_map(const smile_layer_desc &d, const Workspace &ws, const int32_t *group_idx,
                               const int32_t *local_idx, int32_t *pos_in_group, int32_t *slot, void *y,
                               const LossArgs &loss, hipStream_t s)
{
    const int ppr = d.d_model * elem_size(d.dtype) / 16;
    const int B = (d.T + kRouteBlock - 1) / kRouteBlock;
    SMILE_LAUNCH(finalize_map_kernel, dim3(B), dim3(kRouteBlock), 0, s, group_idx, local_idx,
                       ws.block_expert_hist, ws.block_group_hist, ws.rank_in_block, ws.pos_in_block, pos_in_group,
                       slot, ws.slot_token, static_cast<u32x4 *>(y), d.T, ppr, d.n_groups, d.m_local, d.capacity, loss,
                       d.alpha, d.beta);
    return hipGetLastError();
}

hipError_t launch_finalize_map_scan(const smile_layer_desc &d, const Workspace &ws, const int32_t *group_idx,
                                    const int32_t *local_idx, int32_t *pos_in_group, int32_t *slot, void *y,
                                    int32_t *group_count, int32_t *local_count, int32_t *expert_count,
                                    int32_t *kept_count, float *p_sum, float *q_sum, float *loss3, hipStream_t s)
{
    const int ppr = d.d_model * elem_size(d.dtype) / 16;
    const int B = (d.T + kRouteBlock - 1) / kRouteBlock;
    const int n = d.n_groups, m = d.m_local;
    const size_t lds = sizeof(int32_t) * (size_t)(n * m + n + 2 * (n + m));
    SMILE_LAUNCH(finalize_map_scan_kernel, dim3(B), dim3(kRouteBlock), lds, s, group_idx, local_idx,
                       ws.block_expert_hist, ws.block_group_hist, ws.block_p_sum, ws.block_q_sum, ws.rank_in_block,
                       ws.pos_in_block, pos_in_group, slot, ws.slot_token, static_cast<u32x4 *>(y), d.T, ppr, n, m,
                       d.capacity, group_count, local_count, expert_count, kept_count, p_sum, q_sum, loss3, d.alpha,
                       d.beta);
    return hipGetLastError();
}

hipError_t launch_combine(const smile_layer_desc &d, const void *ye, const int32_t *group_idx,
                          const int32_t *local_idx, const int32_t *slot, const float *gate, void *y, hipStream_t s)
{
    const int ppr = d.d_model * elem_size(d.dtype) / 16;
    const int lpr = lanes_per_row(ppr);
    const dim3 grid((d.T + kThreads / lpr - 1) / (kThreads / lpr)), block(kThreads);
#define SMILE_COMBINE(DT)                                                                                          \
    SMILE_LPR_SWITCH(lpr, SMILE_LAUNCH((combine_kernel<DT, L>), grid, block, 0, s,                             \
                                             static_cast<const u32x4 *>(ye), group_idx, local_idx, slot, gate,       \
                                             static_cast<u32x4 *>(y), d.T, ppr, d.m_local, d.capacity))
    if (d.dtype == SMILE_DTYPE_BF16) { SMILE_COMBINE(SMILE_DTYPE_BF16); }
    else if (d.dtype == SMILE_DTYPE_F16) { SMILE_COMBINE(SMILE_DTYPE_F16); }
    else { SMILE_COMBINE(SMILE_DTYPE_F32); }
#undef SMILE_COMBINE
    return hipGetLastError();
}

}  // namespace smile
