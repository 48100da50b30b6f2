// Bi-level top-1 routing with per-expert capacity (Section 3.2.1, Section 3.2.2 statistics,
// Section 4.2 capacity), as three small kernels:
//
//   route_decide   one thread per token: biased logits (both rows fetched at once and kept in registers
//                  for routers of up to 32 columns) -> top-1 group and local expert, the two softmax
//                  probabilities (Eq. 1 read as a softmax), the gate p*q (Eq. 3); per-block column sums
//                  of p and q in a fixed order (wave butterflies for routers of up to 8 columns, an
//                  LDS tile summed in segments otherwise); the token's rank among
//                  EARLIER tokens of the same block with the same group / the same expert (wave64
//                  ballots + per-wave LDS counters combined after one barrier); per-block histograms.
//   route_scan     one wave per histogram column: exclusive scan along the block axis (turning the
//                  histograms into block offsets; 64 blocks per shuffle scan), totals, kept counts,
//                  and the fixed-order sums of p and q.
//   route_finalize one thread per token: global rank = block offset + in-block rank; capacity cut.
//                  (The chained forward pass skips this kernel and does the same inside dispatch.)
//
// With a group capacity (a first-hop buffer of Cg rows per group, Section 3.2.3) two more kernels run
// between the scan and the last step: route_first_hop recomputes the in-block expert ranks over the
// tokens whose stage-1 position is below Cg only (the others get a rank no capacity admits), and
// route_scan_experts scans the new per-block expert histograms.
//
// Everything that decides an integer is integer arithmetic or an fp32 compare of the caller's logits,
// so the result depends only on the logits and the token order, never on the launch geometry.  No
// atomics order, no inter-workgroup waiting, no memory that must be cleared beforehand.
#include <algorithm>

#include "smile_internal.hpp"

namespace smile {

namespace {

__device__ __forceinline__ unsigned long long lanemask_lt()
{
    const unsigned lane = __lane_id();
    return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

// Lanes of this wave (among `valid` ones) holding the same key; key < 2^bits.
__device__ __forceinline__ unsigned long long match_any(int key, int bits, bool valid)
{
    unsigned long long mask = __ballot(valid);
    for (int b = 0; b < bits; ++b) {
        const bool set = (key >> b) & 1;
        const unsigned long long bal = __ballot(valid && set);
        mask &= set ? bal : ~bal;
    }
    return mask;
}

// exp(v) for v <= 0 by the hardware exp2 (v_exp_f32 is accurate to about 1 ulp; the scaling by
// log2(e) adds a relative error of about |v| * 6e-8, far inside the 1e-5 tolerance of the gates).
// The kernel is instruction-bound (one wave per SIMD at T = 65536), which is why this matters.
__device__ __forceinline__ float exp_neg(float v)
{
    return __builtin_amdgcn_exp2f(v * 1.4426950408889634f);
}

constexpr int kLoadChunk = 8;   // logits fetched per lane before any of them is used (loads in flight)

// kLoadChunk biased logits starting at column i0 (one fp32 add each; columns >= len give `fill`).
// All loads are issued before the first use, so a lane waits for memory once per chunk, not per logit.
__device__ __forceinline__ void load_biased(const float *__restrict__ row, const float *__restrict__ bias, int i0,
                                            int len, float fill, float (&a)[kLoadChunk])
{
    float v[kLoadChunk], bv[kLoadChunk];
#pragma unroll
    for (int k = 0; k < kLoadChunk; ++k) {
        const int i = min(i0 + k, len - 1);
        v[k] = row[i];
        bv[k] = bias ? bias[i] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < kLoadChunk; ++k) a[k] = i0 + k < len ? (bias ? __fadd_rn(v[k], bv[k]) : v[k]) : fill;
}

// Top-1 over `len` biased logits: lowest index of the maximum, and 1/sum(exp(a - max)) which is
// the softmax probability of that maximum.  `row` and `bias` (may be null) are read twice.
__device__ __forceinline__ void top1_softmax(const float *__restrict__ row, const float *__restrict__ bias,
                                             int len, int &arg, float &mx, float &inv_z)
{
    arg = 0;
    mx = -INFINITY;
    float a[kLoadChunk];
    for (int i0 = 0; i0 < len; i0 += kLoadChunk) {
        load_biased(row, bias, i0, len, -INFINITY, a);
#pragma unroll
        for (int k = 0; k < kLoadChunk; ++k)
            if (a[k] > mx) { mx = a[k]; arg = i0 + k; }   // strict: the lowest index of the maximum wins
    }
    float z = 0.f;
    for (int i0 = 0; i0 < len; i0 += kLoadChunk) {
        load_biased(row, bias, i0, len, -INFINITY, a);
#pragma unroll
        for (int k = 0; k < kLoadChunk; ++k) z += exp_neg(a[k] - mx);   // exp2(-inf) = 0 for the padding
    }
    inv_z = 1.0f / z;
}

// A whole logit row kept in registers (routers of up to CAP columns): every load is issued before the first
// use, and the argmax, the exp-sum and the per-column probabilities all come from the same registers, so a
// token waits for memory once per router instead of once per pass.  Columns >= len hold -inf.
template <int CAP>
__device__ __forceinline__ void load_row(const float *__restrict__ row, const float *__restrict__ bias, int len,
                                         float (&a)[CAP])
{
    float v[CAP], bv[CAP];
#pragma unroll
    for (int k = 0; k < CAP; ++k) {
        const int i = min(k, len - 1);
        v[k] = row[i];
        bv[k] = bias ? bias[i] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < CAP; ++k) a[k] = k < len ? (bias ? __fadd_rn(v[k], bv[k]) : v[k]) : -INFINITY;
}

template <int CAP>
__device__ __forceinline__ void top1_softmax_row(const float (&a)[CAP], int &arg, float &mx, float &inv_z)
{
    arg = 0;
    mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < CAP; ++k)
        if (a[k] > mx) { mx = a[k]; arg = k; }   // strict: the lowest index of the maximum wins
    float z = 0.f;
#pragma unroll
    for (int k = 0; k < CAP; ++k) z += exp_neg(a[k] - mx);   // exp2(-inf) = 0 for the padding
    inv_z = 1.0f / z;
}

// block_column_sums (below) on a row held in registers
template <int CAP>
__device__ __forceinline__ void block_column_sums_row(const float (&a)[CAP], int len, float mx, float inv_z, bool valid,
                                                      float *__restrict__ part, float *__restrict__ out)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int k = 0; k < CAP; ++k) {
        if (k < len) {   // uniform
            float v = valid ? exp_neg(a[k] - mx) * inv_z : 0.f;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0) part[wave * len + k] = v;
        }
    }
    __syncthreads();
    for (int c = tid; c < len; c += kRouteBlock) {
        float sum = part[c];
#pragma unroll
        for (int w = 1; w < kRouteBlock / 64; ++w) sum += part[w * len + c];
        out[c] = sum;
    }
    __syncthreads();
}

constexpr int kColChunk = 32;   // probability columns summed per LDS pass

// Column sums over the block's tokens of prob[t, c] = exp(a[t,c] - mx_t) * inv_z_t, written to out[c], for
// routers of more than 8 columns: the probabilities go through an LDS tile, 32 columns at a time, and are summed
// in a fixed order (8 segments of 32 tokens serially, then the 8 partials serially).  GET(c) yields the biased
// logit of column c (from registers or from memory).
template <typename Get>
__device__ __forceinline__ void block_column_sums_tile(Get get, int len, float mx, float inv_z, bool valid,
                                                       float (*tile)[kColChunk + 1], float (*part)[kColChunk],
                                                       float *__restrict__ out)
{
    const int tid = threadIdx.x;
    for (int c0 = 0; c0 < len; c0 += kColChunk) {
        const int w = min(kColChunk, len - c0);
        get(c0, w, tile[tid]);   // tile[tid][k] = biased logit of column c0 + k for k < w (valid threads only)
        if (valid) {
            for (int k = 0; k < w; ++k) tile[tid][k] = exp_neg(tile[tid][k] - mx) * inv_z;
        } else {
            for (int k = 0; k < w; ++k) tile[tid][k] = 0.f;
        }
        __syncthreads();
        const int col = tid & (kColChunk - 1), seg = tid / kColChunk;   // 8 segments of 32 tokens
        if (col < w) {
            float s = 0.f;
            for (int j = 0; j < kRouteBlock / 8; ++j) s += tile[seg * (kRouteBlock / 8) + j][col];
            part[seg][col] = s;
        }
        __syncthreads();
        if (tid < w) {
            float s = 0.f;
            for (int sg = 0; sg < 8; ++sg) s += part[sg][tid];
            out[c0 + tid] = s;
        }
        __syncthreads();
    }
}

// PERWAVE: every wave counts into its own copy of the LDS histograms and the copies are combined after one
// barrier (needs 4 x (N + n) counters); otherwise the four waves take turns on one copy.
// CP / CQ: register capacity for the inter / intra logit row (0: rows longer than 32 columns are re-read from
// memory by every pass).
template <bool PERWAVE, int CP, int CQ>
__global__ __launch_bounds__(kRouteBlock) void route_decide_kernel(
    const float *__restrict__ logits_inter, const float *__restrict__ logits_intra,
    const float *__restrict__ bias_inter, const float *__restrict__ bias_intra,
    int T, int n, int m, int bits_n, int bits_N,
    int32_t *__restrict__ group_idx, int32_t *__restrict__ local_idx,
    int32_t *__restrict__ pos_in_block, int32_t *__restrict__ rank_in_block,
    float *__restrict__ gate, float *__restrict__ p_top, float *__restrict__ q_top,
    int32_t *__restrict__ block_expert_hist, int32_t *__restrict__ block_group_hist,
    float *__restrict__ block_p_sum, float *__restrict__ block_q_sum)
{
    // [N] expert counters then [n] group counters (PERWAVE: one such set per wave); reused afterwards as the
    // [4][max(n, m)] partial probability sums (both fit: n, m <= N + n)
    extern __shared__ int32_t hist[];
    __shared__ float tile[kRouteBlock][kColChunk + 1];
    __shared__ float part8[8][kColChunk];
    constexpr int kWaves = kRouteBlock / 64;

    const int N = n * m, NC = N + n;
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int t = b * kRouteBlock + tid;
    const bool valid = t < T;

    for (int i = tid; i < (PERWAVE ? kWaves : 1) * NC; i += kRouteBlock) hist[i] = 0;

    int g = 0, l = 0;
    float mx_p = 0.f, iz_p = 0.f, mx_q = 0.f, iz_q = 0.f;
    const float *rp = logits_inter + (size_t)(valid ? t : 0) * n;
    const float *rq = logits_intra + (size_t)(valid ? t : 0) * m;
    const float *bq = nullptr;
    float ap[CP > 0 ? CP : 1], aq[CQ > 0 ? CQ : 1];
    if (valid) {
        // the intra row does not depend on the chosen group (only its bias row does): fetch both rows at once
        if constexpr (CP > 0) load_row<CP>(rp, bias_inter, n, ap);
        if constexpr (CQ > 0) {
            if (!bias_intra) load_row<CQ>(rq, nullptr, m, aq);
        }
        if constexpr (CP > 0) top1_softmax_row<CP>(ap, g, mx_p, iz_p);
        else top1_softmax(rp, bias_inter, n, g, mx_p, iz_p);
        bq = bias_intra ? bias_intra + (size_t)g * m : nullptr;
        if constexpr (CQ > 0) {
            if (bias_intra) load_row<CQ>(rq, bq, m, aq);
            top1_softmax_row<CQ>(aq, l, mx_q, iz_q);
        } else {
            top1_softmax(rq, bq, m, l, mx_q, iz_q);
        }
        group_idx[t] = g;
        local_idx[t] = l;
        p_top[t] = iz_p;
        q_top[t] = iz_q;
        gate[t] = iz_p * iz_q;
    }
    __syncthreads();   // counters are zero

    // rank among earlier tokens of this block with the same expert / the same group
    const int e = g * m + l;
    const unsigned long long me = match_any(e, bits_N, valid);
    const unsigned long long mg = match_any(g, bits_n, valid);
    const unsigned long long lt = lanemask_lt();
    const int lane = __lane_id();
    const int wave = tid >> 6;
    if constexpr (PERWAVE) {
        int32_t *mine = hist + wave * NC;
        if (valid) {   // the last lane of each matching set publishes the wave's count
            if (63 - __clzll(me) == lane) mine[e] = __popcll(me);
            if (63 - __clzll(mg) == lane) mine[N + g] = __popcll(mg);
        }
        __syncthreads();
        if (valid) {
            int base_e = 0, base_g = 0;
            for (int w = 0; w < wave; ++w) {
                base_e += hist[w * NC + e];
                base_g += hist[w * NC + N + g];
            }
            rank_in_block[t] = base_e + __popcll(me & lt);
            pos_in_block[t] = base_g + __popcll(mg & lt);
        }
        for (int i = tid; i < N; i += kRouteBlock) {
            int c = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) c += hist[w * NC + i];
            block_expert_hist[(size_t)b * N + i] = c;
        }
        for (int i = tid; i < n; i += kRouteBlock) {
            int c = 0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) c += hist[w * NC + N + i];
            block_group_hist[(size_t)b * n + i] = c;
        }
        // per-block counts by local index (summed over groups), stored behind the [B][n] group histograms
        for (int j = tid; j < m; j += kRouteBlock) {
            int c = 0;
            for (int i = 0; i < n; ++i)
#pragma unroll
                for (int w = 0; w < kWaves; ++w) c += hist[w * NC + i * m + j];
            block_group_hist[(size_t)gridDim.x * n + (size_t)b * m + j] = c;
        }
    } else {
        int32_t *ghist = hist + N;
        for (int w = 0; w < kWaves; ++w) {   // the waves take turns in token order
            if (wave == w && valid) {
                const int base_e = hist[e];
                const int base_g = ghist[g];
                rank_in_block[t] = base_e + __popcll(me & lt);
                pos_in_block[t] = base_g + __popcll(mg & lt);
                if (63 - __clzll(me) == lane) hist[e] = base_e + __popcll(me);
                if (63 - __clzll(mg) == lane) ghist[g] = base_g + __popcll(mg);
            }
            __syncthreads();
        }
        for (int i = tid; i < N; i += kRouteBlock) block_expert_hist[(size_t)b * N + i] = hist[i];
        for (int i = tid; i < n; i += kRouteBlock) block_group_hist[(size_t)b * n + i] = ghist[i];
        for (int j = tid; j < m; j += kRouteBlock) {
            int c = 0;
            for (int i = 0; i < n; ++i) c += hist[i * m + j];
            block_group_hist[(size_t)gridDim.x * n + (size_t)b * m + j] = c;
        }
    }
    __syncthreads();   // the counters have been read: the memory becomes the partial-sum buffer

    // per-block column sums of p and q: wave butterflies for routers of at most 8 columns (registers), else
    // through the LDS tile
    float *part = reinterpret_cast<float *>(hist);
    if constexpr (CP == 8) {
        block_column_sums_row<CP>(ap, n, mx_p, iz_p, valid, part, block_p_sum + (size_t)b * n);
    } else if constexpr (CP > 0) {
        block_column_sums_tile([&](int c0, int w, float *dst) {
#pragma unroll
            for (int k = 0; k < CP; ++k)
                if (k >= c0 && k < c0 + w) dst[k - c0] = ap[k];
        }, n, mx_p, iz_p, valid, tile, part8, block_p_sum + (size_t)b * n);
    } else {
        block_column_sums_tile([&](int c0, int w, float *dst) {
            if (!valid) return;
            for (int i0 = 0; i0 < w; i0 += kLoadChunk) {
                float a[kLoadChunk];
                load_biased(rp, bias_inter, c0 + i0, n, -INFINITY, a);
#pragma unroll
                for (int k = 0; k < kLoadChunk; ++k)
                    if (i0 + k < w) dst[i0 + k] = a[k];
            }
        }, n, mx_p, iz_p, valid, tile, part8, block_p_sum + (size_t)b * n);
    }
    if constexpr (CQ == 8) {
        block_column_sums_row<CQ>(aq, m, mx_q, iz_q, valid, part, block_q_sum + (size_t)b * m);
    } else if constexpr (CQ > 0) {
        block_column_sums_tile([&](int c0, int w, float *dst) {
#pragma unroll
            for (int k = 0; k < CQ; ++k)
                if (k >= c0 && k < c0 + w) dst[k - c0] = aq[k];
        }, m, mx_q, iz_q, valid, tile, part8, block_q_sum + (size_t)b * m);
    } else {
        block_column_sums_tile([&](int c0, int w, float *dst) {
            if (!valid) return;
            for (int i0 = 0; i0 < w; i0 += kLoadChunk) {
                float a[kLoadChunk];
                load_biased(rq, bq, c0 + i0, m, -INFINITY, a);
#pragma unroll
                for (int k = 0; k < kLoadChunk; ++k)
                    if (i0 + k < w) dst[i0 + k] = a[k];
            }
        }, m, mx_q, iz_q, valid, tile, part8, block_q_sum + (size_t)b * m);
    }
}

// Exclusive scan along the block axis of one histogram column (64 blocks per step, one per lane,
// Hillis-Steele over the wave); returns the column total.  hist[b*stride + col] is rewritten in place.
__device__ __forceinline__ int wave_scan_column(int32_t *__restrict__ hist, int B, int stride, int col)
{
    const int lane = __lane_id();
    int carry = 0;
    for (int b0 = 0; b0 < B; b0 += 64) {
        const int b = b0 + lane;
        const int v = b < B ? hist[(size_t)b * stride + col] : 0;
        int incl = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        if (b < B) hist[(size_t)b * stride + col] = carry + incl - v;
        carry += __shfl(incl, 63, 64);
    }
    return carry;
}

// One wave per column of the work list
//   [N expert columns | n group columns | n p-sum columns | m q-sum columns | m local-count columns],
// 4 waves per workgroup; the columns are independent, so the grid spreads them over the chip.
constexpr int kScanWaves = 4;

__global__ __launch_bounds__(64 * kScanWaves) void route_scan_kernel(
    int B, int n, int m, int C,
    int32_t *__restrict__ block_expert_hist, int32_t *__restrict__ block_group_hist,
    const float *__restrict__ block_p_sum, const float *__restrict__ block_q_sum,
    int32_t *__restrict__ group_count, int32_t *__restrict__ local_count,
    int32_t *__restrict__ expert_count, int32_t *__restrict__ kept_count,
    float *__restrict__ p_sum, float *__restrict__ q_sum)
{
    const int N = n * m;
    const int lane = threadIdx.x & 63;
    const int w = blockIdx.x * kScanWaves + (threadIdx.x >> 6);
    if (w < N) {
        const int total = wave_scan_column(block_expert_hist, B, N, w);
        if (lane == 0) {
            expert_count[w] = total;
            kept_count[w] = min(total, C);
        }
    } else if (w < N + n) {
        const int total = wave_scan_column(block_group_hist, B, n, w - N);
        if (lane == 0) group_count[w - N] = total;
    } else if (w < N + 2 * n) {
        const float s = wave_sum_column(block_p_sum, B, n, w - N - n);
        if (lane == 0) p_sum[w - N - n] = s;
    } else if (w < N + 2 * n + m) {
        const float s = wave_sum_column(block_q_sum, B, m, w - N - 2 * n);
        if (lane == 0) q_sum[w - N - 2 * n] = s;
    } else if (w < N + 2 * n + 2 * m) {
        // local_count[j] = tokens whose local index is j, over all groups.  The expert columns are
        // being rewritten by other waves, so it is summed from the per-block counts by local index
        // that route_decide stored behind the group histograms.
        const int j = w - N - 2 * n - m;
        int s = 0;
        for (int b = lane; b < B; b += 64) s += block_group_hist[(size_t)B * n + (size_t)b * m + j];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane == 0) local_count[j] = s;
    }
}

// Group capacity, step 1: tokens whose stage-1 position (block offset of the group + in-block
// position) reaches Cg are dropped at the first hop.  The in-block expert ranks and the per-block
// expert histograms are rebuilt over the remaining tokens, overwriting those of route_decide (whose
// totals the first scan has already turned into expert_count).
__global__ __launch_bounds__(kRouteBlock) void route_first_hop_kernel(
    int T, int n, int m, int Cg, int bits_N,
    const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx,
    const int32_t *__restrict__ block_group_off, const int32_t *__restrict__ pos_in_block,
    int32_t *__restrict__ rank_in_block, int32_t *__restrict__ block_expert_hist)
{
    extern __shared__ int32_t hist[];   // [N]
    const int N = n * m;
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int t = b * kRouteBlock + tid;
    for (int i = tid; i < N; i += kRouteBlock) hist[i] = 0;
    int e = 0;
    bool through = false;
    if (t < T) {
        const int g = group_idx[t];
        e = g * m + local_idx[t];
        through = block_group_off[(size_t)b * n + g] + pos_in_block[t] < Cg;
    }
    __syncthreads();
    const unsigned long long me = match_any(e, bits_N, through);
    const unsigned long long lt = lanemask_lt();
    const int lane = __lane_id();
    const int wave = tid >> 6;
    for (int w = 0; w < kRouteBlock / 64; ++w) {
        if (wave == w && through) {
            const int base = hist[e];
            rank_in_block[t] = base + __popcll(me & lt);
            if (63 - __clzll(me) == lane) hist[e] = base + __popcll(me);
        }
        __syncthreads();
    }
    if (t < T && !through) rank_in_block[t] = kHop1Dropped;
    for (int i = tid; i < N; i += kRouteBlock) block_expert_hist[(size_t)b * N + i] = hist[i];
}

// Group capacity, step 2: block offsets of the rebuilt expert histograms; kept_count = tokens that
// reached the expert, cut at C.
__global__ __launch_bounds__(64 * kScanWaves) void route_scan_experts_kernel(
    int B, int N, int C, int32_t *__restrict__ block_expert_hist, int32_t *__restrict__ kept_count)
{
    const int w = blockIdx.x * kScanWaves + (threadIdx.x >> 6);
    if (w >= N) return;
    const int total = wave_scan_column(block_expert_hist, B, N, w);
    if ((threadIdx.x & 63) == 0) kept_count[w] = min(total, C);
}

__global__ __launch_bounds__(kRouteBlock) void route_finalize_kernel(
    int T, int n, int m, int C,
    const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx,
    const int32_t *__restrict__ block_expert_off, const int32_t *__restrict__ block_group_off,
    const int32_t *__restrict__ rank_in_block, const int32_t *__restrict__ pos_in_block,
    int32_t *__restrict__ pos_in_group, int32_t *__restrict__ slot)
{
    const int b = blockIdx.x;
    const int t = b * kRouteBlock + threadIdx.x;
    if (t >= T) return;
    const int g = group_idx[t], l = local_idx[t];
    const int N = n * m;
    const int rank = block_expert_off[(size_t)b * N + g * m + l] + rank_in_block[t];
    slot[t] = rank < C ? rank : -1;
    pos_in_group[t] = block_group_off[(size_t)b * n + g] + pos_in_block[t];
}

int ceil_log2(int v)
{
    int b = 0;
    while ((1 << b) < v) ++b;
    return b;
}

}  // namespace

hipError_t launch_route(const smile_layer_desc &d, const Workspace &ws, const float *logits_inter,
                        const float *logits_intra, const float *bias_inter, const float *bias_intra,
                        int32_t *group_idx, int32_t *local_idx, int32_t *pos_in_group, int32_t *slot, float *gate,
                        float *p_top, float *q_top, int32_t *group_count, int32_t *local_count,
                        int32_t *expert_count, int32_t *kept_count, float *p_sum, float *q_sum, hipStream_t s,
                        bool finalize, bool scan)
{
    const int n = d.n_groups, m = d.m_local, N = n * m;
    const int B = (d.T + kRouteBlock - 1) / kRouteBlock;
    // one histogram copy per wave while four of them fit beside the kernel's static LDS (the probability tile and
    // its partial sums) in the 64 KB a workgroup may have without opting in: N + n <= 1920
    constexpr size_t kStaticLds = sizeof(float) * (kRouteBlock * (kColChunk + 1) + 8 * kColChunk);
    const bool per_wave = (size_t)(N + n) * (kRouteBlock / 64) * sizeof(int32_t) + kStaticLds <= 64 * 1024;
    // the counters' memory is reused for the [4][max(n, m)] partial probability sums
    const size_t counters = (size_t)(N + n) * (per_wave ? kRouteBlock / 64 : 1);
    const size_t lds1 = sizeof(int32_t) * std::max(counters, (size_t)(kRouteBlock / 64) * std::max(n, m));
    const int cp = n <= 8 ? 8 : (n <= 32 ? 32 : 0), cq = m <= 8 ? 8 : (m <= 32 ? 32 : 0);
#define SMILE_DECIDE(PW, CP, CQ)                                                                                     \
    SMILE_LAUNCH((route_decide_kernel<PW, CP, CQ>), dim3(B), dim3(kRouteBlock), lds1, s, logits_inter,          \
                       logits_intra, bias_inter, bias_intra, d.T, n, m, ceil_log2(n), ceil_log2(N), group_idx,        \
                       local_idx, ws.pos_in_block, ws.rank_in_block, gate, p_top, q_top, ws.block_expert_hist,         \
                       ws.block_group_hist, ws.block_p_sum, ws.block_q_sum)
    if (!per_wave) SMILE_DECIDE(false, 0, 0);
    else if (cp == 8 && cq == 8) SMILE_DECIDE(true, 8, 8);
    else if (cp == 32 && cq == 8) SMILE_DECIDE(true, 32, 8);
    else if (cp == 8 && cq == 32) SMILE_DECIDE(true, 8, 32);
    else if (cp == 32 && cq == 32) SMILE_DECIDE(true, 32, 32);
    else SMILE_DECIDE(true, 0, 0);
#undef SMILE_DECIDE
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || !scan) return err;   // !scan: the caller's last step scans the histograms itself
    const int columns = N + 2 * n + 2 * m;
    SMILE_LAUNCH(route_scan_kernel, dim3((columns + kScanWaves - 1) / kScanWaves), dim3(64 * kScanWaves), 0, s, B, n,
                       m, d.capacity, ws.block_expert_hist, ws.block_group_hist, ws.block_p_sum, ws.block_q_sum,
                       group_count, local_count, expert_count, kept_count, p_sum, q_sum);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (d.group_capacity > 0) {
        SMILE_LAUNCH(route_first_hop_kernel, dim3(B), dim3(kRouteBlock), sizeof(int32_t) * (size_t)N, s, d.T, n, m,
                           d.group_capacity, ceil_log2(N), group_idx, local_idx, ws.block_group_hist, ws.pos_in_block,
                           ws.rank_in_block, ws.block_expert_hist);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
        SMILE_LAUNCH(route_scan_experts_kernel, dim3((N + kScanWaves - 1) / kScanWaves), dim3(64 * kScanWaves), 0,
                           s, B, N, d.capacity, ws.block_expert_hist, kept_count);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    if (!finalize) return err;
    SMILE_LAUNCH(route_finalize_kernel, dim3(B), dim3(kRouteBlock), 0, s, d.T, n, m, d.capacity, group_idx,
                       local_idx, ws.block_expert_hist, ws.block_group_hist, ws.rank_in_block, ws.pos_in_block,
                       pos_in_group, slot);
    return hipGetLastError();
}

}  // namespace smile
