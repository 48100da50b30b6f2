// Backward pass of the layer: the chain rule on Eq. 3 and Eq. 4 with the discrete routing decisions and
// the fractions f of Eq. 4 held constant (as for the Switch loss of Section 2), in the reverse order of
// the forward steps:
//
//   combine_backward       dye[row(t)] = gate_t * dy[t],  dgate[t] = <dy[t], ye[row(t)]>     (HBM streaming)
//   route_backward         softmax Jacobians of the two routers: dgate and the Eq. 4 terms -> dlogits
//   expert_ffn_backward    (pre, h) = xe . W1^T   unless saved by the forward pass (one launch of the forward kernel)
//                          dpre = (dye . W2) * act'(pre),  dxe = dpre . W1,
//                          dW2 = dye^T . h,  dW1 = dpre^T . xe   (contraction over the expert's rows)
//                          bf16: four launches of the MFMA kernel that reads operands whose contraction index is
//                          the slow one (transposing LDS reads), nothing transposed in memory;
//                          fp32: the forward kernel on operands transposed by a tiled transpose kernel (zero-padded
//                          along the row axis, so experts with fewer than C rows contribute exact zeros)
//   dispatch_backward      dx[t] = dxe[row(t)] + dlp[t,:] . W_p + dlq[t,:] . W_q
//   gate_weights_backward  dW_p = dlp^T . x, dW_q = dlq^T . x: per-block partial sums, then a fixed-order
//                          reduction over the blocks (bit-reproducible, no atomics)
#include <type_traits>


#include "smile_internal.hpp"

namespace smile {

namespace {

constexpr int kThreads = 256;

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

// A 16-byte piece as 4 (fp32) or 8 (16-bit types) floats and back.  DT: SMILE_DTYPE_*.
template <int DT>
struct Piece {
    static constexpr int kElems = DT == SMILE_DTYPE_F32 ? 4 : 8;
    using H = Half<std::conditional_t<DT == SMILE_DTYPE_F16, _Float16, __bf16>>;
    __device__ static __forceinline__ void unpack(u32x4 v, float (&f)[kElems])
    {
        if constexpr (DT != SMILE_DTYPE_F32) {
#pragma unroll
            for (int k = 0; k < 4; ++k) { f[2 * k] = H::lo(v[k]); f[2 * k + 1] = H::hi(v[k]); }
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) f[k] = __uint_as_float(v[k]);
        }
    }
    __device__ static __forceinline__ u32x4 pack(const float (&f)[kElems])
    {
        u32x4 r;
        if constexpr (DT != SMILE_DTYPE_F32) {
#pragma unroll
            for (int k = 0; k < 4; ++k) r[k] = H::pack(f[2 * k], f[2 * k + 1]);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) r[k] = __float_as_uint(f[k]);
        }
        return r;
    }
};

// ------------------------------------------------------------------------------------ combine backward

// LPR consecutive lanes own one token row (as in the forward dispatch / combine kernels).
template <int DT, int LPR>
__global__ __launch_bounds__(kThreads) void combine_backward_kernel(
    const u32x4 *__restrict__ dy, const u32x4 *__restrict__ ye, const int32_t *__restrict__ group_idx,
    const int32_t *__restrict__ local_idx, const int32_t *__restrict__ slot, const float *__restrict__ gate,
    u32x4 *__restrict__ dye, float *__restrict__ dgate, int T, int ppr, int m, int C)
{
    constexpr int E = Piece<DT>::kElems;
    const int t = blockIdx.x * (kThreads / LPR) + threadIdx.x / LPR, sub = threadIdx.x % LPR;
    // every lane of a row group takes the same branch, and a group never straddles a wave
    if (t >= T) return;
    const int sl = slot[t];
    if (sl < 0) {
        if (sub == 0) dgate[t] = 0.f;
        return;
    }
    const float gt = gate[t];
    const size_t row = (size_t)(group_idx[t] * m + local_idx[t]) * C + sl;
    const u32x4 *src = dy + (size_t)t * ppr, *act = ye + row * ppr;
    u32x4 *dst = dye + row * ppr;
    float dot = 0.f;
    for (int c = sub; c < ppr; c += LPR) {
        float a[E], b[E], o[E];
        Piece<DT>::unpack(src[c], a);
        Piece<DT>::unpack(act[c], b);
#pragma unroll
        for (int k = 0; k < E; ++k) {
            dot = fmaf(a[k], b[k], dot);
            o[k] = a[k] * gt;
        }
        dst[c] = Piece<DT>::pack(o);
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) dot += __shfl_xor(dot, off, 64);
    if (sub == 0) dgate[t] = dot;
}

// ------------------------------------------------------------------------------------ route backward

__device__ __forceinline__ float exp_neg(float v) { return __builtin_amdgcn_exp2f(v * 1.4426950408889634f); }

// One thread per token.  For each router: z = sum exp(a - a_top) (so the top probability is 1/z), then
//   u_k = coef * count_k + [k == top] * extra,   dl_k = p_k * (u_k - sum_i u_i p_i).
__device__ __forceinline__ float softmax_z(const float *__restrict__ row, const float *__restrict__ bias, int len,
                                           int top, float &mx)
{
    mx = bias ? __fadd_rn(row[top], bias[top]) : row[top];
    float z = 0.f;
    for (int i = 0; i < len; ++i) z += exp_neg((bias ? __fadd_rn(row[i], bias[i]) : row[i]) - mx);
    return z;
}

// (row and out may be the same array: element i of out is written after the last read of element i of row)
__device__ __forceinline__ void softmax_backward_row(const float *row, const float *__restrict__ bias,
                                                     int len, int top, float mx, float inv_z, float coef,
                                                     const int32_t *__restrict__ count, float extra, float *out)
{
    float dot = 0.f;
    for (int i = 0; i < len; ++i) {
        const float p = exp_neg((bias ? __fadd_rn(row[i], bias[i]) : row[i]) - mx) * inv_z;
        const float u = coef * (float)count[i] + (i == top ? extra : 0.f);
        dot = fmaf(u, p, dot);
    }
    for (int i = 0; i < len; ++i) {
        const float p = exp_neg((bias ? __fadd_rn(row[i], bias[i]) : row[i]) - mx) * inv_z;
        const float u = coef * (float)count[i] + (i == top ? extra : 0.f);
        out[i] = p * (u - dot);
    }
}

__global__ __launch_bounds__(kThreads) void route_backward_kernel(
    const float *__restrict__ logits_inter, const float *__restrict__ logits_intra,
    const float *__restrict__ bias_inter, const float *__restrict__ bias_intra,
    const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx, const float *__restrict__ dgate,
    const int32_t *__restrict__ group_count, const int32_t *__restrict__ local_count,
    int T, int n, int m, float coef_inter, float coef_intra, float *__restrict__ dlp, float *__restrict__ dlq)
{
    const int t = blockIdx.x * kThreads + threadIdx.x;
    if (t >= T) return;
    const int g = group_idx[t], l = local_idx[t];
    const float *rp = logits_inter + (size_t)t * n, *rq = logits_intra + (size_t)t * m;
    const float *bq = bias_intra ? bias_intra + (size_t)g * m : nullptr;
    float mx_p, mx_q;
    const float iz_p = 1.0f / softmax_z(rp, bias_inter, n, g, mx_p);   // = p[g]
    const float iz_q = 1.0f / softmax_z(rq, bq, m, l, mx_q);           // = q[l]
    const float dg = dgate[t];
    softmax_backward_row(rp, bias_inter, n, g, mx_p, iz_p, coef_inter, group_count, dg * iz_q, dlp + (size_t)t * n);
    softmax_backward_row(rq, bq, m, l, mx_q, iz_q, coef_intra, local_count, dg * iz_p, dlq + (size_t)t * m);
}

// The same arithmetic with coalesced memory traffic: a workgroup's logit rows are contiguous in memory, so they are
// copied to LDS with consecutive lanes on consecutive addresses (a thread reading its own row straight from memory
// touches one cache line per lane and instruction), the gradients replace them in place, and the tile is copied
// back the same way.  Row strides in LDS are odd, so the per-token threads fall on distinct banks.
__global__ __launch_bounds__(kThreads) void route_backward_tiled_kernel(
    const float *__restrict__ logits_inter, const float *__restrict__ logits_intra,
    const float *__restrict__ bias_inter, const float *__restrict__ bias_intra,
    const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx, const float *__restrict__ dgate,
    const int32_t *__restrict__ group_count, const int32_t *__restrict__ local_count,
    int T, int n, int m, float coef_inter, float coef_intra, float *__restrict__ dlp, float *__restrict__ dlq,
    int tokens_per_block)
{
    extern __shared__ float route_bwd_lds[];
    const int sp = n | 1, sq = m | 1;
    float *tp = route_bwd_lds, *tq = route_bwd_lds + (size_t)tokens_per_block * sp;
    const int t0 = blockIdx.x * tokens_per_block, cnt = min(tokens_per_block, T - t0);
    const float *gp = logits_inter + (size_t)t0 * n, *gq = logits_intra + (size_t)t0 * m;
    // element i of the contiguous tile <-> (row i / len, column i % len), advanced without divisions
    auto copy_tile = [&](auto to_lds, float *tile, int stride, const float *src, float *dst, int len) {
        const int dr = kThreads / len, dc = kThreads % len;
        int r = threadIdx.x / len, c = threadIdx.x % len;
        for (int i = threadIdx.x; i < cnt * len; i += kThreads) {
            if constexpr (decltype(to_lds)::value) tile[r * stride + c] = src[i];
            else dst[i] = tile[r * stride + c];
            r += dr, c += dc;
            if (c >= len) c -= len, ++r;
        }
    };
    copy_tile(std::true_type{}, tp, sp, gp, nullptr, n);
    copy_tile(std::true_type{}, tq, sq, gq, nullptr, m);
    __syncthreads();
    if ((int)threadIdx.x < cnt) {
        const int t = t0 + threadIdx.x;
        const int g = group_idx[t], l = local_idx[t];
        float *rp = tp + threadIdx.x * sp, *rq = tq + threadIdx.x * sq;
        const float *bq = bias_intra ? bias_intra + (size_t)g * m : nullptr;
        float mx_p, mx_q;
        const float iz_p = 1.0f / softmax_z(rp, bias_inter, n, g, mx_p);   // = p[g]
        const float iz_q = 1.0f / softmax_z(rq, bq, m, l, mx_q);           // = q[l]
        const float dg = dgate[t];
        softmax_backward_row(rp, bias_inter, n, g, mx_p, iz_p, coef_inter, group_count, dg * iz_q, rp);
        softmax_backward_row(rq, bq, m, l, mx_q, iz_q, coef_intra, local_count, dg * iz_p, rq);
    }
    __syncthreads();
    copy_tile(std::false_type{}, tp, sp, nullptr, dlp + (size_t)t0 * n, n);
    copy_tile(std::false_type{}, tq, sq, nullptr, dlq + (size_t)t0 * m, m);
}

// ------------------------------------------------------------------------------------ transpose

// out[e][c][r] = r < rows_e ? in[e][r][c] : 0   for c < cols, r < rows_out;
// in[N][R][cols], out[N][cols][rows_out], rows_e = kept ? min(kept[e], R) : R.  64 x 64 element tiles
// through LDS, 16-byte global accesses on both sides.  cols and rows_out are multiples of VEC.
template <typename E, int VEC>
__global__ __launch_bounds__(kThreads) void transpose_pad_kernel(
    const E *__restrict__ in, E *__restrict__ out, const int32_t *__restrict__ kept, int R, int cols, int rows_out,
    int row_tiles, int col_tiles)
{
    constexpr int TILE = 64, PPT = TILE / VEC;   // pieces per tile row
    constexpr int PAD = sizeof(E) == 2 ? 2 : 1;   // row stride of 33 / 65 words: conflict-free column reads
    __shared__ E tile[TILE][TILE + PAD];
    typedef E vec_t __attribute__((ext_vector_type(VEC)));

    const int per_e = row_tiles * col_tiles;
    const int e = blockIdx.x / per_e, rem = blockIdx.x - e * per_e;
    const int rt = rem / col_tiles, ct = rem - rt * col_tiles;
    const int rows = kept ? min(kept[e], R) : R;
    const E *src = in + (size_t)e * R * cols;
    E *dst = out + (size_t)e * cols * rows_out;
    const int r0 = rt * TILE, c0 = ct * TILE;

    for (int p = threadIdx.x; p < TILE * PPT; p += kThreads) {
        const int r = p / PPT, cp = (p - r * PPT) * VEC;
        vec_t v = {};
        if (r0 + r < rows && c0 + cp < cols) v = *reinterpret_cast<const vec_t *>(src + (size_t)(r0 + r) * cols + c0 + cp);
#pragma unroll
        for (int k = 0; k < VEC; ++k) tile[r][cp + k] = v[k];
    }
    __syncthreads();
    for (int p = threadIdx.x; p < TILE * PPT; p += kThreads) {
        const int c = p / PPT, rp = (p - c * PPT) * VEC;
        if (c0 + c >= cols || r0 + rp >= rows_out) continue;
        vec_t v;
#pragma unroll
        for (int k = 0; k < VEC; ++k) v[k] = tile[rp + k][c];
        *reinterpret_cast<vec_t *>(dst + (size_t)(c0 + c) * rows_out + r0 + rp) = v;
    }
}

template <typename E, int VEC>
hipError_t launch_transpose(const void *in, void *out, const int32_t *kept, int N, int R, int cols, int rows_out,
                            hipStream_t s)
{
    const int row_tiles = (rows_out + 63) / 64, col_tiles = (cols + 63) / 64;
    SMILE_LAUNCH((transpose_pad_kernel<E, VEC>), dim3((unsigned)((size_t)N * row_tiles * col_tiles)),
                       dim3(kThreads), 0, s, static_cast<const E *>(in), static_cast<E *>(out), kept, R, cols,
                       rows_out, row_tiles, col_tiles);
    return hipGetLastError();
}

hipError_t transpose_pad(int dtype, const void *in, void *out, const int32_t *kept, int N, int R, int cols,
                         int rows_out, hipStream_t s)
{
    if (is_half(dtype)) return launch_transpose<uint16_t, 8>(in, out, kept, N, R, cols, rows_out, s);
    return launch_transpose<float, 4>(in, out, kept, N, R, cols, rows_out, s);
}

// ------------------------------------------------------------------------------------ dispatch backward

// dx[t] = dxe[row(t)] (kept tokens) + sum_i dlp[t,i] W_p[i] + sum_j dlq[t,j] W_q[j], one rounding.
template <int DT, int LPR>
__global__ __launch_bounds__(kThreads) void dispatch_backward_kernel(
    const u32x4 *__restrict__ dxe, const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx,
    const int32_t *__restrict__ slot, const float *__restrict__ dlp, const float *__restrict__ dlq,
    const u32x4 *__restrict__ w_inter, const u32x4 *__restrict__ w_intra, u32x4 *__restrict__ dx,
    int T, int ppr, int n, int m, int C)
{
    constexpr int E = Piece<DT>::kElems;
    const int t = blockIdx.x * (kThreads / LPR) + threadIdx.x / LPR, sub = threadIdx.x % LPR;
    if (t >= T) return;
    const int sl = slot[t];
    const u32x4 *src = sl >= 0 ? dxe + ((size_t)(group_idx[t] * m + local_idx[t]) * C + sl) * ppr : nullptr;
    const float *lp = dlp + (size_t)t * n, *lq = dlq + (size_t)t * m;
    for (int c = sub; c < ppr; c += LPR) {
        float acc[E], w[E];
        if (src) Piece<DT>::unpack(src[c], acc);
        else {
#pragma unroll
            for (int k = 0; k < E; ++k) acc[k] = 0.f;
        }
        // acc += sum_i dl[i] * rows[i][c], eight rows at a time with all their loads issued first
        auto add_rows = [&](const u32x4 *__restrict__ rows, const float *__restrict__ dl, int count) {
            for (int i0 = 0; i0 < count; i0 += 8) {
                u32x4 wp[8];
                float g[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const int i = min(i0 + q, count - 1);
                    wp[q] = rows[(size_t)i * ppr + c];
                    g[q] = dl[i];
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    if (i0 + q < count) {
                        Piece<DT>::unpack(wp[q], w);
#pragma unroll
                        for (int k = 0; k < E; ++k) acc[k] = fmaf(g[q], w[k], acc[k]);
                    }
                }
            }
        };
        add_rows(w_inter, lp, n);
        add_rows(w_intra, lq, m);
        dx[(size_t)t * ppr + c] = Piece<DT>::pack(acc);
    }
}

// ------------------------------------------------------------------------------------ router weights backward

constexpr int kGwTokens = 128;   // tokens per workgroup
constexpr int kGwCols = 64;      // columns of x per workgroup
constexpr int kGwChunk = 16;     // logit columns per pass over the token tile

// partial[b][i][k] = sum over the block's tokens of dl[t][i] * x[t][k], i over the n + m logit columns
// (dlp first, then dlq).  The x tile (fp32) and a chunk of 16 logit-gradient columns sit in LDS; lane =
// column of x, wave w owns logit columns 4w .. 4w+3 of the chunk, so its four dl values of a token come
// from one broadcast LDS read.  Tokens are summed serially: a fixed order.
template <int DT>
__global__ __launch_bounds__(kThreads) void gate_weights_partial_kernel(
    const void *__restrict__ x, const float *__restrict__ dlp, const float *__restrict__ dlq,
    float *__restrict__ partial, int T, int d, int n, int m)
{
    __shared__ float xs[kGwTokens][kGwCols + 1];
    __shared__ __attribute__((aligned(16))) float dls[kGwTokens][kGwChunk];
    const int b = blockIdx.x, k0 = blockIdx.y * kGwCols;
    const int t0 = b * kGwTokens;
    const int cnt = min(kGwTokens, T - t0);
    {
        // x tile: 16-byte pieces, all of a thread's loads issued before the first LDS write (d % 8 == 0)
        constexpr int E = Piece<DT>::kElems, PPT = kGwCols / E, PER = kGwTokens * PPT / kThreads;
        u32x4 v[PER];
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int id = threadIdx.x + q * kThreads, tt = id / PPT, k = (id - tt * PPT) * E;
            v[q] = u32x4{0u, 0u, 0u, 0u};
            if (tt < cnt && k0 + k < d)
                v[q] = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(x) +
                                                        ((size_t)(t0 + tt) * d + k0 + k) * (16 / E));
        }
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int id = threadIdx.x + q * kThreads, tt = id / PPT, k = (id - tt * PPT) * E;
            float f[E];
            Piece<DT>::unpack(v[q], f);
#pragma unroll
            for (int j = 0; j < E; ++j) xs[tt][k + j] = f[j];
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cols = n + m;
    for (int c0 = 0; c0 < cols; c0 += kGwChunk) {
        __syncthreads();   // x tile ready / previous chunk consumed
        for (int id = threadIdx.x; id < kGwTokens * kGwChunk; id += kThreads) {
            const int tt = id / kGwChunk, i = c0 + (id - tt * kGwChunk);
            float v = 0.f;
            if (tt < cnt && i < cols)
                v = i < n ? dlp[(size_t)(t0 + tt) * n + i] : dlq[(size_t)(t0 + tt) * m + (i - n)];
            dls[tt][id - tt * kGwChunk] = v;
        }
        __syncthreads();
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll 8
        for (int tt = 0; tt < cnt; ++tt) {
            const float xv = xs[tt][lane];
            const float4 g = *reinterpret_cast<const float4 *>(&dls[tt][4 * wave]);
            s0 = fmaf(g.x, xv, s0);
            s1 = fmaf(g.y, xv, s1);
            s2 = fmaf(g.z, xv, s2);
            s3 = fmaf(g.w, xv, s3);
        }
        if (k0 + lane < d) {
            const float sv[4] = {s0, s1, s2, s3};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = c0 + 4 * wave + j;
                if (i < cols) partial[((size_t)b * cols + i) * d + k0 + lane] = sv[j];
            }
        }
    }
}

// dw[i][k] = sum_b partial[b][i][k], blocks in index order.
__global__ __launch_bounds__(kThreads) void gate_weights_reduce_kernel(
    const float *__restrict__ partial, float *__restrict__ dw_inter, float *__restrict__ dw_intra, int B, int d, int n,
    int m)
{
    const long long id = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long total = (long long)(n + m) * d;
    if (id >= total) return;
    float s = 0.f;
#pragma unroll 8
    for (int b = 0; b < B; ++b) s += partial[(size_t)b * total + id];
    if (id < (long long)n * d) dw_inter[id] = s;
    else dw_intra[id - (long long)n * d] = s;
}

int lanes_per_row(int ppr)
{
    int l = 8;
    while (l * 2 <= ppr && l < 32) l *= 2;
    return l;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

#define SMILE_BWD_LPR_SWITCH(lpr, CALL)             \
    switch (lpr) {                                  \
    case 8: { constexpr int L = 8; CALL; } break;   \
    case 16: { constexpr int L = 16; CALL; } break; \
    default: { constexpr int L = 32; CALL; } break; \
    }

// CALL with the compile-time constant DT set to the runtime storage type
#define SMILE_DTYPE_SWITCH(dtype, CALL)                                             \
    switch (dtype) {                                                                \
    case SMILE_DTYPE_BF16: { constexpr int DT = SMILE_DTYPE_BF16; CALL; } break;    \
    case SMILE_DTYPE_F16: { constexpr int DT = SMILE_DTYPE_F16; CALL; } break;      \
    default: { constexpr int DT = SMILE_DTYPE_F32; CALL; } break;                   \
    }

BackwardLayout backward_workspace_layout(const smile_layer_desc &d)
{
    BackwardLayout L{};
    const size_t esz = elem_size(d.dtype);
    const size_t N = (size_t)d.n_groups * d.m_local, C = (size_t)d.capacity;
    const size_t dm = (size_t)d.d_model, F = (size_t)d.d_ff;
    L.k_pad = (int32_t)((d.capacity + 63) / 64 * 64);
    L.gw_blocks = (d.T + kGwTokens - 1) / kGwTokens;
    size_t off = 0;
    L.off_pre = off;     off = align_up(off + N * C * F * esz, 256);
    L.off_h = off;       off = align_up(off + N * C * F * esz, 256);
    L.off_dpre = off;    off = align_up(off + N * C * F * esz, 256);
    // transposed copies of the operands: the fp32 path only (the bf16 kernel reads them in place)
    const size_t tr = is_half(d.dtype) ? 0 : 1;
    L.off_h_t = off;     off = align_up(off + tr * N * F * (size_t)L.k_pad * esz, 256);
    L.off_dpre_t = off;  off = align_up(off + tr * N * F * (size_t)L.k_pad * esz, 256);
    L.off_dye_t = off;   off = align_up(off + tr * N * dm * (size_t)L.k_pad * esz, 256);
    L.off_xe_t = off;    off = align_up(off + tr * N * dm * (size_t)L.k_pad * esz, 256);
    L.off_w_t = off;     off = align_up(off + tr * N * dm * F * esz, 256);
    L.off_gw_partial = off;
    off = align_up(off + (size_t)L.gw_blocks * (size_t)(d.n_groups + d.m_local) * dm * sizeof(float), 256);
    L.total = off;
    return L;
}

hipError_t launch_combine_backward(const smile_layer_desc &d, const void *dy, const void *ye, const int32_t *group_idx,
                                   const int32_t *local_idx, const int32_t *slot, const float *gate, void *dye,
                                   float *dgate, hipStream_t s)
{
    const int ppr = d.d_model * elem_size(d.dtype) / 16;
    const int lpr = lanes_per_row(ppr);
    const dim3 grid((d.T + kThreads / lpr - 1) / (kThreads / lpr)), block(kThreads);
    SMILE_DTYPE_SWITCH(d.dtype, SMILE_BWD_LPR_SWITCH(
        lpr, SMILE_LAUNCH((combine_backward_kernel<DT, L>), grid, block, 0, s, static_cast<const u32x4 *>(dy),
                                static_cast<const u32x4 *>(ye), group_idx, local_idx, slot, gate,
                                static_cast<u32x4 *>(dye), dgate, d.T, ppr, d.m_local, d.capacity)));
    return hipGetLastError();
}

hipError_t launch_route_backward(const smile_layer_desc &d, const float *logits_inter, const float *logits_intra,
                                 const float *bias_inter, const float *bias_intra, const int32_t *group_idx,
                                 const int32_t *local_idx, const float *dgate, const int32_t *group_count,
                                 const int32_t *local_count, float dloss, float *dlp, float *dlq, hipStream_t s)
{
    // d(alpha * n * sum_i f_i P_i) / dp[t,i] = alpha * n * (count_i / T) / T
    const float inv_t2 = 1.0f / ((float)d.T * (float)d.T);
    const float ci = dloss * d.alpha * (float)d.n_groups * inv_t2, cq = dloss * d.beta * (float)d.m_local * inv_t2;
    // tokens per workgroup of the tiled kernel: as many as keep its LDS tile within 64 KB; routers too wide even for
    // 64 tokens take the kernel that reads its rows from memory
    const size_t row_bytes = (size_t)((d.n_groups | 1) + (d.m_local | 1)) * sizeof(float);
    int tokens = kThreads;
    while (tokens >= 64 && tokens * row_bytes > 64 * 1024) tokens /= 2;
    if (tokens >= 64 && d.n_groups + d.m_local >= 32) {   // narrower routers: measured faster from memory
        SMILE_LAUNCH(route_backward_tiled_kernel, dim3((d.T + tokens - 1) / tokens), dim3(kThreads),
                           tokens * row_bytes, s, logits_inter, logits_intra, bias_inter, bias_intra, group_idx, local_idx,
                           dgate, group_count, local_count, d.T, d.n_groups, d.m_local, ci, cq, dlp, dlq, tokens);
        return hipGetLastError();
    }
    SMILE_LAUNCH(route_backward_kernel, dim3((d.T + kThreads - 1) / kThreads), dim3(kThreads), 0, s, logits_inter,
                       logits_intra, bias_inter, bias_intra, group_idx, local_idx, dgate, group_count, local_count, d.T,
                       d.n_groups, d.m_local, ci, cq, dlp, dlq);
    return hipGetLastError();
}

hipError_t launch_expert_ffn_backward(const LayerDesc &d, void *workspace, const void *xe,
                                      const int32_t *kept_count, const void *w1, const void *w2, const void *dye,
                                      const void *h_saved, const void *pre_saved, void *dxe, void *dw1, void *dw2,
                                      hipStream_t s)
{
    const BackwardLayout L = backward_workspace_layout(d);
    char *b = static_cast<char *>(workspace);
    void *dpre = b + L.off_dpre, *h_t = b + L.off_h_t;
    void *dpre_t = b + L.off_dpre_t, *dye_t = b + L.off_dye_t, *xe_t = b + L.off_xe_t, *w_t = b + L.off_w_t;
    const int N = d.n_groups * d.m_local, C = d.capacity, dm = d.d_model, F = d.d_ff, Kp = L.k_pad;
    const int act = d.act == SMILE_ACT_RELU ? 1 : 2;
    hipError_t err;
#define SMILE_TRY(call) do { err = (call); if (err != hipSuccess) return err; } while (0)

    // hidden activation and its pre-activation: saved by the forward pass, or recomputed here
    const void *h = h_saved, *pre = pre_saved;
    if (!h) {
        void *h_ws = b + L.off_h, *pre_ws = b + L.off_pre;
        SMILE_TRY(launch_grouped_gemm_nt(d.dtype, GroupedGemm{xe, w1, h_ws, pre_ws, kept_count, N, C, F, dm, act, nullptr, nullptr, nullptr, 0, d.tune}, s));
        h = h_ws;
        pre = pre_ws;
    }
    if (is_half(d.dtype)) {
        // MFMA kernel that reads operands with the contraction index as the slow index: no transposed copies
        const long long cd = (long long)C * dm, cf = (long long)C * F, df = (long long)dm * F;
        // dpre[r,f] = (sum_c dye[r,c] W2[c,f]) * act'(pre[r,f])
        SMILE_TRY(launch_grouped_gemm_t(
            d.dtype, TransposedGemm{dye, w2, dpre, pre, kept_count, nullptr, N, C, F, dm, dm, F, cd, df, cf, false, true, act, d.tune}, s));
        // dW2[c,f] = sum_r dye[r,c] h[r,f]
        SMILE_TRY(launch_grouped_gemm_t(
            d.dtype, TransposedGemm{dye, h, dw2, nullptr, nullptr, kept_count, N, dm, F, C, dm, F, cd, cf, df, true, true, 0, d.tune}, s));
        // dxe[r,k] = sum_f dpre[r,f] W1[f,k]
        SMILE_TRY(launch_grouped_gemm_t(
            d.dtype, TransposedGemm{dpre, w1, dxe, nullptr, kept_count, nullptr, N, C, dm, F, F, dm, cf, df, cd, false, true, 0, d.tune}, s));
        // dW1[f,k] = sum_r dpre[r,f] xe[r,k]
        SMILE_TRY(launch_grouped_gemm_t(
            d.dtype, TransposedGemm{dpre, xe, dw1, nullptr, nullptr, kept_count, N, F, dm, C, F, dm, cf, cd, df, true, true, 0, d.tune}, s));
        return hipSuccess;
    }
    // fp32: the same four products on the x . w^T kernel, with explicitly transposed operands
    // dpre = (dye . W2) * act'(pre)   (W2 is [d][F]: transposed so that the contraction index is contiguous)
    SMILE_TRY(transpose_pad(d.dtype, w2, w_t, nullptr, N, dm, F, dm, s));                      // W2^T [N][F][d]
    {
        GroupedGemm g{dye, w_t, dpre, nullptr, kept_count, N, C, F, dm, 0};
        g.aux = pre;
        g.post = act;
        g.tune = d.tune;
        SMILE_TRY(launch_grouped_gemm_nt(d.dtype, g, s));
    }
    // dW2[c][f] = sum_r dye[r][c] h[r][f]
    SMILE_TRY(transpose_pad(d.dtype, dye, dye_t, kept_count, N, C, dm, Kp, s));                 // [N][d][Kp]
    SMILE_TRY(transpose_pad(d.dtype, h, h_t, kept_count, N, C, F, Kp, s));                      // [N][F][Kp]
    SMILE_TRY(launch_grouped_gemm_nt(d.dtype, GroupedGemm{dye_t, h_t, dw2, nullptr, nullptr, N, dm, F, Kp, 0, nullptr, nullptr, nullptr, 0, d.tune}, s));
    // dxe = dpre . W1   (W1 is [F][d])
    SMILE_TRY(transpose_pad(d.dtype, w1, w_t, nullptr, N, F, dm, F, s));                        // W1^T [N][d][F]
    SMILE_TRY(launch_grouped_gemm_nt(d.dtype, GroupedGemm{dpre, w_t, dxe, nullptr, kept_count, N, C, dm, F, 0, nullptr, nullptr, nullptr, 0, d.tune}, s));
    // dW1[f][k] = sum_r dpre[r][f] xe[r][k]
    SMILE_TRY(transpose_pad(d.dtype, dpre, dpre_t, kept_count, N, C, F, Kp, s));                // [N][F][Kp]
    SMILE_TRY(transpose_pad(d.dtype, xe, xe_t, kept_count, N, C, dm, Kp, s));                   // [N][d][Kp]
    SMILE_TRY(launch_grouped_gemm_nt(d.dtype, GroupedGemm{dpre_t, xe_t, dw1, nullptr, nullptr, N, F, dm, Kp, 0, nullptr, nullptr, nullptr, 0, d.tune}, s));
#undef SMILE_TRY
    return hipSuccess;
}

hipError_t launch_dispatch_backward(const LayerDesc &d, const void *dxe, const int32_t *group_idx,
                                    const int32_t *local_idx, const int32_t *slot, const float *dlp, const float *dlq,
                                    const void *w_inter, const void *w_intra, void *dx, hipStream_t s)
{
    // Tuning::router_grad_mfma = 0 keeps the vector-ALU kernels (tuning / comparison runs)
    if (dispatch_backward_mfma_applies(d) && d.tune.router_grad_mfma != 0)
        return launch_dispatch_backward_mfma(d, dxe, group_idx, local_idx, slot, dlp, dlq, w_inter, w_intra, dx, s);
    const int ppr = d.d_model * elem_size(d.dtype) / 16;
    const int lpr = lanes_per_row(ppr);
    const dim3 grid((d.T + kThreads / lpr - 1) / (kThreads / lpr)), block(kThreads);
    SMILE_DTYPE_SWITCH(d.dtype, SMILE_BWD_LPR_SWITCH(
        lpr, SMILE_LAUNCH((dispatch_backward_kernel<DT, L>), grid, block, 0, s, static_cast<const u32x4 *>(dxe),
                                group_idx, local_idx, slot, dlp, dlq, static_cast<const u32x4 *>(w_inter),
                                static_cast<const u32x4 *>(w_intra), static_cast<u32x4 *>(dx), d.T, ppr, d.n_groups,
                                d.m_local, d.capacity)));
    return hipGetLastError();
}

hipError_t launch_gate_weights_backward(const LayerDesc &d, void *workspace, const void *x, const float *dlp,
                                        const float *dlq, float *dw_inter, float *dw_intra, hipStream_t s)
{
    const BackwardLayout L = backward_workspace_layout(d);
    float *partial = reinterpret_cast<float *>(static_cast<char *>(workspace) + L.off_gw_partial);
    int blocks = L.gw_blocks;
    hipError_t err;
    if (gate_weights_mfma_applies(d) && d.tune.router_grad_mfma != 0) {
        const int tokens = gate_weights_mfma_block_tokens(d, kGwTokens);
        blocks = (d.T + tokens - 1) / tokens;   // <= L.gw_blocks: the partial sums fit the same scratch area
        err = launch_gate_weights_mfma(d, x, dlp, dlq, partial, blocks, tokens, s);
    } else {
        const dim3 grid(L.gw_blocks, (d.d_model + kGwCols - 1) / kGwCols), block(kThreads);
        SMILE_DTYPE_SWITCH(d.dtype, SMILE_LAUNCH(gate_weights_partial_kernel<DT>, grid, block, 0, s, x, dlp, dlq,
                                                       partial, d.T, d.d_model, d.n_groups, d.m_local));
        err = hipGetLastError();
    }
    if (err != hipSuccess) return err;
    const long long total = (long long)(d.n_groups + d.m_local) * d.d_model;
    SMILE_LAUNCH(gate_weights_reduce_kernel, dim3((unsigned)((total + kThreads - 1) / kThreads)), dim3(kThreads), 0, s,
                       partial, dw_inter, dw_intra, blocks, d.d_model, d.n_groups, d.m_local);
    return hipGetLastError();
}

}  // namespace smile
