// The two skinny products of the backward pass that involve the router weights, on the matrix cores (bf16 storage):
//
//   dx[t,:]   = dxe[row(t),:] + dlp[t,:] . W_p + dlq[t,:] . W_q           (chain rule through Eq. 1 of both levels)
//   dW_p[i,:] = sum_t dlp[t,i] x[t,:],   dW_q[j,:] = sum_t dlq[t,j] x[t,:]
//
// The logit gradients are fp32 and have to stay fp32-accurate, the weights and tokens are bf16.  An fp32 value is
// the exact sum of three bf16 values (8 + 8 + 8 mantissa bits: hi = bf16(v), mid = bf16(v - hi), lo = bf16(v - hi -
// mid)) and a bf16 x bf16 product is exact in the fp32 accumulator of v_mfma_f32_32x32x16_bf16, so three MFMAs per
// 16 logit columns give the fp32 product, at 1/20 of the vector-ALU time of the FMA formulation (which has to
// widen every bf16 weight for every token).
//
// MFMA operand layout used below (same as the expert GEMMs): for D = A . B, lane l supplies 8 consecutive k of
// row (l & 31) of A and of column (l & 31) of B, k-group l >> 5; accumulator element v of lane l is row
// 8*(v/4) + 4*(l>>5) + v%4, column l & 31 of D.
#include "smile_internal.hpp"

namespace smile {

namespace {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef Half<__bf16>::vec8 bf16x8;

constexpr int kThreads = 256;

// v = hi + mid + lo exactly (up to 2^-24 relative), each representable in bf16
__device__ __forceinline__ void split3(float v, __bf16 &hi, __bf16 &mid, __bf16 &lo)
{
    hi = (__bf16)v;
    const float r1 = v - (float)hi;
    mid = (__bf16)r1;
    lo = (__bf16)(r1 - (float)mid);
}

// ------------------------------------------------------------------------------------ dx

// columns of d per workgroup: 256, or 128 when the transposed weights of 256 would leave room for one workgroup per CU
constexpr int dx_cols(int kc) { return kc <= 6 ? 256 : 128; }
constexpr int kDxTokens = 128;   // tokens per workgroup: 32 per wave
constexpr int kDxMaxChunks = 10; // 16-wide chunks of logit columns (inter, then intra) kept in registers

// Row i of an MFMA A tile holds weight column perm(i) of the 32-column tile, so that a lane's 16 accumulator
// elements are 16 CONSECUTIVE columns (16 * (lane >> 5) + v) of its token: two 16-byte pieces per tile.
__device__ __forceinline__ int perm_col(int i) { return 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3); }

// Workgroup = 128 tokens x 256 (or 128) columns.  The weight rows of the column range are transposed into LDS once
// (wt[column][logit column], bf16); each wave splits the logit gradients of its 32 tokens into bf16 planes once
// (registers) and then walks the column range 64 columns at a time: 2*KC*3 MFMAs, add the expert-buffer row, round,
// store; rows are read and written whole (128 bytes of a row per 8 lanes), through a per-wave LDS tile.
template <int KC>
__global__ __launch_bounds__(kThreads) void dispatch_backward_mfma_kernel(
    const __bf16 *__restrict__ dxe, const int32_t *__restrict__ group_idx, const int32_t *__restrict__ local_idx,
    const int32_t *__restrict__ slot, const float *__restrict__ dlp, const float *__restrict__ dlq,
    const __bf16 *__restrict__ w_inter, const __bf16 *__restrict__ w_intra, __bf16 *__restrict__ dx, int T, int d,
    int n, int m, int C, int kp)
{
    constexpr int kDxCols = dx_cols(KC);
    constexpr int RS = KC * 16 + 8;   // row stride of wt in elements (+8: bank spread, keeps 16-byte alignment)
    __shared__ __attribute__((aligned(16))) __bf16 wt[kDxCols * RS];
    __shared__ u32x4 io[kThreads / 64][32 * 9];   // per wave: 32 rows x 8 pieces (+1: bank spread)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c_base = blockIdx.y * kDxCols;

    // ---- weights of this column range, transposed: piece = 8 columns of one weight row
    for (int p = tid; p < KC * 16 * (kDxCols / 8); p += kThreads) {
        const int r = p / (kDxCols / 8), c8 = (p - r * (kDxCols / 8)) * 8;
        const int ri = r < kp * 16 ? r : r - kp * 16;                    // row inside its router
        const bool inter = r < kp * 16;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (c_base + c8 < d && ri < (inter ? n : m))
            v = *reinterpret_cast<const u32x4 *>((inter ? w_inter : w_intra) + (size_t)ri * d + c_base + c8);
        const __bf16 *e = reinterpret_cast<const __bf16 *>(&v);
#pragma unroll
        for (int j = 0; j < 8; ++j) wt[(c8 + j) * RS + r] = e[j];
    }

    // ---- logit gradients of this wave's tokens as bf16 planes: lane = (token lane & 31, k-group lane >> 5)
    const int t = blockIdx.x * kDxTokens + wave * 32 + (lane & 31), g = lane >> 5;
    const bool t_ok = t < T;
    bf16x8 plane[KC][3];
#pragma unroll
    for (int ch = 0; ch < KC; ++ch) {
        const bool inter = ch < kp;
        const int r0 = (inter ? ch : ch - kp) * 16 + 8 * g, cnt = inter ? n : m;
        const float *dl = inter ? dlp + (size_t)t * n : dlq + (size_t)t * m;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float v = (t_ok && r0 + j < cnt) ? dl[r0 + j] : 0.f;
            __bf16 hi, mid, lo;
            split3(v, hi, mid, lo);
            plane[ch][0][j] = hi, plane[ch][1][j] = mid, plane[ch][2][j] = lo;
        }
    }
    const int sl = t_ok ? slot[t] : -1;
    const __bf16 *src = sl >= 0 ? dxe + ((size_t)(group_idx[t] * m + local_idx[t]) * C + sl) * d : nullptr;

    // ---- memory side: 64 columns (128 bytes of a row) at a time, whole rows per instruction.  Lane = (row lane / 8 +
    // 8 it, 16-byte piece lane % 8) for it = 0..3; the rows' source pointers live in the lanes that own the tokens
    // and are fetched from there once.  The tile goes through a per-wave LDS buffer to the lanes that hold the
    // matching accumulators (token lane & 31, columns 32 u + 16 g + 8 h of the 64: piece 4 u + 2 g + h) and back.
    const int mrow = lane >> 3, mpiece = lane & 7;
    const __bf16 *msrc[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const unsigned long long p = reinterpret_cast<unsigned long long>(src);
        const unsigned lo = __shfl((unsigned)p, mrow + 8 * it, 64), hi = __shfl((unsigned)(p >> 32), mrow + 8 * it, 64);
        msrc[it] = reinterpret_cast<const __bf16 *>(((unsigned long long)hi << 32) | lo);
    }
    const int t_wave = blockIdx.x * kDxTokens + wave * 32;   // first token of the wave
    u32x4 *tile = io[wave];
    __syncthreads();

    const int arow = perm_col(lane & 31);
    u32x4 in[4];
    auto fetch = [&](int c0) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            in[it] = u32x4{0u, 0u, 0u, 0u};
            if (msrc[it]) in[it] = *reinterpret_cast<const u32x4 *>(msrc[it] + c0 + mpiece * 8);
        }
    };
    if (c_base < d) fetch(c_base);
#pragma unroll 1
    for (int cs = 0; cs < kDxCols / 64; ++cs) {
        const int c0 = c_base + cs * 64;
        if (c0 >= d) break;   // uniform (d is a multiple of 64)
#pragma unroll
        for (int it = 0; it < 4; ++it) tile[(mrow + 8 * it) * 9 + mpiece] = in[it];
        if (c0 + 64 < d && cs + 1 < kDxCols / 64) fetch(c0 + 64);   // in flight during the MFMAs
        f32x16 acc[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[u][v] = 0.f;
#pragma unroll
            for (int ch = 0; ch < KC; ++ch) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&wt[(cs * 64 + u * 32 + arow) * RS + ch * 16 + 8 * g]);
#pragma unroll
                for (int p = 0; p < 3; ++p) acc[u] = Half<__bf16>::mfma_32x32x16(a, plane[ch][p], acc[u]);
            }
        }
        // lane holds columns c0 + 32 u + 16 g + 0..15 of token (lane & 31): add the expert-buffer row, round once
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                u32x4 *cell = &tile[(lane & 31) * 9 + 4 * u + 2 * g + h];
                const u32x4 v = *cell;
                u32x4 o;
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    o[k] = Half<__bf16>::pack(Half<__bf16>::lo(v[k]) + acc[u][8 * h + 2 * k],
                                              Half<__bf16>::hi(v[k]) + acc[u][8 * h + 2 * k + 1]);
                *cell = o;
            }
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int row = mrow + 8 * it;
            const u32x4 o = tile[row * 9 + mpiece];
            if (t_wave + row < T) *reinterpret_cast<u32x4 *>(dx + (size_t)(t_wave + row) * d + c0 + mpiece * 8) = o;
        }
    }
}

template <int KC>
hipError_t launch_dx(const smile_layer_desc &d, const void *dxe, const int32_t *group_idx, const int32_t *local_idx,
                     const int32_t *slot, const float *dlp, const float *dlq, const void *w_inter, const void *w_intra,
                     void *dx, int kp, hipStream_t s)
{
    const dim3 grid((d.T + kDxTokens - 1) / kDxTokens, (d.d_model + dx_cols(KC) - 1) / dx_cols(KC)), block(kThreads);
    SMILE_LAUNCH(dispatch_backward_mfma_kernel<KC>, grid, block, 0, s, static_cast<const __bf16 *>(dxe), group_idx,
                       local_idx, slot, dlp, dlq, static_cast<const __bf16 *>(w_inter),
                       static_cast<const __bf16 *>(w_intra), static_cast<__bf16 *>(dx), d.T, d.d_model, d.n_groups,
                       d.m_local, d.capacity, kp);
    return hipGetLastError();
}


// ------------------------------------------------------------------------------------ dW_p, dW_q

constexpr int kGwCb = 256;         // columns of x per workgroup
constexpr int kGwMaxRowTiles = 5;  // 32-wide tiles of logit columns (inter and intra concatenated)
typedef short s16x4 __attribute__((ext_vector_type(4)));

// partial[b][r][c] = sum over the tokens of block b of dl[t][r] * x[t][c], r over the n + m logit columns (dlp first,
// then dlq).  D = A . B with A = x^T (row = column c of x, k = token) and B = the bf16 planes of dl (column = logit
// column r, k = token).  Both are stored token-major, i.e. with k as the slow index:
//   * the x tile (64 tokens x 256 columns) is written to LDS as it is in memory and its fragments are fetched with
//     the transposing LDS read (ds_read_b64_tr_b16: within 16 lanes, lane 4a+b receives element b of the 8-byte
//     rows addressed by lanes a, a+4, a+8, a+12; so lane i addresses token i/4 and the 4-column block i%4 and ends
//     up with 4 consecutive tokens of its own column).  A token row's 16-byte pieces are rotated by 4*(token&3)
//     positions so that the 8 token rows a wave touches per read spread over all banks;
//   * the planes are written transposed, pl[plane][r][token], by the threads that split the values.
// The next tile's global loads are in flight while the current one is multiplied.  Tokens are summed in a fixed
// order and the blocks are added by the reduce kernel in index order: deterministic.
template <int RT>
__global__ __launch_bounds__(kThreads) void gate_weights_mfma_kernel(
    const __bf16 *__restrict__ x, const float *__restrict__ dlp, const float *__restrict__ dlq,
    float *__restrict__ partial, int T, int d, int n, int m, int tokens_per_block)
{
    constexpr int PPK = kGwCb / 8;   // 16-byte pieces per token row of the tile
    constexpr int PS = 64 + 8;       // row stride of a plane in elements (+8: bank spread, keeps 16-byte alignment)
    constexpr int XP = 64 * PPK / kThreads;   // x pieces per thread
    constexpr int DLV = (64 * RT * 32 + kThreads - 1) / kThreads;   // dl values per thread (upper bound)
    __shared__ u32x4 xs[64 * PPK];
    __shared__ __attribute__((aligned(16))) __bf16 pl[3][RT * 32][PS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c_base = blockIdx.y * kGwCb, R = n + m;
    const int t_begin = blockIdx.x * tokens_per_block, t_end = min(T, t_begin + tokens_per_block);

    // rows of the planes beyond the n + m logit columns stay zero
    for (int i = tid; i < 3 * RT * 32 * PS / 8; i += kThreads) reinterpret_cast<u32x4 *>(&pl[0][0][0])[i] = u32x4{0u, 0u, 0u, 0u};

    f32x16 acc[2][RT];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[u][rt][v] = 0.f;

    // fragment addressing of the x tile: lane = 16 tg + 4 tj + ta addresses token 8 (tg / 2) + tj (+4: second read,
    // +16 per k-step) and the 4 columns 16 (tg % 2) + 4 ta of its 32-column tile
    const int tg = lane >> 4, tj = (lane >> 2) & 3, ta = lane & 3;
    const int tk0 = 8 * (tg >> 1) + tj;
    int xoff[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int col = (wave * 2 + u) * 32 + 16 * (tg & 1) + 4 * ta;
        xoff[u] = (tk0 * PPK + ((col >> 3) + 4 * tj) % PPK) * 16 + (col & 4) * 2;
    }

    u32x4 xr[XP];
    float dv[DLV];
    // (index arithmetic is redone from an opaque copy of the thread id wherever it is needed, so that the compiler
    // does not keep two dozen precomputed addresses in registers across the token loop)
    auto opaque_tid = [&]() {
        int v = tid;
        asm volatile("" : "+v"(v));
        return v;
    };
    auto prefetch = [&](int t0) {
        const int tid = opaque_tid();
#pragma unroll
        for (int q = 0; q < XP; ++q) {
            const int id = tid + q * kThreads, k = id / PPK, p = id - k * PPK;
            xr[q] = u32x4{0u, 0u, 0u, 0u};
            if (t0 + k < t_end && c_base + p * 8 < d)
                xr[q] = *reinterpret_cast<const u32x4 *>(x + (size_t)(t0 + k) * d + c_base + p * 8);
        }
#pragma unroll
        for (int q = 0; q < DLV; ++q) {
            const int id = tid + q * kThreads, k = id / R, r = id - k * R;
            dv[q] = 0.f;
            if (k < 64 && t0 + k < t_end) dv[q] = r < n ? dlp[(size_t)(t0 + k) * n + r] : dlq[(size_t)(t0 + k) * m + r - n];
        }
    };
    prefetch(t_begin);
    for (int t0 = t_begin; t0 < t_end; t0 += 64) {
        __syncthreads();   // the previous tile has been read by every wave (first pass: the zero fill is complete)
        const int tid = opaque_tid();
#pragma unroll
        for (int q = 0; q < XP; ++q) {
            const int id = tid + q * kThreads, k = id / PPK, p = id - k * PPK;
            xs[k * PPK + (p + 4 * (k & 3)) % PPK] = xr[q];
        }
#pragma unroll
        for (int q = 0; q < DLV; ++q) {
            const int id = tid + q * kThreads, k = id / R, r = id - k * R;
            if (k < 64) {
                __bf16 hi, mid, lo;
                split3(dv[q], hi, mid, lo);
                pl[0][r][k] = hi, pl[1][r][k] = mid, pl[2][r][k] = lo;
            }
        }
        __syncthreads();
        if (t0 + 64 < t_end) prefetch(t0 + 64);
        const char *xb = reinterpret_cast<const char *>(xs);
#pragma unroll 1
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 a[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const char *p = xb + xoff[u] + kk * 16 * PPK * 16;
                struct { s16x4 lo, hi; } t;
                t.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
                t.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p + 4 * PPK * 16));
                a[u] = __builtin_bit_cast(bf16x8, t);
            }
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    const bf16x8 b = *reinterpret_cast<const bf16x8 *>(&pl[p][rt * 32 + (lane & 31)][16 * kk + 8 * (lane >> 5)]);
#pragma unroll
                    for (int u = 0; u < 2; ++u) acc[u][rt] = Half<__bf16>::mfma_32x32x16(a[u], b, acc[u][rt]);
                }
        }
    }

    // accumulator element v of a lane: logit column rt*32 + (lane & 31), x column 8*(v/4) + 4*(lane>>5) + v%4
    float *out = partial + (size_t)blockIdx.x * R * d;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int r = rt * 32 + (lane & 31);
        if (r >= R) continue;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = c_base + (wave * 2 + u) * 32 + 8 * q + 4 * (lane >> 5);
                if (c < d)
                    *reinterpret_cast<f32x4 *>(out + (size_t)r * d + c) =
                        f32x4{acc[u][rt][4 * q], acc[u][rt][4 * q + 1], acc[u][rt][4 * q + 2], acc[u][rt][4 * q + 3]};
            }
    }
}

template <int RT>
hipError_t launch_gw(const smile_layer_desc &d, const void *x, const float *dlp, const float *dlq, float *partial,
                     int blocks, int tokens_per_block, hipStream_t s)
{
    const dim3 grid(blocks, (d.d_model + kGwCb - 1) / kGwCb), block(kThreads);
    SMILE_LAUNCH(gate_weights_mfma_kernel<RT>, grid, block, 0, s, static_cast<const __bf16 *>(x), dlp, dlq, partial,
                       d.T, d.d_model, d.n_groups, d.m_local, tokens_per_block);
    return hipGetLastError();
}

}  // namespace

bool dispatch_backward_mfma_applies(const smile_layer_desc &d)
{
    const int kc = (d.n_groups + 15) / 16 + (d.m_local + 15) / 16;
    return d.dtype == SMILE_DTYPE_BF16 && kc <= kDxMaxChunks && d.d_model % 8 == 0;
}

hipError_t launch_dispatch_backward_mfma(const smile_layer_desc &d, const void *dxe, const int32_t *group_idx,
                                         const int32_t *local_idx, const int32_t *slot, const float *dlp,
                                         const float *dlq, const void *w_inter, const void *w_intra, void *dx,
                                         hipStream_t s)
{
    const int kp = (d.n_groups + 15) / 16, kc = kp + (d.m_local + 15) / 16;
#define SMILE_DX_CASE(K) \
    case K: return launch_dx<K>(d, dxe, group_idx, local_idx, slot, dlp, dlq, w_inter, w_intra, dx, kp, s);
    switch (kc) {
        SMILE_DX_CASE(2) SMILE_DX_CASE(3) SMILE_DX_CASE(4) SMILE_DX_CASE(5) SMILE_DX_CASE(6) SMILE_DX_CASE(7)
        SMILE_DX_CASE(8) SMILE_DX_CASE(9) SMILE_DX_CASE(10)
    default: return hipErrorInvalidValue;
    }
#undef SMILE_DX_CASE
}

bool gate_weights_mfma_applies(const smile_layer_desc &d)
{
    return d.dtype == SMILE_DTYPE_BF16 && (d.n_groups + d.m_local + 31) / 32 <= kGwMaxRowTiles && d.d_model % 8 == 0;
}

// Tokens per partial-sum block: a multiple of `granule` (the block size the workspace was laid out for, so that
// fewer, larger blocks always fit), grown until the grid is down to about four workgroups per CU.
int gate_weights_mfma_block_tokens(const smile_layer_desc &d, int granule)
{
    const long long col_blocks = (d.d_model + kGwCb - 1) / kGwCb;
    int k = 1;
    while (k < 8 && ((long long)d.T / (granule * 2 * k)) * col_blocks >= 1024) k *= 2;
    return granule * k;
}

hipError_t launch_gate_weights_mfma(const smile_layer_desc &d, const void *x, const float *dlp, const float *dlq,
                                    float *partial, int blocks, int tokens_per_block, hipStream_t s)
{
    switch ((d.n_groups + d.m_local + 31) / 32) {
    case 1: return launch_gw<1>(d, x, dlp, dlq, partial, blocks, tokens_per_block, s);
    case 2: return launch_gw<2>(d, x, dlp, dlq, partial, blocks, tokens_per_block, s);
    case 3: return launch_gw<3>(d, x, dlp, dlq, partial, blocks, tokens_per_block, s);
    case 4: return launch_gw<4>(d, x, dlp, dlq, partial, blocks, tokens_per_block, s);
    case 5: return launch_gw<5>(d, x, dlp, dlq, partial, blocks, tokens_per_block, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace smile
