// Expert FFN E_e of Eq. 3 (Section 4.1: hidden -> intermediate -> hidden with GELU) for all N
// experts at once, as two grouped "NT" GEMMs with device-resident, ragged row counts:
//
//   h [e] = act(xe[e] . w1[e]^T + b1[e])      rows r < kept[e],  xe[e]: [C,d],  w1[e]: [F,d]
//   ye[e] =      h[e] . w2[e]^T + b2[e]                          h[e]:  [C,F],  w2[e]: [d,F]
//
// Both operands of either product are K-contiguous, which is exactly the MFMA register layout
// (8 consecutive k per lane), so tiles go global -> LDS -> registers as 16-byte pieces with no
// transposition anywhere.
//
// bf16 kernel (the hot kernel of the layer): one workgroup computes a BM x BN tile of one expert
// with v_mfma_f32_32x32x16_bf16, fp32 accumulators, K stepped in 64-element (128-byte) slabs that
// are double-buffered in LDS: the global loads of slab k+1 are issued before the MFMAs of slab k
// and written to the other LDS buffer after them, one barrier per slab.  LDS rows are 128 bytes;
// the 16-byte piece index is XOR-ed with (row & 7) so that the 32 rows a wave reads for one MFMA
// operand fall on distinct banks.  The weight tile is the MFMA "A" operand and the token tile the
// "B" operand, so a lane ends up holding 4 consecutive output columns of one token row and the
// epilogue (bias, activation, round to bf16) stores 8 bytes at a time.
//
// The grid covers every (expert, column tile, row tile); tiles whose first row is >= kept[e] exit
// at once, so no host synchronisation on the routing result is needed.  Workgroup ids are dealt
// round-robin to the 8 XCDs by the hardware; the id is remapped so that each XCD (own L2) works
// on a contiguous range of tiles: the row tiles sharing a weight tile and the column tiles
// sharing a token tile then meet in the same L2.
//
// fp32 kernel (small / reference-precision configurations): classic LDS-tiled FMA GEMM.
#include <cstdlib>

#include "smile_internal.hpp"

namespace smile {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kXcds = 8;

template <int ACT>
__device__ __forceinline__ float activate(float v)
{
    if constexpr (ACT == 1) return v > 0.f ? v : 0.f;
    else if constexpr (ACT == 2) return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f));
    else return v;
}

// ------------------------------------------------------------------------------------ bf16 / MFMA

struct GemmArgs {
    const void *x;          // [N][C][K]
    const void *w;          // [N][Nout][K]
    const void *bias;       // [N][Nout] or null
    void *y;                // [N][C][Nout]
    const int32_t *kept;    // [N]
    int C, Nout, K;
    int row_tiles, col_tiles, tiles;   // tiles = N*row_tiles*col_tiles
};

template <int BM, int BN, int WGM, int WGN, int ACT>
__global__ __launch_bounds__(WGM *WGN * 64) void grouped_gemm_nt_bf16_kernel(GemmArgs a)
{
    constexpr int NT = WGM * WGN * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;        // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;          // MFMA tiles per wave
    constexpr int XP = BM * 8 / NT, WP = BN * 8 / NT;  // 16-byte pieces per thread per slab
    static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "wave tile must be a multiple of 32");
    static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0 && NT % 8 == 0, "slab must divide over the threads");

    __shared__ u32x4 lds_x[2][BM * 8];
    __shared__ u32x4 lds_w[2][BN * 8];

    // ---- which tile (XCD-aware remap of the hardware's round-robin workgroup placement)
    const int per_xcd = (a.tiles + kXcds - 1) / kXcds;
    const int lid = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (lid >= a.tiles) return;
    const int per_expert = a.row_tiles * a.col_tiles;
    const int e = lid / per_expert;
    const int rem = lid - e * per_expert;
    const int ct = rem / a.row_tiles, rt = rem - ct * a.row_tiles;
    const int rows = min(a.kept[e], a.C);   // never trust a count beyond the buffer
    if (rt * BM >= rows) return;

    const int K = a.K, Nout = a.Nout;
    const __bf16 *X = static_cast<const __bf16 *>(a.x) + (size_t)e * a.C * K;
    const __bf16 *W = static_cast<const __bf16 *>(a.w) + (size_t)e * Nout * K;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WGM, wn = wave / WGM;

    // ---- global -> LDS: thread moves piece (tid & 7) of rows (tid >> 3) + i * NT/8
    const int piece = tid & 7, prow = tid >> 3;
    const __bf16 *xg[XP];
    const __bf16 *wg[WP];
    int xl[XP], wl[WP];
#pragma unroll
    for (int i = 0; i < XP; ++i) {
        const int r = prow + i * (NT / 8);
        xg[i] = X + (size_t)min(rt * BM + r, rows - 1) * K + piece * 8;   // rows past the end re-read the last one
        xl[i] = r * 8 + (piece ^ (r & 7));
    }
#pragma unroll
    for (int i = 0; i < WP; ++i) {
        const int r = prow + i * (NT / 8);
        wg[i] = W + (size_t)min(ct * BN + r, Nout - 1) * K + piece * 8;
        wl[i] = r * 8 + (piece ^ (r & 7));
    }

    // ---- LDS -> MFMA operands: lane reads row (lane & 31), pieces 2*kk + (lane >> 5)
    const int frow = lane & 31, fhi = lane >> 5, fsw = lane & 7;
    const int xbase = (wm * WM + frow) * 8, wbase = (wn * WN + frow) * 8;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    u32x4 xr[XP], wr[WP];
#pragma unroll
    for (int i = 0; i < XP; ++i) xr[i] = *reinterpret_cast<const u32x4 *>(xg[i]);
#pragma unroll
    for (int i = 0; i < WP; ++i) wr[i] = *reinterpret_cast<const u32x4 *>(wg[i]);
#pragma unroll
    for (int i = 0; i < XP; ++i) lds_x[0][xl[i]] = xr[i];
#pragma unroll
    for (int i = 0; i < WP; ++i) lds_w[0][wl[i]] = wr[i];
    __syncthreads();

    const int slabs = K / 64;
    for (int kt = 0; kt < slabs; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < slabs;
        if (more) {
            const int k0 = (kt + 1) * 64;
#pragma unroll
            for (int i = 0; i < XP; ++i) xr[i] = *reinterpret_cast<const u32x4 *>(xg[i] + k0);
#pragma unroll
            for (int i = 0; i < WP; ++i) wr[i] = *reinterpret_cast<const u32x4 *>(wg[i] + k0);
        }
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            bf16x8 xf[TM], wf[TN];
            const int p = (2 * kk + fhi) ^ fsw;
#pragma unroll
            for (int j = 0; j < TM; ++j) xf[j] = __builtin_bit_cast(bf16x8, lds_x[cur][xbase + j * 256 + p]);
#pragma unroll
            for (int i = 0; i < TN; ++i) wf[i] = __builtin_bit_cast(bf16x8, lds_w[cur][wbase + i * 256 + p]);
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
#pragma unroll
            for (int i = 0; i < XP; ++i) lds_x[cur ^ 1][xl[i]] = xr[i];
#pragma unroll
            for (int i = 0; i < WP; ++i) lds_w[cur ^ 1][wl[i]] = wr[i];
        }
        __syncthreads();
    }

    // ---- epilogue: accumulator element v of a lane is (column 8*(v/4) + 4*(lane/32) + v%4, row lane%32)
    __bf16 *Y = static_cast<__bf16 *>(a.y) + (size_t)e * a.C * Nout;
    const __bf16 *bias = a.bias ? static_cast<const __bf16 *>(a.bias) + (size_t)e * Nout : nullptr;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int row = rt * BM + wm * WM + j * 32 + frow;
        if (row >= rows) continue;
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = ct * BN + wn * WN + i * 32 + 8 * q + 4 * fhi;
                if (col >= Nout) continue;
                bf16x4 out;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    float f = acc[i][j][4 * q + v];
                    if (bias) f += (float)bias[col + v];
                    out[v] = (__bf16)activate<ACT>(f);
                }
                *reinterpret_cast<bf16x4 *>(Y + (size_t)row * Nout + col) = out;
            }
        }
    }
}

template <int BM, int BN, int WGM, int WGN>
hipError_t launch_bf16_tile(GemmArgs a, int N, int act, hipStream_t s)
{
    a.row_tiles = (a.C + BM - 1) / BM;
    a.col_tiles = (a.Nout + BN - 1) / BN;
    a.tiles = N * a.row_tiles * a.col_tiles;
    const int per_xcd = (a.tiles + kXcds - 1) / kXcds;
    const dim3 grid(per_xcd * kXcds), block(WGM * WGN * 64);
    if (act == 0) hipLaunchKernelGGL((grouped_gemm_nt_bf16_kernel<BM, BN, WGM, WGN, 0>), grid, block, 0, s, a);
    else if (act == 1) hipLaunchKernelGGL((grouped_gemm_nt_bf16_kernel<BM, BN, WGM, WGN, 1>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((grouped_gemm_nt_bf16_kernel<BM, BN, WGM, WGN, 2>), grid, block, 0, s, a);
    return hipGetLastError();
}

// Tile shapes: id -> (BM, BN, waves along M, waves along N)
hipError_t launch_bf16(const GemmArgs &a, int N, int act, int tile, hipStream_t s)
{
    switch (tile) {
    case 0: return launch_bf16_tile<128, 128, 2, 2>(a, N, act, s);
    case 1: return launch_bf16_tile<256, 128, 2, 2>(a, N, act, s);
    case 2: return launch_bf16_tile<128, 256, 2, 2>(a, N, act, s);
    case 3: return launch_bf16_tile<256, 256, 2, 2>(a, N, act, s);
    case 4: return launch_bf16_tile<256, 256, 2, 4>(a, N, act, s);
    case 5: return launch_bf16_tile<64, 128, 1, 4>(a, N, act, s);
    default: return hipErrorInvalidValue;
    }
}

// Heuristic tile choice: the largest tile that still gives every CU at least ~2 tiles of real work.
int pick_tile(int N, int C, int Nout)
{
    if (const char *env = std::getenv("SMILE_FFN_TILE")) return std::atoi(env);
    (void)N; (void)C; (void)Nout;
    return 0;
}

// ------------------------------------------------------------------------------------ fp32 / FMA

template <int ACT>
__global__ __launch_bounds__(256) void grouped_gemm_nt_f32_kernel(
    const float *__restrict__ x, const float *__restrict__ w, const float *__restrict__ bias,
    float *__restrict__ y, const int32_t *__restrict__ kept, int C, int Nout, int K, int row_tiles, int col_tiles)
{
    constexpr int BT = 64, BK = 16;
    __shared__ float xs[BK][BT + 4];
    __shared__ float wsh[BK][BT + 4];

    const int per_expert = row_tiles * col_tiles;
    const int e = blockIdx.x / per_expert;
    const int rem = blockIdx.x - e * per_expert;
    const int ct = rem / row_tiles, rt = rem - ct * row_tiles;
    const int rows = min(kept[e], C);
    if (rt * BT >= rows) return;

    const float *X = x + (size_t)e * C * K;
    const float *W = w + (size_t)e * Nout * K;
    const int tid = threadIdx.x;
    const int lr = tid >> 2, lk = (tid & 3) * 4;            // loader: row lr, 4 floats at k offset lk
    const int xrow = min(rt * BT + lr, rows - 1), wrow = min(ct * BT + lr, Nout - 1);
    const int ty = tid >> 4, tx = tid & 15;                  // compute: rows ty*4.., cols tx*4..

    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += BK) {
        f32x4 xv = {0.f, 0.f, 0.f, 0.f}, wv = {0.f, 0.f, 0.f, 0.f};
        if (k0 + lk < K) {
            xv = *reinterpret_cast<const f32x4 *>(X + (size_t)xrow * K + k0 + lk);
            wv = *reinterpret_cast<const f32x4 *>(W + (size_t)wrow * K + k0 + lk);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) { xs[lk + i][lr] = xv[i]; wsh[lk + i][lr] = wv[i]; }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float xa[4], wb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { xa[i] = xs[k][ty * 4 + i]; wb[i] = wsh[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(xa[i], wb[j], acc[i][j]);
        }
        __syncthreads();
    }
    float *Y = y + (size_t)e * C * Nout;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = rt * BT + ty * 4 + i;
        if (row >= rows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = ct * BT + tx * 4 + j;
            if (col >= Nout) continue;
            float f = acc[i][j];
            if (bias) f += bias[(size_t)e * Nout + col];
            Y[(size_t)row * Nout + col] = activate<ACT>(f);
        }
    }
}

hipError_t launch_f32(const float *x, const float *w, const float *bias, float *y, const int32_t *kept, int N,
                      int C, int Nout, int K, int act, hipStream_t s)
{
    const int row_tiles = (C + 63) / 64, col_tiles = (Nout + 63) / 64;
    const dim3 grid(N * row_tiles * col_tiles), block(256);
    if (act == 0)
        hipLaunchKernelGGL(grouped_gemm_nt_f32_kernel<0>, grid, block, 0, s, x, w, bias, y, kept, C, Nout, K, row_tiles, col_tiles);
    else if (act == 1)
        hipLaunchKernelGGL(grouped_gemm_nt_f32_kernel<1>, grid, block, 0, s, x, w, bias, y, kept, C, Nout, K, row_tiles, col_tiles);
    else
        hipLaunchKernelGGL(grouped_gemm_nt_f32_kernel<2>, grid, block, 0, s, x, w, bias, y, kept, C, Nout, K, row_tiles, col_tiles);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_expert_ffn_up(const smile_layer_desc &d, const Workspace &ws, const void *xe,
                                const int32_t *kept_count, const void *w1, const void *b1, hipStream_t s)
{
    const int N = d.n_groups * d.m_local;
    const int act = d.act == SMILE_ACT_RELU ? 1 : 2;
    if (d.dtype == SMILE_DTYPE_BF16) {
        GemmArgs g{xe, w1, b1, ws.hidden, kept_count, d.capacity, d.d_ff, d.d_model, 0, 0, 0};
        return launch_bf16(g, N, act, pick_tile(N, d.capacity, d.d_ff), s);
    }
    return launch_f32(static_cast<const float *>(xe), static_cast<const float *>(w1),
                      static_cast<const float *>(b1), static_cast<float *>(ws.hidden), kept_count, N, d.capacity,
                      d.d_ff, d.d_model, act, s);
}

hipError_t launch_expert_ffn_down(const smile_layer_desc &d, const Workspace &ws, const int32_t *kept_count,
                                  const void *w2, const void *b2, void *ye, hipStream_t s)
{
    const int N = d.n_groups * d.m_local;
    if (d.dtype == SMILE_DTYPE_BF16) {
        GemmArgs g{ws.hidden, w2, b2, ye, kept_count, d.capacity, d.d_model, d.d_ff, 0, 0, 0};
        return launch_bf16(g, N, 0, pick_tile(N, d.capacity, d.d_model), s);
    }
    return launch_f32(static_cast<const float *>(ws.hidden), static_cast<const float *>(w2),
                      static_cast<const float *>(b2), static_cast<float *>(ye), kept_count, N, d.capacity,
                      d.d_model, d.d_ff, 0, s);
}

}  // namespace smile
