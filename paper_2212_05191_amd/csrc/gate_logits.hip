// Router logits r(x) = W_r x (Section 2, text before Eq. 1) for the inter router W_p[n,d] and the
// intra router W_q[m,d] (Section 3.2.1: two tied routers reading the same token), computed as one
// skinny product [T,d] x [d,n+m].  n+m is 10-40 in the paper-shaped workloads (up to 257 for the flat
// one-level router the paper compares against), so the kernel is
// bound by the single read of x from HBM; the weights (<= 80 KB) stay in L2.
//
// bf16 / fp16: one workgroup of 4 waves owns RT x 16 token rows; the waves split the K (d) range in
// 64-wide chunks, each feeding v_mfma_f32_16x16x32_bf16 (or _f16) straight from global memory (a lane reads
// 32 contiguous bytes of its row, so 4 lanes cover a full 128-byte line), then the 4 partial
// accumulators are summed through LDS in a fixed order.  Every workgroup re-reads the router
// weights from L2, so RT grows with T (weight traffic / RT) while keeping >= 512 workgroups:
// RT = 1 for the smallest paper-shaped batch (T = 8192), 4 from T = 32768.
// fp32: plain FMA kernel, one thread per (token, column), 4 partial sums.
#include <algorithm>

#include "smile_internal.hpp"

namespace smile {

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kRows = 16;      // token rows per workgroup
constexpr int kWaves = 4;      // K-split factor

// CT = number of 16-column tiles covering the n+m logits columns; RT = 16-row tiles per workgroup.
// E: __bf16 or _Float16.
template <typename E, int CT, int RT>
__global__ __launch_bounds__(64 * kWaves) void gate_logits_half_kernel(
    const E *__restrict__ x, const E *__restrict__ w_inter, const E *__restrict__ w_intra,
    float *__restrict__ logits_inter, float *__restrict__ logits_intra, int T, int d, int n, int m, int col0)
{
    typedef typename Half<E>::vec8 bf16x8;   // 8 elements: one MFMA operand
    __shared__ f32x4 red[kWaves - 1][RT][CT][64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, kg = lane >> 4;
    const int row0 = blockIdx.x * kRows * RT;
    const E *xrow[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) xrow[rt] = x + (size_t)min(row0 + rt * kRows + r, T - 1) * d;

    // the weight row this lane feeds as the B operand of column tile ct (null: padding column)
    const E *wrow[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const int c = col0 + ct * 16 + r;
        wrow[ct] = c < n ? w_inter + (size_t)c * d : (c < n + m ? w_intra + (size_t)(c - n) * d : nullptr);
    }

    f32x4 acc[RT][CT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) acc[rt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};

    const bf16x8 zero = {};
    const int chunks = d / 64;
    const int iters = (chunks - wave + kWaves - 1) / kWaves;   // this wave's chunks: wave, wave + 4, ...
    for (int it = 0; it < iters; ++it) {
        // the contraction index may be visited in any order as long as A and B agree: lane group kg
        // takes k0 + kg*16 + [0,8) for the first MFMA and + [8,16) for the second
        const int k = (wave + it * kWaves) * 64 + kg * 16;
        bf16x8 a0[RT], a1[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            a0[rt] = *reinterpret_cast<const bf16x8 *>(xrow[rt] + k);
            a1[rt] = *reinterpret_cast<const bf16x8 *>(xrow[rt] + k + 8);
        }
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const bf16x8 b0 = wrow[ct] ? *reinterpret_cast<const bf16x8 *>(wrow[ct] + k) : zero;
            const bf16x8 b1 = wrow[ct] ? *reinterpret_cast<const bf16x8 *>(wrow[ct] + k + 8) : zero;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                acc[rt][ct] = Half<E>::mfma_16x16x32(a0[rt], b0, acc[rt][ct]);
                acc[rt][ct] = Half<E>::mfma_16x16x32(a1[rt], b1, acc[rt][ct]);
            }
        }
    }

    if (wave > 0) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) red[wave - 1][rt][ct][lane] = acc[rt][ct];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                f32x4 s = acc[rt][ct];
#pragma unroll
                for (int w = 0; w < kWaves - 1; ++w) s += red[w][rt][ct][lane];
                // accumulator element i of this lane is (row kg*4 + i, column r) of the 16x16 tile
                const int c = col0 + ct * 16 + r;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = row0 + rt * kRows + kg * 4 + i;
                    if (row < T) {
                        if (c < n) logits_inter[(size_t)row * n + c] = s[i];
                        else if (c < n + m) logits_intra[(size_t)row * m + (c - n)] = s[i];
                    }
                }
            }
    }
}

__global__ __launch_bounds__(256) void gate_logits_f32_kernel(
    const float *__restrict__ x, const float *__restrict__ w_inter, const float *__restrict__ w_intra,
    float *__restrict__ logits_inter, float *__restrict__ logits_intra, int T, int d, int n, int m)
{
    const long long id = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int cols = n + m;
    if (id >= (long long)T * cols) return;
    const int t = (int)(id / cols), c = (int)(id - (long long)t * cols);
    const f32x4 *xr = reinterpret_cast<const f32x4 *>(x + (size_t)t * d);
    const f32x4 *wr = reinterpret_cast<const f32x4 *>(c < n ? w_inter + (size_t)c * d : w_intra + (size_t)(c - n) * d);
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < d / 4; ++k) s += xr[k] * wr[k];
    const float v = (s[0] + s[1]) + (s[2] + s[3]);
    if (c < n) logits_inter[(size_t)t * n + c] = v;
    else logits_intra[(size_t)t * m + (c - n)] = v;
}

template <int CT, int RT>
void launch_half_rt(const smile_layer_desc &d, const void *x, const void *w_inter, const void *w_intra,
                    float *logits_inter, float *logits_intra, int col0, hipStream_t s)
{
    const int blocks = (d.T + kRows * RT - 1) / (kRows * RT);
    if (d.dtype == SMILE_DTYPE_BF16)
        SMILE_LAUNCH((gate_logits_half_kernel<__bf16, CT, RT>), dim3(blocks), dim3(64 * kWaves), 0, s,
                           static_cast<const __bf16 *>(x), static_cast<const __bf16 *>(w_inter),
                           static_cast<const __bf16 *>(w_intra), logits_inter, logits_intra, d.T, d.d_model,
                           d.n_groups, d.m_local, col0);
    else
        SMILE_LAUNCH((gate_logits_half_kernel<_Float16, CT, RT>), dim3(blocks), dim3(64 * kWaves), 0, s,
                           static_cast<const _Float16 *>(x), static_cast<const _Float16 *>(w_inter),
                           static_cast<const _Float16 *>(w_intra), logits_inter, logits_intra, d.T, d.d_model,
                           d.n_groups, d.m_local, col0);
}

// columns [col0, col0 + 16*CT)
template <int CT>
void launch_half(const smile_layer_desc &d, const void *x, const void *w_inter, const void *w_intra,
                 float *logits_inter, float *logits_intra, int col0, hipStream_t s)
{
    // the accumulators of RT x CT tiles must stay in registers: RT * CT <= 16
    if (d.T >= 32768 && CT <= 4) launch_half_rt<CT, 4>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s);
    else if (d.T >= 16384) launch_half_rt<CT, 2>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s);
    else launch_half_rt<CT, 1>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s);
}

}  // namespace

hipError_t launch_gate_logits(const smile_layer_desc &d, const void *x, const void *w_inter, const void *w_intra,
                              float *logits_inter, float *logits_intra, hipStream_t s)
{
    const int cols = d.n_groups + d.m_local;
    if (is_half(d.dtype)) {
        // up to 128 columns per pass over x (8 accumulator tiles); wider routers (a flat one-level
        // router over all N experts) take several passes
        for (int col0 = 0; col0 < cols; col0 += 128) {
            switch ((std::min(cols - col0, 128) + 15) / 16) {
            case 1: launch_half<1>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s); break;
            case 2: launch_half<2>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s); break;
            case 3: launch_half<3>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s); break;
            case 4: launch_half<4>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s); break;
            case 5: launch_half<5>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s); break;
            case 6: launch_half<6>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s); break;
            case 7: launch_half<7>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s); break;
            default: launch_half<8>(d, x, w_inter, w_intra, logits_inter, logits_intra, col0, s); break;
            }
        }
    } else {
        const long long total = (long long)d.T * cols;
        SMILE_LAUNCH(gate_logits_f32_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           static_cast<const float *>(x), static_cast<const float *>(w_inter),
                           static_cast<const float *>(w_intra), logits_inter, logits_intra, d.T, d.d_model,
                           d.n_groups, d.m_local);
    }
    return hipGetLastError();
}

}  // namespace smile
