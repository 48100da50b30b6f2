// Device-side pieces shared by the grouped expert GEMM kernels (HIP, gfx950): vector types, the activation
// functions of the epilogues, the kernel argument block, direct-to-LDS load helpers and the LDS bank swizzle.
#pragma once

#include "smile_internal.hpp"

namespace smile {

// Arguments of the 16-bit grouped GEMM kernels (one block for every variant).
struct GemmArgs {
    const void *x;          // [N][C][K]; with x_rows: the token matrix [T][K]
    const void *w;          // [N][Nout][K]
    const void *bias;       // [N][Nout] or null
    void *y;                // [N][C][Nout], or null when only the scattered output is wanted
    const int32_t *kept;    // [N]
    int C, Nout, K;
    int row_tiles, col_tiles, tiles;   // tiles = N*row_tiles*col_tiles
    // Permutation fused into the GEMM (both optional, [N][C] token index of each buffer row):
    const int32_t *x_rows;  // gather: input row r of expert e is x[x_rows[e*C + r]]  (dispatch fused in)
    const int32_t *y_rows;  // scatter: output row also goes to y_tok[y_rows[e*C + r]] * gate  (combine fused in)
    void *y_tok;            // [T][Nout]
    const float *gate;      // [T]
    void *y2 = nullptr;     // [N][C][Nout]: the same product without the activation (DUAL kernels only)
    const void *aux = nullptr;   // [N][C][Nout]: POST kernels multiply the output by act'(aux)
    int N = 0;                   // experts (PERSIST kernels walk the live row tiles of all of them)
};

namespace {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

constexpr int kXcds = 8;

// ACT: 0 none, 1 ReLU, 2 GELU (erff; fp32 path), 3 GELU (rational erfc; 16-bit path)
template <int ACT>
__device__ __forceinline__ float activate(float v)
{
    if constexpr (ACT == 1) return v > 0.f ? v : 0.f;
    else if constexpr (ACT == 2) return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f));
    else if constexpr (ACT == 3) {
        // GELU(v) = v * Phi(v) = max(v,0) - |v| * erfc(|v|/sqrt2)/2, with erfc from the rational
        // approximation 7.1.26 of Abramowitz & Stegun (|error| < 1.5e-7, far below bf16 resolution):
        // erfc(z) = (a1 t + ... + a5 t^5) exp(-z^2), t = 1/(1 + p z).  ~14 VALU ops, no branches.
        const float av = fabsf(v);
        const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, av, 1.0f));
        float poly = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
        poly = fmaf(poly, t, 0.5f * 1.421413741f);
        poly = fmaf(poly, t, 0.5f * -0.284496736f);
        poly = fmaf(poly, t, 0.5f * 0.254829592f);
        const float ex = __builtin_amdgcn_exp2f(v * v * (-0.5f * 1.4426950408889634f));
        return fmaxf(v, 0.f) - av * (poly * t * ex);
    } else return v;
}

// Derivative of the activation at v.  POST 1: ReLU, 2: GELU, d/dv [v Phi(v)] = Phi(v) + v phi(v), with
// Phi from the same rational erfc approximation as above (|error| < 1.5e-7) and phi sharing its exp.
template <int POST>
__device__ __forceinline__ float activate_grad(float v)
{
    if constexpr (POST == 1) return v > 0.f ? 1.f : 0.f;
    else {
        const float av = fabsf(v);
        const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, av, 1.0f));
        float poly = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
        poly = fmaf(poly, t, 0.5f * 1.421413741f);
        poly = fmaf(poly, t, 0.5f * -0.284496736f);
        poly = fmaf(poly, t, 0.5f * 0.254829592f);
        const float ex = __builtin_amdgcn_exp2f(v * v * (-0.5f * 1.4426950408889634f));
        const float q = poly * t * ex;                      // 1 - Phi(|v|)
        const float cdf = v >= 0.f ? 1.0f - q : q;
        return fmaf(v * 0.3989422804014327f, ex, cdf);
    }
}

// ------------------------------------------------------------------------------------ bf16 / fp16: MFMA

// One 16-byte piece (8 elements) times a gate: fp32 product, rounded to the storage type (nearest even) --
// the same arithmetic as the stand-alone combine kernel.
template <typename E>
__device__ __forceinline__ u32x4 scale_x8(u32x4 v, float g)
{
    u32x4 r;
#pragma unroll
    for (int k = 0; k < 4; ++k) r[k] = Half<E>::pack(Half<E>::lo(v[k]) * g, Half<E>::hi(v[k]) * g);
    return r;
}

#define SMILE_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define SMILE_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);   // expcnt, lgkmcnt: no wait
}

// Swizzle term of a row: rows are BK*2 bytes; consecutive rows must land on different banks.
template <int BK, int SWZ>
__device__ __forceinline__ int swz(int row)
{
    if (BK == 64) return SWZ == 0 ? (row & 7) : ((row >> 1) & 7);
    return SWZ == 0 ? ((row >> 1) & 3) : ((row >> 2) & 3);
}

}  // namespace

}  // namespace smile
