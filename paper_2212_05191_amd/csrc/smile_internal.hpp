// Internal declarations shared by the translation units of libsmile (HIP, gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>

#include "smile.h"

namespace smile {

// bytes per element of a storage type, and whether it is one of the 16-bit types of the MFMA kernels
inline int elem_size(int dtype) { return dtype == SMILE_DTYPE_F32 ? 4 : 2; }
inline bool is_half(int dtype) { return dtype == SMILE_DTYPE_BF16 || dtype == SMILE_DTYPE_F16; }

// The two 16-bit storage types: element, 8-element MFMA operand, the MFMA instructions, and conversion of a
// 32-bit word holding two elements to and from fp32 (round to nearest even).
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float mfma_f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float mfma_f32x16;

template <typename E>
struct Half;

template <>
struct Half<__bf16> {
    typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 vec8;
    __device__ static __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }   // upper half of an fp32
    __device__ static __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
    __device__ static __forceinline__ uint32_t pack(float a, float b)
    {
        typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 vec2;
        vec2 p;
        p[0] = (__bf16)a;
        p[1] = (__bf16)b;
        return __builtin_bit_cast(uint32_t, p);
    }
    __device__ static __forceinline__ mfma_f32x16 mfma_32x32x16(vec8 a, vec8 b, mfma_f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ mfma_f32x4 mfma_16x16x32(vec8 a, vec8 b, mfma_f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};

template <>
struct Half<_Float16> {
    typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 vec8;
    typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 vec2;
    __device__ static __forceinline__ float lo(uint32_t w) { return (float)__builtin_bit_cast(vec2, w)[0]; }
    __device__ static __forceinline__ float hi(uint32_t w) { return (float)__builtin_bit_cast(vec2, w)[1]; }
    __device__ static __forceinline__ uint32_t pack(float a, float b)
    {
        vec2 p;
        p[0] = (_Float16)a;
        p[1] = (_Float16)b;
        return __builtin_bit_cast(uint32_t, p);
    }
    __device__ static __forceinline__ mfma_f32x16 mfma_32x32x16(vec8 a, vec8 b, mfma_f32x16 c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ mfma_f32x4 mfma_16x16x32(vec8 a, vec8 b, mfma_f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};

// tokens handled by one workgroup of the routing kernels
constexpr int kRouteBlock = 256;

// in-block rank given to a token dropped at the first hop (group capacity): any block offset added to
// it stays at or above every legal capacity and below 2^31 (T <= 2^30 is enforced with a group capacity)
constexpr int32_t kHop1Dropped = 1 << 30;

struct Workspace {
    // routing: per-block histograms turned into exclusive block offsets by the scan kernel
    int32_t *block_expert_hist;   // [B][N]
    int32_t *block_group_hist;    // [B][n] per group, then [B][m] per local index
    float *block_p_sum;           // [B][n]
    float *block_q_sum;           // [B][m]
    int32_t *rank_in_block;       // [T] rank among earlier tokens of the same block with the same expert
    int32_t *pos_in_block;        // [T] ... with the same group
    int32_t *slot_token;          // [N][C] token sitting in each expert-buffer row (rows < kept only)
    // expert FFN: hidden activation between the two grouped GEMMs, ctx dtype
    void *hidden;                 // [N][C][F]
};

struct Layout {
    size_t off_block_expert_hist, off_block_group_hist, off_block_p_sum, off_block_q_sum, off_rank_in_block,
        off_pos_in_block, off_slot_token, off_hidden, total;
    int32_t route_blocks;
};

Layout workspace_layout(const smile_layer_desc &d);

// Eq. 4 on one wave (64 lanes): lane-strided serial sums, fixed butterfly.  Shared by the stand-alone
// loss kernel and the routing scan kernel so that both give identical bits.
__device__ __forceinline__ void aux_loss_wave(const int32_t *group_count, const int32_t *local_count,
                                              const float *p_sum, const float *q_sum, int T, int n, int m,
                                              float alpha, float beta, float *out3)
{
    const int lane = threadIdx.x & 63;
    const float inv_t = 1.0f / (float)T;
    float a = 0.f, b = 0.f;
    for (int i = lane; i < n; i += 64) a += ((float)group_count[i] * inv_t) * (p_sum[i] * inv_t);
    for (int j = lane; j < m; j += 64) b += ((float)local_count[j] * inv_t) * (q_sum[j] * inv_t);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        a += __shfl_xor(a, off, 64);
        b += __shfl_xor(b, off, 64);
    }
    a *= (float)n;
    b *= (float)m;
    if (lane == 0) {
        out3[0] = a;
        out3[1] = b;
        out3[2] = alpha * a + beta * b;
    }
}

// Sum over blocks of one column of per-block partial sums, in a fixed order: lane l adds blocks
// l, l+64, ... serially, then a fixed butterfly over the wave.
__device__ __forceinline__ float wave_sum_column(const float *__restrict__ part, int B, int stride, int col)
{
    float s = 0.f;
    for (int b = __lane_id(); b < B; b += 64) s += part[(size_t)b * stride + col];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    return s;
}

// Walk of a persistent workgroup over the LIVE tiles of a grouped GEMM whose groups (experts) have ragged,
// device-resident row counts: row tile rt of group e is live when rt*BM < rows[e].  The grid is one workgroup per
// slot the chip can hold; tiles of empty buffer rows are never scheduled (with a plain grid each of them is a
// workgroup that has to wait for a free slot before it can exit).  Every wave finds the live row tiles for
// itself, in registers, with no LDS and no extra launch: lane c holds the live row tiles of groups 64c .. 64c+63
// (hence N <= 4096) and the group of a ticket is located with two ballots.  Tickets are ordered (group, column
// tile, row tile) so that the row tiles sharing a weight tile and the column tiles sharing a token tile run
// side by side.  The 8 XCDs (own L2 each; workgroup ids are dealt round-robin to them by the hardware) take
// chunks of consecutive tickets in turn.  One chunk per XCD (a contiguous eighth of the tickets) keeps the tiles that
// share operands in one L2 and is what the forward GEMMs want (interleaving their tickets costs 5-15 %).  8 k
// equal chunks of at most 128 tickets (`interleave`) spread groups whose tiles cost more over all XCDs; the
// weight-gradient GEMMs, whose contraction length is the group's row count, want that (13 % on a skewed
// 256-expert workload).
// All results are wave-uniform and equal in every wave of a workgroup.
template <int BM>
struct LiveTileWalk {
    const int32_t *rows;   // [N] or null: `cap` rows in every group
    int N, cap, col_tiles;
    int lane;
    int chunk_tiles, chunk_incl;           // lane c: live row tiles of groups 64c..64c+63, and their inclusive prefix
    int cur_chunk, cur_cnt, cur_incl;      // the chunk the last ticket fell in: lane l = group 64*cur_chunk + l
    int local, local_step, xcd, tickets, chunk;   // position in the XCD's own sequence of tickets; chunk size

    __device__ __forceinline__ int live_row_tiles(int g) const
    {
        if (g >= N) return 0;
        const int r = rows ? min(max(rows[g], 0), cap) : cap;
        return (r + BM - 1) / BM;
    }
    __device__ __forceinline__ int scan(int v) const   // inclusive prefix sum over the 64 lanes
    {
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(v, off, 64);
            if (lane >= off) v += o;
        }
        return v;
    }
    __device__ __forceinline__ void init(const int32_t *rows_, int N_, int cap_, int col_tiles_, bool interleave)
    {
        rows = rows_, N = N_, cap = cap_, col_tiles = col_tiles_;
        lane = threadIdx.x & 63;
        chunk_tiles = 0, cur_chunk = -1, cur_cnt = 0, cur_incl = 0;
        const int nchunks = (N + 63) / 64;
        for (int c0 = 0; c0 < nchunks; c0 += 4) {   // four chunks at a time: their loads overlap
            int v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = live_row_tiles((c0 + u) * 64 + lane);   // 0 beyond N
#pragma unroll
            for (int u = 0; u < 4; ++u) {
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) v[u] += __shfl_xor(v[u], off, 64);
                if (lane == c0 + u) chunk_tiles = v[u];
            }
        }
        chunk_incl = scan(chunk_tiles);
        tickets = __builtin_amdgcn_readlane(chunk_incl, 63) * col_tiles;
        // 8 k chunks of equal size: k = 1 (contiguous eighths), or enough for chunks of at most 128 tickets
        const int k = interleave ? max(1, (tickets + 1023) / 1024) : 1;
        chunk = max(1, (tickets + 8 * k - 1) / (8 * k));
        xcd = blockIdx.x % 8;
        local = blockIdx.x / 8;
        local_step = gridDim.x / 8;
    }
    // the tile of the current ticket; false when this workgroup has no ticket left
    __device__ __forceinline__ bool tile(int &e, int &rt, int &ct)
    {
        // the XCD's local-th ticket: chunk (local / chunk) * 8 + xcd, offset local % chunk; increasing in local
        const int ticket = ((local / chunk) * 8 + xcd) * chunk + local % chunk;
        if (ticket >= tickets) return false;
        const int I = ticket / col_tiles;   // index of the live row tile
        const int c = __builtin_ctzll(__ballot(chunk_incl > I));
        const int cbase = __builtin_amdgcn_readlane(chunk_incl - chunk_tiles, c);
        if (c != cur_chunk) {
            cur_cnt = live_row_tiles(c * 64 + lane);
            cur_incl = scan(cur_cnt);
            cur_chunk = c;
        }
        const int l = __builtin_ctzll(__ballot(cbase + cur_incl > I));
        const int first = cbase + __builtin_amdgcn_readlane(cur_incl - cur_cnt, l);
        const int cnt = __builtin_amdgcn_readlane(cur_cnt, l);
        const int u = ticket - first * col_tiles;   // 0 .. cnt*col_tiles-1, row tile fastest
        e = c * 64 + l;
        ct = u / cnt;
        rt = u - ct * cnt;
        return true;
    }
    __device__ __forceinline__ void advance() { local += local_step; }
};

// Kernel timing (smile_kernel_timing): while a library call runs on a ctx with events attached, every kernel it
// launches takes the next caller-owned event pair, which receives the begin / end timestamps of that kernel
// itself (no launch gaps).  The entry points install the ctx's timer for the duration of the call on the calling
// thread; launch sites go through SMILE_LAUNCH.
constexpr int kMaxTimedKernels = 32;
struct KernelTimer {
    hipEvent_t *events = nullptr;   // 2 * pairs handles: start, stop, start, stop, ...
    int pairs = 0, used = 0;
    const char *names[kMaxTimedKernels] = {};
};
extern thread_local KernelTimer *tls_kernel_timer;

template <typename Kernel, typename... Args>
inline void launch_kernel(const char *name, Kernel kernel, dim3 grid, dim3 block, size_t lds, hipStream_t s, Args... args)
{
    KernelTimer *t = tls_kernel_timer;
    if (t && t->used < t->pairs) {
        hipExtLaunchKernelGGL(kernel, grid, block, lds, s, t->events[2 * t->used], t->events[2 * t->used + 1], 0, args...);
        t->names[t->used++] = name;
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
    }
}
#define SMILE_LAUNCH(kernel, ...) ::smile::launch_kernel(#kernel, kernel, __VA_ARGS__)

// Tuning overrides and the device's size, fixed when a ctx is created (smile_create reads the SMILE_* environment
// variables once and asks the runtime for the compute-unit count); -1 = the library's own choice.
struct Tuning {
    int ffn_tile = -1;           // SMILE_FFN_TILE: tile shape of the forward expert GEMMs
    int tgemm_tile = -1;         // SMILE_TGEMM_TILE: tile shape of the gradient GEMMs
    int persist = -1;            // SMILE_FFN_PERSIST: 0 plain grid, 1 persistent grid
    int router_grad_mfma = -1;   // SMILE_ROUTER_GRAD_MFMA: 0 keeps the vector-ALU router-gradient kernels
    int cus = 256;               // compute units of the device the ctx was created on
};

// the validated layer description of a ctx plus its tuning state
struct LayerDesc : smile_layer_desc {
    Tuning tune;
};

// Workgroup slots of the chip for a kernel of `waves` waves per workgroup that was compiled for `occ` waves per SIMD
// and uses `lds_bytes` of LDS: CUs x min(register budget, LDS budget), rounded down to a multiple of the 8 XCDs
// (the persistent tile walk deals tickets to gridDim / 8 workgroups per XCD).
constexpr int kLdsPerCu = 160 * 1024;
constexpr int workgroups_per_cu(int waves, int occ, int lds_bytes)
{
    const int by_regs = occ * 4 / waves > 0 ? occ * 4 / waves : 1;
    const int by_lds = kLdsPerCu / lds_bytes;
    return by_regs < by_lds ? by_regs : by_lds;
}
inline int workgroup_slots(const Tuning &t, int per_cu)
{
    const int slots = (t.cus > 0 ? t.cus : 256) * per_cu / 8 * 8;
    return slots < 8 ? 8 : slots;
}

// Persistent launch or the plain grid?  Persistent when the plain grid would be several times the number of slots:
// then workgroups of empty buffer rows would take turns with the live ones.  With at most a few tiles per slot the
// two are equal within 1-2 %.  Tuning::persist overrides the choice.
bool use_persistent_grid(const Tuning &t, int N, long long tiles, int slots);

}  // namespace smile

struct smile_ctx {
    smile::LayerDesc desc;
    smile::Workspace ws;
    void *base;
    size_t bytes;
    bool owns;
    smile::KernelTimer timer;
};

namespace smile {

struct LossArgs {
    const int32_t *group_count, *local_count;
    const float *p_sum, *q_sum;
    float *out3;   // null: no loss
};

// Launchers: enqueue on `s`, return the launch status.  Shapes were validated by the caller.
hipError_t launch_gate_logits(const smile_layer_desc &d, const void *x, const void *w_inter, const void *w_intra,
                              float *logits_inter, float *logits_intra, hipStream_t s);

// finalize = false leaves pos_in_group / slot unwritten (the block-local ranks stay in the workspace
// for launch_dispatch_finalize).  scan = false (needs finalize = false, no group capacity) also leaves the
// per-block histograms and partial sums unscanned and the counts / sums unwritten: launch_finalize_map_scan
// does both.
hipError_t launch_route(const smile_layer_desc &d, const Workspace &ws, const float *logits_inter,
                        const float *logits_intra, const float *bias_inter, const float *bias_intra,
                        int32_t *group_idx, int32_t *local_idx, int32_t *pos_in_group, int32_t *slot, float *gate,
                        float *p_top, float *q_top, int32_t *group_count, int32_t *local_count,
                        int32_t *expert_count, int32_t *kept_count, float *p_sum, float *q_sum, hipStream_t s,
                        bool finalize = true, bool scan = true);

hipError_t launch_dispatch(const smile_layer_desc &d, const void *x, const int32_t *group_idx,
                           const int32_t *local_idx, const int32_t *slot, void *xe, hipStream_t s);

// the same move in the two hops of Section 3.2.3 through a group buffer xg[n, group_rows, d]
hipError_t launch_dispatch_hop1(const smile_layer_desc &d, const void *x, const int32_t *group_idx,
                                const int32_t *pos_in_group, int group_rows, void *xg, hipStream_t s);
hipError_t launch_dispatch_hop2(const smile_layer_desc &d, const void *xg, const int32_t *group_idx,
                                const int32_t *local_idx, const int32_t *pos_in_group, const int32_t *slot,
                                int group_rows, void *xe, hipStream_t s);

// dispatch fused with the last routing step: computes pos_in_group / slot from the workspace ranks
// and block offsets, writes them, moves the rows, records the slot -> token map in ws.slot_token and
// zeroes the rows of dropped tokens in y; loss != nullptr: one wave also evaluates Eq. 4 from the
// routing statistics (saves the separate loss launch)
hipError_t launch_dispatch_finalize(const smile_layer_desc &d, const Workspace &ws, const void *x,
                                    const int32_t *group_idx, const int32_t *local_idx, int32_t *pos_in_group,
                                    int32_t *slot, void *xe, void *y, const LossArgs &loss, hipStream_t s);

hipError_t launch_combine(const smile_layer_desc &d, const void *ye, const int32_t *group_idx,
                          const int32_t *local_idx, const int32_t *slot, const float *gate, void *y, hipStream_t s);

// up: hidden = act(xe . w1^T + b1) into ws.hidden;  down: ye = hidden . w2^T + b2
// t0/t1: optional events receiving the begin/end timestamps of the up kernel itself (both or neither)
// x_tokens != nullptr: gather the input rows from the token matrix x[T,d] through ws.slot_token (xe unused)
// h_save / pre_save (both or neither): write act(.) there instead of ws.hidden, and the pre-activation too
hipError_t launch_expert_ffn_up(const LayerDesc &d, const Workspace &ws, const void *xe,
                                const int32_t *kept_count, const void *w1, const void *b1, hipStream_t s,
                                hipEvent_t t0 = nullptr, hipEvent_t t1 = nullptr, const void *x_tokens = nullptr,
                                void *h_save = nullptr, void *pre_save = nullptr);
// y_tokens != nullptr: also write gate[t] * row to y_tokens[t] for the token t of each row (ye may be null)
hipError_t launch_expert_ffn_down(const LayerDesc &d, const Workspace &ws, const int32_t *kept_count,
                                  const void *w2, const void *b2, void *ye, hipStream_t s,
                                  void *y_tokens = nullptr, const float *gate = nullptr,
                                  const void *h_saved = nullptr);

// One grouped product y[e] = act(x[e] . w[e]^T) over N groups: x[N][C][K], w[N][Nout][K], y[N][C][Nout], rows
// below kept[e] only (kept == nullptr: all C rows).  act: 0 none, 1 ReLU, 2 GELU.  y2 != nullptr: the product
// without the activation goes there as well.  bf16 needs K % 64 == 0 and Nout % 8 == 0, fp32 K % 4 == 0.
// bias: [N][Nout] or null.  x_rows != nullptr: input row r of group e is row x_rows[e*C + r] of the matrix x[.][K].
// post (1 ReLU, 2 GELU; needs act == 0 and aux[N][C][Nout]): the output is multiplied by act'(aux).
struct GroupedGemm {
    const void *x, *w;
    void *y, *y2;
    const int32_t *kept;
    int N, C, Nout, K, act;
    const void *bias = nullptr;
    const int32_t *x_rows = nullptr;
    const void *aux = nullptr;
    int post = 0;
    Tuning tune = {};
};
hipError_t launch_grouped_gemm_nt(int dtype, const GroupedGemm &g, hipStream_t s);

// One grouped 16-bit (bf16 / fp16) product y[e][i][j] = sum_k X(i,k) W(j,k) whose operands may have the contraction index as
// their slow index (x_transposed: x[e] is [K][Mrows]; w_transposed: w[e] is [K][Nout]); a normal x is
// [Mrows][K].  ldx / ldw: leading dimensions, sx / sw / sy: per-group strides, all in elements.
// rows_valid[e] (or Mrows) output rows are computed; k_valid[e] (or K) terms are summed (transposed operands
// only: a normal operand needs K % 64 == 0 and full K).  post (1 ReLU, 2 GELU): times act'(aux), aux shaped as y.
struct TransposedGemm {
    const void *x, *w;
    void *y;
    const void *aux;
    const int32_t *rows_valid, *k_valid;
    int N, Mrows, Nout, K, ldx, ldw;
    long long sx, sw, sy;
    bool x_transposed, w_transposed;
    int post;
    Tuning tune = {};
};
hipError_t launch_grouped_gemm_t(int dtype, const TransposedGemm &g, hipStream_t s);

// Last routing step for the fully fused forward pass: pos_in_group / slot as launch_route's finalize
// kernel, plus the slot -> token map in ws.slot_token, zero output rows for dropped tokens in y, and
// (loss.out3 != nullptr) the Eq. 4 loss.
hipError_t launch_finalize_map(const smile_layer_desc &d, const Workspace &ws, const int32_t *group_idx,
                               const int32_t *local_idx, int32_t *pos_in_group, int32_t *slot, void *y,
                               const LossArgs &loss, hipStream_t s);

// ---- backward pass.  Its workspace is separate from the ctx's and supplied by the caller per call.
struct BackwardLayout {
    size_t off_pre, off_h, off_dpre, off_h_t, off_dpre_t, off_dye_t, off_xe_t, off_w_t, off_gw_partial, total;
    int32_t k_pad;       // capacity rounded up to the GEMM slab depth: contraction length of the weight-gradient GEMMs
    int32_t gw_blocks;   // token blocks of the router-weight gradient
};
BackwardLayout backward_workspace_layout(const smile_layer_desc &d);

hipError_t launch_combine_backward(const smile_layer_desc &d, const void *dy, const void *ye, const int32_t *group_idx,
                                   const int32_t *local_idx, const int32_t *slot, const float *gate, void *dye,
                                   float *dgate, hipStream_t s);
hipError_t launch_route_backward(const smile_layer_desc &d, const float *logits_inter, const float *logits_intra,
                                 const float *bias_inter, const float *bias_intra, const int32_t *group_idx,
                                 const int32_t *local_idx, const float *dgate, const int32_t *group_count,
                                 const int32_t *local_count, float dloss, float *dlp, float *dlq, hipStream_t s);
// h / pre (both or neither): the hidden activation and pre-activation saved by the forward pass; null: recomputed
hipError_t launch_expert_ffn_backward(const LayerDesc &d, void *workspace, const void *xe,
                                      const int32_t *kept_count, const void *w1, const void *w2, const void *dye,
                                      const void *h, const void *pre, void *dxe, void *dw1, void *dw2, hipStream_t s);
hipError_t launch_dispatch_backward(const LayerDesc &d, const void *dxe, const int32_t *group_idx,
                                    const int32_t *local_idx, const int32_t *slot, const float *dlp, const float *dlq,
                                    const void *w_inter, const void *w_intra, void *dx, hipStream_t s);
// bf16 storage and at most 10 chunks of 16 logit columns: the same product on the matrix cores
bool dispatch_backward_mfma_applies(const smile_layer_desc &d);
hipError_t launch_dispatch_backward_mfma(const smile_layer_desc &d, const void *dxe, const int32_t *group_idx,
                                         const int32_t *local_idx, const int32_t *slot, const float *dlp,
                                         const float *dlq, const void *w_inter, const void *w_intra, void *dx,
                                         hipStream_t s);
// bf16 storage and at most 160 logit columns: the per-block partial sums on the matrix cores
bool gate_weights_mfma_applies(const smile_layer_desc &d);
int gate_weights_mfma_block_tokens(const smile_layer_desc &d, int granule);
hipError_t launch_gate_weights_mfma(const smile_layer_desc &d, const void *x, const float *dlp, const float *dlq,
                                    float *partial, int blocks, int tokens_per_block, hipStream_t s);
hipError_t launch_gate_weights_backward(const LayerDesc &d, void *workspace, const void *x, const float *dlp,
                                        const float *dlq, float *dw_inter, float *dw_intra, hipStream_t s);

// The same for small batches, without the separate scan kernel: every block sums the histogram rows of the
// blocks before it (at most kScanInFinalizeBlocks - 1 rows), and the last block produces the counts, the
// probability sums (same summation order as the scan kernel: identical bits) and the loss.
constexpr int kScanInFinalizeBlocks = 64;
hipError_t launch_finalize_map_scan(const smile_layer_desc &d, const Workspace &ws, const int32_t *group_idx,
                                    const int32_t *local_idx, int32_t *pos_in_group, int32_t *slot, void *y,
                                    int32_t *group_count, int32_t *local_count, int32_t *expert_count,
                                    int32_t *kept_count, float *p_sum, float *q_sum, float *loss3, hipStream_t s);

hipError_t launch_aux_loss(const smile_layer_desc &d, const int32_t *group_count, const int32_t *local_count,
                           const float *p_sum, const float *q_sum, float *out3, hipStream_t s);

}  // namespace smile
