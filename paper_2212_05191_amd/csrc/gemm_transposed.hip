// Grouped 16-bit (bf16 / fp16) MFMA GEMM whose operands may be stored with the contraction index as the SLOW index
// ("transposed"): the four gradient GEMMs of the expert FFN backward pass,
//
//     dpre[r,f] = sum_c dye[r,c] W2[c,f]      x normal,      w transposed      (K = d)
//     dxe [r,k] = sum_f dpre[r,f] W1[f,k]     x normal,      w transposed      (K = F)
//     dW2 [c,f] = sum_r dye[r,c] h[r,f]       x transposed,  w transposed      (K = rows of the expert)
//     dW1 [f,k] = sum_r dpre[r,f] xe[r,k]     x transposed,  w transposed      (K = rows of the expert)
//
// without materialising any transposed copy.  y[e][i][j] = sum_k X(i,k) W(j,k) per group e, where a
// normal operand is stored [i][k] (k contiguous) and a transposed one [k][i] (i contiguous).
//
// Design (gfx950):
//   * global -> LDS with the direct 16-byte loads of the forward kernel, STAGES-deep ring of K slabs
//     (BK = 64).  A normal operand lands as [row][64 k] (8 pieces per row, XOR-swizzled); a transposed
//     one lands as it is in memory, [k][BM or BN columns] (16 or 32 pieces per row).
//   * MFMA 32x32x16 bf16 wants, per lane, 8 consecutive k of one row/column.  From a normal tile that
//     is one 16-byte LDS read.  From a transposed tile it is two transposing LDS reads
//     (ds_read_b64_tr_b16): within each group of 16 lanes, lane 4a+b receives element b of the four
//     8-byte rows addressed by lanes a, a+4, a+8, a+12.  Lane i of a group therefore addresses
//     k-row (i / 4) [+4 for the second read] and the 4-column block (i % 4) of its 16-column span,
//     and every lane ends up with k, k+1, k+2, k+3 of its own column -- the same k order as a
//     normal operand, so the two kinds mix in one MFMA.
//   * transposed tiles are swizzled by k: a row's pieces are rotated by 4 * (k & 3) positions.  The 8
//     k-rows a wave touches in one read then cover all 64 banks twice, the minimum for 512 bytes
//     (rows of 16, 24 or 32 pieces alike; with 24 the last group of four pieces wraps onto a used bank).
//   * the contraction length of the weight-gradient GEMMs is the expert's row count: slabs beyond it
//     are skipped, and k-rows beyond it inside the last slab are loaded from a zero block instead
//     (no zero-padded copies, no work on empty buffer rows).
//   * epilogue as in the forward kernel: fp32 -> bf16, staged through LDS, row-contiguous 16-byte
//     stores; POST multiplies by act'(aux) there (the gradient at the pre-activation).
#include <type_traits>

#include "smile_internal.hpp"

namespace smile {

namespace {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int kXcds = 8;
constexpr int BK = 64;

__device__ __attribute__((aligned(16))) const uint32_t kZeroPiece[4] = {0u, 0u, 0u, 0u};

#define SMILE_GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define SMILE_LPTR(p) ((__attribute__((address_space(3))) void *)(p))

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);   // expcnt, lgkmcnt: no wait
}

template <int POST>
__device__ __forceinline__ float activate_grad(float v)
{
    if constexpr (POST == 1) return v > 0.f ? 1.f : 0.f;
    else {
        // d/dv [v Phi(v)] = Phi(v) + v phi(v); Phi from the rational erfc approximation 7.1.26 of
        // Abramowitz & Stegun (|error| < 1.5e-7), phi sharing its exponential
        const float av = fabsf(v);
        const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f * 0.70710678118654752f, av, 1.0f));
        float poly = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
        poly = fmaf(poly, t, 0.5f * 1.421413741f);
        poly = fmaf(poly, t, 0.5f * -0.284496736f);
        poly = fmaf(poly, t, 0.5f * 0.254829592f);
        const float ex = __builtin_amdgcn_exp2f(v * v * (-0.5f * 1.4426950408889634f));
        const float q = poly * t * ex;   // 1 - Phi(|v|)
        return fmaf(v * 0.3989422804014327f, ex, v >= 0.f ? 1.0f - q : q);
    }
}

// E: the 16-bit storage type (__bf16 or _Float16)
template <typename E>
struct TGemmArgs {
    const E *x, *w;
    E *y;
    const E *aux;             // POST: [N][rows][Nout] like y
    const int32_t *rows_valid;   // [N] valid output rows per group, or null: Mrows for all
    const int32_t *k_valid;      // [N] valid contraction length per group, or null: K for all
    int Mrows, Nout, K;          // output extents per group and the full contraction length
    int ldx, ldw;                // leading dimensions (elements) of x and w
    long long sx, sw, sy;        // per-group strides (elements) of x, w and y / aux
    int row_tiles, col_tiles, tiles;
    int N;                       // groups
};

// One operand tile of a stage, as seen by the loader and by the MFMA fragment reader.
//   T == false: [EXT rows][8 pieces], piece ^= (row >> 1) & 7
//   T == true : [64 k][EXT / 8 pieces], position = (piece + 4 * (k & 3)) mod (EXT / 8)
template <typename E, int EXT, bool T>
struct OperandTile {
    static constexpr int kPieces = EXT * BK / 8;
    static constexpr int kPiecesPerK = EXT / 8;

    // global source of linear LDS piece q (slab 0) and whether / how it depends on k
    __device__ static __forceinline__ const E *source(const E *base, int q, int tile0, int ext_valid, int ld,
                                                      int &k_row)
    {
        if constexpr (!T) {
            const int row = q >> 3, piece = (q & 7) ^ ((row >> 1) & 7);
            k_row = -1;   // all k of this piece are inside the slab; no k bound needed (K % 64 == 0)
            return base + (size_t)min(tile0 + row, ext_valid - 1) * ld + piece * 8;
        } else {
            const int k = q / kPiecesPerK, pos = q - k * kPiecesPerK;
            const int piece = pos - 4 * (k & 3) + (pos < 4 * (k & 3) ? kPiecesPerK : 0);   // the piece rotated to pos
            k_row = k;
            return base + (size_t)k * ld + min(tile0 + piece * 8, ext_valid - 8);
        }
    }
};

template <typename E, int BM, int BN, int WGM, int WGN, int STAGES, int OCC, bool XT, bool WT, int POST, bool PERSIST = false>
__global__ __launch_bounds__(WGM *WGN * 64, OCC) void grouped_gemm_t_kernel(TGemmArgs<E> a)
{
    typedef typename Half<E>::vec8 bf16x8;                              // one MFMA operand: 8 elements
    typedef __attribute__((__vector_size__(4 * sizeof(E)))) E bf16x4;   // 4 rounded outputs
    constexpr int NW = WGM * WGN, NT = NW * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    using XTile = OperandTile<E, BM, XT>;
    using WTile = OperandTile<E, BN, WT>;
    constexpr int XI = XTile::kPieces / 64, WI = WTile::kPieces / 64;   // load instructions per slab
    constexpr int GPW = (XI + WI) / NW;
    constexpr int STAGE = XTile::kPieces + WTile::kPieces;
    constexpr int OROWS = WGM * 32, OSTRIDE = BN / 8 + 1, OPR = BN / 8;
    static_assert((XI + WI) % NW == 0, "load instructions must divide over the waves");
    static_assert(BM % 32 == 0 && BN % 32 == 0 && BM >= 128 && BN >= 128, "rotation swizzle: rows of at least 16 pieces");
    static_assert(STAGES >= 2 && STAGES <= 4 && (STAGES - 2) * GPW < 64, "pipeline depth");
    static_assert(OROWS * OSTRIDE <= STAGES * STAGE, "epilogue staging must fit in the pipeline buffers");

    __shared__ u32x4 lds[STAGES * STAGE];

    // ---- which tile(s): one per workgroup (plain grid, ids remapped so that each XCD gets a contiguous range) or
    // PERSIST: one workgroup per slot of the chip walks the live tiles (LiveTileWalk) and requests the first
    // slabs of its next tile before the epilogue of the current one (PREFETCH), which then stages its output in
    // the one pipeline buffer those loads do not touch.
    constexpr bool PREFETCH = PERSIST && OROWS * OSTRIDE <= STAGE;
    constexpr int STG = PREFETCH ? (STAGES - 1) * STAGE : 0;   // staging area, in 16-byte units
    LiveTileWalk<BM> walk;
    if constexpr (PERSIST) walk.init(a.rows_valid, a.N, a.Mrows, a.col_tiles, XT && WT);
    struct Tile {
        int e, rt, ct, rows, kv;
    };
    auto select = [&](Tile &t) {
        if constexpr (PERSIST) {
            if (!walk.tile(t.e, t.rt, t.ct)) return false;
        } else {
            const int per_xcd = (a.tiles + kXcds - 1) / kXcds;
            const int lid = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
            if (lid >= a.tiles) return false;
            const int per_group = a.row_tiles * a.col_tiles;
            t.e = lid / per_group;
            const int rem = lid - t.e * per_group;
            t.ct = rem / a.row_tiles, t.rt = rem - t.ct * a.row_tiles;
        }
        t.rows = a.rows_valid ? min(a.rows_valid[t.e], a.Mrows) : a.Mrows;
        t.kv = a.k_valid ? min(a.k_valid[t.e], a.K) : a.K;
        return t.rt * BM < t.rows;
    };

    // ---- loader: this lane's source of each of the wave's load instructions (slab 0), the k-row it
    // holds (transposed operands; -1 otherwise) and its advance per slab
    // Instruction wave + i*NW of a slab: the first XI / NW values of i fill the x tile for every wave, the
    // rest the w tile (both counts are multiples of NW), so the kind of each load is known at compile time.
    static_assert(XI % NW == 0, "x tile instructions must divide over the waves");
    constexpr int XG = XI / NW;
    // The contraction length is ragged only in the weight-gradient GEMMs (both operands transposed).
    constexpr bool KRAGGED = XT && WT;
    const E *src[GPW];
    int krow[GPW];
    int kv = 0;   // contraction length of the tile whose loads are being issued
    const size_t adv_x = XT ? (size_t)BK * a.ldx : (size_t)BK, adv_w = WT ? (size_t)BK * a.ldw : (size_t)BK;
    const E *zero = reinterpret_cast<const E *>(kZeroPiece);
    // load instruction i of slab `slab` into `stage`
    auto load_one = [&](int wave, int i, int slab, int stage) {
        const E *p = src[i] + (size_t)slab * (i < XG ? adv_x : adv_w);
        if (KRAGGED && slab * BK + krow[i] >= kv) p = zero;   // beyond the contraction length
        __builtin_amdgcn_global_load_lds(SMILE_GPTR(p), SMILE_LPTR(&lds[stage * STAGE + (wave + i * NW) * 64]), 16, 0, 0);
    };
    // Per-lane indices are derived afresh wherever they are needed (PERSIST: through an opaque copy of the
    // thread id), so that nothing computed from them stays in registers from one tile to the next.
    auto thread_id = [&]() {
        int tid = threadIdx.x;
        if constexpr (PERSIST) asm volatile("" : "+v"(tid));
        return tid;
    };
    // source addresses of a tile and the requests for its first STAGES-1 slabs
    auto start_tile = [&](const Tile &t) {
        const int tid = thread_id(), lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const E *X = a.x + (size_t)t.e * a.sx;
        const E *W = a.w + (size_t)t.e * a.sw;
        kv = t.kv;
        const int slabs = (t.kv + BK - 1) / BK;
#pragma unroll
        for (int i = 0; i < GPW; ++i) {
            const int inst = wave + i * NW;
            if (i < XG) {
                // a transposed x holds the output rows along its fast index: all Mrows columns exist in memory
                src[i] = XTile::source(X, inst * 64 + lane, t.rt * BM, XT ? a.Mrows : t.rows, a.ldx, krow[i]);
            } else {
                src[i] = WTile::source(W, (inst - XI) * 64 + lane, t.ct * BN, a.Nout, a.ldw, krow[i]);
            }
        }
#pragma unroll
        for (int s = 0; s < STAGES - 1; ++s)
            if (s < slabs) {
#pragma unroll
                for (int i = 0; i < GPW; ++i) load_one(wave, i, s, s);
            }
    };

    Tile cur;
    if (!select(cur)) return;
    start_tile(cur);
    for (;;) {
    const int e = cur.e, rt = cur.rt, ct = cur.ct, rows = cur.rows;
    const int slabs = (cur.kv + BK - 1) / BK;
    const int tid = thread_id(), lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;

    // ---- fragment addressing
    // normal: lane reads row (lane & 31), pieces 2*kk + (lane >> 5)
    const int frow = lane & 31, fhi = lane >> 5, fsw = (frow >> 1) & 7;
    // transposed: lane = 16 g + 4 j + a addresses k-row 8 (g / 2) + j (+4: second read, +16 kk) and the
    // 4 columns 16 (g % 2) + 4 a of the 32-column tile
    const int tg = lane >> 4, tj = (lane >> 2) & 3, ta = lane & 3;
    const int tk0 = 8 * (tg >> 1) + tj;
    const int tcol = 16 * (tg & 1) + 4 * ta;   // column inside the 32-column tile
    int xoff[TM], woff[TN];                    // byte offsets inside the stage for kk = 0, first read
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        if constexpr (XT) {
            const int col = wm * WM + j * 32 + tcol;
            xoff[j] = (tk0 * XTile::kPiecesPerK + ((col >> 3) + 4 * tj) % XTile::kPiecesPerK) * 16 + (col & 4) * 2;
        } else {
            xoff[j] = ((wm * WM + j * 32 + frow) * 8) * 16;
        }
    }
#pragma unroll
    for (int i = 0; i < TN; ++i) {
        if constexpr (WT) {
            const int col = wn * WN + i * 32 + tcol;
            woff[i] = (XTile::kPieces + tk0 * WTile::kPiecesPerK + ((col >> 3) + 4 * tj) % WTile::kPiecesPerK) * 16 +
                      (col & 4) * 2;
        } else {
            woff[i] = ((XTile::kPieces + (wn * WN + i * 32 + frow) * 8)) * 16;
        }
    }

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const bool wave_live = rt * BM + wm * WM < rows;   // wave-uniform
    int stage = 0;
    // One K slab.  ISSUE: this iteration also issues the loads of slab kt+STAGES-1.  As in the forward kernel
    // the fragments of k-step kk+1 are fetched while the MFMAs of k-step kk run, the next slab's load
    // instructions are spread over the k-steps, and the instruction order is pinned.
    auto slab_step = [&](auto issue_tag, int kt) {
        constexpr bool ISSUE = decltype(issue_tag)::value;
        if (ISSUE) {
            // a prefetched tile's first slabs were requested before the previous tile's stores: wait for all
            if (PREFETCH && STAGES > 2 && kt == 0) wait_vmcnt<0>();
            else wait_vmcnt<(STAGES - 2) * GPW>();
        } else {
            const int ahead = slabs - 1 - kt;   // 0 .. STAGES-2 slabs were issued after this one
            if (PREFETCH && kt == 0) wait_vmcnt<0>();
            else if (STAGES >= 4 && ahead == 2) wait_vmcnt<2 * GPW>();
            else if (STAGES >= 3 && ahead == 1) wait_vmcnt<GPW>();
            else wait_vmcnt<0>();
        }
        __builtin_amdgcn_s_barrier();
        const int nstage = stage == 0 ? STAGES - 1 : stage - 1;
        const int nxt = kt + STAGES - 1;
        const char *cur_stage = reinterpret_cast<const char *>(lds + stage * STAGE);
        bf16x8 xf[2][TM], wf[2][TN];
        auto fetch = [&](int buf, int kk) {
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                if constexpr (XT) {
                    const char *p = cur_stage + xoff[j] + kk * 16 * XTile::kPiecesPerK * 16;
                    struct { s16x4 lo, hi; } t;
                    t.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
                    t.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4 *)(p + 4 * XTile::kPiecesPerK * 16));
                    xf[buf][j] = __builtin_bit_cast(bf16x8, t);
                } else {
                    xf[buf][j] = *reinterpret_cast<const bf16x8 *>(cur_stage + xoff[j] + (((2 * kk + fhi) ^ fsw) * 16));
                }
            }
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                if constexpr (WT) {
                    const char *p = cur_stage + woff[i] + kk * 16 * WTile::kPiecesPerK * 16;
                    struct { s16x4 lo, hi; } t;
                    t.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)p);
                    t.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4 *)(p + 4 * WTile::kPiecesPerK * 16));
                    wf[buf][i] = __builtin_bit_cast(bf16x8, t);
                } else {
                    wf[buf][i] = *reinterpret_cast<const bf16x8 *>(cur_stage + woff[i] + (((2 * kk + fhi) ^ fsw) * 16));
                }
            }
        };
        auto issue_part = [&](int l0, int l1) {
#pragma unroll
            for (int i = 0; i < GPW; ++i)
                if (i >= l0 && i < l1) load_one(wave, i, nxt, nstage);
        };
        constexpr int KS = BK / 16;
        if (!wave_live) {
            if (ISSUE) issue_part(0, GPW);   // none of this wave's rows exists: it only helps loading
            stage = stage + 1 == STAGES ? 0 : stage + 1;
            return;
        }
        fetch(0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            const int l0 = GPW * kk / KS, l1 = GPW * (kk + 1) / KS;
            if (kk + 1 < KS) fetch((kk + 1) & 1, kk + 1);
            if (ISSUE) issue_part(l0, l1);
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = Half<E>::mfma_32x32x16(wf[kk & 1][i], xf[kk & 1][j], acc[i][j]);
            // order inside the k-step: MFMA, LDS read(s), MFMA, ... then MFMA + global loads
            constexpr int NM = TM * TN, ND = (XT ? 2 : 1) * TM + (WT ? 2 : 1) * TN;
            constexpr int DPM = (ND + NM - 1) / NM;   // LDS reads placed after each MFMA
#pragma unroll
            for (int r = 0; r < NM; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
#pragma unroll
                for (int q = 0; q < DPM; ++q)
                    if (kk + 1 < KS && r * DPM + q < ND) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if (ISSUE && r >= NM - (l1 - l0)) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        stage = stage + 1 == STAGES ? 0 : stage + 1;
    };
    // the next tile is chosen before the main loop, so that the loads of its row counts are long back when
    // the epilogue needs them
    Tile nxt_tile;
    bool more = false;
    if constexpr (PERSIST) {
        walk.advance();
        more = select(nxt_tile);
    }
    int kt = 0;
    for (; kt + STAGES - 1 < slabs; ++kt) slab_step(std::true_type{}, kt);
    for (; kt < slabs; ++kt) slab_step(std::false_type{}, kt);

    // ---- epilogue.  Accumulator element v of a lane is (column 8*(v/4) + 4*(lane/32) + v%4, row lane%32)
    // of its 32x32 tile: rounded to bf16, staged as a [OROWS][BN] tile, stored row-contiguously.
    E *Y = a.y + (size_t)e * a.sy;
    u32x2 *stg = reinterpret_cast<u32x2 *>(lds + STG);
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wave's LDS reads are done
        __builtin_amdgcn_s_barrier();
        if (PREFETCH && j == 0 && more) start_tile(nxt_tile);
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int lcol = wn * WN + i * 32 + 8 * q + 4 * fhi;
                bf16x4 out;
#pragma unroll
                for (int v = 0; v < 4; ++v) out[v] = (E)acc[i][j][4 * q + v];
                stg[((wm * 32 + frow) * OSTRIDE) * 2 + (lcol >> 2)] = __builtin_bit_cast(u32x2, out);
            }
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        // all of the thread's staged pieces are read before the first store, so that the LDS latencies overlap
        constexpr int NIT = (OROWS * OPR + NT - 1) / NT;
        u32x4 outv[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int id = min(tid + it * NT, OROWS * OPR - 1);
            const int orow = id / OPR, piece = id - orow * OPR;
            outv[it] = lds[STG + orow * OSTRIDE + piece];
        }
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int id = tid + it * NT;
            const int orow = id / OPR, piece = id - orow * OPR;
            const int row = rt * BM + (orow >> 5) * WM + j * 32 + (orow & 31);
            const int col = ct * BN + piece * 8;
            if (id < OROWS * OPR && row < rows && col < a.Nout) {
                u32x4 v = outv[it];
                if constexpr (POST != 0) {
                    const u32x4 p = *reinterpret_cast<const u32x4 *>(a.aux + (size_t)e * a.sy + (size_t)row * a.Nout + col);
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        v[k] = Half<E>::pack(Half<E>::lo(v[k]) * activate_grad<POST>(Half<E>::lo(p[k])),
                                             Half<E>::hi(v[k]) * activate_grad<POST>(Half<E>::hi(p[k])));
                }
                u32x4 *dst = reinterpret_cast<u32x4 *>(Y + (size_t)row * a.Nout + col);
                // weight gradients are not read again soon: keep them out of the way of the operands in L2
                if constexpr (KRAGGED) __builtin_nontemporal_store(v, dst);
                else *dst = v;
            }
        }
    }
    if (!more) return;
    if constexpr (!PREFETCH) {
        // the next tile's first loads overwrite the staging area: every wave must be done reading it
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        start_tile(nxt_tile);
    }
    cur = nxt_tile;
    }   // tile loop
}

template <typename E, int BM, int BN, int STAGES, int OCC, bool XT, bool WT, int POST>
hipError_t launch_tile(TGemmArgs<E> a, int N, const Tuning &tune, hipStream_t s)
{
    a.row_tiles = (a.Mrows + BM - 1) / BM;
    a.col_tiles = (a.Nout + BN - 1) / BN;
    a.tiles = N * a.row_tiles * a.col_tiles;
    a.N = N;
    const int slots = workgroup_slots(tune, workgroups_per_cu(4, OCC, STAGES * (BM + BN) * BK * 2));
    if (use_persistent_grid(tune, N, a.tiles, slots)) {
        SMILE_LAUNCH((grouped_gemm_t_kernel<E, BM, BN, 2, 2, STAGES, OCC, XT, WT, POST, true>), dim3(slots), dim3(256),
                           0, s, a);
    } else {
        const int per_xcd = (a.tiles + kXcds - 1) / kXcds;
        SMILE_LAUNCH((grouped_gemm_t_kernel<E, BM, BN, 2, 2, STAGES, OCC, XT, WT, POST>), dim3(per_xcd * kXcds),
                           dim3(256), 0, s, a);
    }
    return hipGetLastError();
}

// Tile shapes: id -> (BM, BN, stages, workgroups per CU).  Measured on the backward pass of the bf16
// workloads: two co-resident workgroups with a two-stage ring beat one workgroup with a larger tile or a
// deeper ring for all four products; 128 x 192 (fewer LDS bytes per MFMA) wins when it still gives every CU
// its two workgroups and does not pad the columns much, else 128 x 128.  Tuning::tgemm_tile (0..3) overrides the choice for tuning runs.
template <typename E, bool XT, bool WT, int POST>
hipError_t launch_shape(const TGemmArgs<E> &a, int N, const Tuning &tune, hipStream_t s)
{
    const long long wide = (long long)N * ((a.Mrows + 127) / 128) * ((a.Nout + 191) / 192);
    int tile = wide >= 512 ? 3 : 2;
    // 192-wide column tiles that would be padded by more than a tenth over 128-wide ones (e.g. 1024 columns: 6 x 192
    // against 8 x 128): the narrower tile wins (6 % on 64 experts of 320 x 1024 x 4096)
    if ((a.Nout + 191) / 192 * 192 * 10 > (a.Nout + 127) / 128 * 128 * 11) tile = 2;
    if (tune.tgemm_tile >= 0 && tune.tgemm_tile <= 3) tile = tune.tgemm_tile;
    if (tile == 0) return launch_tile<E, 128, 256, 3, 1, XT, WT, POST>(a, N, tune, s);
    if (tile == 1) return launch_tile<E, 128, 128, 4, 1, XT, WT, POST>(a, N, tune, s);
    if (tile == 2) return launch_tile<E, 128, 128, 2, 2, XT, WT, POST>(a, N, tune, s);
    return launch_tile<E, 128, 192, 2, 2, XT, WT, POST>(a, N, tune, s);
}

template <typename E>
hipError_t launch_typed(const TransposedGemm &g, hipStream_t s)
{
    TGemmArgs<E> a{static_cast<const E *>(g.x), static_cast<const E *>(g.w), static_cast<E *>(g.y),
                   static_cast<const E *>(g.aux), g.rows_valid, g.k_valid, g.Mrows, g.Nout, g.K, g.ldx, g.ldw,
                   g.sx, g.sw, g.sy, 0, 0, 0, g.N};
    if (g.x_transposed) return launch_shape<E, true, true, 0>(a, g.N, g.tune, s);
    if (g.post == 1) return launch_shape<E, false, true, 1>(a, g.N, g.tune, s);
    if (g.post == 2) return launch_shape<E, false, true, 2>(a, g.N, g.tune, s);
    return launch_shape<E, false, true, 0>(a, g.N, g.tune, s);
}

}  // namespace

hipError_t launch_grouped_gemm_t(int dtype, const TransposedGemm &g, hipStream_t s)
{
    if (!is_half(dtype)) return hipErrorInvalidValue;
    if (g.K < 1 || g.Mrows < 1 || g.Nout % 8 || g.ldx % 8 || g.ldw % 8) return hipErrorInvalidValue;
    if (!g.x_transposed && g.K % BK) return hipErrorInvalidValue;   // a normal operand is read in whole 64-k slabs
    if (!g.w_transposed) return hipErrorInvalidValue;               // not needed by any caller
    if (g.x_transposed && (g.Mrows % 8 || g.post)) return hipErrorInvalidValue;
    if (dtype == SMILE_DTYPE_BF16) return launch_typed<__bf16>(g, s);
    return launch_typed<_Float16>(g, s);
}

}  // namespace smile
