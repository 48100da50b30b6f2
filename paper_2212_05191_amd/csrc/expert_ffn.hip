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
// 16-bit kernel (bf16 or fp16 storage; the hot kernel of the layer).  One workgroup computes a BM x BN tile
// of one expert with v_mfma_f32_32x32x16_bf16 / _f16 and fp32 accumulators.
//   * K is cut into slabs of BK elements.  A slab travels global -> LDS directly
//     (global_load_lds_dwordx4: no staging registers, no ds_write) into a ring of STAGES buffers
//     with STAGES-1 slabs in flight.  Per slab: wait until this wave's part has landed (s_waitcnt
//     vmcnt), one s_barrier (every wave's part landed, and every wave is done reading the buffer
//     about to be refilled), issue the loads of the slab STAGES-1 ahead, then the MFMAs.
//   * A direct load writes 64 lanes x 16 bytes to consecutive LDS addresses, i.e. whole rows of a
//     slab.  The bank swizzle is therefore applied on the global side: the lane that fills position
//     p of a row fetches piece p ^ f(row), so piece c of a row sits at position c ^ f(row) and the
//     32 rows a wave reads for one MFMA operand fall on distinct banks.
//   * The weight tile is the MFMA "A" operand and the token tile the "B" operand, so a lane ends up
//     with 4 consecutive output columns of one token row.  The epilogue (bias, activation, round
//     to the storage type) writes them to LDS and the workgroup then stores whole rows, 16 bytes per lane, so
//     every global store instruction covers full cache lines.
//   * Traffic L2 -> LDS per flop falls as 1/BM + 1/BN; that path (about 64 B/clk per CU at best)
//     and not HBM is what bounds small tiles, so tiles are as large as the workload can still
//     spread over 256 CUs.
//
// Plain grid (at most a few tiles per workgroup slot of the chip): it covers every (expert, column tile,
// row tile); tiles whose first row is >= kept[e] exit at once, so no host synchronisation on the routing
// result is needed.  Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the id is remapped
// so that each XCD (own L2) works on a contiguous range of tiles: the row tiles sharing a weight tile and
// the column tiles sharing a token tile then meet in the same L2.
// Persistent grid (many tiles per slot): one workgroup per slot walks the live tiles only, in the same
// order (LiveTileWalk), again without any host knowledge of the row counts.  When experts are far below
// capacity this is up to 25 % faster: a workgroup of an empty tile still has to wait for a free slot (its
// LDS) before it can exit, in turn with the live ones.
//
// fp32 kernel (small / reference-precision configurations): classic LDS-tiled FMA GEMM.
#include <type_traits>

#include <hip/hip_ext.h>

#include "gemm_device.hpp"

namespace smile {

namespace {

// OCC: waves per SIMD the register allocation must leave room for (workgroups per CU when the
// workgroup has 4 waves).
// DUAL: the epilogue runs twice, storing act(product) to y and the bare product to y2 (the hidden
// activation and its pre-activation from one GEMM, for the backward pass).
// POST (1 ReLU, 2 GELU): the rounded output is multiplied by act'(aux) on its way out (the gradient at the
// pre-activation, dh * act'(pre)); aux is read with the same row-contiguous 16-byte accesses as the store.
// E: the 16-bit storage type (__bf16 or _Float16).
template <typename E, int BM, int BN, int WGM, int WGN, int BK, int STAGES, int OCC, int SWZ, int ACT,
          bool DUAL = false, int POST = 0, bool PERSIST = false>
__global__ __launch_bounds__(WGM *WGN * 64, OCC) void grouped_gemm_nt_kernel(GemmArgs a)
{
    typedef typename Half<E>::vec8 bf16x8;                                  // one MFMA operand: 8 elements
    typedef __attribute__((__vector_size__(4 * sizeof(E)))) E bf16x4;       // 4 rounded outputs
    constexpr int NW = WGM * WGN, NT = NW * 64;
    constexpr int WM = BM / WGM, WN = BN / WGN;   // wave tile
    constexpr int TM = WM / 32, TN = WN / 32;     // MFMA tiles per wave
    constexpr int PPR = BK / 8;                   // 16-byte pieces per LDS row
    constexpr int RPI = 64 / PPR;                 // rows filled by one direct-load instruction
    constexpr int ROWS = BM + BN;                 // LDS rows per stage: token tile, then weight tile
    constexpr int GPW = ROWS / RPI / NW;          // load instructions per wave per slab
    constexpr int STAGE = ROWS * PPR;             // 16-byte units per stage
    constexpr int OROWS = WGM * 32;               // output rows staged per epilogue pass
    constexpr int OSTRIDE = BN / 8 + 1;           // staged row length in 16-byte units (+1: bank spread)
    static_assert(BK == 64 || BK == 32, "slab depth");
    static_assert(BM % (WGM * 32) == 0 && BN % (WGN * 32) == 0, "wave tile must be a multiple of 32");
    static_assert(ROWS % (RPI * NW) == 0 && BM % RPI == 0, "slab must divide into load instructions over the waves");
    static_assert(STAGES >= 2 && STAGES <= 4 && (STAGES - 2) * GPW < 64, "pipeline depth");
    static_assert(OROWS * OSTRIDE <= STAGES * STAGE, "epilogue staging must fit in the pipeline buffers");

    __shared__ u32x4 lds[STAGES * STAGE];

    const int K = a.K, Nout = a.Nout;
    const int slabs = K / BK;

    // ---- which tile(s).
    // Plain kernels: one tile per workgroup; the id is remapped so that each XCD gets a contiguous range
    // (the hardware deals workgroup ids round-robin to the 8 XCDs).
    // PERSIST kernels: one workgroup per slot of the chip walks the live tiles (LiveTileWalk).  The first
    // slabs of the next tile are requested before the epilogue of the current one (PREFETCH), which then
    // stages its output in the one pipeline buffer those loads do not touch.
    constexpr bool PREFETCH = PERSIST && OROWS * OSTRIDE <= STAGE;
    constexpr int STG = PREFETCH ? (STAGES - 1) * STAGE : 0;   // staging area, in 16-byte units
    LiveTileWalk<BM> walk;
    if constexpr (PERSIST) walk.init(a.kept, a.N, a.C, a.col_tiles, false);
    struct Tile {
        int e, rt, ct, rows;
    };
    // the tile of the current ticket (PERSIST) / of this workgroup (plain); false when there is none
    auto select = [&](Tile &t) {
        if constexpr (PERSIST) {
            if (!walk.tile(t.e, t.rt, t.ct)) return false;
        } else {
            const int per_xcd = (a.tiles + kXcds - 1) / kXcds;
            const int lid = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
            if (lid >= a.tiles) return false;
            const int per_expert = a.row_tiles * a.col_tiles;
            t.e = lid / per_expert;
            const int rem = lid - t.e * per_expert;
            t.ct = rem / a.row_tiles, t.rt = rem - t.ct * a.row_tiles;
        }
        t.rows = a.kept ? min(a.kept[t.e], a.C) : a.C;   // never trust a count beyond the buffer
        return t.rt * BM < t.rows;
    };

    // ---- loads.  src: this lane's source address in each of the wave's load instructions of a slab.
    const E *src[GPW];
    auto issue = [&](int wave, int slab, int stage) {
#pragma unroll
        for (int i = 0; i < GPW; ++i)
            __builtin_amdgcn_global_load_lds(SMILE_GPTR(src[i] + slab * BK),
                                             SMILE_LPTR(&lds[stage * STAGE + (wave + i * NW) * 64]), 16, 0, 0);
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
        const int lr = lane / PPR, lp = lane % PPR;
        const E *X = static_cast<const E *>(a.x) + (a.x_rows ? (size_t)0 : (size_t)t.e * a.C * K);
        const E *W = static_cast<const E *>(a.w) + (size_t)t.e * Nout * K;
        const int32_t *x_rows = a.x_rows ? a.x_rows + (size_t)t.e * a.C : nullptr;
#pragma unroll
        for (int i = 0; i < GPW; ++i) {
            const int row = (wave + i * NW) * RPI + lr;            // row of the stage
            const int piece = lp ^ swz<BK, SWZ>(row);
            // rows past the end of the expert's tokens / of the weight matrix re-read the last valid one
            if (row < BM) {
                const int xr = min(t.rt * BM + row, t.rows - 1);
                src[i] = X + (size_t)(x_rows ? x_rows[xr] : xr) * K + piece * 8;
            } else {
                src[i] = W + (size_t)min(t.ct * BN + row - BM, Nout - 1) * K + piece * 8;
            }
        }
#pragma unroll
        for (int s = 0; s < STAGES - 1; ++s)
            if (s < slabs) issue(wave, s, s);
    };

    Tile cur;
    if (!select(cur)) return;
    start_tile(cur);
    for (;;) {
    const int e = cur.e, rt = cur.rt, ct = cur.ct, rows = cur.rows;
    const int tid = thread_id(), lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WGM, wn = wave / WGM;
    // LDS -> MFMA operands: lane reads row (lane & 31), pieces 2*kk + (lane >> 5)
    const int frow = lane & 31, fhi = lane >> 5, fsw = swz<BK, SWZ>(lane);   // tile bases are multiples of 32
    const int xbase = (wm * WM + frow) * PPR, wbase = (BM + wn * WN + frow) * PPR;

    f32x16 acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    int stage = 0;
    const bool wave_live = rt * BM + wm * WM < rows;   // wave-uniform
    // One K slab.  ISSUE: this iteration also issues the loads of slab kt+STAGES-1 (always true in
    // the steady state, false in the last STAGES-1 iterations).  The loads are spread over the
    // k-steps and the instruction order is pinned (sched_group_barrier: one MFMA, one LDS read, ...,
    // then the k-step's share of the global loads) so that the three pipes stay busy together
    // instead of in bursts.
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
        const u32x4 *cur_stage = lds + stage * STAGE;
        bf16x8 xf[2][TM], wf[2][TN];
        auto fetch = [&](int buf, int kk) {
            const int p = (2 * kk + fhi) ^ fsw;
#pragma unroll
            for (int j = 0; j < TM; ++j) xf[buf][j] = __builtin_bit_cast(bf16x8, cur_stage[xbase + j * 32 * PPR + p]);
#pragma unroll
            for (int i = 0; i < TN; ++i) wf[buf][i] = __builtin_bit_cast(bf16x8, cur_stage[wbase + i * 32 * PPR + p]);
        };
        constexpr int KS = BK / 16;
        if (!wave_live) {
            // none of this wave's token rows exists (ragged tile): it only helps loading
            if (ISSUE) issue(wave, nxt, nstage);
            stage = stage + 1 == STAGES ? 0 : stage + 1;
            return;
        }
        fetch(0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            // this k-step's share of the next slab's load instructions
            const int l0 = GPW * kk / KS, l1 = GPW * (kk + 1) / KS;
            if (kk + 1 < KS) fetch((kk + 1) & 1, kk + 1);
            if (ISSUE) {
#pragma unroll
                for (int i = 0; i < GPW; ++i)
                    if (i >= l0 && i < l1)
                        __builtin_amdgcn_global_load_lds(SMILE_GPTR(src[i] + nxt * BK),
                                                         SMILE_LPTR(&lds[nstage * STAGE + (wave + i * NW) * 64]), 16, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = Half<E>::mfma_32x32x16(wf[kk & 1][i], xf[kk & 1][j], acc[i][j]);
            // order inside the k-step: MFMA, LDS read, MFMA, LDS read, ... then MFMA + global loads
            constexpr int NM = TM * TN, ND = TM + TN;
#pragma unroll
            for (int r = 0; r < NM; ++r) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // 1 MFMA
                if (kk + 1 < KS && r < ND) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // 1 LDS read
                if (ISSUE && r >= NM - (l1 - l0) ) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // 1 global load
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        stage = stage + 1 == STAGES ? 0 : stage + 1;
    };
    // the next tile is chosen before the main loop, so that the loads of its row counts are long back when
    // the epilogue needs them (after it where registers are short: DUAL)
    Tile nxt_tile;
    bool more = false;
    if constexpr (PERSIST && !DUAL) {
        walk.advance();
        more = select(nxt_tile);
    }
    int kt = 0;
    for (; kt + STAGES - 1 < slabs; ++kt) slab_step(std::true_type{}, kt);
    for (; kt < slabs; ++kt) slab_step(std::false_type{}, kt);
    if constexpr (PERSIST && DUAL) {
        walk.advance();
        more = select(nxt_tile);
    }

    // ---- epilogue.  Accumulator element v of a lane is (column 8*(v/4) + 4*(lane/32) + v%4,
    // row lane%32) of its 32x32 tile.  One pass per 32-row slice of the wave tiles: bias +
    // activation + rounding, 8-byte writes into a [OROWS][BN] staging tile, then row-contiguous
    // 16-byte global stores by the whole workgroup.
    const int32_t *y_rows = a.y_rows ? a.y_rows + (size_t)e * a.C : nullptr;
    const E *bias = a.bias ? static_cast<const E *>(a.bias) + (size_t)e * Nout : nullptr;
    u32x2 *stg = reinterpret_cast<u32x2 *>(lds + STG);
    constexpr int OPR = BN / 8;   // 16-byte pieces per output row
#pragma unroll
    for (int pass = 0; pass < (DUAL ? 2 : 1); ++pass) {
        void *dst = pass == 0 ? a.y : a.y2;
        E *Y = dst ? static_cast<E *>(dst) + (size_t)e * a.C * Nout : nullptr;
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): this wave's LDS reads are done
            __builtin_amdgcn_s_barrier();          // main-loop reads / the previous pass's stores are finished
            if (PREFETCH && pass == 0 && j == 0 && more) start_tile(nxt_tile);
#pragma unroll
            for (int i = 0; i < TN; ++i) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int lcol = wn * WN + i * 32 + 8 * q + 4 * fhi;      // column inside the tile
                    bf16x4 out;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float f = acc[i][j][4 * q + v];
                        if (bias) f += (float)bias[min(ct * BN + lcol + v, Nout - 1)];
                        out[v] = (E)(pass == 0 ? activate<ACT>(f) : f);
                    }
                    stg[((wm * 32 + frow) * OSTRIDE) * 2 + (lcol >> 2)] = __builtin_bit_cast(u32x2, out);
                }
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
            // staged piece `id` (already read into v) -> global memory
            auto store_piece = [&](int id, u32x4 v) {
                const int orow = id / OPR, piece = id - orow * OPR;
                const int row = rt * BM + (orow >> 5) * WM + j * 32 + (orow & 31);
                const int col = ct * BN + piece * 8;
                if (id < OROWS * OPR && row < rows && col < Nout) {
                    if constexpr (POST != 0) {
                        const u32x4 p = *reinterpret_cast<const u32x4 *>(
                            static_cast<const E *>(a.aux) + ((size_t)e * a.C + row) * Nout + col);
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            v[k] = Half<E>::pack(Half<E>::lo(v[k]) * activate_grad<POST>(Half<E>::lo(p[k])),
                                                 Half<E>::hi(v[k]) * activate_grad<POST>(Half<E>::hi(p[k])));
                    }
                    if (Y) *reinterpret_cast<u32x4 *>(Y + (size_t)row * Nout + col) = v;
                    if (pass == 0 && y_rows) {   // gate-weighted return to token order (Eq. 3), fused
                        const int tok = y_rows[row];
                        *reinterpret_cast<u32x4 *>(static_cast<E *>(a.y_tok) + (size_t)tok * Nout + col) =
                            scale_x8<E>(v, a.gate[tok]);
                    }
                }
            };
            if constexpr (DUAL) {
                // the accumulators are needed again: registers are short, one piece at a time
                for (int id = tid; id < OROWS * OPR; id += NT) {
                    const int orow = id / OPR;
                    store_piece(id, lds[STG + orow * OSTRIDE + id - orow * OPR]);
                }
            } else {
                // all of the thread's staged pieces are read before the first store, so that the LDS latencies overlap
                constexpr int NIT = (OROWS * OPR + NT - 1) / NT;
                u32x4 outv[NIT];
#pragma unroll
                for (int it = 0; it < NIT; ++it) {
                    const int id = min(tid + it * NT, OROWS * OPR - 1);
                    const int orow = id / OPR;
                    outv[it] = lds[STG + orow * OSTRIDE + id - orow * OPR];
                }
#pragma unroll
                for (int it = 0; it < NIT; ++it) store_piece(tid + it * NT, outv[it]);
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

// t0/t1 (both or neither): events that receive the begin / end timestamps of the kernel itself.
template <typename Kernel>
void launch_timed(Kernel k, dim3 grid, dim3 block, hipStream_t s, hipEvent_t t0, hipEvent_t t1, const GemmArgs &a)
{
    if (t0 && t1) hipExtLaunchKernelGGL(k, grid, block, 0, s, t0, t1, 0, a);
    else launch_kernel("grouped_gemm_nt_kernel", k, grid, block, 0, s, a);
}

template <typename E, int BM, int BN, int WGM, int WGN, int BK, int STAGES, int OCC = 1, int SWZ = 1>
hipError_t launch_half_tile(GemmArgs a, int N, int act, const Tuning &tune, hipStream_t s, hipEvent_t t0, hipEvent_t t1)
{
    a.row_tiles = (a.C + BM - 1) / BM;
    a.col_tiles = (a.Nout + BN - 1) / BN;
    a.tiles = N * a.row_tiles * a.col_tiles;
    a.N = N;
    const int slots = workgroup_slots(tune, workgroups_per_cu(WGM * WGN, OCC, STAGES * (BM + BN) * BK * 2));
    const dim3 block(WGM * WGN * 64);
    if (use_persistent_grid(tune, N, a.tiles, slots)) {
        const dim3 grid(slots);
        if (act == 0) launch_timed(grouped_gemm_nt_kernel<E, BM, BN, WGM, WGN, BK, STAGES, OCC, SWZ, 0, false, 0, true>, grid, block, s, t0, t1, a);
        else if (act == 1) launch_timed(grouped_gemm_nt_kernel<E, BM, BN, WGM, WGN, BK, STAGES, OCC, SWZ, 1, false, 0, true>, grid, block, s, t0, t1, a);
        else launch_timed(grouped_gemm_nt_kernel<E, BM, BN, WGM, WGN, BK, STAGES, OCC, SWZ, 3, false, 0, true>, grid, block, s, t0, t1, a);
        return hipGetLastError();
    }
    const dim3 grid((a.tiles + kXcds - 1) / kXcds * kXcds);
    if (act == 0) launch_timed(grouped_gemm_nt_kernel<E, BM, BN, WGM, WGN, BK, STAGES, OCC, SWZ, 0>, grid, block, s, t0, t1, a);
    else if (act == 1) launch_timed(grouped_gemm_nt_kernel<E, BM, BN, WGM, WGN, BK, STAGES, OCC, SWZ, 1>, grid, block, s, t0, t1, a);
    else launch_timed(grouped_gemm_nt_kernel<E, BM, BN, WGM, WGN, BK, STAGES, OCC, SWZ, 3>, grid, block, s, t0, t1, a);
    return hipGetLastError();
}

// The two epilogue variants of the backward pass, on the up-projection tile shape only:
//   a.y2 given: act(product) and the bare product in one launch;   post != 0: output times act'(a.aux).
template <typename E>
hipError_t launch_half_special_typed(GemmArgs a, int N, int act, int post, const Tuning &tune, hipStream_t s)
{
    constexpr int BM = 128, BN = 192;
    a.row_tiles = (a.C + BM - 1) / BM;
    a.col_tiles = (a.Nout + BN - 1) / BN;
    a.tiles = N * a.row_tiles * a.col_tiles;
    a.N = N;
    const int slots = workgroup_slots(tune, workgroups_per_cu(4, 2, 2 * (BM + BN) * 64 * 2));
    const bool persist = use_persistent_grid(tune, N, a.tiles, slots);
    const dim3 plain((a.tiles + kXcds - 1) / kXcds * kXcds), grid(persist ? dim3(slots) : plain), block(256);
    if (a.y2) {
        if (act == 1 && persist) SMILE_LAUNCH((grouped_gemm_nt_kernel<E, BM, BN, 2, 2, 64, 2, 2, 1, 1, true, 0, true>), grid, block, 0, s, a);
        else if (act == 1) SMILE_LAUNCH((grouped_gemm_nt_kernel<E, BM, BN, 2, 2, 64, 2, 2, 1, 1, true>), grid, block, 0, s, a);
        else if (persist) SMILE_LAUNCH((grouped_gemm_nt_kernel<E, BM, BN, 2, 2, 64, 2, 2, 1, 3, true, 0, true>), grid, block, 0, s, a);
        else SMILE_LAUNCH((grouped_gemm_nt_kernel<E, BM, BN, 2, 2, 64, 2, 2, 1, 3, true>), grid, block, 0, s, a);
    } else if (post == 1) {
        SMILE_LAUNCH((grouped_gemm_nt_kernel<E, BM, BN, 2, 2, 64, 2, 2, 1, 0, false, 1>), plain, block, 0, s, a);
    } else {
        SMILE_LAUNCH((grouped_gemm_nt_kernel<E, BM, BN, 2, 2, 64, 2, 2, 1, 0, false, 2>), plain, block, 0, s, a);
    }
    return hipGetLastError();
}

// Tile shapes: id -> (BM, BN, waves along M, waves along N, BK, stages, waves/SIMD budget).
// Measured on the four bf16 workloads (T = 8192..65536 tokens, 16..256 experts):
//   * up-projection (short K = d_model, wide output, GELU epilogue): 128x192 with two stages and two
//     co-resident workgroups per CU wins everywhere -- the second workgroup's MFMAs cover the first
//     one's prologue latency and activation epilogue;
//   * down-projection (long K = d_ff, narrow output): a single workgroup per CU with a deeper ring
//     wins -- four stages of 128x192 when the grid has at most one tile per CU, else three stages
//     of 128x256 (fewer weight bytes through L2 per flop).  256x128 tiles with eight waves (one tile per
//     expert and column tile when buffers hold at most 256 rows) were the choice for many small buffers while
//     every tile was a workgroup of its own; with the persistent walk over live tiles 128x256 is equal or
//     better on every shape measured (256 experts at 21 % / 50 % / 95 % fill: 386 / 440 / 653 us against
//     418 / 496 / 651), so they are only reachable through the override now.
// Larger tiles (256x128 .. 256x256) move fewer bytes L2 -> LDS per flop but were never faster here.
template <typename E>
hipError_t launch_half_typed(const GemmArgs &a, int N, int act, int tile, const Tuning &tune, hipStream_t s,
                             hipEvent_t t0 = nullptr, hipEvent_t t1 = nullptr)
{
    switch (tile) {
    case 0: return launch_half_tile<E, 128, 192, 2, 2, 64, 2, 2>(a, N, act, tune, s, t0, t1);
    case 1: return launch_half_tile<E, 128, 192, 2, 2, 64, 4, 1>(a, N, act, tune, s, t0, t1);
    case 2: return launch_half_tile<E, 128, 256, 2, 2, 64, 3, 1>(a, N, act, tune, s, t0, t1);
    case 3: return launch_half_tile<E, 256, 128, 4, 2, 64, 3, 2>(a, N, act, tune, s, t0, t1);
    case 4: return launch_half_tile<E, 128, 128, 2, 2, 32, 4, 2>(a, N, act, tune, s, t0, t1);
    case 5: return launch_half_tile<E, 64, 256, 1, 4, 64, 2, 2>(a, N, act, tune, s, t0, t1);
    case 6: return launch_half_tile<E, 256, 256, 2, 4, 32, 4, 2>(a, N, act, tune, s, t0, t1);
    default: return hipErrorInvalidValue;
    }
}
constexpr int kNumTiles = 7;

// Tile choice; Tuning::ffn_tile (0..6) overrides it for tuning runs.
int pick_tile(const Tuning &tune, int N, int C, int Nout, int K)
{
    if (tune.ffn_tile >= 0 && tune.ffn_tile < kNumTiles) return tune.ffn_tile;
    if (Nout >= K) return 0;
    const long long tiles = (long long)N * ((C + 127) / 128) * ((Nout + 191) / 192);
    return tiles <= 256 ? 1 : 2;
}

// ------------------------------------------------------------------------------------ fp32 / FMA

template <int ACT>
__global__ __launch_bounds__(256) void grouped_gemm_nt_f32_kernel(
    const float *__restrict__ x, const float *__restrict__ w, const float *__restrict__ bias,
    float *__restrict__ y, const int32_t *__restrict__ kept, int C, int Nout, int K, int row_tiles, int col_tiles,
    const int32_t *__restrict__ x_rows, const int32_t *__restrict__ y_rows, float *__restrict__ y_tok,
    const float *__restrict__ gate, float *__restrict__ y2, const float *__restrict__ aux, int post)
{
    constexpr int BT = 64, BK = 16;
    __shared__ float xs[BK][BT + 4];
    __shared__ float wsh[BK][BT + 4];

    const int per_expert = row_tiles * col_tiles;
    const int e = blockIdx.x / per_expert;
    const int rem = blockIdx.x - e * per_expert;
    const int ct = rem / row_tiles, rt = rem - ct * row_tiles;
    const int rows = kept ? min(kept[e], C) : C;
    if (rt * BT >= rows) return;

    const float *X = x + (x_rows ? (size_t)0 : (size_t)e * C * K);
    const float *W = w + (size_t)e * Nout * K;
    const int tid = threadIdx.x;
    const int lr = tid >> 2, lk = (tid & 3) * 4;            // loader: row lr, 4 floats at k offset lk
    const int xr = min(rt * BT + lr, rows - 1);
    const int xrow = x_rows ? x_rows[(size_t)e * C + xr] : xr, wrow = min(ct * BT + lr, Nout - 1);
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
    float *Y = y ? y + (size_t)e * C * Nout : nullptr;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = rt * BT + ty * 4 + i;
        if (row >= rows) continue;
        const int tok = y_rows ? y_rows[(size_t)e * C + row] : 0;
        const float g = y_rows ? gate[tok] : 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = ct * BT + tx * 4 + j;
            if (col >= Nout) continue;
            float f = acc[i][j];
            if (bias) f += bias[(size_t)e * Nout + col];
            if (y2) y2[((size_t)e * C + row) * Nout + col] = f;   // the bare product as well
            if (post) {   // times act'(aux), with the exact erf form in fp32
                const float p = aux[((size_t)e * C + row) * Nout + col];
                f *= post == 1 ? (p > 0.f ? 1.f : 0.f)
                               : 0.5f * (1.0f + erff(p * 0.70710678118654752f)) +
                                     p * 0.3989422804014327f * expf(-0.5f * p * p);
            }
            f = activate<ACT>(f);
            if (Y) Y[(size_t)row * Nout + col] = f;
            if (y_rows) y_tok[(size_t)tok * Nout + col] = f * g;
        }
    }
}

hipError_t launch_f32(const float *x, const float *w, const float *bias, float *y, const int32_t *kept, int N,
                      int C, int Nout, int K, int act, hipStream_t s, const int32_t *x_rows = nullptr,
                      const int32_t *y_rows = nullptr, float *y_tok = nullptr, const float *gate = nullptr,
                      float *y2 = nullptr, const float *aux = nullptr, int post = 0)
{
    const int row_tiles = (C + 63) / 64, col_tiles = (Nout + 63) / 64;
    const dim3 grid(N * row_tiles * col_tiles), block(256);
    if (act == 0)
        SMILE_LAUNCH(grouped_gemm_nt_f32_kernel<0>, grid, block, 0, s, x, w, bias, y, kept, C, Nout, K, row_tiles, col_tiles,
                           x_rows, y_rows, y_tok, gate, y2, aux, post);
    else if (act == 1)
        SMILE_LAUNCH(grouped_gemm_nt_f32_kernel<1>, grid, block, 0, s, x, w, bias, y, kept, C, Nout, K, row_tiles, col_tiles,
                           x_rows, y_rows, y_tok, gate, y2, aux, post);
    else
        SMILE_LAUNCH(grouped_gemm_nt_f32_kernel<2>, grid, block, 0, s, x, w, bias, y, kept, C, Nout, K, row_tiles, col_tiles,
                           x_rows, y_rows, y_tok, gate, y2, aux, post);
    return hipGetLastError();
}


// dtype dispatch of the two MFMA launchers
hipError_t launch_half(int dtype, const GemmArgs &a, int N, int act, int tile, const Tuning &tune, hipStream_t s,
                       hipEvent_t t0 = nullptr, hipEvent_t t1 = nullptr)
{
    if (dtype == SMILE_DTYPE_BF16) return launch_half_typed<__bf16>(a, N, act, tile, tune, s, t0, t1);
    return launch_half_typed<_Float16>(a, N, act, tile, tune, s, t0, t1);
}

hipError_t launch_half_special(int dtype, const GemmArgs &a, int N, int act, int post, const Tuning &tune, hipStream_t s)
{
    if (dtype == SMILE_DTYPE_BF16) return launch_half_special_typed<__bf16>(a, N, act, post, tune, s);
    return launch_half_special_typed<_Float16>(a, N, act, post, tune, s);
}

}  // namespace

bool use_persistent_grid(const Tuning &tune, int N, long long tiles, int slots)
{
    if (N > 4096) return false;   // the tile walk keeps one lane per 64 groups
    if (tune.persist >= 0) return tune.persist != 0;
    return tiles >= 4LL * slots;
}

hipError_t launch_grouped_gemm_nt(int dtype, const GroupedGemm &g, hipStream_t s)
{
    const int act = g.act == 0 ? 0 : (g.act == 1 ? 1 : 2);
    if ((g.y2 && act == 0) || (g.post && (act != 0 || g.y2 || !g.aux))) return hipErrorInvalidValue;
    if (is_half(dtype)) {
        if (g.K % 64 || g.Nout % 8) return hipErrorInvalidValue;
        GemmArgs a{g.x, g.w, g.bias, g.y, g.kept, g.C, g.Nout, g.K, 0, 0, 0, g.x_rows, nullptr, nullptr, nullptr, g.y2, g.aux};
        if (g.y2 || g.post) return launch_half_special(dtype, a, g.N, act, g.post, g.tune, s);
        return launch_half(dtype, a, g.N, act, pick_tile(g.tune, g.N, g.C, g.Nout, g.K), g.tune, s);
    }
    if (g.K % 4) return hipErrorInvalidValue;
    return launch_f32(static_cast<const float *>(g.x), static_cast<const float *>(g.w),
                      static_cast<const float *>(g.bias), static_cast<float *>(g.y), g.kept, g.N, g.C, g.Nout, g.K, act,
                      s, g.x_rows, nullptr, nullptr, nullptr, static_cast<float *>(g.y2),
                      static_cast<const float *>(g.aux), g.post);
}

hipError_t launch_expert_ffn_up(const LayerDesc &d, const Workspace &ws, const void *xe,
                                const int32_t *kept_count, const void *w1, const void *b1, hipStream_t s,
                                hipEvent_t t0, hipEvent_t t1, const void *x_tokens, void *h_save, void *pre_save)
{
    const int N = d.n_groups * d.m_local;
    const int act = d.act == SMILE_ACT_RELU ? 1 : 2;
    // x_tokens: read the rows straight from the token matrix through the slot -> token map
    const int32_t *x_rows = x_tokens ? ws.slot_token : nullptr;
    const void *src = x_tokens ? x_tokens : xe;
    if (h_save) {   // training: the hidden activation and its pre-activation go to the caller's buffers
        if (t0 && t1) (void)hipEventRecord(t0, s);
        const hipError_t err = launch_grouped_gemm_nt(
            d.dtype, GroupedGemm{src, w1, h_save, pre_save, kept_count, N, d.capacity, d.d_ff, d.d_model, act, b1, x_rows,
                                 nullptr, 0, d.tune}, s);
        if (t0 && t1) (void)hipEventRecord(t1, s);
        return err;
    }
    if (is_half(d.dtype)) {
        GemmArgs g{src, w1, b1, ws.hidden, kept_count, d.capacity, d.d_ff, d.d_model, 0, 0, 0, x_rows, nullptr, nullptr, nullptr};
        return launch_half(d.dtype, g, N, act, pick_tile(d.tune, N, d.capacity, d.d_ff, d.d_model), d.tune, s, t0, t1);
    }
    if (t0 && t1) (void)hipEventRecord(t0, s);
    const hipError_t err = launch_f32(static_cast<const float *>(src), static_cast<const float *>(w1),
                                      static_cast<const float *>(b1), static_cast<float *>(ws.hidden), kept_count, N,
                                      d.capacity, d.d_ff, d.d_model, act, s, x_rows);
    if (t0 && t1) (void)hipEventRecord(t1, s);
    return err;
}

hipError_t launch_expert_ffn_down(const LayerDesc &d, const Workspace &ws, const int32_t *kept_count,
                                  const void *w2, const void *b2, void *ye, hipStream_t s, void *y_tokens,
                                  const float *gate, const void *h_saved)
{
    const int N = d.n_groups * d.m_local;
    const void *hidden = h_saved ? h_saved : ws.hidden;
    // y_tokens: also (or, with ye == null, only) return the rows to token order, times the gate
    const int32_t *y_rows = y_tokens ? ws.slot_token : nullptr;
    if (is_half(d.dtype)) {
        GemmArgs g{hidden, w2, b2, ye, kept_count, d.capacity, d.d_model, d.d_ff, 0, 0, 0, nullptr, y_rows, y_tokens, gate};
        return launch_half(d.dtype, g, N, 0, pick_tile(d.tune, N, d.capacity, d.d_model, d.d_ff), d.tune, s);
    }
    return launch_f32(static_cast<const float *>(hidden), static_cast<const float *>(w2),
                      static_cast<const float *>(b2), static_cast<float *>(ye), kept_count, N, d.capacity,
                      d.d_model, d.d_ff, 0, s, nullptr, y_rows, static_cast<float *>(y_tokens), gate);
}

}  // namespace smile
