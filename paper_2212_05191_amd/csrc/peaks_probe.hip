// Stand-alone microbenchmark of the rates an MI355X (gfx950) actually delivers, for the denominators of the
// "fraction of measured peak" figures that bench.py reports beside the nominal ones (8 TB/s HBM, 2.5 PFLOP/s dense
// bf16).  It shares no code with the library.  Every kernel is a bounded loop over in-bounds addresses.
//
//   copy          plain device copy, 1 GiB read + 1 GiB written (16 bytes per lane)
//   read          read-only stream of 2 GiB (register loads, 16 bytes per lane, 8 loads in flight per lane)
//   fill          store-only stream of 2 GiB (16 bytes per lane, no reads)
//   weight-tiles  the expert GEMM's weight access pattern, read-only, through direct-to-LDS loads: a workgroup
//                 streams tiles of 192 rows x K bf16, slab after slab (128 bytes of every row at a K*2-byte
//                 stride), `depth - 1` slabs in flight; the same bytes laid out contiguously per slab for
//                 comparison
//   weight-frags  the same bytes streamed straight into registers by independent waves (no LDS, no barrier), in the
//                 MFMA operand layout (a lane's 16 bytes of its own row) and in the coalesced layout
//   l2            L2-resident data (a window of a few MB per XCD) read by register loads and by direct-to-LDS loads
//   lds           ds_read_b128 issue rate (bytes per second out of LDS, chip-wide)
//   mfma          back-to-back v_mfma_f32_32x32x16_bf16 with no memory traffic, 1 and 2 waves per SIMD
//
// Usage: peaks_probe [section ...]   (no argument: all sections).  Prints one line per measurement.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

#define CK(x)                                                                              \
    do {                                                                                   \
        hipError_t e_ = (x);                                                               \
        if (e_ != hipSuccess) {                                                            \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);          \
            exit(1);                                                                       \
        }                                                                                  \
    } while (0)
#define GPTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define LPTR(p) ((__attribute__((address_space(3))) void *)(p))

static int g_cus = 256;

// ------------------------------------------------------------------------------------------ HBM streams
__global__ __launch_bounds__(256) void copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// stores only: the ceiling of a kernel whose traffic is its output (the weight-gradient GEMMs of small experts)
__global__ __launch_bounds__(256) void fill_kernel(u32x4 *__restrict__ dst, size_t n16, uint32_t value)
{
    const size_t stride = (size_t)gridDim.x * 256;
    const u32x4 v = {value, value, value, value};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = v;
}

__global__ __launch_bounds__(256) void read_kernel(const u32x4 *__restrict__ src, size_t n16, uint32_t *out)
{
    const size_t stride = (size_t)gridDim.x * 256;
    u32x4 acc = {0, 0, 0, 0};
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    for (; i < n16; i += stride) acc ^= src[i];
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) out[0] = 1;   // keeps the loads alive
}

// MODE 0: tile rows K elements apart (the GEMM operand as it lies in memory); 1: each slab contiguous
template <int MODE, int DEPTH>
__global__ __launch_bounds__(256) void weight_tile_kernel(const u32x4 *w, int K, int tiles, uint32_t *out)
{
    constexpr int ROWS = 192, GPW = ROWS / 8 / 4;   // 6 load instructions per wave and slab (24 KB per slab)
    __shared__ u32x4 lds[DEPTH][ROWS * 8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slabs = K / 64;
    const size_t tile_pieces = (size_t)ROWS * K / 8;
    for (int t = blockIdx.x; t < tiles; t += gridDim.x) {
        const u32x4 *base = w + (size_t)t * tile_pieces;
        auto issue = [&](int s, int st) {
#pragma unroll
            for (int i = 0; i < GPW; ++i) {
                const int grp = wave + i * 4;   // group of 8 rows
                const int row = grp * 8 + (lane >> 3), piece = lane & 7;
                const size_t idx = MODE == 0 ? (size_t)row * (K / 8) + (size_t)s * 8 + piece
                                             : (size_t)s * (ROWS * 8) + (size_t)row * 8 + piece;
                __builtin_amdgcn_global_load_lds(GPTR(base + idx), LPTR(&lds[st][grp * 64]), 16, 0, 0);
            }
        };
        for (int s = 0; s < DEPTH - 1 && s < slabs; ++s) issue(s, s);
        for (int s = 0; s < slabs; ++s) {
            if (s + DEPTH - 1 < slabs) {
                issue(s + DEPTH - 1, (s + DEPTH - 1) % DEPTH);
                constexpr int left = (DEPTH - 1) * GPW;   // loads that may still be in flight
                __builtin_amdgcn_s_waitcnt(0x0F70 | (left & 15) | ((left >> 4) << 14));
            } else {
                __builtin_amdgcn_s_waitcnt(0x0F70);
            }
            __builtin_amdgcn_s_barrier();
        }
    }
    out[blockIdx.x * 256 + tid] = lds[0][tid][0];
}

// Weight rows streamed straight into registers, no LDS: every wave owns 64 rows of K bf16 (rows K*2 bytes apart)
// and keeps DEPTH 64-deep slabs (8 loads of 16 bytes per lane each) in flight.
//   MODE 0: MFMA operand layout -- lane (r = lane % 32, h = lane / 32) loads 16 bytes of row r (or 32 + r) at
//           k-offset 16*kk + 8*h: an instruction touches 32 rows x 32 bytes
//   MODE 1: coalesced layout -- 8 consecutive lanes cover 128 bytes of one row: an instruction touches 8 rows
template <int MODE, int DEPTH>
__global__ __launch_bounds__(256) void weight_frag_kernel(const u32x4 *w, int K, int tiles, uint32_t *out)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int slabs = K / 64, row16 = K / 8;   // 16-byte units per row
    u32x4 acc = {0, 0, 0, 0};
    for (int t = blockIdx.x * 4 + wave; t < tiles; t += gridDim.x * 4) {
        const u32x4 *base = w + (size_t)t * 64 * row16;
        auto addr = [&](int s, int i) {   // i-th load of slab s
            if (MODE == 0) return base + (size_t)((i >> 2) * 32 + (lane & 31)) * row16 + s * 8 + (i & 3) * 2 + (lane >> 5);
            return base + (size_t)(i * 8 + (lane >> 3)) * row16 + s * 8 + (lane & 7);
        };
        u32x4 buf[DEPTH][8];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
#pragma unroll
            for (int i = 0; i < 8; ++i) buf[d][i] = *addr(d < slabs ? d : slabs - 1, i);
        for (int s = 0; s < slabs; s += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
#pragma unroll
                for (int i = 0; i < 8; ++i) acc ^= buf[d][i];
                const int nx = s + d + DEPTH < slabs ? s + d + DEPTH : slabs - 1;
#pragma unroll
                for (int i = 0; i < 8; ++i) buf[d][i] = *addr(nx, i);
            }
        }
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc ^= buf[d][i];
    }
    out[blockIdx.x * 256 + tid] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

// ------------------------------------------------------------------------------------------ L2 -> CU
// every workgroup streams from a window shared by the workgroups of its XCD (ids are dealt round-robin to the XCDs)
template <int MODE>
__global__ __launch_bounds__(256) void l2_kernel(const u32x4 *buf, size_t window16, int iters, uint32_t *out)
{
    __shared__ u32x4 lds[2048];
    const int xcd = blockIdx.x % 8;
    const u32x4 *base = buf + (size_t)xcd * window16;
    const int tid = threadIdx.x, wave = tid >> 6;
    size_t off = ((size_t)(blockIdx.x / 8) * 977 * 256) % window16;
    u32x4 acc = {0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t idx = (off + (size_t)u * 256 + tid) % window16;
            if (MODE == 0) acc ^= base[idx];
            else __builtin_amdgcn_global_load_lds(GPTR(base + idx), LPTR(&lds[(u * 4 + wave) * 64]), 16, 0, 0);
        }
        off = (off + 8 * 256) % window16;
        if (MODE == 1) __builtin_amdgcn_s_waitcnt(0x0F70);
    }
    if (MODE == 1) {
        __syncthreads();
        acc = lds[tid];
    }
    out[blockIdx.x * 256 + tid] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

// ------------------------------------------------------------------------------------------ LDS reads
__global__ __launch_bounds__(256) void lds_kernel(int iters, uint32_t *out)
{
    __shared__ u32x4 lds[4096];   // 64 KB
    const int tid = threadIdx.x;
    for (int i = tid; i < 4096; i += 256) lds[i] = u32x4{(uint32_t)i, 1u, 2u, 3u};
    __syncthreads();
    u32x4 acc = {0, 0, 0, 0};
    int p = tid;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) acc ^= lds[(p + u * 256) & 4095];   // consecutive lanes, consecutive 16-byte words
        p = (p + 64) & 4095;
    }
    out[blockIdx.x * 256 + tid] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

// ------------------------------------------------------------------------------------------ MFMA issue rate
__global__ __launch_bounds__(256) void mfma_kernel(int iters, float *out)
{
    bf16x8 a, b;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        a[k] = (__bf16)(float)((threadIdx.x + k) & 3);
        b[k] = (__bf16)(float)((threadIdx.x * 3 + k) & 3);
    }
    f32x16 acc[6];
#pragma unroll
    for (int i = 0; i < 6; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 6; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 6; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// ------------------------------------------------------------------------------------------ host side
template <typename F>
static double time_us(F launch, int reps = 3)
{
    hipEvent_t s, t;
    CK(hipEventCreate(&s));
    CK(hipEventCreate(&t));
    launch();   // warm-up
    CK(hipDeviceSynchronize());
    double best = 1e30;
    for (int r = 0; r < reps; ++r) {
        CK(hipEventRecord(s));
        launch();
        CK(hipEventRecord(t));
        CK(hipDeviceSynchronize());
        float ms = 0.f;
        CK(hipEventElapsedTime(&ms, s, t));
        if (ms * 1e3 < best) best = ms * 1e3;
    }
    CK(hipEventDestroy(s));
    CK(hipEventDestroy(t));
    return best;
}

static bool wanted(int argc, char **argv, const char *name)
{
    if (argc <= 1) return true;
    for (int i = 1; i < argc; ++i)
        if (!strcmp(argv[i], name)) return true;
    return false;
}

template <int MODE, int DEPTH>
static void run_weight_frags(const char *name, const u32x4 *w, int K, int tiles, int per_cu, uint32_t *out)
{
    const dim3 grid(g_cus * per_cu);
    const double us = time_us([&] { hipLaunchKernelGGL((weight_frag_kernel<MODE, DEPTH>), grid, dim3(256), 0, 0, w, K, tiles, out); });
    const double bytes = (double)tiles * 64 * K * 2;   // the repeats of a tile's last slabs are cache hits
    printf("weight-frags  %-30s slabs in flight %d  workgroups/CU %d : %8.1f us  %6.2f TB/s\n", name, DEPTH, per_cu, us,
           bytes / us / 1e6);
}

template <int MODE, int DEPTH>
static void run_weight_tiles(const char *name, const u32x4 *w, int K, int tiles, int per_cu, uint32_t *out)
{
    const dim3 grid(g_cus * per_cu);
    const double us = time_us([&] { hipLaunchKernelGGL((weight_tile_kernel<MODE, DEPTH>), grid, dim3(256), 0, 0, w, K, tiles, out); });
    const double bytes = (double)tiles * 192 * K * 2;
    printf("weight-tiles  %-30s slabs in flight %d  workgroups/CU %d : %8.1f us  %6.2f TB/s\n", name, DEPTH - 1, per_cu, us,
           bytes / us / 1e6);
}

int main(int argc, char **argv)
{
    int dev = 0;
    CK(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, dev));
    g_cus = prop.multiProcessorCount;
    printf("device %s  CUs %d  clock %d MHz  memory clock %d MHz\n", prop.gcnArchName, g_cus, prop.clockRate / 1000,
           prop.memoryClockRate / 1000);
    uint32_t *out;
    CK(hipMalloc(&out, (size_t)g_cus * 8 * 256 * 4));

    if (wanted(argc, argv, "copy") || wanted(argc, argv, "read") || wanted(argc, argv, "fill")) {
        const size_t bytes = (size_t)1 << 30;
        u32x4 *a, *b;
        CK(hipMalloc(&a, 2 * bytes));
        CK(hipMemset(a, 1, 2 * bytes));
        b = a + bytes / 16;
        if (wanted(argc, argv, "copy"))
            for (int per_cu : {4, 8, 16}) {
                const double us = time_us([&] { hipLaunchKernelGGL(copy_kernel, dim3(g_cus * per_cu), dim3(256), 0, 0, a, b, bytes / 16); });
                printf("copy          1 GiB read + 1 GiB written      workgroups/CU %2d : %8.1f us  %6.2f TB/s (read + written)\n",
                       per_cu, us, 2.0 * bytes / us / 1e6);
            }
        if (wanted(argc, argv, "read"))
            for (int per_cu : {4, 8, 16}) {
                const double us = time_us([&] { hipLaunchKernelGGL(read_kernel, dim3(g_cus * per_cu), dim3(256), 0, 0, a, 2 * bytes / 16, out); });
                printf("read          2 GiB, register loads            workgroups/CU %2d : %8.1f us  %6.2f TB/s\n", per_cu, us,
                       2.0 * bytes / us / 1e6);
            }
        if (wanted(argc, argv, "fill"))
            for (int per_cu : {4, 8, 16}) {
                const double us = time_us([&] { hipLaunchKernelGGL(fill_kernel, dim3(g_cus * per_cu), dim3(256), 0, 0, a, 2 * bytes / 16, 7u); });
                printf("fill          2 GiB written, no reads          workgroups/CU %2d : %8.1f us  %6.2f TB/s\n", per_cu, us,
                       2.0 * bytes / us / 1e6);
            }
        CK(hipFree(a));
    }

    if (wanted(argc, argv, "weight-tiles")) {
        const int K = 1024, tiles = 5632;   // 5632 tiles x 384 KB = 2.2 GB: one projection of 256 experts of 1024 x 4096
        u32x4 *w;
        const size_t bytes = (size_t)tiles * 192 * K * 2;
        CK(hipMalloc(&w, bytes));
        CK(hipMemset(w, 1, bytes));
        run_weight_tiles<0, 2>("rows 2 KB apart (as stored)", w, K, tiles, 2, out);
        run_weight_tiles<1, 2>("slab-contiguous", w, K, tiles, 2, out);
        run_weight_tiles<0, 3>("rows 2 KB apart (as stored)", w, K, tiles, 2, out);
        run_weight_tiles<1, 3>("slab-contiguous", w, K, tiles, 2, out);
        run_weight_tiles<0, 4>("rows 2 KB apart (as stored)", w, K, tiles, 1, out);
        run_weight_tiles<0, 6>("rows 2 KB apart (as stored)", w, K, tiles, 1, out);
        run_weight_tiles<1, 6>("slab-contiguous", w, K, tiles, 1, out);
        CK(hipFree(w));
    }

    if (wanted(argc, argv, "weight-frags")) {
        const int K = 1024, tiles = 16896;   // 16896 wave tiles x 128 KB = 2.2 GB
        u32x4 *w;
        const size_t bytes = (size_t)tiles * 64 * K * 2;
        CK(hipMalloc(&w, bytes));
        CK(hipMemset(w, 1, bytes));
        run_weight_frags<0, 2>("MFMA layout, 32 rows x 32 B", w, K, tiles, 2, out);
        run_weight_frags<0, 3>("MFMA layout, 32 rows x 32 B", w, K, tiles, 2, out);
        run_weight_frags<0, 4>("MFMA layout, 32 rows x 32 B", w, K, tiles, 2, out);
        run_weight_frags<1, 2>("coalesced, 8 rows x 128 B", w, K, tiles, 2, out);
        run_weight_frags<1, 3>("coalesced, 8 rows x 128 B", w, K, tiles, 2, out);
        run_weight_frags<1, 4>("coalesced, 8 rows x 128 B", w, K, tiles, 2, out);
        run_weight_frags<1, 3>("coalesced, 8 rows x 128 B", w, K, tiles, 1, out);
        CK(hipFree(w));
    }

    if (wanted(argc, argv, "l2")) {
        u32x4 *buf;
        const size_t total = (size_t)8 * 16 << 20;
        CK(hipMalloc(&buf, total));
        CK(hipMemset(buf, 1, total));
        const int iters = 2000;
        for (size_t window : {(size_t)1 << 20, (size_t)3 << 20})
            for (int per_cu : {2, 4, 8}) {
                const dim3 grid(g_cus * per_cu);
                const double bytes = (double)grid.x * iters * 8 * 256 * 16;
                double us = time_us([&] { hipLaunchKernelGGL(l2_kernel<0>, grid, dim3(256), 0, 0, buf, window / 16, iters, out); });
                printf("l2            register loads   window/XCD %4.1f MB  workgroups/CU %d : %6.2f TB/s\n", window / 1048576.0, per_cu,
                       bytes / us / 1e6);
                us = time_us([&] { hipLaunchKernelGGL(l2_kernel<1>, grid, dim3(256), 0, 0, buf, window / 16, iters, out); });
                printf("l2            direct-to-LDS    window/XCD %4.1f MB  workgroups/CU %d : %6.2f TB/s\n", window / 1048576.0, per_cu,
                       bytes / us / 1e6);
            }
        CK(hipFree(buf));
    }

    if (wanted(argc, argv, "lds")) {
        const int iters = 4000;
        for (int per_cu : {1, 2}) {
            const dim3 grid(g_cus * per_cu);
            const double us = time_us([&] { hipLaunchKernelGGL(lds_kernel, grid, dim3(256), 0, 0, iters, out); });
            const double bytes = (double)grid.x * 256 * iters * 16 * 16;
            printf("lds           ds_read_b128                      workgroups/CU %d : %6.1f TB/s chip-wide, %5.1f B/clk/CU at %d MHz\n",
                   per_cu, bytes / us / 1e6, bytes / us / 1e6 * 1e12 / g_cus / (prop.clockRate * 1e3), prop.clockRate / 1000);
        }
    }

    if (wanted(argc, argv, "mfma")) {
        const int iters = 20000;
        float *fout;
        CK(hipMalloc(&fout, (size_t)g_cus * 2 * 256 * 4));
        for (int per_cu : {1, 2}) {
            const dim3 grid(g_cus * per_cu);
            const double us = time_us([&] { hipLaunchKernelGGL(mfma_kernel, grid, dim3(256), 0, 0, iters, fout); });
            const double flop = (double)grid.x * 4 * iters * 24 * 2.0 * 32 * 32 * 16;
            printf("mfma          v_mfma_f32_32x32x16_bf16, no loads   waves/SIMD %d : %8.1f us  %7.1f TFLOP/s\n", per_cu, us,
                   flop / us / 1e6);
        }
        CK(hipFree(fout));
    }
    CK(hipFree(out));
    return 0;
}
