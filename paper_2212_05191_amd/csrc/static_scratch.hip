// smile_route_bilevel_static: the routing step for callers that cannot allocate (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc).  Same kernels and results as smile_route_bilevel; the
// routing workspace (per-block histograms, partial probability sums, block-local ranks) lives in a file-scope
// device array instead of a ctx's hipMalloc'ed workspace, and there is no ctx at all.
//
// Every device the library runs on holds its own copy of the array at its own address until the process ends.
// In host code the array's name is only a stand-in for the symbol: its device address is fetched once per
// device with hipGetSymbolAddress and that pointer is what the kernels receive.  The array keeps the previous
// call's contents; the routing kernels overwrite every element they later read, so nothing has to be cleared.
// Calls that overlap on one device (two streams, two threads) share the array and race.
#include <mutex>

#include "smile_internal.hpp"

namespace smile {

namespace {

constexpr size_t kStaticScratchBytes = SMILE_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once known

// The device address of this device's copy of the array (null on failure).  The first call on a device asks
// the runtime; later calls only read the table.
void *scratch_address()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return nullptr;
    }
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool bad(const void *p) { return p == nullptr || !aligned16(p); }
bool bad_opt(const void *p) { return p != nullptr && !aligned16(p); }

}  // namespace

}  // namespace smile

using namespace smile;

extern "C" smile_status smile_route_bilevel_static(const smile_layer_desc *desc, const float *logits_inter,
                                                   const float *logits_intra, const float *bias_inter,
                                                   const float *bias_intra, int32_t *group_idx, int32_t *local_idx,
                                                   int32_t *pos_in_group, int32_t *slot, float *gate, float *p_top,
                                                   float *q_top, int32_t *group_count, int32_t *local_count,
                                                   int32_t *expert_count, int32_t *kept_count, float *p_sum,
                                                   float *q_sum, void *stream)
{
    const smile_status st = smile_validate_desc(desc);
    if (st != SMILE_OK) return st;
    if (bad(logits_inter) || bad(logits_intra) || bad_opt(bias_inter) || bad_opt(bias_intra) || bad(group_idx) ||
        bad(local_idx) || bad(pos_in_group) || bad(slot) || bad(gate) || bad(p_top) || bad(q_top) ||
        bad(group_count) || bad(local_count) || bad(expert_count) || bad(kept_count) || bad(p_sum) || bad(q_sum))
        return SMILE_INVALID_ARG;
    // the routing part of the workspace layout ends where the slot -> token map begins
    const Layout L = workspace_layout(*desc);
    if (L.off_slot_token > kStaticScratchBytes) return SMILE_WORKSPACE;
    char *base = static_cast<char *>(scratch_address());
    if (!base) return SMILE_HIP_ERROR;
    Workspace ws{};
    ws.block_expert_hist = reinterpret_cast<int32_t *>(base + L.off_block_expert_hist);
    ws.block_group_hist = reinterpret_cast<int32_t *>(base + L.off_block_group_hist);
    ws.block_p_sum = reinterpret_cast<float *>(base + L.off_block_p_sum);
    ws.block_q_sum = reinterpret_cast<float *>(base + L.off_block_q_sum);
    ws.rank_in_block = reinterpret_cast<int32_t *>(base + L.off_rank_in_block);
    ws.pos_in_block = reinterpret_cast<int32_t *>(base + L.off_pos_in_block);
    const hipError_t err = launch_route(*desc, ws, logits_inter, logits_intra, bias_inter, bias_intra, group_idx,
                                        local_idx, pos_in_group, slot, gate, p_top, q_top, group_count, local_count,
                                        expert_count, kept_count, p_sum, q_sum, static_cast<hipStream_t>(stream));
    if (err == hipSuccess) return SMILE_OK;
    (void)hipGetLastError();
    return SMILE_HIP_ERROR;
}
