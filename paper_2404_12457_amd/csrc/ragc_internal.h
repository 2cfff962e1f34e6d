// Internal launch interface between the C-ABI front end (ragc_api.cpp) and the
// gfx950 kernels.  Not installed; the public contract is include/ragc.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ragc {

constexpr int kBlock = 16;  // tokens per paged block

// Records the text that ragc_last_error() returns on this thread; returns `code`.
int set_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Everything a device kernel needs to find the K/V of a batch.
struct PagedBatch {
    const void* pool_k;
    const void* pool_v;
    int64_t block_stride;  // elements between blocks of one plane
    const int32_t* prefix_len;
    const int32_t* new_len;
    const int32_t* new_start;
    const int32_t* block_table;
    int32_t table_stride;
    int32_t num_reqs;
    int32_t kv_heads;
    int32_t head_dim;
};

struct AttnLaunch {
    PagedBatch b;
    const void* q;
    const void* k_new;
    const void* v_new;
    void* out;
    void* pool_k_w;  // writable aliases of the pool planes (fused append)
    void* pool_v_w;
    void* partial;   // workspace for the partial results of work items split along the keys (bf16 path)
    int32_t q_heads;
    int32_t group;      // q_heads / kv_heads
    uint32_t group_magic;  // ceil(2^32 / group), 0 for group 1: row / group by one multiply in the kernels
    float scale_log2e;  // softmax_scale * log2(e)
    int32_t fused_append;
    int32_t max_new;  // max over requests of new_len (host-side)
    int32_t total_new;
};

hipError_t launch_attn_f32(const AttnLaunch& a, hipStream_t s);

// bf16 path: the host orders the (request, row tile) work items by cost and passes
// them in the kernel argument buffer (no device staging); long lists go out in
// several launches.
constexpr int kAttnRowsPerItem = 128;
constexpr int kAttnMaxItems = 224;
// One work item carries the request's lengths, so a workgroup needs no memory round trip
// before it can look up its first block ids.
struct AttnItem {
    uint32_t req_tile;   // request << 16 | row tile
    int32_t prefix_len;
    int32_t new_len;
    int32_t new_start;
};
// bytes of one partial result: O [rows][D] fp32, then (max, sum) per row
inline int64_t attn_partial_bytes(int head_dim) { return (int64_t)kAttnRowsPerItem * (head_dim + 2) * 4; }
constexpr int kAttnMaxSplits = 16;
// With `splits` = S > 1 every work item appears S times in a row (entry e is copy e % S) and
// entry e leaves its partial result in slot part_base + e of the workspace.
struct AttnWorkList {
    int32_t n;
    int32_t splits;
    int32_t part_base;
    int32_t pad;
    AttnItem item[kAttnMaxItems];
};
enum AttnVariant {
    kAttnVariantOneGroup = 0,   // 4 waves per workgroup, two workgroups per CU
    kAttnVariantTwoGroups = 1,  // 8 waves per workgroup on alternating key tiles
    kAttnVariantCount = 2
};
// number of 64-key tiles the work item (row tile `tile` of kAttnRowsPerItem rows) walks
int attn_bf16_item_cost(int prefix, int new_len, int group, int tile);
hipError_t launch_attn_bf16(const AttnLaunch& a, const AttnWorkList& wl, int variant, hipStream_t s);
// second pass after a launch of split items: `wl` lists copy 0 of every item; combines the partial results into `out`
hipError_t launch_attn_bf16_merge(const AttnLaunch& a, const AttnWorkList& wl, hipStream_t s);

hipError_t launch_append(const PagedBatch& b, void* pool_k, void* pool_v, const void* k_new, const void* v_new,
                         int32_t total_new, int esize, hipStream_t s);
hipError_t launch_gather(const PagedBatch& b, int32_t req, int32_t length, void* k_out, void* v_out, int esize,
                         hipStream_t s);

// Block copies between the device pool and a host-mapped pinned pool.  Pairs are
// passed by value in the kernel argument buffer, so no device staging is needed.
constexpr int kSwapPairsPerLaunch = 384;
struct SwapPairs {
    int32_t dev[kSwapPairsPerLaunch];
    int32_t slot[kSwapPairsPerLaunch];
};
hipError_t launch_swap(char* dev_k, char* dev_v, int64_t dev_block_bytes_stride, char* host_k, char* host_v,
                       int64_t host_block_bytes_stride, int64_t plane_block_bytes, const SwapPairs& pairs, int32_t n,
                       int to_device, hipStream_t s);

}  // namespace ragc
