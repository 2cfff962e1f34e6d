// Byte-moving kernels of the paged K/V store: append of fresh K/V rows into
// their paged slots (paper Sec. 4: the tensors of the accessed documents are
// cached after the first token), gather of a request's logical sequence (test
// helper), and whole-block copies between the device pool and a host-mapped
// pinned pool (Sec. 5.1 "Swap out only once").  All three are HBM- or
// host-link-bound copies in 16-byte units; values are never interpreted.
#include "ragc_internal.h"

namespace ragc {
namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Request that owns packed row t: largest r with new_start[r] <= t (new_start is
// increasing and new_start[0] <= t < new_start[num_reqs]).
__device__ __forceinline__ int find_request(const int32_t* __restrict__ new_start, int num_reqs, int t) {
    int lo = 0, hi = num_reqs;  // invariant: new_start[lo] <= t < new_start[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (new_start[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// Append.  A workgroup owns 16 consecutive packed rows (tokens) and a run of kv heads: 1024
// 16-byte chunks per plane, four of K and four of V per thread, all loads issued before the
// first store.  For one head the 16 rows land next to each other in the pool (a 16-token block
// is contiguous per head), so a wave writes whole 1 KiB runs and the workgroup reads 16 row
// pieces of 1 KiB or more; both sides stay within a few DRAM pages.  The rows are resolved to
// their paged slots once per workgroup (16 threads) and shared through LDS.  Loads and stores
// are nontemporal: nothing here is touched twice.
constexpr int kAppendRows = 16;
constexpr int kAppendUnroll = 4;
constexpr int kAppendChunksPerGroup = 256 * kAppendUnroll;

__global__ __launch_bounds__(256) void append_kernel(PagedBatch b, char* __restrict__ pool_k, char* __restrict__ pool_v,
                                                     const char* __restrict__ k_new, const char* __restrict__ v_new,
                                                     int total_new, int esize, int head_groups) {
    __shared__ long long slot_off[kAppendRows];  // byte offset of (block, head 0, slot) of each row; -1: no such row
    const int first_row = b.new_start[0];  // a sub-batch may start anywhere in the packed arrays
    // the head group varies fastest, so workgroups that run together cover whole source rows
    const int hg = blockIdx.x % head_groups;
    const int t0 = (blockIdx.x / head_groups) * kAppendRows;
    const int head_bytes = b.head_dim * esize;
    if (threadIdx.x < kAppendRows) {
        const int t_rel = t0 + threadIdx.x;
        long long off = -1;
        if (t_rel < total_new) {
            const int t = first_row + t_rel;
            const int r = find_request(b.new_start, b.num_reqs, t);
            const int pos = b.prefix_len[r] + (t - b.new_start[r]);
            const int blk = b.block_table[(long long)r * b.table_stride + (pos >> 4)];
            off = ((long long)blk * b.block_stride + (long long)(pos & 15) * b.head_dim) * esize;
        }
        slot_off[threadIdx.x] = off;
    }
    __syncthreads();
    // chunks per head is 8, 16 or 32 (head_dim 64 or 128, 2 or 4 bytes per element)
    const int cph_shift = __ffs(head_bytes >> 4) - 1;
    const int per_head_shift = cph_shift + 4;  // chunks of one head over the 16 rows
    const int total = b.kv_heads << per_head_shift;
    const long long row_bytes = (long long)b.kv_heads * head_bytes;
    const long long src0 = (long long)(first_row + t0) * row_bytes;
    const long long dst_head_stride = (long long)kBlock * head_bytes;
    u32x4 kk[kAppendUnroll], vv[kAppendUnroll];
    long long dst[kAppendUnroll];
#pragma unroll
    for (int u = 0; u < kAppendUnroll; ++u) {
        const int idx = hg * kAppendChunksPerGroup + u * 256 + threadIdx.x;  // (head, row, chunk), chunk fastest
        dst[u] = -1;
        if (idx < total) {
            const int g = idx >> per_head_shift;
            const int row = (idx >> cph_shift) & (kAppendRows - 1);
            const int ch = idx & ((1 << cph_shift) - 1);
            const long long so = slot_off[row];
            if (so >= 0) {
                dst[u] = so + g * dst_head_stride + (ch << 4);
                const long long src = src0 + row * row_bytes + (long long)g * head_bytes + (ch << 4);
                kk[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(k_new + src));
                vv[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(v_new + src));
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kAppendUnroll; ++u) {
        if (dst[u] >= 0) {
            __builtin_nontemporal_store(kk[u], reinterpret_cast<u32x4*>(pool_k + dst[u]));
            __builtin_nontemporal_store(vv[u], reinterpret_cast<u32x4*>(pool_v + dst[u]));
        }
    }
}

__global__ __launch_bounds__(256) void gather_kernel(PagedBatch b, int req, int length, char* __restrict__ k_out,
                                                     char* __restrict__ v_out, int esize) {
    const int head_bytes = b.head_dim * esize;
    const int chunks_per_head = head_bytes >> 4;
    const int chunks_per_row = b.kv_heads * chunks_per_head;
    const long long total = (long long)length * chunks_per_row;
    const char* pk = static_cast<const char*>(b.pool_k);
    const char* pv = static_cast<const char*>(b.pool_v);
    for (long long c = (long long)blockIdx.x * blockDim.x + threadIdx.x; c < total; c += (long long)gridDim.x * blockDim.x) {
        const int pos = (int)(c / chunks_per_row);
        const int in_row = (int)(c - (long long)pos * chunks_per_row);
        const int g = in_row / chunks_per_head;
        const int ch = in_row - g * chunks_per_head;
        const int blk = b.block_table[(long long)req * b.table_stride + (pos >> 4)];
        const long long src = ((long long)blk * b.block_stride + ((long long)g * kBlock + (pos & 15)) * b.head_dim) * esize + (ch << 4);
        *reinterpret_cast<u32x4*>(k_out + (c << 4)) = *reinterpret_cast<const u32x4*>(pk + src);
        *reinterpret_cast<u32x4*>(v_out + (c << 4)) = *reinterpret_cast<const u32x4*>(pv + src);
    }
}

// One unit = kSwapSeg bytes of one plane of one block (four 16-byte loads in flight per thread
// before the stores); unit index = (pair * 2 + plane) * segs + seg.  The workgroups stride over
// the units: the host link needs only a few dozen workgroups' worth of loads in flight, and a
// small grid leaves the compute units to an attention kernel running next to the copies.
constexpr int kSwapSeg = 256 * 16 * 4;
constexpr int kSwapMaxWorkgroups = 32;  // measured: 16-64 reach the link's rate, 8 do not, hundreds block co-running kernels

__global__ __launch_bounds__(256) void swap_kernel(char* __restrict__ dev_k, char* __restrict__ dev_v, long long dev_stride,
                                                   char* __restrict__ host_k, char* __restrict__ host_v, long long host_stride,
                                                   long long plane_bytes, int segs, int units, SwapPairs pairs, int to_device) {
    for (int unit = blockIdx.x; unit < units; unit += gridDim.x) {
        const int seg = unit % segs;
        const int plane = (unit / segs) & 1;
        const int pair = unit / (2 * segs);
        char* d = (plane ? dev_v : dev_k) + (long long)pairs.dev[pair] * dev_stride;
        char* h = (plane ? host_v : host_k) + (long long)pairs.slot[pair] * host_stride;
        const char* src = to_device ? h : d;
        char* dst = to_device ? d : h;
        const long long base = (long long)seg * kSwapSeg + ((long long)threadIdx.x << 4);
        u32x4 tmp[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const long long off = base + (long long)i * 4096;
            if (off < plane_bytes) tmp[i] = *reinterpret_cast<const u32x4*>(src + off);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const long long off = base + (long long)i * 4096;
            if (off < plane_bytes) *reinterpret_cast<u32x4*>(dst + off) = tmp[i];
        }
    }
}

inline int grid_for(long long items, int per_block, int cap) {
    long long g = (items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

}  // namespace

hipError_t launch_append(const PagedBatch& b, void* pool_k, void* pool_v, const void* k_new, const void* v_new,
                         int32_t total_new, int esize, hipStream_t s) {
    if (total_new <= 0) return hipSuccess;
    const int chunks_per_group_of_rows = kAppendRows * b.kv_heads * ((b.head_dim * esize) >> 4);
    const int head_groups = (chunks_per_group_of_rows + kAppendChunksPerGroup - 1) / kAppendChunksPerGroup;
    const long long grid = (long long)((total_new + kAppendRows - 1) / kAppendRows) * head_groups;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(append_kernel, dim3((unsigned)grid), dim3(256), 0, s, b, static_cast<char*>(pool_k),
                       static_cast<char*>(pool_v), static_cast<const char*>(k_new), static_cast<const char*>(v_new),
                       total_new, esize, head_groups);
    return hipGetLastError();
}

hipError_t launch_gather(const PagedBatch& b, int32_t req, int32_t length, void* k_out, void* v_out, int esize,
                         hipStream_t s) {
    if (length <= 0) return hipSuccess;
    const long long chunks = (long long)length * b.kv_heads * ((b.head_dim * esize) >> 4);
    const int grid = grid_for(chunks, 256, 256 * 64);
    hipLaunchKernelGGL(gather_kernel, dim3(grid), dim3(256), 0, s, b, req, length, static_cast<char*>(k_out),
                       static_cast<char*>(v_out), esize);
    return hipGetLastError();
}

hipError_t launch_swap(char* dev_k, char* dev_v, int64_t dev_block_bytes_stride, char* host_k, char* host_v,
                       int64_t host_block_bytes_stride, int64_t plane_block_bytes, const SwapPairs& pairs, int32_t n,
                       int to_device, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    const int segs = (int)((plane_block_bytes + kSwapSeg - 1) / kSwapSeg);
    const int units = n * 2 * segs;
    hipLaunchKernelGGL(swap_kernel, dim3(units < kSwapMaxWorkgroups ? units : kSwapMaxWorkgroups), dim3(256), 0, s, dev_k, dev_v, (long long)dev_block_bytes_stride,
                       host_k, host_v, (long long)host_block_bytes_stride, (long long)plane_block_bytes, segs, units, pairs,
                       to_device);
    return hipGetLastError();
}

}  // namespace ragc
