// C-ABI front end: argument validation, error reporting and dispatch to the
// gfx950 kernels.  Every check runs on the host before anything is enqueued.
#include "../../include/ragc.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "ragc_internal.h"

namespace {
thread_local char g_err[512] = "";
// test overrides of the launch plan (ragc_debug_set_attn_plan); -1 / 0 = the library decides
std::atomic<int> g_force_variant{-1};
std::atomic<int> g_force_splits{0};
}

namespace ragc {
int set_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
}  // namespace ragc

namespace {

int (&fail)(int, const char*, ...) = ragc::set_error;

int esize_of(int32_t dtype) { return dtype == RAGC_DTYPE_BF16 ? 2 : dtype == RAGC_DTYPE_F32 ? 4 : 0; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_pool(const ragc_kv_pool* pool) {
    if (!pool) return fail(RAGC_ERR_NULL, "pool is NULL");
    if (!pool->k || !pool->v) return fail(RAGC_ERR_NULL, "pool->k / pool->v is NULL");
    if (pool->block_size != RAGC_BLOCK_SIZE) return fail(RAGC_ERR_SHAPE, "block_size %d (must be 16)", pool->block_size);
    if (pool->head_dim != 64 && pool->head_dim != 128) return fail(RAGC_ERR_SHAPE, "head_dim %d (must be 64 or 128)", pool->head_dim);
    if (esize_of(pool->dtype) == 0) return fail(RAGC_ERR_SHAPE, "dtype %d unknown", pool->dtype);
    if (pool->reserved != 0) return fail(RAGC_ERR_SHAPE, "pool->reserved must be 0");
    if (pool->kv_heads <= 0 || pool->kv_heads > 65535) return fail(RAGC_ERR_SHAPE, "kv_heads %d", pool->kv_heads);
    if (pool->num_blocks <= 0) return fail(RAGC_ERR_SHAPE, "num_blocks %d", pool->num_blocks);
    const int64_t min_stride = (int64_t)pool->kv_heads * RAGC_BLOCK_SIZE * pool->head_dim;
    if (pool->block_stride_elems < min_stride)
        return fail(RAGC_ERR_SHAPE, "block_stride_elems %lld < kv_heads*16*head_dim = %lld", (long long)pool->block_stride_elems, (long long)min_stride);
    if (!aligned16(pool->k) || !aligned16(pool->v) || (pool->block_stride_elems * esize_of(pool->dtype)) % 16 != 0)
        return fail(RAGC_ERR_ALIGN, "pool planes and block stride must be 16-byte aligned");
    return RAGC_OK;
}

struct BatchInfo {
    int64_t total_new = 0;
    int32_t max_new = 0;
};

// Host view of the batch metadata.  The h_* arrays of the batch are used when given; an array
// that is missing is read back from its device copy (a synchronous copy, the slow path).
struct HostMeta {
    const int32_t* prefix_len = nullptr;
    const int32_t* new_len = nullptr;
    const int32_t* new_start = nullptr;
    const int32_t* block_table = nullptr;  // may stay NULL: then block ids are not range-checked
    std::vector<int32_t> own_prefix, own_new, own_start, own_table;
};

int hip_fail(hipError_t e, const char* what) { return fail(RAGC_ERR_HIP, "%s: %s", what, hipGetErrorString(e)); }

int read_back(std::vector<int32_t>* dst, const int32_t* dev, size_t n, const char* what) {
    if (!dev) return fail(RAGC_ERR_NULL, "%s: neither the host copy nor the device array is given", what);
    dst->resize(n);
    const hipError_t e = hipMemcpy(dst->data(), dev, n * sizeof(int32_t), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return hip_fail(e, what);
    return RAGC_OK;
}

// want_table: read the block table back as well when no host copy is given (validation mode).
int resolve_host(const ragc_batch* b, bool want_table, HostMeta* h) {
    const size_t R = (size_t)b->num_reqs;
    h->prefix_len = b->h_prefix_len;
    h->new_len = b->h_new_len;
    h->new_start = b->h_new_start;
    h->block_table = b->h_block_table;
    if (!h->prefix_len) {
        if (int rc = read_back(&h->own_prefix, b->prefix_len, R, "prefix_len")) return rc;
        h->prefix_len = h->own_prefix.data();
    }
    if (!h->new_len) {
        if (int rc = read_back(&h->own_new, b->new_len, R, "new_len")) return rc;
        h->new_len = h->own_new.data();
    }
    if (!h->new_start) {
        if (int rc = read_back(&h->own_start, b->new_start, R, "new_start")) return rc;
        h->new_start = h->own_start.data();
    }
    if (!h->block_table && want_table) {
        if (b->table_stride <= 0) return fail(RAGC_ERR_SHAPE, "table_stride %d", b->table_stride);
        if (int rc = read_back(&h->own_table, b->block_table, R * (size_t)b->table_stride, "block_table")) return rc;
        h->block_table = h->own_table.data();
    }
    return RAGC_OK;
}

// Host-side checks of the batch metadata.  need_device: the device arrays are required.
int check_batch(const ragc_kv_pool* pool, const ragc_batch* b, bool need_device, bool want_table, HostMeta* h, BatchInfo* info) {
    if (!b) return fail(RAGC_ERR_NULL, "batch is NULL");
    if (b->num_reqs < 0 || b->num_reqs > 65535) return fail(RAGC_ERR_SHAPE, "num_reqs %d", b->num_reqs);
    if (b->num_reqs == 0) return RAGC_OK;
    if (need_device && (!b->prefix_len || !b->new_len || !b->new_start || !b->block_table))
        return fail(RAGC_ERR_NULL, "a device array of the batch is NULL");
    if (b->table_stride <= 0) return fail(RAGC_ERR_SHAPE, "table_stride %d", b->table_stride);
    if (int rc = resolve_host(b, want_table, h)) return rc;
    for (int r = 0; r < b->num_reqs; ++r) {
        const int64_t p = h->prefix_len[r], n = h->new_len[r];
        if (p < 0 || n < 0) return fail(RAGC_ERR_RANGE, "request %d: prefix_len %lld, new_len %lld", r, (long long)p, (long long)n);
        if (h->new_start[r] < 0) return fail(RAGC_ERR_RANGE, "request %d: new_start %d", r, h->new_start[r]);
        const int64_t blocks = (p + n + RAGC_BLOCK_SIZE - 1) / RAGC_BLOCK_SIZE;
        if (blocks > b->table_stride)
            return fail(RAGC_ERR_RANGE, "request %d: %lld tokens need %lld table entries, table_stride is %d", r, (long long)(p + n), (long long)blocks, b->table_stride);
        if (h->block_table) {
            const int32_t* row = h->block_table + (int64_t)r * b->table_stride;
            for (int64_t i = 0; i < blocks; ++i)
                if (row[i] < 0 || row[i] >= pool->num_blocks)
                    return fail(RAGC_ERR_RANGE, "request %d: block_table[%lld] = %d outside [0, %d)", r, (long long)i, row[i], pool->num_blocks);
        }
        info->total_new += n;
        info->max_new = std::max<int32_t>(info->max_new, (int32_t)n);
    }
    if (info->total_new > (int64_t)1 << 30) return fail(RAGC_ERR_RANGE, "sum of new_len %lld too large", (long long)info->total_new);
    return RAGC_OK;
}

// new_start must be the running sum of new_len (what the append kernel's row search assumes)
int check_packed(const ragc_batch* b, const HostMeta& h) {
    for (int r = 0; r + 1 < b->num_reqs; ++r)
        if ((int64_t)h.new_start[r + 1] != (int64_t)h.new_start[r] + h.new_len[r])
            return fail(RAGC_ERR_RANGE, "request %d: new_start[%d] = %d, expected new_start[%d] + new_len[%d] = %lld (rows must be packed in request order)",
                        r + 1, r + 1, h.new_start[r + 1], r, r, (long long)h.new_start[r] + h.new_len[r]);
    return RAGC_OK;
}

// Debug validation of what the device side cannot check: the device arrays equal their host
// copies, and (writes = true) every block that receives new tokens appears once, in one
// request, and in no request's read-only prefix.
int validate_batch(const ragc_kv_pool* pool, const ragc_batch* b, const HostMeta& h, bool writes) {
    const size_t R = (size_t)b->num_reqs;
    std::vector<int32_t> dev;
    struct { const int32_t* host; const int32_t* device; size_t n; const char* name; } arrays[] = {
        {b->h_prefix_len, b->prefix_len, R, "prefix_len"},
        {b->h_new_len, b->new_len, R, "new_len"},
        {b->h_new_start, b->new_start, R, "new_start"},
    };
    for (auto& a : arrays) {
        if (!a.host || !a.device) continue;  // nothing to compare (a missing host copy was read from the device anyway)
        if (int rc = read_back(&dev, a.device, a.n, a.name)) return rc;
        for (size_t i = 0; i < a.n; ++i)
            if (dev[i] != a.host[i]) return fail(RAGC_ERR_RANGE, "%s[%zu]: device copy %d differs from host copy %d", a.name, i, dev[i], a.host[i]);
    }
    if (b->h_block_table && b->block_table) {
        if (int rc = read_back(&dev, b->block_table, R * (size_t)b->table_stride, "block_table")) return rc;
        for (size_t r = 0; r < R; ++r) {
            const int64_t blocks = ((int64_t)h.prefix_len[r] + h.new_len[r] + RAGC_BLOCK_SIZE - 1) / RAGC_BLOCK_SIZE;
            for (int64_t i = 0; i < blocks; ++i) {
                const size_t at = r * (size_t)b->table_stride + (size_t)i;
                if (dev[at] != b->h_block_table[at])
                    return fail(RAGC_ERR_RANGE, "block_table[%zu][%lld]: device copy %d differs from host copy %d", r, (long long)i, dev[at], b->h_block_table[at]);
            }
        }
    }
    if (!writes || !h.block_table) return RAGC_OK;
    // owner[block]: -1 untouched, r >= 0: receives new tokens of request r, -2: read as prefix by some request
    std::vector<int32_t> owner((size_t)pool->num_blocks, -1);
    for (size_t r = 0; r < R; ++r) {  // pass 1: write targets
        const int64_t p = h.prefix_len[r], n = h.new_len[r];
        if (n == 0) continue;
        const int32_t* row = h.block_table + r * (size_t)b->table_stride;
        for (int64_t i = p / RAGC_BLOCK_SIZE; i < (p + n + RAGC_BLOCK_SIZE - 1) / RAGC_BLOCK_SIZE; ++i) {
            if (owner[row[i]] != -1)
                return fail(RAGC_ERR_RANGE, "block %d receives new tokens of request %zu (table entry %lld) and of request %d: append targets must be exclusive",
                            row[i], r, (long long)i, owner[row[i]]);
            owner[row[i]] = (int32_t)r;
        }
    }
    for (size_t r = 0; r < R; ++r) {  // pass 2: read-only prefix blocks (whole blocks below the first write target)
        const int32_t* row = h.block_table + r * (size_t)b->table_stride;
        const int64_t full = (h.new_len[r] == 0 ? ((int64_t)h.prefix_len[r] + RAGC_BLOCK_SIZE - 1) : (int64_t)h.prefix_len[r]) / RAGC_BLOCK_SIZE;
        for (int64_t i = 0; i < full; ++i)
            if (owner[row[i]] >= 0)
                return fail(RAGC_ERR_RANGE, "block %d is read as cached prefix by request %zu (table entry %lld) and receives new tokens of request %d",
                            row[i], r, (long long)i, owner[row[i]]);
    }
    return RAGC_OK;
}

ragc::PagedBatch make_paged(const ragc_kv_pool* pool, const ragc_batch* b) {
    ragc::PagedBatch pb;
    pb.pool_k = pool->k;
    pb.pool_v = pool->v;
    pb.block_stride = pool->block_stride_elems;
    pb.prefix_len = b->prefix_len;
    pb.new_len = b->new_len;
    pb.new_start = b->new_start;
    pb.block_table = b->block_table;
    pb.table_stride = b->table_stride;
    pb.num_reqs = b->num_reqs;
    pb.kv_heads = pool->kv_heads;
    pb.head_dim = pool->head_dim;
    return pb;
}

// compute units of the current device (queried once per thread)
int cu_count() {
    thread_local int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

// How the bf16 path will run a batch: the (request, 128-row tile) work items, most key tiles
// first so the long ones start early; how many copies of each item share its keys; which
// kernel shape; and the workspace the copies need.  ragc_prefill_attn_workspace and
// ragc_prefill_attn both call this, so they always agree.
struct Bf16Item {
    int32_t cost;  // key tiles
    ragc::AttnItem it;
};
struct Bf16Plan {
    std::vector<Bf16Item> items;
    int splits = 1;
    int variant = ragc::kAttnVariantOneGroup;
    int64_t workspace = 0;
};

int plan_bf16(const ragc_kv_pool* pool, const ragc_batch* batch, const HostMeta& h, int group, uint32_t flags, Bf16Plan* plan) {
    for (int r = 0; r < batch->num_reqs; ++r) {
        const int n = h.new_len[r], p = h.prefix_len[r];
        const int64_t rows = (int64_t)n * group;
        const int64_t tiles = (rows + ragc::kAttnRowsPerItem - 1) / ragc::kAttnRowsPerItem;
        if (tiles > 65535) return fail(RAGC_ERR_RANGE, "request %d: new_len * group too large", r);
        for (int t = 0; t < (int)tiles; ++t)
            plan->items.push_back({ragc::attn_bf16_item_cost(p, n, group, t),
                                   ragc::AttnItem{(uint32_t)r << 16 | (uint32_t)t, p, n, h.new_start[r]}});
    }
    // Order: requests by their most expensive row tile, longest first, and the row tiles of one
    // request next to each other (longest first).  Long items start early, and the workgroups that
    // run at the same time on an XCD walk the key tiles of the same few requests at about the same
    // pace, so a tile fetched by one row tile is still in that XCD's L2 for the others.
    std::vector<int32_t> req_cost(batch->num_reqs, 0);
    for (const Bf16Item& it : plan->items) {
        int32_t& c = req_cost[it.it.req_tile >> 16];
        c = std::max(c, it.cost);
    }
    std::stable_sort(plan->items.begin(), plan->items.end(), [&](const Bf16Item& x, const Bf16Item& y) {
        const uint32_t rx = x.it.req_tile >> 16, ry = y.it.req_tile >> 16;
        if (rx != ry) return req_cost[rx] != req_cost[ry] ? req_cost[rx] > req_cost[ry] : rx < ry;
        return x.cost > y.cost;
    });
    const int64_t wgs = (int64_t)plan->items.size() * pool->kv_heads;
    const int64_t cus = cu_count();
    // Fewer work items than CUs: split each along its keys until every CU has one, keeping at
    // least three key tiles per copy of the longest item (measured on eight small shapes: with the
    // one-round-trip merge pass, copies of three to four tiles are still worth their fixed cost).
    // ragc_debug_set_attn_plan overrides (tests).
    int splits = 1;
    if (!(flags & RAGC_ATTN_NO_SPLIT) && wgs > 0) {
        splits = (int)std::min<int64_t>(cus / wgs, ragc::kAttnMaxSplits);
        splits = std::min(splits, plan->items.front().cost / 3);
        if (const int force = g_force_splits.load(std::memory_order_relaxed); force > 0) splits = std::min(force, ragc::kAttnMaxSplits);
        if (splits < 1) splits = 1;
    }
    plan->splits = splits;
    // With at least two workgroups per CU two 4-wave workgroups share a CU; otherwise one 8-wave
    // workgroup divides its key tiles between two wave groups -- unless the items are already split
    // along their keys (measured: 4-wave workgroups are then as fast or faster, 23.8 against 26.3 us
    // on four decode requests of 4096 keys).  ragc_debug_set_attn_plan overrides (tests).
    plan->variant = (splits > 1 || wgs >= 2 * cus) ? ragc::kAttnVariantOneGroup : ragc::kAttnVariantTwoGroups;
    if (const int force = g_force_variant.load(std::memory_order_relaxed); force >= 0) plan->variant = force;
    plan->workspace = splits > 1 ? (int64_t)plan->items.size() * splits * pool->kv_heads * ragc::attn_partial_bytes(pool->head_dim) : 0;
    return 0;
}

constexpr uint32_t kAttnFlags = RAGC_ATTN_APPEND_FUSED | RAGC_ATTN_NO_SPLIT | RAGC_ATTN_VALIDATE;

// Enqueue the launches of a planned bf16 batch: every copy of an item is a list entry of its
// own and a launch takes kAttnMaxItems entries, so a long list goes out in several launches
// (each followed by its merge pass when the items are split).
int run_bf16_plan(ragc::AttnLaunch& a, const Bf16Plan& plan, hipStream_t s) {
    const int S = plan.splits;
    const size_t per_launch = (size_t)ragc::kAttnMaxItems / S;
    for (size_t i = 0; i < plan.items.size(); i += per_launch) {
        ragc::AttnWorkList wl{}, leads{};
        wl.splits = leads.splits = S;
        wl.part_base = leads.part_base = (int32_t)(i * S);
        const size_t cnt = std::min(per_launch, plan.items.size() - i);
        for (size_t j = 0; j < cnt; ++j) {
            for (int c = 0; c < S; ++c) wl.item[wl.n++] = plan.items[i + j].it;
            leads.item[leads.n++] = plan.items[i + j].it;
        }
        hipError_t e = ragc::launch_attn_bf16(a, wl, plan.variant, s);
        if (e == hipSuccess && S > 1) e = ragc::launch_attn_bf16_merge(a, leads, s);
        if (e != hipSuccess)
            return fail(RAGC_ERR_HIP, "prefill attention launch %zu of %zu: %s (earlier launches of this call stay enqueued)",
                        i / per_launch + 1, (plan.items.size() + per_launch - 1) / per_launch, hipGetErrorString(e));
    }
    return RAGC_OK;
}

// ---- partial results of key-split work items for callers that cannot allocate --------------
// One array per GPU (every device that loads the library holds its own copy until the process
// ends).  Host code must never pass the array's name to a kernel: that name is a host-side
// stand-in; the device address comes from hipGetSymbolAddress, once per device.
constexpr int64_t kStaticScratchBytes = 256 * 128 * (128 + 2) * 4;  // 256 partial results at head_dim 128: 17,039,360 bytes
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(RAGC_ERR_RANGE, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // address of THIS device's copy
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return fail(RAGC_ERR_ALIGN, "static scratch is not 256-byte aligned");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return RAGC_OK;
}

int prefill_attn_impl(const ragc_kv_pool* pool, const ragc_batch* batch, const void* q, const void* k_new,
                      const void* v_new, void* out, int32_t q_heads, float softmax_scale, uint32_t flags,
                      void* workspace, size_t workspace_bytes, bool use_static_scratch, void* stream) {
    g_err[0] = 0;
    if (int rc = check_pool(pool)) return rc;
    if (flags & ~kAttnFlags) return fail(RAGC_ERR_SHAPE, "unknown flags 0x%x", flags);
    if (q_heads <= 0 || q_heads % pool->kv_heads != 0)
        return fail(RAGC_ERR_SHAPE, "q_heads %d not a multiple of kv_heads %d", q_heads, pool->kv_heads);
    if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale))
        return fail(RAGC_ERR_SHAPE, "softmax_scale must be positive and finite");
    const bool validate = (flags & RAGC_ATTN_VALIDATE) != 0;
    if (use_static_scratch) {
        // nothing in this mode may allocate or synchronise: no read-backs
        if (validate) return fail(RAGC_ERR_SHAPE, "RAGC_ATTN_VALIDATE reads device arrays back; not available in ragc_prefill_attn_static");
        if (batch && batch->num_reqs > 0 && (!batch->h_prefix_len || !batch->h_new_len || !batch->h_new_start))
            return fail(RAGC_ERR_NULL, "ragc_prefill_attn_static needs h_prefix_len, h_new_len and h_new_start");
    }
    BatchInfo info;
    HostMeta h;
    if (int rc = check_batch(pool, batch, true, validate, &h, &info)) return rc;
    if (batch->num_reqs == 0 || info.total_new == 0) return RAGC_OK;
    if (!q || !k_new || !v_new || !out) return fail(RAGC_ERR_NULL, "q / k_new / v_new / out is NULL");
    if (!aligned16(q) || !aligned16(k_new) || !aligned16(v_new) || !aligned16(out))
        return fail(RAGC_ERR_ALIGN, "q / k_new / v_new / out must be 16-byte aligned");
    if (validate)
        if (int rc = validate_batch(pool, batch, h, (flags & RAGC_ATTN_APPEND_FUSED) != 0)) return rc;

    ragc::AttnLaunch a;
    a.b = make_paged(pool, batch);
    a.q = q;
    a.k_new = k_new;
    a.v_new = v_new;
    a.out = out;
    a.pool_k_w = pool->k;
    a.pool_v_w = pool->v;
    a.partial = nullptr;
    a.q_heads = q_heads;
    a.group = q_heads / pool->kv_heads;
    a.group_magic = a.group == 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) + a.group - 1) / a.group);
    a.scale_log2e = softmax_scale * 1.44269504088896340736f;
    a.fused_append = (flags & RAGC_ATTN_APPEND_FUSED) ? 1 : 0;
    a.max_new = info.max_new;
    a.total_new = (int32_t)info.total_new;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (pool->dtype == RAGC_DTYPE_F32) {
        const hipError_t e = ragc::launch_attn_f32(a, s);
        if (e != hipSuccess) return hip_fail(e, "prefill attention launch");
        return RAGC_OK;
    }
    Bf16Plan plan;
    if (int rc = plan_bf16(pool, batch, h, a.group, flags, &plan)) return rc;
    if (plan.workspace > 0) {
        if (use_static_scratch) {
            if (plan.workspace > kStaticScratchBytes)
                return fail(RAGC_ERR_WORKSPACE, "this batch needs %lld bytes for its partial results; the static scratch holds %lld",
                            (long long)plan.workspace, (long long)kStaticScratchBytes);
            if (int rc = static_scratch(&a.partial)) return rc;
        } else {
            if (!workspace || (int64_t)workspace_bytes < plan.workspace)
                return fail(RAGC_ERR_WORKSPACE, "workspace of %lld bytes needed (ragc_prefill_attn_workspace), %zu given",
                            (long long)plan.workspace, workspace_bytes);
            if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(RAGC_ERR_ALIGN, "workspace must be 256-byte aligned");
            a.partial = workspace;
        }
    }
    return run_bf16_plan(a, plan, s);
}

}  // namespace

extern "C" {

int ragc_version(void) { return 100; }

const char* ragc_last_error(void) { return g_err; }

int64_t ragc_kv_bytes_per_token(int32_t layers, int32_t kv_heads, int32_t head_dim, int32_t dtype) {
    const int es = esize_of(dtype);
    if (layers <= 0 || kv_heads <= 0 || head_dim <= 0 || es == 0) return 0;
    return (int64_t)2 * layers * kv_heads * head_dim * es;
}

int ragc_debug_set_attn_plan(int32_t variant, int32_t splits) {
    g_err[0] = 0;
    if (variant < -1 || variant >= ragc::kAttnVariantCount) return fail(RAGC_ERR_SHAPE, "variant %d unknown", variant);
    if (splits < 0 || splits > ragc::kAttnMaxSplits) return fail(RAGC_ERR_SHAPE, "splits %d outside [0, %d]", splits, ragc::kAttnMaxSplits);
    g_force_variant.store(variant, std::memory_order_relaxed);
    g_force_splits.store(splits, std::memory_order_relaxed);
    return RAGC_OK;
}

int ragc_batch_validate(const ragc_kv_pool* pool, const ragc_batch* batch, int32_t writes_new_tokens) {
    g_err[0] = 0;
    if (int rc = check_pool(pool)) return rc;
    BatchInfo info;
    HostMeta h;
    if (int rc = check_batch(pool, batch, true, true, &h, &info)) return rc;
    if (batch->num_reqs == 0) return RAGC_OK;
    return validate_batch(pool, batch, h, writes_new_tokens != 0);
}

int64_t ragc_prefill_attn_workspace(const ragc_kv_pool* pool, const ragc_batch* batch, int32_t q_heads, uint32_t flags) {
    g_err[0] = 0;
    if (int rc = check_pool(pool)) return rc;
    if (flags & ~kAttnFlags) return fail(RAGC_ERR_SHAPE, "unknown flags 0x%x", flags);
    if (q_heads <= 0 || q_heads % pool->kv_heads != 0)
        return fail(RAGC_ERR_SHAPE, "q_heads %d not a multiple of kv_heads %d", q_heads, pool->kv_heads);
    BatchInfo info;
    HostMeta h;
    if (int rc = check_batch(pool, batch, false, false, &h, &info)) return rc;
    if (pool->dtype != RAGC_DTYPE_BF16 || batch->num_reqs == 0 || info.total_new == 0) return 0;
    Bf16Plan plan;
    if (int rc = plan_bf16(pool, batch, h, q_heads / pool->kv_heads, flags, &plan)) return rc;
    return plan.workspace;
}

int ragc_prefill_attn(const ragc_kv_pool* pool, const ragc_batch* batch, const void* q, const void* k_new,
                      const void* v_new, void* out, int32_t q_heads, float softmax_scale, uint32_t flags,
                      void* workspace, size_t workspace_bytes, void* stream) {
    return prefill_attn_impl(pool, batch, q, k_new, v_new, out, q_heads, softmax_scale, flags, workspace, workspace_bytes,
                             false, stream);
}

int ragc_prefill_attn_static(const ragc_kv_pool* pool, const ragc_batch* batch, const void* q, const void* k_new,
                             const void* v_new, void* out, int32_t q_heads, float softmax_scale, uint32_t flags,
                             void* stream) {
    return prefill_attn_impl(pool, batch, q, k_new, v_new, out, q_heads, softmax_scale, flags, nullptr, 0, true, stream);
}

int ragc_kv_append(const ragc_kv_pool* pool, const ragc_batch* batch, const void* k_new, const void* v_new, void* stream) {
    g_err[0] = 0;
    if (int rc = check_pool(pool)) return rc;
    BatchInfo info;
    HostMeta h;
    if (int rc = check_batch(pool, batch, true, false, &h, &info)) return rc;
    if (batch->num_reqs == 0 || info.total_new == 0) return RAGC_OK;
    if (int rc = check_packed(batch, h)) return rc;
    if (!k_new || !v_new) return fail(RAGC_ERR_NULL, "k_new / v_new is NULL");
    if (!aligned16(k_new) || !aligned16(v_new)) return fail(RAGC_ERR_ALIGN, "k_new / v_new must be 16-byte aligned");
    const hipError_t e = ragc::launch_append(make_paged(pool, batch), pool->k, pool->v, k_new, v_new, (int32_t)info.total_new,
                                             esize_of(pool->dtype), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "append launch");
    return RAGC_OK;
}

int ragc_kv_gather(const ragc_kv_pool* pool, const ragc_batch* batch, int32_t req, int32_t length, void* k_out,
                   void* v_out, void* stream) {
    g_err[0] = 0;
    if (int rc = check_pool(pool)) return rc;
    if (!batch) return fail(RAGC_ERR_NULL, "batch is NULL");
    if (!batch->block_table) return fail(RAGC_ERR_NULL, "block_table is NULL");
    if (req < 0 || req >= batch->num_reqs) return fail(RAGC_ERR_RANGE, "req %d outside [0, %d)", req, batch->num_reqs);
    if (length < 0 || (int64_t)length > (int64_t)batch->table_stride * RAGC_BLOCK_SIZE)
        return fail(RAGC_ERR_RANGE, "length %d exceeds table capacity %lld", length, (long long)batch->table_stride * RAGC_BLOCK_SIZE);
    if (batch->h_block_table) {
        const int32_t* row = batch->h_block_table + (int64_t)req * batch->table_stride;
        for (int i = 0; i < (length + RAGC_BLOCK_SIZE - 1) / RAGC_BLOCK_SIZE; ++i)
            if (row[i] < 0 || row[i] >= pool->num_blocks)
                return fail(RAGC_ERR_RANGE, "block_table[%d] = %d outside [0, %d)", i, row[i], pool->num_blocks);
    }
    if (length == 0) return RAGC_OK;
    if (!k_out || !v_out) return fail(RAGC_ERR_NULL, "k_out / v_out is NULL");
    if (!aligned16(k_out) || !aligned16(v_out)) return fail(RAGC_ERR_ALIGN, "k_out / v_out must be 16-byte aligned");
    const hipError_t e = ragc::launch_gather(make_paged(pool, batch), req, length, k_out, v_out, esize_of(pool->dtype),
                                             static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "gather launch");
    return RAGC_OK;
}

int ragc_kv_swap(const ragc_kv_pool* pool, void* host_k, void* host_v, int64_t host_block_stride_elems,
                 int32_t num_host_slots, const int32_t* dev_block_ids, const int32_t* host_slots, int32_t n,
                 int32_t direction, uint32_t flags, void* stream) {
    g_err[0] = 0;
    if (int rc = check_pool(pool)) return rc;
    if (!host_k || !host_v) return fail(RAGC_ERR_NULL, "host_k / host_v is NULL");
    if (n < 0) return fail(RAGC_ERR_RANGE, "n %d", n);
    if (direction != RAGC_SWAP_TO_DEVICE && direction != RAGC_SWAP_TO_HOST) return fail(RAGC_ERR_SHAPE, "direction %d", direction);
    if (flags > RAGC_SWAP_KERNEL) return fail(RAGC_ERR_SHAPE, "unknown swap flags 0x%x", flags);
    const int es = esize_of(pool->dtype);
    const int64_t plane_elems = (int64_t)pool->kv_heads * RAGC_BLOCK_SIZE * pool->head_dim;
    if (host_block_stride_elems < plane_elems)
        return fail(RAGC_ERR_SHAPE, "host_block_stride_elems %lld < %lld", (long long)host_block_stride_elems, (long long)plane_elems);
    if (!aligned16(host_k) || !aligned16(host_v) || (host_block_stride_elems * es) % 16 != 0)
        return fail(RAGC_ERR_ALIGN, "host planes and stride must be 16-byte aligned");
    if (num_host_slots <= 0) return fail(RAGC_ERR_SHAPE, "num_host_slots %d", num_host_slots);
    if (n == 0) return RAGC_OK;
    if (!dev_block_ids || !host_slots) return fail(RAGC_ERR_NULL, "dev_block_ids / host_slots is NULL");
    for (int i = 0; i < n; ++i) {
        if (dev_block_ids[i] < 0 || dev_block_ids[i] >= pool->num_blocks)
            return fail(RAGC_ERR_RANGE, "dev_block_ids[%d] = %d outside [0, %d)", i, dev_block_ids[i], pool->num_blocks);
        if (host_slots[i] < 0 || host_slots[i] >= num_host_slots)
            return fail(RAGC_ERR_RANGE, "host_slots[%d] = %d outside [0, %d)", i, host_slots[i], num_host_slots);
    }
    {  // two pairs must not write the same destination
        std::vector<int32_t> dst(direction == RAGC_SWAP_TO_DEVICE ? dev_block_ids : host_slots,
                                 (direction == RAGC_SWAP_TO_DEVICE ? dev_block_ids : host_slots) + n);
        std::sort(dst.begin(), dst.end());
        if (std::adjacent_find(dst.begin(), dst.end()) != dst.end())
            return fail(RAGC_ERR_RANGE, "two pairs write the same destination block");
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t plane_bytes = plane_elems * es;
    const int64_t dev_stride = pool->block_stride_elems * es;
    const int64_t host_stride = host_block_stride_elems * es;
    const bool to_dev = direction == RAGC_SWAP_TO_DEVICE;

    if (flags == RAGC_SWAP_MEMCPY) {
        // one copy per plane and run of pairs that are adjacent on both sides
        const bool dense = dev_stride == plane_bytes && host_stride == plane_bytes;
        int i = 0;
        while (i < n) {
            int j = i + 1;
            while (dense && j < n && dev_block_ids[j] == dev_block_ids[j - 1] + 1 && host_slots[j] == host_slots[j - 1] + 1) ++j;
            const size_t bytes = (size_t)(j - i) * plane_bytes;
            for (int plane = 0; plane < 2; ++plane) {
                char* d = static_cast<char*>(plane ? pool->v : pool->k) + (int64_t)dev_block_ids[i] * dev_stride;
                char* h = static_cast<char*>(plane ? host_v : host_k) + (int64_t)host_slots[i] * host_stride;
                const hipError_t e = to_dev ? hipMemcpyAsync(d, h, bytes, hipMemcpyHostToDevice, s)
                                            : hipMemcpyAsync(h, d, bytes, hipMemcpyDeviceToHost, s);
                if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync");
            }
            i = j;
        }
        return RAGC_OK;
    }

    // copy kernel over the host-mapped pinned pool
    void *hk_dev = nullptr, *hv_dev = nullptr;
    hipError_t e = hipHostGetDevicePointer(&hk_dev, host_k, 0);
    if (e != hipSuccess) return hip_fail(e, "host_k is not pinned, device-mapped memory (hipHostGetDevicePointer)");
    e = hipHostGetDevicePointer(&hv_dev, host_v, 0);
    if (e != hipSuccess) return hip_fail(e, "host_v is not pinned, device-mapped memory (hipHostGetDevicePointer)");
    for (int i = 0; i < n; i += ragc::kSwapPairsPerLaunch) {
        const int cnt = std::min(ragc::kSwapPairsPerLaunch, n - i);
        ragc::SwapPairs pairs{};
        std::memcpy(pairs.dev, dev_block_ids + i, sizeof(int32_t) * cnt);
        std::memcpy(pairs.slot, host_slots + i, sizeof(int32_t) * cnt);
        e = ragc::launch_swap(static_cast<char*>(pool->k), static_cast<char*>(pool->v), dev_stride,
                              static_cast<char*>(hk_dev), static_cast<char*>(hv_dev), host_stride, plane_bytes, pairs, cnt,
                              to_dev ? 1 : 0, s);
        if (e != hipSuccess) return hip_fail(e, "swap kernel launch");
    }
    return RAGC_OK;
}

}  // extern "C"
