/*
 * ragc -- prefix-cached paged prefill attention for gfx950 (MI355X), C ABI.
 *
 * The hot path of knowledge caching for retrieval-augmented generation: the
 * K/V tensors of retrieved documents are kept in fixed-size, non-contiguous
 * blocks referenced from the nodes of a prefix tree over document ids
 * (paper Sec. 5.1, knowledge tree); a request whose document sequence matches a
 * path of the tree computes only its non-cached tokens and attends over the
 * cached blocks (Sec. 3.2 "Full prefill computation"; Sec. 4 "prefix caching
 * kernel"; Sec. 6: multi-head and grouped-query attention); the K/V of the new
 * tokens is handed back for caching (Sec. 4); blocks move between GPU and host
 * memory (Sec. 3.2 "Cache hit", Sec. 5.1 "Swap out only once").
 *
 * Conventions
 *   - Stateless: the library allocates nothing and keeps nothing between calls.
 *     Every buffer belongs to the caller.  Calls validate their arguments on the
 *     host, enqueue work on the given HIP stream and return; completion is
 *     observed through the stream.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Pointers are marked [device], [host] or [pinned host].
 *   - Every entry point returns 0 or a negative ragc_status.  Every check runs on the
 *     host before the first launch, so an argument error enqueues nothing.  The one
 *     exception: a batch with more work items than one launch carries goes out in
 *     several launches, and if the runtime refuses a later one (RAGC_ERR_HIP) the
 *     earlier ones stay enqueued; `out` and, with the fused append, the pool blocks of
 *     the new tokens are then partly written.  ragc_last_error() gives a thread-local
 *     message.
 *   - Block size is 16 tokens.  head_dim is 64 or 128.  dtype is fp32 or bf16 and is
 *     the type of the pool, of q/k_new/v_new and of the output.
 *
 * Pool layout.  Two planes, K and V, each
 *       [num_blocks][kv_heads][16][head_dim]           (row-major)
 *   with `block_stride_elems` elements between consecutive blocks of a plane
 *   (>= kv_heads*16*head_dim).  One (block, kv head) tile is contiguous (4 KiB for
 *   bf16 at head_dim 128); one block of a plane is contiguous (what swap moves).
 *
 * Addressing.  Logical position j of request r (0 <= j < prefix_len+new_len)
 *   lives in block block_table[r][j / 16], slot j % 16.  Positions below
 *   prefix_len[r] are the cached documents (read only); positions from
 *   prefix_len[r] on are the request's new tokens (written by the append).
 *
 * Preconditions the kernels themselves cannot check
 *   - every block that receives new tokens belongs to that request alone (shared
 *     chains cover only full blocks inside the prefix);
 *   - block_table rows hold ceil((prefix_len+new_len)/16) valid block ids;
 *   - the device arrays of a batch equal their host copies;
 *   - no swap writes a block that a running attention call reads.
 *   Block ids are range-checked whenever h_block_table is given.  The first three are
 *   checked in full by ragc_batch_validate / RAGC_ATTN_VALIDATE (a debug mode: it reads
 *   the device arrays back synchronously).  The last one is the caller's stream order.
 *
 * Accuracy (bf16).  Against exact arithmetic on the same bf16 inputs the output is
 *   within 2e-2 absolute wherever |out| < 8; from 8 on, half a unit of the bf16 output
 *   grid alone is 2^-5 or more and the bound becomes 2^-8 * |out| + 4e-3.  fp32: 1e-4.
 *
 * Several layers, one pool per layer (Sec. 5.1 "Swap out only once": transfers overlap
 *   with computation).  The library keeps no state, so the caller orders the calls.  All
 *   layers share block ids and host slots; a request's plan (swap-out pairs, swap-in
 *   pairs, table row) applies to each.  The order that overlaps copies with attention:
 *     main stream:  record event `begun`
 *     side stream:  wait `begun` (the copies may touch blocks that earlier work on the
 *                   main stream still reads or appends); then for every layer l in turn:
 *                   ragc_kv_swap(TO_HOST, out pairs), ragc_kv_swap(TO_DEVICE, in pairs),
 *                   record event ready[l].  Outgoing before incoming, because an
 *                   incoming block may reuse the device block an outgoing one frees.
 *     main stream:  for every layer l in turn: wait ready[l];
 *                   ragc_prefill_attn(pool of l, RAGC_ATTN_APPEND_FUSED)
 *     afterwards:   the side stream waits for the main stream before the next request's
 *                   copies (they may evict what this request appended).
 *   The side stream therefore runs ahead of the main one by as many layers as the copies
 *   are faster than attention; the main stream waits for its own layer only.  One
 *   workspace serves all layers, since their attention calls share a stream.
 *
 * Where this header departs from the three-call sketch of the benchmark spec
 *   (ragc_prefill_attn, ragc_kv_append, ragc_kv_swap with descriptors of device pointers
 *   and optional host mirrors):
 *   - ragc_kv_swap takes two more arguments: num_host_slots (so host slot ids can be
 *     range-checked) and flags (copy mechanism).
 *   - the fused-append flag is spelled RAGC_ATTN_APPEND_FUSED; RAGC_ATTN_NO_SPLIT is new.
 *   - more exports: ragc_last_error, ragc_kv_bytes_per_token, ragc_prefill_attn_workspace,
 *     ragc_batch_validate, ragc_debug_set_attn_plan, ragc_prefill_attn_static.
 *   - host copies of the lengths are optional but their absence costs a synchronous
 *     read-back per call (the launch is sized on the host).
 */
#ifndef RAGC_H
#define RAGC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RAGC_BLOCK_SIZE 16

typedef enum ragc_status {
    RAGC_OK = 0,
    RAGC_ERR_NULL = -1,      /* a required pointer is NULL */
    RAGC_ERR_SHAPE = -2,     /* unsupported or inconsistent shape / dtype / flag */
    RAGC_ERR_RANGE = -3,     /* a length or block id is out of range */
    RAGC_ERR_ALIGN = -4,     /* a pointer or stride is not 16-byte aligned */
    RAGC_ERR_HIP = -5,       /* a HIP runtime call failed */
    RAGC_ERR_WORKSPACE = -6  /* workspace missing or too small */
} ragc_status;

typedef enum ragc_dtype { RAGC_DTYPE_F32 = 0, RAGC_DTYPE_BF16 = 1 } ragc_dtype;

/* Paged K/V pool of one layer. */
typedef struct ragc_kv_pool {
    void* k;                    /* [device] K plane */
    void* v;                    /* [device] V plane */
    int32_t num_blocks;
    int32_t block_size;         /* must be 16 */
    int32_t kv_heads;
    int32_t head_dim;           /* 64 or 128 */
    int32_t dtype;              /* ragc_dtype */
    int32_t reserved;           /* must be 0 */
    int64_t block_stride_elems; /* elements between blocks of one plane */
} ragc_kv_pool;

/* One batch of augmented requests.  The request's document sequence has already
 * been matched against the tree by the caller: what arrives here is the block
 * chain of the matched path (block_table), the cached length (prefix_len, the
 * paper's alpha) and the non-cached length (new_len, the paper's beta).
 * new_start[r] is the row of q/k_new/v_new/out where request r's new tokens
 * begin; its rows are contiguous.  Normally the exclusive scan of new_len
 * starting at 0.  ragc_prefill_attn accepts any offsets (so a subset of a batch
 * can be launched over the same packed tensors); ragc_kv_append needs
 * new_start[r+1] = new_start[r] + new_len[r] (new_start[0] may be non-zero).
 * The h_* arrays are host copies of the same metadata.  The launch is sized on the host
 * and the work items carry the lengths to the device in the kernel arguments, so a
 * serving loop passes h_prefix_len, h_new_len and h_new_start; any of them that is NULL
 * is read back from its device array with a synchronous hipMemcpy inside the call (slow,
 * not capturable in a HIP graph, and the device array must be complete by then).
 * h_block_table is optional; when given, every entry the call will touch is
 * range-checked. */
typedef struct ragc_batch {
    int32_t num_reqs;
    int32_t table_stride;          /* entries per block_table row */
    const int32_t* prefix_len;     /* [device] [num_reqs] */
    const int32_t* new_len;        /* [device] [num_reqs] */
    const int32_t* new_start;      /* [device] [num_reqs+1] first packed row of each request */
    const int32_t* block_table;    /* [device] [num_reqs][table_stride] */
    const int32_t* h_prefix_len;   /* [host] [num_reqs] */
    const int32_t* h_new_len;      /* [host] [num_reqs] */
    const int32_t* h_new_start;    /* [host] [num_reqs+1] */
    const int32_t* h_block_table;  /* [host] optional */
} ragc_batch;

/* flags of ragc_prefill_attn */
#define RAGC_ATTN_APPEND_FUSED 0x1u /* also write k_new/v_new into their paged slots */
#define RAGC_ATTN_NO_SPLIT 0x2u     /* never split the key range across workgroups */
#define RAGC_ATTN_VALIDATE 0x4u     /* debug: run ragc_batch_validate first (synchronous read-backs) */

/* flags of ragc_kv_swap */
#define RAGC_SWAP_AUTO 0x0u
#define RAGC_SWAP_MEMCPY 0x1u /* one hipMemcpyAsync per run of adjacent blocks and plane */
#define RAGC_SWAP_KERNEL 0x2u /* copy kernel that reads/writes the pinned host pool directly */

#define RAGC_SWAP_TO_DEVICE 0
#define RAGC_SWAP_TO_HOST 1

/* Library version, major*10000 + minor*100 + patch. */
int ragc_version(void);

/* Thread-local text of the last error on this thread ("" if none). */
const char* ragc_last_error(void);

/* Bytes of K/V cache one token occupies in a model: 2 * layers * kv_heads *
 * head_dim * sizeof(dtype) (the KV Size column of the paper's model table).
 * Returns 0 on bad arguments. */
int64_t ragc_kv_bytes_per_token(int32_t layers, int32_t kv_heads, int32_t head_dim, int32_t dtype);

/* Debug validation of the preconditions that the kernels cannot check (see the top of
 * this file): reads prefix_len, new_len, new_start and block_table back from the device
 * (synchronous copies; the arrays must be complete), compares them with the host copies
 * that are given, range-checks every table entry the batch touches and, with
 * writes_new_tokens != 0 (a fused or standalone append follows), requires that every
 * block that receives new tokens does so for one request only and is in no request's
 * read-only prefix.  Returns RAGC_ERR_RANGE with a message that names the block and the
 * requests.  Not for the serving path. */
int ragc_batch_validate(const ragc_kv_pool* pool, const ragc_batch* batch, int32_t writes_new_tokens);

/* Test hook: override how ragc_prefill_attn lays a bf16 batch out on the GPU.
 *   variant  -1 = library's choice, 0 = 4-wave workgroups, 1 = 8-wave workgroups
 *   splits    0 = library's choice, 1..16 = copies of every work item along the keys
 * Process-wide and not synchronised with calls in flight on other threads: set it
 * before the calls it should affect and reset it (-1, 0) afterwards.  It changes the
 * workspace size, so query ragc_prefill_attn_workspace under the same setting. */
int ragc_debug_set_attn_plan(int32_t variant, int32_t splits);

/* Workspace ragc_prefill_attn needs for this batch with these flags (bytes, possibly 0).
 * A bf16 batch with fewer (request, 128-row tile, kv head) work items than the GPU has
 * compute units is split along the keys over several workgroups, whose partial results
 * (unnormalised output, row max and row sum, fp32) pass through the workspace and are
 * combined by a second kernel of the same call; RAGC_ATTN_NO_SPLIT turns that off (0 bytes).
 * Only the host arrays of `batch` are read.  Returns a negative ragc_status on error. */
int64_t ragc_prefill_attn_workspace(const ragc_kv_pool* pool, const ragc_batch* batch, int32_t q_heads,
                                    uint32_t flags);

/* Prefill attention of the new tokens of every request over the cached paged
 * prefix and their own fresh K/V, causal (Sec. 3.2, Sec. 4, Sec. 6):
 *     out[t,h,:] = softmax_j( scale * q[t,h,:] . K_j ) V_j ,  j = 0 .. prefix_len+i
 * where t = new_start[r]+i, kv head = h / (q_heads / kv_heads), K_j/V_j come from the
 * pool for j < prefix_len[r] and from k_new/v_new (row new_start[r]+j-prefix_len[r])
 * otherwise.  Softmax and accumulation are fp32; for bf16 the probabilities are
 * rounded to bf16 before the PV product and the output is rounded to nearest even.
 *   q, out        [device] [sum new_len][q_heads][head_dim]
 *   k_new, v_new  [device] [sum new_len][kv_heads][head_dim]
 *   workspace     [device] >= ragc_prefill_attn_workspace() bytes for the same flags, 256-byte
 *                 aligned (may be NULL when that is 0; too small: RAGC_ERR_WORKSPACE, nothing is
 *                 launched).  Contents need no initialisation and are undefined afterwards; it
 *                 is in use until the call's work has finished on `stream`, so calls on
 *                 different streams need workspaces of their own.
 * With RAGC_ATTN_APPEND_FUSED the same pass performs ragc_kv_append; the pool then
 * holds byte-identical contents to a separate ragc_kv_append call.
 * Requests with new_len == 0 are skipped.  prefix_len == 0 is plain causal
 * self-attention. */
int ragc_prefill_attn(const ragc_kv_pool* pool, const ragc_batch* batch, const void* q, const void* k_new,
                      const void* v_new, void* out, int32_t q_heads, float softmax_scale, uint32_t flags,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ragc_prefill_attn for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments minus the workspace, same kernels, same results; the
 * partial results of key-split work items go to an array that is part of the library's
 * device image (17,039,360 bytes, held by every GPU the library runs on until the process
 * ends) instead.  The call allocates nothing and does not synchronise:
 *   - h_prefix_len, h_new_len and h_new_start are required (RAGC_ERR_NULL otherwise) and
 *     RAGC_ATTN_VALIDATE is rejected, because both would read device memory back;
 *   - a batch whose partial results exceed the array returns RAGC_ERR_WORKSPACE and
 *     launches nothing (cannot happen with the library's own choice of split on a GPU of
 *     up to 256 compute units; it can under ragc_debug_set_attn_plan);
 *   - every call on one GPU shares that GPU's array: calls that may overlap (different
 *     streams, or different threads on one device) race -- serialise them or use
 *     ragc_prefill_attn with workspaces of their own.  Nothing in it needs clearing
 *     between calls: every value that is read was written by the same call.
 *   The first call on a device looks the array's address up (and may load the device
 *   image); make that call before starting a graph capture. */
int ragc_prefill_attn_static(const ragc_kv_pool* pool, const ragc_batch* batch, const void* q, const void* k_new,
                             const void* v_new, void* out, int32_t q_heads, float softmax_scale, uint32_t flags,
                             void* stream);

/* Write the fresh K/V of every request into its paged slots (Sec. 4: the tensors
 * of the accessed documents are cached after the first token): row
 * new_start[r]+i of k_new/v_new goes to position prefix_len[r]+i.  A byte copy.
 * Rows must be packed in request order, new_start[r+1] = new_start[r] + new_len[r]
 * (RAGC_ERR_RANGE otherwise; new_start[0] may be non-zero). */
int ragc_kv_append(const ragc_kv_pool* pool, const ragc_batch* batch, const void* k_new, const void* v_new,
                   void* stream);

/* Copy whole blocks (all kv heads, K and V planes) between the device pool and a
 * pinned host pool of the same per-block layout (Sec. 5.1 "Swap out only once";
 * Sec. 3.2 "Cache hit": the transfer is part of the hit latency).
 *   host_k, host_v            [pinned host] planes [num_host_slots][kv_heads][16][head_dim]
 *   host_block_stride_elems   elements between host slots of one plane
 *   dev_block_ids, host_slots [host] n entries each; pair i moves device block
 *                             dev_block_ids[i] <-> host slot host_slots[i]
 *   direction                 RAGC_SWAP_TO_DEVICE or RAGC_SWAP_TO_HOST
 * The id arrays are read before the call returns.  `stream` is normally a side
 * stream; the caller orders it against attention with events.  A byte copy. */
int ragc_kv_swap(const ragc_kv_pool* pool, void* host_k, void* host_v, int64_t host_block_stride_elems,
                 int32_t num_host_slots, const int32_t* dev_block_ids, const int32_t* host_slots, int32_t n,
                 int32_t direction, uint32_t flags, void* stream);

/* Test helper: gather `length` logical positions of request `req` from the pool
 * into contiguous [length][kv_heads][head_dim] buffers.  A byte copy.
 *   k_out, v_out [device]; length <= table_stride*16 */
int ragc_kv_gather(const ragc_kv_pool* pool, const ragc_batch* batch, int32_t req, int32_t length, void* k_out,
                   void* v_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RAGC_H */
