/* ragc_ctl.h — host-side controller of the paged K/V cache: knowledge tree, prefix matching,
 * PGDSF replacement over a GPU tier and a host tier, swap-out-only-once bookkeeping and the
 * cost model T(alpha, beta), and the cache-aware request queue.  Plain C ABI, CPU only, no GPU call is made here: the functions
 * turn a request's document sequence into the inputs of ragc_prefill_attn / ragc_kv_swap
 * (block table row, cached length, swap lists).  Everything is host memory; arrays passed in
 * are read during the call only, arrays passed out are caller-owned with stated capacities.
 * Not thread-safe per tree: one controller thread, as in the paper.  Errors: the negative
 * RAGC_ERR_* codes of ragc.h, text from ragc_last_error().
 *
 * Readings of the paper taken here:
 *  - A node is one document at one place in a path of documents (paper Sec. 5.1, knowledge
 *    tree).  K/V is addressed flatly over a request's sequence in 16-token blocks; a node
 *    covering tokens [b, e) of its path owns the blocks whose last token lies in [b, e),
 *    i.e. floor(e/16) - floor(b/16) blocks.  The cached prefix handed to the kernels is
 *    alpha = 16 * floor(end of the last matched node / 16); up to 15 tail tokens of the matched
 *    path are recomputed with the request.
 *  - Priority = Clock + AvgCost * Frequency (Sec. 5.1, Formula 1 with the Cost/Size of
 *    Formula 3; Algorithm 1).  One clock and one priority per tier; both priorities are set on
 *    every retrieval.  A node's statistics live and die with the node.
 *  - Eviction from the GPU tier takes the lowest-priority GPU leaf (a node in GPU memory with
 *    no child in GPU memory), ties to the node created first, and raises the clock to the
 *    priority of each evicted node (Formula 2; Algorithm 1, EVICT_IN_GPU).  Nodes of requests
 *    between begin and end are never candidates.  The host tier works the same way on nodes
 *    that live in host memory only and have no children; what it evicts leaves the cache.
 *  - Swap out only once (Sec. 5.1): the first GPU eviction of a node copies its blocks to host
 *    slots, which the node keeps while it is in the tree; later GPU evictions copy nothing.
 *    When the host tier cannot make room for a first copy the node and its subtree are freed.
 *    A first copy is struck from the request's list again when, later in the same request, the
 *    host tier drops that node: its slot may already be promised to another node.
 *  - Device block ids and host slot ids come from LIFO free lists that start as 0, 1, 2, ...
 *  - T(alpha, beta): bilinear interpolation in the profiled grid (Algorithm 1, interpolation
 *    steps); outside the grid the outermost cell is extended linearly.
 */
#ifndef RAGC_CTL_H
#define RAGC_CTL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Profiled prefill time T[i * n_beta + j] = T(alpha[i], beta[j]); alpha and beta strictly
 * increasing, at least two grid lines each.  All three arrays are copied by ragc_tree_create. */
typedef struct ragc_cost_grid {
    int32_t n_alpha;
    int32_t n_beta;
    const double* alpha; /* cached tokens */
    const double* beta;  /* non-cached tokens */
    const double* t;     /* any time unit */
} ragc_cost_grid;

/* T(alpha, beta) by bilinear interpolation (paper Sec. 5.1, Algorithm 1).  Returns 0 and writes
 * *t_out, or RAGC_ERR_NULL / RAGC_ERR_SHAPE for a missing or malformed grid. */
int ragc_cost_interp(const ragc_cost_grid* grid, double alpha, double beta, double* t_out);

typedef struct ragc_tree ragc_tree; /* opaque */

/* A tree over `gpu_blocks` device blocks and `host_slots` host slots (both may be any size >= 0;
 * ids handed out are 0 .. n-1).  NULL on error. */
ragc_tree* ragc_tree_create(int32_t gpu_blocks, int32_t host_slots, const ragc_cost_grid* grid);
void ragc_tree_destroy(ragc_tree* tree);

/* What one request needs, as counts; the lists are fetched with ragc_tree_plan_read. */
typedef struct ragc_plan {
    int64_t request_id;
    int32_t matched_docs;   /* documents found by prefix matching (paper Sec. 5.1) */
    int32_t alpha;          /* cached tokens = prefix_len for ragc_prefill_attn, a multiple of 16 */
    int32_t beta;           /* non-cached tokens = new_len: tail of the matched path, new documents, question */
    int32_t n_blocks;       /* block table entries: ceil((alpha + beta) / 16) */
    int32_t n_swap_out;     /* (device block, host slot) copies to run first, device -> host */
    int32_t n_swap_in;      /* then these, host -> device; then attention */
    int32_t n_evicted_gpu;  /* nodes that left GPU memory for this request, in order */
    int32_t n_evicted_host; /* nodes that left the cache, in order */
} ragc_plan;

/* A request arrives with its retrieved documents in order (ids and token counts; a document id
 * always comes with the same count) and `question_len` further tokens.  Matches the prefix,
 * makes room (evictions, swap lists), gives every non-cached document a node, assigns blocks
 * for all alpha + beta tokens and updates frequency, cost and priority of every document of the
 * request (Algorithm 1, UPDATE_NODE_IN_GPU with the request's alpha and beta).  The nodes of the
 * request stay in GPU memory until ragc_tree_end.  RAGC_ERR_RANGE if the request cannot fit even
 * after evicting everything that is not in use: then nothing has changed.
 * Requests in flight together (the paper batches several per prefill iteration, Sec. 7): a node
 * created by a request that has not ended yet has its blocks reserved but its K/V not written, so
 * it is not a cached prefix for anyone else.  Matching stops at such a node; this request then
 * computes that document and everything after it in blocks of its own (they return to the free
 * list at ragc_tree_end), gives none of them a node, and counts as one more computation in the
 * statistics of the nodes that exist.  Plans of requests in flight together therefore never share
 * a block that one of them writes, and may be launched in one batch or in any order. */
int ragc_tree_begin(ragc_tree* tree, const int64_t* doc_ids, const int32_t* doc_lens, int32_t n_docs,
                    int32_t question_len, ragc_plan* plan);

/* Caller-owned arrays for the lists of a plan; a NULL array is skipped, a capacity below the
 * plan's count is RAGC_ERR_RANGE (nothing is written). */
typedef struct ragc_plan_buffers {
    int32_t* block_table;   int32_t table_cap;
    int32_t* swap_out_dev;  int32_t* swap_out_slot;
    int32_t* swap_in_dev;   int32_t* swap_in_slot;  int32_t swap_cap;
    int64_t* evicted_gpu;   int64_t* evicted_host;  int32_t evicted_cap;
} ragc_plan_buffers;
int ragc_tree_plan_read(const ragc_tree* tree, int64_t request_id, const ragc_plan_buffers* out);

/* The request is done (its K/V has been appended): the nodes it created become usable as cached
 * prefix, its nodes may be evicted again and the blocks that no node owns (tail of the last
 * document, question, documents it computed next to a request in flight) return to the free
 * list.  Call it only after the attention call that appends the request's K/V has been enqueued
 * on the stream every later reader uses (or has completed). */
int ragc_tree_end(ragc_tree* tree, int64_t request_id);

typedef struct ragc_tree_stats {
    double clock_gpu, clock_host;
    int64_t nodes, nodes_in_gpu;
    int64_t free_gpu_blocks, free_host_slots;
    int64_t docs_requested, docs_hit;      /* hit rate = docs_hit / docs_requested (paper Sec. 7.3) */
    int64_t blocks_swapped_out, blocks_swapped_in, zero_copy_evictions;
} ragc_tree_stats;
int ragc_tree_get_stats(const ragc_tree* tree, ragc_tree_stats* out);

typedef struct ragc_node_info {
    int64_t id;          /* creation order, 1, 2, ... */
    int32_t in_gpu;      /* 1: GPU memory, 0: host memory only */
    int32_t host_valid;  /* a host copy exists */
    int32_t length;      /* tokens */
    int32_t n_owned;     /* blocks */
    int32_t pins;        /* requests in flight that use it */
    int32_t computed;    /* 1 once the request that created the node has ended (its K/V is written) */
    int64_t frequency, num_computed;
    double avg_cost, priority_gpu, priority_host;
} ragc_node_info;
/* The node reached by the document path; RAGC_ERR_RANGE if that path is not cached. */
int ragc_tree_find(const ragc_tree* tree, const int64_t* doc_path, int32_t n, ragc_node_info* out);

/* Frequencies count retrievals within a time window (Sec. 5.1): start a new window. */
int ragc_tree_reset_frequencies(ragc_tree* tree);

/* Cached length alpha and computation length beta the request would get from ragc_tree_begin now;
 * nothing changes. */
int ragc_tree_peek(const ragc_tree* tree, const int64_t* doc_ids, const int32_t* doc_lens, int32_t n_docs,
                   int32_t question_len, int32_t* alpha, int32_t* beta);

/* Cache-aware reordering (paper Sec. 5.2): waiting requests are served by
 * OrderPriority = cached length / computation length, evaluated against the tree at the moment of
 * the choice; equal priorities go to the request that arrived first.  Starvation window (the paper
 * says there is one, not how it counts): a request that has seen `window` later arrivals served
 * before it is served next, oldest first; window 0 is arrival order. */
typedef struct ragc_queue ragc_queue; /* opaque */
ragc_queue* ragc_queue_create(int32_t window);
void ragc_queue_destroy(ragc_queue* queue);
/* The arrays are copied; `tag` is the caller's name for the request. */
int ragc_queue_push(ragc_queue* queue, int64_t tag, const int64_t* doc_ids, const int32_t* doc_lens, int32_t n_docs,
                    int32_t question_len);
/* Removes the request to serve next and writes its tag; RAGC_ERR_RANGE if nothing waits. */
int ragc_queue_pop(ragc_queue* queue, const ragc_tree* tree, int64_t* tag);
int32_t ragc_queue_size(const ragc_queue* queue);

#ifdef __cplusplus
}
#endif
#endif
