// Host-side controller of the paged K/V cache (declared in include/ragc_ctl.h): knowledge tree
// with prefix matching, PGDSF replacement over a GPU tier and a host tier, swap-out-only-once
// bookkeeping, block allocation and the cost model T(alpha, beta) (paper Sec. 5.1, Formulas
// 1-3, Algorithm 1).  CPU only.
//
// Candidates for eviction are kept in two ordered sets keyed by (priority, node id), one per
// tier, and membership is re-evaluated whenever one of the things it depends on changes (tier,
// pins, number of children in GPU memory, priority), so an eviction costs O(log nodes).
#include "../../include/ragc_ctl.h"

#include <algorithm>
#include <cstdio>
#include <deque>
#include <map>
#include <memory>
#include <set>
#include <unordered_map>
#include <utility>
#include <vector>

#include "../../include/ragc.h"
#include "ragc_internal.h"

using ragc::set_error;

namespace {

constexpr int kBlk = ragc::kBlock;
enum Tier { kGpu = 0, kHost = 1 };

struct CostGrid {
    std::vector<double> alpha, beta, t;  // t[i * beta.size() + j]

    static int validate(const ragc_cost_grid* g) {
        if (!g || !g->alpha || !g->beta || !g->t) return set_error(RAGC_ERR_NULL, "cost grid or one of its arrays is NULL");
        if (g->n_alpha < 2 || g->n_beta < 2) return set_error(RAGC_ERR_SHAPE, "cost grid needs at least 2 x 2 points (got %d x %d)", g->n_alpha, g->n_beta);
        for (int i = 1; i < g->n_alpha; ++i)
            if (!(g->alpha[i] > g->alpha[i - 1])) return set_error(RAGC_ERR_SHAPE, "cost grid: alpha is not strictly increasing at %d", i);
        for (int j = 1; j < g->n_beta; ++j)
            if (!(g->beta[j] > g->beta[j - 1])) return set_error(RAGC_ERR_SHAPE, "cost grid: beta is not strictly increasing at %d", j);
        return 0;
    }

    // lower grid line of the cell used for x; the outermost cells also serve points outside the grid
    static int cell(const double* axis, int n, double x) {
        const int l = (int)(std::upper_bound(axis, axis + n, x) - axis) - 1;
        return std::min(std::max(l, 0), n - 2);
    }

    // Algorithm 1, interpolation steps: along alpha on the low and the high beta line, then along beta
    static double interp(const double* alpha, int na, const double* beta, int nb, const double* t, double a, double b) {
        const int i = cell(alpha, na, a), j = cell(beta, nb, b);
        const double al = alpha[i], ah = alpha[i + 1], bl = beta[j], bh = beta[j + 1];
        const double t_ll = t[i * nb + j], t_hl = t[(i + 1) * nb + j], t_lh = t[i * nb + j + 1], t_hh = t[(i + 1) * nb + j + 1];
        const double t_l = t_ll + (a - al) / (ah - al) * (t_hl - t_ll);
        const double t_h = t_lh + (a - al) / (ah - al) * (t_hh - t_lh);
        return t_l + (b - bl) / (bh - bl) * (t_h - t_l);
    }

    double operator()(double a, double b) const {
        return interp(alpha.data(), (int)alpha.size(), beta.data(), (int)beta.size(), t.data(), a, b);
    }
};

struct Node {
    int64_t id = 0;
    int64_t doc = -1;
    int32_t length = 0;
    int64_t tok_begin = 0;
    Node* parent = nullptr;
    std::map<int64_t, Node*> children;
    int tier = kGpu;
    bool host_valid = false;
    std::vector<int32_t> dev, host;  // owned blocks in GPU memory / their host slots
    int64_t frequency = 0, num_computed = 0;
    double total_cost = 0.0, avg_cost = 0.0;
    double priority[2] = {0.0, 0.0};
    int pins = 0;
    bool computed = false;  // its K/V has been written: set when the request that created the node ends
    int gpu_children = 0;
    bool listed[2] = {false, false};  // member of the candidate set of the tier
    double listed_key[2] = {0.0, 0.0};

    int64_t tok_end() const { return tok_begin + length; }
    int32_t n_owned() const { return (int32_t)(tok_end() / kBlk - tok_begin / kBlk); }
};

struct Request {
    std::vector<Node*> nodes;       // matched and new, in path order (all pinned)
    std::vector<Node*> created;     // the new ones: computed once this request has ended
    std::vector<int32_t> unowned;   // blocks no node owns
    std::vector<int32_t> table, out_dev, out_slot, in_dev, in_slot;
    std::vector<int64_t> evicted_gpu, evicted_host;
};

}  // namespace

struct ragc_tree {
    CostGrid grid;
    std::vector<int32_t> free_dev, free_host;  // LIFO
    double clock[2] = {0.0, 0.0};
    Node root;
    int64_t next_id = 1, next_request = 1;
    int64_t n_nodes = 0, n_nodes_gpu = 0;
    std::set<std::pair<double, int64_t>> candidates[2];
    std::unordered_map<int64_t, Node*> by_id;
    std::unordered_map<int64_t, Request> requests;
    int64_t docs_requested = 0, docs_hit = 0, swapped_out = 0, swapped_in = 0, zero_copy = 0;

    // ---- candidate sets
    bool eligible(const Node* n, int tier) const {
        if (n == &root || n->pins != 0) return false;
        if (tier == kGpu) return n->tier == kGpu && n->gpu_children == 0;
        return n->tier == kHost && n->children.empty();
    }
    void refresh(Node* n) {
        for (int tier = 0; tier < 2; ++tier) {
            if (n->listed[tier]) {
                candidates[tier].erase({n->listed_key[tier], n->id});
                n->listed[tier] = false;
            }
            if (eligible(n, tier)) {
                n->listed_key[tier] = n->priority[tier];
                candidates[tier].insert({n->listed_key[tier], n->id});
                n->listed[tier] = true;
            }
        }
    }
    void unlist(Node* n) {
        for (int tier = 0; tier < 2; ++tier)
            if (n->listed[tier]) {
                candidates[tier].erase({n->listed_key[tier], n->id});
                n->listed[tier] = false;
            }
    }
    void set_tier(Node* n, int tier) {
        if (n->tier == tier) return;
        n->tier = tier;
        const int d = tier == kGpu ? 1 : -1;
        n_nodes_gpu += d;
        if (n->parent) {
            n->parent->gpu_children += d;
            refresh(n->parent);
        }
        refresh(n);
    }
    void pin(Node* n, int d) {
        n->pins += d;
        refresh(n);
    }

    int32_t take(std::vector<int32_t>& list) {
        const int32_t b = list.back();
        list.pop_back();
        return b;
    }

    // a node leaves the cache together with everything below it
    void remove_subtree(Node* n, Request* rq) {
        // children in the order they were created (ids grow with creation)
        std::vector<Node*> kids;
        for (const auto& kv : n->children) kids.push_back(kv.second);
        std::sort(kids.begin(), kids.end(), [](const Node* a, const Node* b) { return a->id < b->id; });
        for (Node* c : kids) remove_subtree(c, rq);
        unlist(n);
        if (n->tier == kGpu) {
            free_dev.insert(free_dev.end(), n->dev.begin(), n->dev.end());
            --n_nodes_gpu;
            --n->parent->gpu_children;
        }
        if (n->host_valid) {
            // a copy to the host that this same request asked for a moment ago is void now
            if (rq && !n->host.empty()) {
                size_t kept = 0;
                for (size_t i = 0; i < rq->out_slot.size(); ++i) {
                    if (std::find(n->host.begin(), n->host.end(), rq->out_slot[i]) != n->host.end()) continue;
                    rq->out_dev[kept] = rq->out_dev[i];
                    rq->out_slot[kept] = rq->out_slot[i];
                    ++kept;
                }
                swapped_out -= (int64_t)(rq->out_slot.size() - kept);
                rq->out_dev.resize(kept);
                rq->out_slot.resize(kept);
            }
            free_host.insert(free_host.end(), n->host.begin(), n->host.end());
        }
        Node* p = n->parent;
        p->children.erase(n->doc);
        if (rq) rq->evicted_host.push_back(n->id);
        by_id.erase(n->id);
        --n_nodes;
        delete n;
        refresh(p);
    }

    // host tier: free slots by dropping host-only leaves, lowest priority first
    bool evict_in_host(size_t required, Request* rq) {
        while (free_host.size() < required) {
            if (candidates[kHost].empty()) return false;
            const auto top = *candidates[kHost].begin();
            clock[kHost] = std::max(clock[kHost], top.first);
            remove_subtree(by_id.at(top.second), rq);
        }
        return true;
    }

    // Algorithm 1, EVICT_IN_GPU, plus the swap-out-only-once rule
    void evict_in_gpu(int64_t required, Request& rq) {
        int64_t freed = 0;
        while (freed < required) {
            const auto top = *candidates[kGpu].begin();  // begin() has checked that enough can be freed
            Node* n = by_id.at(top.second);
            clock[kGpu] = std::max(clock[kGpu], top.first);
            rq.evicted_gpu.push_back(n->id);
            const int32_t owned = n->n_owned();
            freed += owned;
            if (n->host_valid) {
                ++zero_copy;
            } else if (owned == 0) {
                n->host_valid = true;
            } else {
                // its own slot must not be taken from under it: the node is not a host candidate yet
                if (!evict_in_host((size_t)owned, &rq)) {
                    remove_subtree(n, &rq);
                    continue;
                }
                for (int32_t i = 0; i < owned; ++i) {
                    n->host.push_back(take(free_host));
                    rq.out_dev.push_back(n->dev[i]);
                    rq.out_slot.push_back(n->host[i]);
                }
                swapped_out += owned;
                n->host_valid = true;
            }
            free_dev.insert(free_dev.end(), n->dev.begin(), n->dev.end());
            n->dev.clear();
            set_tier(n, kHost);
        }
    }

    // (n can be evicted from the GPU tier eventually, blocks that evictions at and below n can free)
    std::pair<bool, int64_t> freeable(const Node* n) const {
        bool ok = n != &root && n->tier == kGpu && n->pins == 0;
        int64_t blocks = 0;
        for (const auto& kv : n->children) {
            if (kv.second->tier != kGpu) continue;
            const auto c = freeable(kv.second);
            blocks += c.second;
            ok = ok && c.first;
        }
        if (ok) blocks += n->n_owned();
        return {ok, blocks};
    }

    // Algorithm 1, UPDATE_NODE_IN_GPU with the request's alpha and beta
    void update_node(Node* n, bool is_cached, int32_t alpha, int32_t beta) {
        n->frequency += 1;
        if (!is_cached) {
            const double t = grid((double)alpha, (double)beta);
            n->total_cost += t / (double)beta;
            n->num_computed += 1;
            n->avg_cost = n->total_cost / (double)n->num_computed;
        }
        for (int tier = 0; tier < 2; ++tier) n->priority[tier] = clock[tier] + n->avg_cost * (double)n->frequency;
        refresh(n);
    }

    ~ragc_tree() {
        for (auto& kv : requests)
            for (Node* n : kv.second.nodes) n->pins = 0;
        while (!root.children.empty()) remove_subtree(root.children.begin()->second, nullptr);
    }
};

extern "C" {

int ragc_cost_interp(const ragc_cost_grid* grid, double alpha, double beta, double* t_out) {
    if (!t_out) return set_error(RAGC_ERR_NULL, "t_out is NULL");
    if (int rc = CostGrid::validate(grid)) return rc;
    *t_out = CostGrid::interp(grid->alpha, grid->n_alpha, grid->beta, grid->n_beta, grid->t, alpha, beta);
    return 0;
}

ragc_tree* ragc_tree_create(int32_t gpu_blocks, int32_t host_slots, const ragc_cost_grid* grid) {
    if (gpu_blocks < 0 || host_slots < 0) {
        set_error(RAGC_ERR_RANGE, "gpu_blocks %d / host_slots %d must not be negative", gpu_blocks, host_slots);
        return nullptr;
    }
    if (CostGrid::validate(grid)) return nullptr;
    ragc_tree* t = new ragc_tree();
    t->grid.alpha.assign(grid->alpha, grid->alpha + grid->n_alpha);
    t->grid.beta.assign(grid->beta, grid->beta + grid->n_beta);
    t->grid.t.assign(grid->t, grid->t + (size_t)grid->n_alpha * grid->n_beta);
    for (int32_t b = gpu_blocks - 1; b >= 0; --b) t->free_dev.push_back(b);   // back() is 0, then 1, ...
    for (int32_t s = host_slots - 1; s >= 0; --s) t->free_host.push_back(s);
    t->root.pins = 1;
    t->root.computed = true;
    return t;
}

void ragc_tree_destroy(ragc_tree* tree) { delete tree; }

int ragc_tree_begin(ragc_tree* tree, const int64_t* doc_ids, const int32_t* doc_lens, int32_t n_docs, int32_t question_len,
                    ragc_plan* plan) {
    if (!tree || !plan) return set_error(RAGC_ERR_NULL, "tree or plan is NULL");
    if (n_docs < 0 || question_len < 0) return set_error(RAGC_ERR_RANGE, "n_docs %d / question_len %d must not be negative", n_docs, question_len);
    if (n_docs > 0 && (!doc_ids || !doc_lens)) return set_error(RAGC_ERR_NULL, "doc_ids or doc_lens is NULL");
    int64_t docs_total = 0;
    for (int32_t i = 0; i < n_docs; ++i) {
        if (doc_lens[i] <= 0) return set_error(RAGC_ERR_RANGE, "document %d has %d tokens", i, doc_lens[i]);
        for (int32_t j = 0; j < i; ++j)
            if (doc_ids[j] == doc_ids[i]) return set_error(RAGC_ERR_SHAPE, "document id %lld appears twice in one request", (long long)doc_ids[i]);
        docs_total += doc_lens[i];
    }
    const int64_t total = docs_total + question_len;
    if (total <= 0 || total > 0x7fffffff) return set_error(RAGC_ERR_RANGE, "request has %lld tokens", (long long)total);

    // prefix matching along the path of documents (O(height))
    std::vector<Node*> path;
    Node* cur = &tree->root;
    // A node whose request is still in flight has its blocks reserved but its K/V not written: it
    // cannot serve as a cached prefix, so matching stops there as well.
    for (int32_t i = 0; i < n_docs; ++i) {
        const auto it = cur->children.find(doc_ids[i]);
        if (it == cur->children.end() || !it->second->computed) break;
        if (it->second->length != doc_lens[i])
            return set_error(RAGC_ERR_SHAPE, "document id %lld comes with %d tokens, cached with %d", (long long)doc_ids[i], doc_lens[i], it->second->length);
        path.push_back(it->second);
        cur = it->second;
    }
    const int32_t m = (int32_t)path.size();
    // The next documents have nodes that are being computed elsewhere: this request computes them
    // for itself in blocks of its own and adds nothing to the tree below that point.
    std::vector<Node*> in_progress;
    {
        const Node* nxt = cur;
        for (int32_t i = m; i < n_docs; ++i) {
            const auto it = nxt->children.find(doc_ids[i]);
            if (it == nxt->children.end()) break;
            if (it->second->length != doc_lens[i])
                return set_error(RAGC_ERR_SHAPE, "document id %lld comes with %d tokens, cached with %d", (long long)doc_ids[i], doc_lens[i], it->second->length);
            in_progress.push_back(it->second);
            nxt = it->second;
        }
    }
    const bool blocked = !in_progress.empty();
    for (Node* n : path) tree->pin(n, +1);
    const int64_t matched_end = path.empty() ? 0 : path.back()->tok_end();
    const int32_t alpha = (int32_t)(matched_end / kBlk * kBlk);
    const int32_t beta = (int32_t)(total - alpha);
    const int64_t blocks_total = (total + kBlk - 1) / kBlk;
    const int64_t cacheable = blocked ? alpha / kBlk : docs_total / kBlk;
    int64_t need = blocks_total - alpha / kBlk;
    for (Node* n : path)
        if (n->tier == kHost) need += n->n_owned();
    const int64_t have = (int64_t)tree->free_dev.size();
    if (need > have && need > have + tree->freeable(&tree->root).second) {  // the walk over the tree only when room is short
        for (Node* n : path) tree->pin(n, -1);
        return set_error(RAGC_ERR_RANGE, "request needs %lld blocks: %lld free, the rest is in use", (long long)need, (long long)have);
    }

    const int64_t rid = tree->next_request++;
    Request& rq = tree->requests[rid];
    if (need > have) tree->evict_in_gpu(need - have, rq);

    // matched nodes that live in host memory come back (the host copy stays valid)
    for (Node* n : path) {
        if (n->tier != kHost) continue;
        const int32_t owned = n->n_owned();
        for (int32_t i = 0; i < owned; ++i) {
            n->dev.push_back(tree->take(tree->free_dev));
            rq.in_dev.push_back(n->dev[i]);
            rq.in_slot.push_back(n->host[i]);
        }
        tree->swapped_in += owned;
        tree->set_tier(n, kGpu);
    }
    // a node for every document that was not matched
    rq.nodes = path;
    int64_t tok = matched_end;
    for (int32_t i = m; i < (blocked ? m : n_docs); ++i) {
        Node* n = new Node();
        n->id = tree->next_id++;
        n->doc = doc_ids[i];
        n->length = doc_lens[i];
        n->tok_begin = tok;
        n->parent = cur;
        n->pins = 1;
        const int32_t owned = n->n_owned();
        for (int32_t k = 0; k < owned; ++k) n->dev.push_back(tree->take(tree->free_dev));
        cur->children[n->doc] = n;
        cur->gpu_children += 1;
        tree->refresh(cur);
        tree->by_id[n->id] = n;
        ++tree->n_nodes;
        ++tree->n_nodes_gpu;
        rq.nodes.push_back(n);
        rq.created.push_back(n);
        cur = n;
        tok += n->length;
    }
    for (int64_t i = cacheable; i < blocks_total; ++i) rq.unowned.push_back(tree->take(tree->free_dev));
    for (Node* n : rq.nodes) rq.table.insert(rq.table.end(), n->dev.begin(), n->dev.end());
    rq.table.insert(rq.table.end(), rq.unowned.begin(), rq.unowned.end());

    // retrieval updates every document's node
    for (size_t i = 0; i < rq.nodes.size(); ++i) tree->update_node(rq.nodes[i], (int32_t)i < m, alpha, beta);
    for (Node* n : in_progress) tree->update_node(n, false, alpha, beta);  // computed once more, by this request
    tree->docs_requested += n_docs;
    tree->docs_hit += m;

    plan->request_id = rid;
    plan->matched_docs = m;
    plan->alpha = alpha;
    plan->beta = beta;
    plan->n_blocks = (int32_t)rq.table.size();
    plan->n_swap_out = (int32_t)rq.out_dev.size();
    plan->n_swap_in = (int32_t)rq.in_dev.size();
    plan->n_evicted_gpu = (int32_t)rq.evicted_gpu.size();
    plan->n_evicted_host = (int32_t)rq.evicted_host.size();
    return 0;
}

int ragc_tree_plan_read(const ragc_tree* tree, int64_t request_id, const ragc_plan_buffers* out) {
    if (!tree || !out) return set_error(RAGC_ERR_NULL, "tree or out is NULL");
    const auto it = tree->requests.find(request_id);
    if (it == tree->requests.end()) return set_error(RAGC_ERR_RANGE, "request %lld is not in flight", (long long)request_id);
    const Request& rq = it->second;
    if (out->block_table && out->table_cap < (int32_t)rq.table.size())
        return set_error(RAGC_ERR_RANGE, "table_cap %d < %zu entries", out->table_cap, rq.table.size());
    const size_t n_swap = std::max(rq.out_dev.size(), rq.in_dev.size());
    if ((out->swap_out_dev || out->swap_out_slot || out->swap_in_dev || out->swap_in_slot) && (size_t)std::max(out->swap_cap, 0) < n_swap)
        return set_error(RAGC_ERR_RANGE, "swap_cap %d < %zu pairs", out->swap_cap, n_swap);
    const size_t n_ev = std::max(rq.evicted_gpu.size(), rq.evicted_host.size());
    if ((out->evicted_gpu || out->evicted_host) && (size_t)std::max(out->evicted_cap, 0) < n_ev)
        return set_error(RAGC_ERR_RANGE, "evicted_cap %d < %zu nodes", out->evicted_cap, n_ev);
    if (out->block_table) std::copy(rq.table.begin(), rq.table.end(), out->block_table);
    if (out->swap_out_dev) std::copy(rq.out_dev.begin(), rq.out_dev.end(), out->swap_out_dev);
    if (out->swap_out_slot) std::copy(rq.out_slot.begin(), rq.out_slot.end(), out->swap_out_slot);
    if (out->swap_in_dev) std::copy(rq.in_dev.begin(), rq.in_dev.end(), out->swap_in_dev);
    if (out->swap_in_slot) std::copy(rq.in_slot.begin(), rq.in_slot.end(), out->swap_in_slot);
    if (out->evicted_gpu) std::copy(rq.evicted_gpu.begin(), rq.evicted_gpu.end(), out->evicted_gpu);
    if (out->evicted_host) std::copy(rq.evicted_host.begin(), rq.evicted_host.end(), out->evicted_host);
    return 0;
}

int ragc_tree_end(ragc_tree* tree, int64_t request_id) {
    if (!tree) return set_error(RAGC_ERR_NULL, "tree is NULL");
    const auto it = tree->requests.find(request_id);
    if (it == tree->requests.end()) return set_error(RAGC_ERR_RANGE, "request %lld is not in flight", (long long)request_id);
    for (Node* n : it->second.nodes) tree->pin(n, -1);
    for (Node* n : it->second.created) n->computed = true;  // the request has run: the K/V of its new documents is in their blocks
    tree->free_dev.insert(tree->free_dev.end(), it->second.unowned.begin(), it->second.unowned.end());
    tree->requests.erase(it);
    return 0;
}

int ragc_tree_get_stats(const ragc_tree* tree, ragc_tree_stats* out) {
    if (!tree || !out) return set_error(RAGC_ERR_NULL, "tree or out is NULL");
    out->clock_gpu = tree->clock[kGpu];
    out->clock_host = tree->clock[kHost];
    out->nodes = tree->n_nodes;
    out->nodes_in_gpu = tree->n_nodes_gpu;
    out->free_gpu_blocks = (int64_t)tree->free_dev.size();
    out->free_host_slots = (int64_t)tree->free_host.size();
    out->docs_requested = tree->docs_requested;
    out->docs_hit = tree->docs_hit;
    out->blocks_swapped_out = tree->swapped_out;
    out->blocks_swapped_in = tree->swapped_in;
    out->zero_copy_evictions = tree->zero_copy;
    return 0;
}

int ragc_tree_find(const ragc_tree* tree, const int64_t* doc_path, int32_t n, ragc_node_info* out) {
    if (!tree || !out || (n > 0 && !doc_path)) return set_error(RAGC_ERR_NULL, "tree, doc_path or out is NULL");
    if (n <= 0) return set_error(RAGC_ERR_RANGE, "empty path");
    const Node* cur = &tree->root;
    for (int32_t i = 0; i < n; ++i) {
        const auto it = cur->children.find(doc_path[i]);
        if (it == cur->children.end()) return set_error(RAGC_ERR_RANGE, "path is not cached beyond %d documents", i);
        cur = it->second;
    }
    out->id = cur->id;
    out->in_gpu = cur->tier == kGpu;
    out->host_valid = cur->host_valid;
    out->length = cur->length;
    out->n_owned = cur->n_owned();
    out->pins = cur->pins;
    out->computed = cur->computed ? 1 : 0;
    out->frequency = cur->frequency;
    out->num_computed = cur->num_computed;
    out->avg_cost = cur->avg_cost;
    out->priority_gpu = cur->priority[kGpu];
    out->priority_host = cur->priority[kHost];
    return 0;
}

// cached and computation length of a request against the tree as it is (no state change)
static void peek_lengths(const ragc_tree* tree, const int64_t* doc_ids, const int32_t* doc_lens, int32_t n_docs,
                         int32_t question_len, int64_t* alpha, int64_t* beta) {
    const Node* cur = &tree->root;
    int64_t matched_end = 0, total = question_len;
    for (int32_t i = 0; i < n_docs; ++i) total += doc_lens[i];
    for (int32_t i = 0; i < n_docs; ++i) {
        const auto it = cur->children.find(doc_ids[i]);
        if (it == cur->children.end() || !it->second->computed) break;
        cur = it->second;
        matched_end = cur->tok_end();
    }
    *alpha = matched_end / kBlk * kBlk;
    *beta = total - *alpha;
}

int ragc_tree_peek(const ragc_tree* tree, const int64_t* doc_ids, const int32_t* doc_lens, int32_t n_docs,
                   int32_t question_len, int32_t* alpha, int32_t* beta) {
    if (!tree || !alpha || !beta || (n_docs > 0 && (!doc_ids || !doc_lens))) return set_error(RAGC_ERR_NULL, "a required pointer is NULL");
    if (n_docs < 0 || question_len < 0) return set_error(RAGC_ERR_RANGE, "n_docs %d / question_len %d must not be negative", n_docs, question_len);
    int64_t a = 0, b = 0;
    peek_lengths(tree, doc_ids, doc_lens, n_docs, question_len, &a, &b);
    *alpha = (int32_t)a;
    *beta = (int32_t)b;
    return 0;
}

int ragc_tree_reset_frequencies(ragc_tree* tree) {
    if (!tree) return set_error(RAGC_ERR_NULL, "tree is NULL");
    for (auto& kv : tree->by_id) kv.second->frequency = 0;
    return 0;
}

// ---- cache-aware reordering (paper Sec. 5.2)
struct ragc_queue {
    struct Waiting {
        int64_t tag;
        std::vector<int64_t> ids;
        std::vector<int32_t> lens;
        int32_t question_len;
        int32_t passed_over;
    };
    int32_t window = 0;
    std::deque<Waiting> waiting;  // in arrival order
};

ragc_queue* ragc_queue_create(int32_t window) {
    if (window < 0) {
        set_error(RAGC_ERR_RANGE, "window %d must not be negative", window);
        return nullptr;
    }
    ragc_queue* q = new ragc_queue();
    q->window = window;
    return q;
}

void ragc_queue_destroy(ragc_queue* queue) { delete queue; }

int ragc_queue_push(ragc_queue* queue, int64_t tag, const int64_t* doc_ids, const int32_t* doc_lens, int32_t n_docs,
                    int32_t question_len) {
    if (!queue || (n_docs > 0 && (!doc_ids || !doc_lens))) return set_error(RAGC_ERR_NULL, "a required pointer is NULL");
    if (n_docs < 0 || question_len < 0) return set_error(RAGC_ERR_RANGE, "n_docs %d / question_len %d must not be negative", n_docs, question_len);
    ragc_queue::Waiting w;
    w.tag = tag;
    w.ids.assign(doc_ids, doc_ids + n_docs);
    w.lens.assign(doc_lens, doc_lens + n_docs);
    w.question_len = question_len;
    w.passed_over = 0;
    queue->waiting.push_back(std::move(w));
    return 0;
}

int ragc_queue_pop(ragc_queue* queue, const ragc_tree* tree, int64_t* tag) {
    if (!queue || !tree || !tag) return set_error(RAGC_ERR_NULL, "queue, tree or tag is NULL");
    if (queue->waiting.empty()) return set_error(RAGC_ERR_RANGE, "no request is waiting");
    size_t pick = queue->waiting.size();
    for (size_t i = 0; i < queue->waiting.size(); ++i)
        if (queue->waiting[i].passed_over >= queue->window) {
            pick = i;  // the oldest request whose window is used up
            break;
        }
    if (pick == queue->waiting.size()) {
        // OrderPriority = cached / computation length, compared as a fraction; ties keep the earlier arrival
        int64_t best_a = 0, best_b = 1;
        bool have = false;
        for (size_t i = 0; i < queue->waiting.size(); ++i) {
            const auto& w = queue->waiting[i];
            int64_t a = 0, b = 0;
            peek_lengths(tree, w.ids.data(), w.lens.data(), (int32_t)w.ids.size(), w.question_len, &a, &b);
            const bool better = !have || (b == 0 ? (best_b != 0) : (best_b != 0 && a * best_b > best_a * b));
            if (better) {
                have = true;
                best_a = a;
                best_b = b;
                pick = i;
            }
        }
    }
    for (size_t i = 0; i < pick; ++i) queue->waiting[i].passed_over += 1;
    *tag = queue->waiting[pick].tag;
    queue->waiting.erase(queue->waiting.begin() + (long)pick);
    return 0;
}

int32_t ragc_queue_size(const ragc_queue* queue) { return queue ? (int32_t)queue->waiting.size() : 0; }

}  // extern "C"
