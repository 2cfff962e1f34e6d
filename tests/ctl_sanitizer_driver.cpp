// Replays a request trace through the controller's C ABI (include/ragc_ctl.h) and prints every
// decision.  tests/test_controller_sanitizers.py builds this file together with ragc_ctl.cpp for
// the CPU with -fsanitize=address,undefined, runs it on seeded traces and compares the printed
// decisions with what the shipped library returns for the same trace.  CPU only.
//
// Trace format (text, whitespace separated):
//   gpu_blocks host_slots n_alpha n_beta  alpha[n_alpha]  beta[n_beta]  t[n_alpha*n_beta]
//   then operations:  B n_docs question_len (id len)*n_docs   -- ragc_tree_begin
//                     E k                                     -- ragc_tree_end of the k-th live request
//                     R                                       -- ragc_tree_reset_frequencies
//                     P n_docs question_len (id len)*n_docs   -- ragc_tree_peek
//                     Q window n (tag n_docs question_len (id len)*n_docs)*n  -- queue: push all, pop all
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../include/ragc.h"
#include "../include/ragc_ctl.h"

namespace ragc {
// the library's error recorder lives in the C-ABI front end, which is not part of this build
int set_error(int code, const char* fmt, ...) {
    (void)fmt;
    return code;
}
}  // namespace ragc

int main(int argc, char** argv) {
    if (argc != 2) return 2;
    FILE* f = std::fopen(argv[1], "r");
    if (!f) return 2;
    int gpu_blocks, host_slots, na, nb;
    if (std::fscanf(f, "%d %d %d %d", &gpu_blocks, &host_slots, &na, &nb) != 4) return 2;
    std::vector<double> alpha(na), beta(nb), t((size_t)na * nb);
    for (double& x : alpha) if (std::fscanf(f, "%lf", &x) != 1) return 2;
    for (double& x : beta) if (std::fscanf(f, "%lf", &x) != 1) return 2;
    for (double& x : t) if (std::fscanf(f, "%lf", &x) != 1) return 2;
    ragc_cost_grid grid{na, nb, alpha.data(), beta.data(), t.data()};
    ragc_tree* tree = ragc_tree_create(gpu_blocks, host_slots, &grid);
    if (!tree) return 3;
    std::vector<int64_t> live;
    char op;
    auto read_docs = [&](std::vector<int64_t>& ids, std::vector<int32_t>& lens, int& qlen) {
        int n;
        if (std::fscanf(f, "%d %d", &n, &qlen) != 2) std::exit(2);
        ids.resize(n);
        lens.resize(n);
        for (int i = 0; i < n; ++i) {
            long long id;
            int len;
            if (std::fscanf(f, "%lld %d", &id, &len) != 2) std::exit(2);
            ids[i] = id;
            lens[i] = len;
        }
    };
    while (std::fscanf(f, " %c", &op) == 1) {
        std::vector<int64_t> ids;
        std::vector<int32_t> lens;
        int qlen = 0;
        if (op == 'B') {
            read_docs(ids, lens, qlen);
            ragc_plan plan{};
            const int rc = ragc_tree_begin(tree, ids.data(), lens.data(), (int32_t)ids.size(), qlen, &plan);
            std::printf("B %d", rc);
            if (rc == 0) {
                std::vector<int32_t> table(plan.n_blocks), od(plan.n_swap_out), os(plan.n_swap_out), id(plan.n_swap_in), is(plan.n_swap_in);
                std::vector<int64_t> eg(plan.n_evicted_gpu), eh(plan.n_evicted_host);
                const int cap_s = plan.n_swap_out > plan.n_swap_in ? plan.n_swap_out : plan.n_swap_in;
                const int cap_e = plan.n_evicted_gpu > plan.n_evicted_host ? plan.n_evicted_gpu : plan.n_evicted_host;
                od.resize(cap_s); os.resize(cap_s); id.resize(cap_s); is.resize(cap_s); eg.resize(cap_e); eh.resize(cap_e);
                ragc_plan_buffers buf{table.data(), plan.n_blocks, od.data(), os.data(), id.data(), is.data(), cap_s, eg.data(), eh.data(), cap_e};
                if (ragc_tree_plan_read(tree, plan.request_id, &buf) != 0) return 4;
                std::printf(" %lld %d %d %d T", (long long)plan.request_id, plan.matched_docs, plan.alpha, plan.beta);
                for (int i = 0; i < plan.n_blocks; ++i) std::printf(" %d", table[i]);
                std::printf(" O");
                for (int i = 0; i < plan.n_swap_out; ++i) std::printf(" %d:%d", od[i], os[i]);
                std::printf(" I");
                for (int i = 0; i < plan.n_swap_in; ++i) std::printf(" %d:%d", id[i], is[i]);
                std::printf(" G");
                for (int i = 0; i < plan.n_evicted_gpu; ++i) std::printf(" %lld", (long long)eg[i]);
                std::printf(" H");
                for (int i = 0; i < plan.n_evicted_host; ++i) std::printf(" %lld", (long long)eh[i]);
                live.push_back(plan.request_id);
            }
            std::printf("\n");
        } else if (op == 'E') {
            int k;
            if (std::fscanf(f, "%d", &k) != 1) return 2;
            const int rc = ragc_tree_end(tree, live.at(k));
            live.erase(live.begin() + k);
            std::printf("E %d\n", rc);
        } else if (op == 'R') {
            std::printf("R %d\n", ragc_tree_reset_frequencies(tree));
        } else if (op == 'P') {
            read_docs(ids, lens, qlen);
            int32_t a = -1, b = -1;
            const int rc = ragc_tree_peek(tree, ids.data(), lens.data(), (int32_t)ids.size(), qlen, &a, &b);
            std::printf("P %d %d %d\n", rc, a, b);
        } else if (op == 'Q') {
            int window, n;
            if (std::fscanf(f, "%d %d", &window, &n) != 2) return 2;
            ragc_queue* q = ragc_queue_create(window);
            if (!q) return 3;
            for (int i = 0; i < n; ++i) {
                long long tag;
                if (std::fscanf(f, "%lld", &tag) != 1) return 2;
                read_docs(ids, lens, qlen);
                if (ragc_queue_push(q, tag, ids.data(), lens.data(), (int32_t)ids.size(), qlen) != 0) return 4;
            }
            std::printf("Q");
            while (ragc_queue_size(q) > 0) {
                int64_t tag = -1;
                if (ragc_queue_pop(q, tree, &tag) != 0) return 4;
                std::printf(" %lld", (long long)tag);
            }
            std::printf("\n");
            ragc_queue_destroy(q);
        } else {
            return 2;
        }
    }
    ragc_tree_stats s{};
    if (ragc_tree_get_stats(tree, &s) != 0) return 4;
    std::printf("S %lld %lld %lld %lld %lld %lld %lld %lld %lld\n", (long long)s.nodes, (long long)s.nodes_in_gpu, (long long)s.free_gpu_blocks,
                (long long)s.free_host_slots, (long long)s.docs_requested, (long long)s.docs_hit, (long long)s.blocks_swapped_out,
                (long long)s.blocks_swapped_in, (long long)s.zero_copy_evictions);
    // requests still in flight are dropped with the tree: destroy must free everything
    ragc_tree_destroy(tree);
    std::fclose(f);
    return 0;
}
