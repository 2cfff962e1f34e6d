"""Pins for the controller oracle (oracle/knowledge_tree.py): what the paper and the
arithmetic fix about the knowledge tree, PGDSF and the cost model (Sec. 5.1, Formulas 1-3,
Algorithm 1, "Swap out only once"; hit-rate example of Sec. 7.3)."""
import os
import random

import numpy as np
import pytest

from oracle import knowledge_tree as KT

HERE = os.path.dirname(os.path.abspath(__file__))

UNIT = ([0.0, 1.0e6], [1.0, 1.0e6 + 1.0])  # grid lines for synthetic cost models


def _grid(f, alphas, betas):
    return [[f(a, b) for b in betas] for a in alphas]


def _tree(gpu_blocks, host_slots, f=lambda a, b: 1.0 * b):
    return KT.KnowledgeTree(gpu_blocks, host_slots, UNIT[0], UNIT[1], _grid(f, *UNIT))


# ---------------------------------------------------------------- cost model
def test_bilinear_hand_worked_example():
    rows = {}
    for line in open(os.path.join(HERE, "golden", "bilinear_worked_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        rows[k] = [float(x) for x in v]
    T = [rows["T"][0:2], rows["T"][2:4]]
    got = KT.bilinear(rows["alphas"], rows["betas"], T, *rows["query"])
    assert got == rows["expect"][0]


def test_bilinear_is_exact_on_grid_points_and_on_bilinear_functions():
    alphas, betas = [0, 256, 1024, 4096], [16, 64, 100, 512, 2048]
    f = lambda a, b: 3.0 + 0.002 * a + 0.05 * b + 1.5e-5 * a * b
    T = _grid(f, alphas, betas)
    for i, a in enumerate(alphas):
        for j, b in enumerate(betas):
            assert KT.bilinear(alphas, betas, T, a, b) == pytest.approx(T[i][j], rel=1e-15)
    rng = random.Random(3)
    for _ in range(200):  # inside and outside the grid: a bilinear function is reproduced everywhere
        a, b = rng.uniform(-500, 6000), rng.uniform(1, 3000)
        assert KT.bilinear(alphas, betas, T, a, b) == pytest.approx(f(a, b), rel=1e-12)


def test_bilinear_reduces_to_linear_interpolation_along_a_grid_line():
    alphas, betas = [0.0, 100.0, 400.0, 900.0], [10.0, 20.0, 80.0]
    rng = np.random.default_rng(5)
    T = rng.uniform(1, 50, (4, 3))
    for a in (0.0, 33.0, 100.0, 250.0, 899.0):
        assert KT.bilinear(alphas, betas, T.tolist(), a, 20.0) == pytest.approx(np.interp(a, alphas, T[:, 1]), rel=1e-13)
    for b in (10.0, 15.0, 50.0, 80.0):
        assert KT.bilinear(alphas, betas, T.tolist(), 400.0, b) == pytest.approx(np.interp(b, betas, T[2]), rel=1e-13)


# ---------------------------------------------------------------- prefix matching
def test_hit_rate_example_of_the_ablation_study():
    """Stored [D1, D2], requested [D1, D3]: one of two retrieved documents hits (Sec. 7.3)."""
    t = _tree(64, 64)
    p = t.begin([1, 2], [32, 32], 10)
    t.end(p.request_id)
    t.docs_requested = t.docs_hit = 0
    p = t.begin([1, 3], [32, 32], 10)
    assert p.matched_docs == 1 and t.hit_rate() == 0.5


def test_matching_stops_at_the_first_missing_document_and_order_matters():
    t = _tree(64, 64)
    t.end(t.begin([1, 2, 3], [16, 16, 16], 4).request_id)
    assert t.begin([1, 3, 2], [16, 16, 16], 4).matched_docs == 1  # D3 is cached only behind [D1, D2]
    assert t.begin([2, 1], [16, 16], 4).matched_docs == 0
    assert t.begin([1, 2, 3], [16, 16, 16], 4).matched_docs == 3
    assert t.find([1, 3, 2]) is not None and t.find([1, 3, 2]) is not t.find([1, 2, 3])


def test_cached_prefix_is_counted_in_whole_blocks():
    t = _tree(64, 64)
    p = t.begin([7, 8], [40, 30], 9)  # 79 tokens: 5 blocks, docs cover 70 tokens = 4 whole blocks
    assert (p.matched_docs, p.alpha, p.beta, len(p.block_table)) == (0, 0, 79, 5)
    assert t.find([7]).n_owned == 2 and t.find([7, 8]).n_owned == 2  # tokens 0-39 | 40-69: blocks {0,1} | {2,3}
    t.end(p.request_id)
    q = t.begin([7, 9], [40, 20], 5)  # D7 matched: 40 tokens -> 32 cached, 8 recomputed with the request
    assert (q.matched_docs, q.alpha, q.beta) == (1, 32, 65 - 32)
    assert q.block_table[:2] == p.block_table[:2] and len(q.block_table) == 5
    assert not set(q.block_table[2:]) & set(p.block_table[:4])  # D8's blocks are still cached, not reused
    t.check_invariants()


# ---------------------------------------------------------------- PGDSF
def test_priority_is_clock_plus_avgcost_times_frequency():
    """Formula 1 with Cost/Size of Formula 3: one computing request, T = 3*beta -> AvgCost = 3."""
    t = _tree(64, 64, lambda a, b: 3.0 * b)
    for k in range(1, 4):
        p = t.begin([5], [32], 8)
        t.end(p.request_id)
        n = t.find([5])
        assert (n.Frequency, n.numComputed, n.AvgCost) == (k, 1, pytest.approx(3.0))
        assert n.Priority[KT.GPU] == pytest.approx(0.0 + 3.0 * k)


def test_cost_per_token_uses_the_requests_cached_and_noncached_sizes():
    f = lambda a, b: 2.0 + 0.001 * a + 0.01 * b + 1e-6 * a * b
    t = _tree(256, 64, f)
    t.end(t.begin([1], [160], 16).request_id)
    p = t.begin([1, 2], [160, 100], 20)  # alpha = 160, beta = 120
    assert (p.alpha, p.beta) == (160, 120)
    assert t.find([1, 2]).AvgCost == pytest.approx(f(160, 120) / 120, rel=1e-12)
    assert t.find([1]).AvgCost == pytest.approx(f(0, 176) / 176, rel=1e-12)  # unchanged by the cached access
    assert t.find([1]).Frequency == 2


def test_eviction_takes_the_lowest_priority_gpu_leaf_and_advances_the_clock():
    t = _tree(8, 64, lambda a, b: 1.0 * b)  # AvgCost = 1 for everything: priority = clock + frequency
    for d, times in ((1, 3), (2, 1), (3, 2)):
        for _ in range(times):
            t.end(t.begin([d], [32], 0).request_id)  # 2 blocks each, 6 of 8 used
    assert [t.find([d]).Priority[KT.GPU] for d in (1, 2, 3)] == [3.0, 1.0, 2.0]
    p = t.begin([4], [64], 0)  # needs 4 blocks, 2 free: evict D2 (priority 1)
    assert p.evicted_gpu == [t.find([2]).ident] and t.Clock[KT.GPU] == 1.0
    assert t.find([2]).where == KT.HOST and len(p.swap_out) == 2
    assert t.find([4]).Priority[KT.GPU] == 1.0 + 1.0  # set from the advanced clock (aging)
    t.end(p.request_id)
    p = t.begin([5], [96], 0)  # 6 blocks, 0 free: D3 and D4 both stand at 2 (the older node first), D1 at 3 stays
    assert p.evicted_gpu == [t.find([3]).ident, t.find([4]).ident] and t.find([1]).where == KT.GPU
    assert t.Clock[KT.GPU] == 2.0  # Formula 2: the largest priority among the evicted
    t.end(p.request_id)
    p = t.begin([6], [32], 0)  # D1 (3) against D5 (clock 2 + 1 = 3): a tie, the older node goes
    assert p.evicted_gpu == [t.find([1]).ident] and t.Clock[KT.GPU] == 3.0
    t.check_invariants()


def test_a_parent_becomes_a_candidate_only_after_its_last_gpu_child_left():
    t = _tree(6, 64, lambda a, b: 1.0 * b)
    t.end(t.begin([1, 2], [32, 32], 0).request_id)
    t.end(t.begin([1, 3], [32, 32], 0).request_id)  # D1 has two children, 6 blocks used
    for _ in range(5):
        t.end(t.begin([1, 3], [32, 32], 0).request_id)  # D1 and [D1,D3] hot, [D1,D2] cold
    t.end(t.begin([1], [32], 0).request_id)  # priorities now: D1 8, [D1,D2] 1, [D1,D3] 6
    n1, n2, n3 = t.find([1]), t.find([1, 2]), t.find([1, 3])
    p = t.begin([9], [64], 0)  # 4 blocks: [D1,D2] first, then [D1,D3]; D1 itself only if more were needed
    assert p.evicted_gpu == [n2.ident, n3.ident] and n1.where == KT.GPU
    t.end(p.request_id)
    p = t.begin([8], [32], 0)  # 2 more: D9 stands at clock 6 + 1 = 7, D1 (now a GPU leaf) at 8 -> D9 goes
    assert p.evicted_gpu == [t.find([9]).ident] and n1.where == KT.GPU
    t.check_invariants()


def test_nodes_of_requests_in_flight_are_not_evicted():
    t = _tree(4, 64)
    a = t.begin([1], [32], 0)
    with pytest.raises(KT.NoRoom):
        t.begin([2], [64], 0)  # would need D1's blocks
    t.check_invariants()
    t.end(a.request_id)
    assert t.begin([2], [64], 0).evicted_gpu == [t.find([1]).ident]


def test_a_document_still_being_computed_is_not_a_cached_prefix_for_a_second_request():
    """Two requests in flight that share a NEW document: the first one's node has its blocks reserved but
    nothing written, so the second must not attend over them.  It computes the document for itself in
    blocks of its own, the node counts two computations, and once the first request has ended a third
    request finds the document cached.  Costs by hand: T = 2*beta, so a request that computes b tokens
    charges 2*b / b = 2 per token each time."""
    t = _tree(64, 64, lambda a, b: 2.0 * b)
    free0 = len(t.free_dev)
    a = t.begin([7, 8], [40, 24], 8)          # creates nodes [7] and [7, 8]: 72 tokens, 4 owned + 1 private block
    assert (a.matched_docs, a.alpha, a.beta) == (0, 0, 72)
    assert not t.find([7]).computed and t.peek([7], [40], 8) == (0, 48)
    b = t.begin([7, 9], [40, 16], 8)          # [7] exists but is in flight: nothing is cached for b
    assert (b.matched_docs, b.alpha, b.beta) == (0, 0, 64)
    assert not set(a.block_table) & set(b.block_table) and len(b.block_table) == 4
    assert t.find([7, 9]) is None             # b adds nothing below the node it had to wait for
    n7 = t.find([7])
    assert (n7.Frequency, n7.numComputed, n7.pins) == (2, 2, 1) and n7.AvgCost == pytest.approx(2.0)
    assert t.find([7, 8]).numComputed == 1    # b does not go through [7, 8]
    t.check_invariants()
    t.end(b.request_id)
    assert len(t.free_dev) == free0 - 5       # all of b's blocks are back; a still holds its five
    assert not t.find([7]).computed
    t.end(a.request_id)
    assert t.find([7]).computed and t.find([7, 8]).computed
    c = t.begin([7, 9], [40, 16], 8)          # now [7] serves as prefix: alpha = 32 (whole blocks of 40 tokens)
    assert (c.matched_docs, c.alpha, c.beta) == (1, 32, 32)
    assert c.block_table[:2] == a.block_table[:2]
    assert t.find([7]).numComputed == 2 and t.find([7]).Frequency == 3
    assert t.find([7, 9]).numComputed == 1 and not t.find([7, 9]).computed
    t.check_invariants()


def test_a_chain_in_flight_blocks_every_document_below_it_and_charges_each_node_once():
    t = _tree(64, 64, lambda a, b: 1.0 * b)
    a = t.begin([1, 2, 3], [16, 16, 16], 4)
    b = t.begin([1, 2, 4], [16, 16, 16], 4)   # [1] and [1, 2] are in flight, [1, 2, 4] does not exist
    assert (b.matched_docs, b.alpha) == (0, 0) and t.find([1, 2, 4]) is None
    assert [t.find(p).numComputed for p in ([1], [1, 2], [1, 2, 3])] == [2, 2, 1]
    t.end(a.request_id)
    t.end(b.request_id)
    c = t.begin([1, 2, 4], [16, 16, 16], 4)
    assert (c.matched_docs, c.alpha, c.beta) == (2, 32, 20)
    t.check_invariants()


def test_cheaper_and_rarer_documents_go_first():
    f = lambda a, b: 1.0 * b + 0.01 * a * b  # per-token cost grows with the cached prefix in front
    t = _tree(10, 64, f)
    t.end(t.begin([1], [32], 0).request_id)          # AvgCost 1
    t.end(t.begin([1, 2], [32, 32], 0).request_id)   # AvgCost 1 + 0.32, deeper prefix -> dearer
    t.end(t.begin([3], [32], 0).request_id)          # AvgCost 1
    t.end(t.begin([3], [32], 0).request_id)          # frequency 2
    t.end(t.begin([4], [32], 0).request_id)          # AvgCost 1, frequency 1
    p = t.begin([5], [96], 0)  # 8 used of 10, 6 needed: leaves are [1,2] (1.32), 3 (2.0), 4 (1.0) -> 4, then [1,2]
    assert p.evicted_gpu == [t.find([4]).ident, t.find([1, 2]).ident]


# ---------------------------------------------------------------- host tier
def test_swap_out_only_once():
    t = _tree(4, 64)
    t.end(t.begin([1], [64], 0).request_id)
    p = t.begin([2], [64], 0)
    assert len(p.swap_out) == 4 and t.blocks_swapped_out == 4  # first eviction copies
    t.end(p.request_id)
    p = t.begin([1], [64], 0)  # D1 comes back from the host: swap-in, and D2 is copied out (its first time)
    assert p.matched_docs == 1 and len(p.swap_in) == 4 and len(p.swap_out) == 4 and p.beta == 0
    assert [s for _, s in p.swap_in] == t.find([1]).host_slots
    t.end(p.request_id)
    p = t.begin([2], [64], 0)  # D2 back in, D1 evicted a second time: nothing is copied out
    assert len(p.swap_in) == 4 and p.swap_out == [] and t.zero_copy_evictions == 1
    assert t.blocks_swapped_out == 8 and t.find([1]).where == KT.HOST and t.find([1]).host_valid
    t.check_invariants()


def test_host_tier_drops_its_own_lowest_priority_leaves_and_keeps_the_hierarchy():
    t = _tree(4, 6)  # host holds one 4-block document and a half
    for d in (1, 2, 3):
        t.end(t.begin([d], [64], 0).request_id)  # each arrival pushes the previous one to the host
    # D1 went to the host first, then D2 needed 4 slots with 2 free: D1 (a host leaf) left the cache
    assert t.find([1]) is None and t.find([2]).where == KT.HOST and t.find([3]).where == KT.GPU
    assert t.Clock[KT.HOST] == 1.0
    t.check_invariants()


def test_a_document_that_cannot_be_copied_out_leaves_the_cache_with_its_subtree():
    t = _tree(6, 2)
    t.end(t.begin([1, 2], [32, 32], 0).request_id)
    t.end(t.begin([3], [32], 0).request_id)  # 6 blocks used, host has 2 slots
    p = t.begin([4], [64], 0)  # needs 4: [1,2] -> host (2 slots), then 3 or 1: no slot left and no host leaf but [1,2]
    assert t.find([4]) is not None
    t.check_invariants()
    assert len(p.evicted_gpu) == 2


def test_without_host_room_an_evicted_document_is_simply_freed():
    t = _tree(4, 0)
    t.end(t.begin([1], [64], 0).request_id)
    p = t.begin([2], [64], 0)
    assert p.swap_out == [] and p.evicted_host == [1] and t.find([1]) is None and t.find([2]) is not None
    t.check_invariants()


def test_a_copy_is_struck_from_the_list_when_its_node_leaves_the_cache_in_the_same_request():
    t = _tree(4, 2)
    t.end(t.begin([1], [32], 0).request_id)
    t.end(t.begin([2], [32], 0).request_id)
    b_blocks = list(t.find([2]).dev_blocks)
    p = t.begin([3], [64], 0)  # D1 goes to the host (2 slots), then D2 needs them: D1 leaves the cache
    assert p.evicted_gpu == [1, 2] and p.evicted_host == [1] and t.find([1]) is None
    assert [d for d, _ in p.swap_out] == b_blocks and sorted(s for _, s in p.swap_out) == [0, 1]
    assert t.blocks_swapped_out == 2
    t.check_invariants()


def test_random_trace_keeps_every_invariant():
    rng = random.Random(11)
    t = _tree(40, 60, lambda a, b: 5.0 + 0.01 * b + 1e-5 * a * b)
    lens = {d: rng.randrange(5, 90) for d in range(30)}
    live = []
    for step in range(600):
        if live and (len(live) >= 3 or rng.random() < 0.4):
            t.end(live.pop(rng.randrange(len(live))))
        k = rng.randrange(1, 4)
        docs = [min(int(rng.paretovariate(1.1)) - 1, 29) for _ in range(k)]
        docs = list(dict.fromkeys(docs))
        try:
            p = t.begin(docs, [lens[d] for d in docs], rng.randrange(1, 40))
        except KT.NoRoom:
            t.check_invariants()
            continue
        total = sum(lens[d] for d in docs)
        assert p.alpha % 16 == 0 and p.alpha <= total and len(set(p.block_table)) == len(p.block_table)
        live.append(p.request_id)
        t.check_invariants()
    assert t.zero_copy_evictions > 0 and t.blocks_swapped_in > 0 and 0.0 < t.hit_rate() < 1.0


# ---------------------------------------------------------------- cache-aware reordering (Sec. 5.2)
def _serve(t, q):
    order, hits = [], 0
    while q.waiting:
        tag, ids, lens, ql = q.pop(t)
        p = t.begin(ids, lens, ql)
        hits += p.matched_docs
        t.end(p.request_id)
        order.append(tag)
    return order, hits


def test_reordering_example_of_the_paper():
    """Requests alternate between D1 and D2, the cache holds one document: in arrival order nothing
    hits; by OrderPriority the order is Q1 Q3 Q5 Q2 Q4 Q6 and 4 of 6 hit (the paper's 66 %)."""
    def six(window):
        t = _tree(4, 0)  # one 64-token document
        q = KT.ReorderQueue(window)
        for i in range(1, 7):
            q.push(i, [1 if i % 2 else 2], [64], 0)
        return _serve(t, q)

    assert six(window=100) == ([1, 3, 5, 2, 4, 6], 4)
    assert six(window=0) == ([1, 2, 3, 4, 5, 6], 0)  # no reordering allowed: arrival order, zero hits


def test_larger_cached_part_and_shorter_computation_go_first():
    t = _tree(64, 64)
    t.end(t.begin([1], [32], 0).request_id)
    t.end(t.begin([2], [64], 0).request_id)
    q = KT.ReorderQueue(100)
    q.push(10, [1], [32], 32)   # cached 32, compute 32 -> 1
    q.push(11, [2], [64], 32)   # cached 64, compute 32 -> 2: same computation, more cached
    q.push(12, [2], [64], 16)   # cached 64, compute 16 -> 4: same cached, less computation
    q.push(13, [3], [64], 16)   # nothing cached -> 0
    assert [q.pop(t)[0] for _ in range(4)] == [12, 11, 10, 13]


def test_starvation_window_bounds_how_often_a_request_is_passed_over():
    t = _tree(64, 64)
    t.end(t.begin([1], [64], 0).request_id)
    q = KT.ReorderQueue(2)
    q.push(1, [9], [64], 8)  # never cached: always the lowest priority
    for i in range(2, 7):
        q.push(i, [1], [64], 8)
    assert [q.pop(t)[0] for _ in range(6)] == [2, 3, 1, 4, 5, 6]  # passed over twice, then served
