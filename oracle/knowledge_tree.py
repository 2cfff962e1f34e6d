"""Oracle for the RAG controller's cache bookkeeping: knowledge tree, prefix matching,
PGDSF replacement over a GPU tier and a host tier, swap-out-only-once, and the cost model
T(alpha, beta) by bilinear interpolation (paper Sec. 5.1: knowledge tree, Formulas 1-3,
Algorithm 1, "Swap out only once").  Test infrastructure only: plain Python objects, lists
and dicts, linear scans instead of heaps, the paper's names (Frequency, TotalCost,
numComputed, AvgCost, Priority, Clock).  It shares no code with the C++ controller.

What the paper leaves open, and the reading taken here (the C++ side documents the same):

* Unit of storage.  K/V lives in 16-token blocks addressed flatly over a request's logical
  sequence (position j -> table[j // 16], slot j % 16).  A node (one document at one place in
  a path) covers tokens [tok_begin, tok_end) of its path and OWNS the blocks whose last token
  falls in that range: floor(tok_end/16) - floor(tok_begin/16) blocks.  The cached prefix of a
  request is therefore a multiple of 16: alpha = 16 * floor(tok_end of the last matched node
  / 16); up to 15 tail tokens of the matched path are recomputed with the request.
* Size in Formula 1 is the document's token count; capacity is counted in blocks.
* Two clocks, one per tier (Sec. 5.1).  A node carries one priority per tier, both set on
  every retrieval from that tier's clock: Priority = Clock + AvgCost * Frequency.
* EVICT_IN_GPU works on the GPU leaves (nodes in GPU memory none of whose children is in GPU
  memory); nodes of requests in flight are not candidates.  Ties in priority go to the node
  created first.  The host tier is handled the same way over the leaves of the whole tree
  that live in host memory only; a node evicted there leaves the cache.
* Swap out only once: a node's blocks are copied to host slots at its first GPU eviction and
  the host copy is kept while the node is in the tree; later GPU evictions copy nothing.  If
  the host tier cannot make room for a first copy, the node and everything below it leave the
  cache.  A first copy that a request asked for is struck from its list again when, later in
  the same request, the host tier drops that node (its slot may already be promised to another).
* Requests in flight together.  A node created by a request that has not ended yet has its
  blocks reserved but its K/V not written; it cannot serve another request as cached prefix
  (the paper batches several requests per prefill iteration, Sec. 7, and says nothing about
  this).  Prefix matching therefore stops at such a node; the second request computes that
  document and everything after it for itself in blocks of its own, adds nothing to the tree
  below that point, and counts as one more computation of the nodes that exist (numComputed).
* Block ids come from a LIFO free list that starts as 0, 1, 2, ... (so results are
  reproducible); this order is part of what the C++ side is compared on.
* Outside the profiled grid T is extrapolated linearly from the two nearest grid lines of
  each axis (the paper's formula with the outermost cell), never clamped.
"""
from __future__ import annotations

from bisect import bisect_right
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

BLOCK = 16
GPU, HOST = 0, 1


# ----------------------------------------------------------------------------- cost model
def bilinear(alphas: Sequence[float], betas: Sequence[float], T: Sequence[Sequence[float]], alpha: float,
             beta: float) -> float:
    """T(alpha, beta) from the profiled grid T[i][j] = T(alphas[i], betas[j]) (Algorithm 1, the
    three interpolation steps): find the enclosing grid lines, interpolate along alpha on the
    low and the high beta line, then along beta."""

    def cell(axis: Sequence[float], x: float) -> int:
        # index l of the lower grid line; the outermost cells also serve points outside the grid
        l = bisect_right(list(axis), x) - 1
        return min(max(l, 0), len(axis) - 2)

    i, j = cell(alphas, alpha), cell(betas, beta)
    al, ah, bl, bh = alphas[i], alphas[i + 1], betas[j], betas[j + 1]
    t_l = T[i][j] + (alpha - al) / (ah - al) * (T[i + 1][j] - T[i][j])
    t_h = T[i][j + 1] + (alpha - al) / (ah - al) * (T[i + 1][j + 1] - T[i][j + 1])
    return t_l + (beta - bl) / (bh - bl) * (t_h - t_l)


# ----------------------------------------------------------------------------- tree
@dataclass
class Node:
    ident: int
    doc: int
    length: int
    tok_begin: int
    parent: Optional["Node"]
    children: Dict[int, "Node"] = field(default_factory=dict)
    where: int = GPU
    host_valid: bool = False
    dev_blocks: List[int] = field(default_factory=list)
    host_slots: List[int] = field(default_factory=list)
    Frequency: int = 0
    TotalCost: float = 0.0
    numComputed: int = 0
    AvgCost: float = 0.0
    Priority: List[float] = field(default_factory=lambda: [0.0, 0.0])  # per tier
    pins: int = 0
    computed: bool = False  # its K/V has been written: set when the request that created the node ends

    @property
    def tok_end(self) -> int:
        return self.tok_begin + self.length

    @property
    def n_owned(self) -> int:
        return self.tok_end // BLOCK - self.tok_begin // BLOCK


@dataclass
class Plan:
    request_id: int
    matched_docs: int
    alpha: int
    beta: int
    block_table: List[int]
    swap_out: List[Tuple[int, int]]  # (device block, host slot), to run before anything else
    swap_in: List[Tuple[int, int]]   # (device block, host slot), after the swap-outs
    evicted_gpu: List[int]           # node idents in eviction order
    evicted_host: List[int]          # node idents that left the cache, in order


class NoRoom(Exception):
    pass


class KnowledgeTree:
    def __init__(self, gpu_blocks: int, host_slots: int, alphas, betas, T):
        self.alphas, self.betas, self.T = list(alphas), list(betas), [list(r) for r in T]
        self.free_dev = list(range(gpu_blocks - 1, -1, -1))    # pop() gives 0, 1, 2, ...
        self.free_host = list(range(host_slots - 1, -1, -1))
        self.Clock = [0.0, 0.0]
        self.root = Node(0, -1, 0, 0, None)
        self.root.pins = 1  # never a candidate
        self.root.computed = True
        self.next_ident = 1
        self.next_request = 1
        self.requests: Dict[int, Tuple[List[Node], List[int]]] = {}
        self.docs_requested = 0
        self.docs_hit = 0
        self.blocks_swapped_out = 0
        self.blocks_swapped_in = 0
        self.zero_copy_evictions = 0

    # ---- helpers
    def _all_nodes(self) -> List[Node]:
        out, stack = [], [self.root]
        while stack:
            n = stack.pop()
            out.append(n)
            stack.extend(n.children.values())
        return out

    def _gpu_leaves(self) -> List[Node]:
        return [n for n in self._all_nodes()
                if n is not self.root and n.where == GPU and n.pins == 0
                and not any(c.where == GPU for c in n.children.values())]

    def _host_leaves(self) -> List[Node]:
        return [n for n in self._all_nodes()
                if n is not self.root and n.where == HOST and n.pins == 0 and not n.children]

    def _remove_subtree(self, n: Node, plan: Plan) -> None:
        for c in list(n.children.values()):
            self._remove_subtree(c, plan)
        assert n.pins == 0
        if n.where == GPU:
            self.free_dev.extend(n.dev_blocks)
        if n.host_valid:
            # a copy to the host that this same request asked for a moment ago is void now
            mine = set(n.host_slots)
            kept = [(d, s) for d, s in plan.swap_out if s not in mine]
            self.blocks_swapped_out -= len(plan.swap_out) - len(kept)
            plan.swap_out[:] = kept
            self.free_host.extend(n.host_slots)
        del n.parent.children[n.doc]
        plan.evicted_host.append(n.ident)

    # ---- Algorithm 1, UPDATE_NODE_IN_GPU (both tiers' priorities are refreshed, see the header)
    def _update_node(self, node: Node, is_cached: bool, alpha: int, beta: int) -> None:
        node.Frequency += 1
        if not is_cached:
            t = bilinear(self.alphas, self.betas, self.T, alpha, beta)
            node.TotalCost += t / beta
            node.numComputed += 1
            node.AvgCost = node.TotalCost / node.numComputed
        for tier in (GPU, HOST):
            node.Priority[tier] = self.Clock[tier] + node.AvgCost * node.Frequency

    def _freeable(self, n: Node) -> Tuple[bool, int]:
        """(can n itself be evicted from the GPU eventually, blocks that evictions below and at n can free):
        a node can go once every child in GPU memory has gone, and nodes of requests in flight stay."""
        ok = n.where == GPU and n.pins == 0
        blocks = 0
        for c in n.children.values():
            if c.where == GPU:
                c_ok, c_blocks = self._freeable(c)
                blocks += c_blocks
                ok = ok and c_ok
        if ok:
            blocks += n.n_owned
        return ok, blocks

    # ---- host tier: make `required` slots free by dropping host-only leaves
    def _evict_in_host(self, required: int, plan: Plan) -> bool:
        while len(self.free_host) < required:
            S = self._host_leaves()
            if not S:
                return False
            n = min(S, key=lambda x: (x.Priority[HOST], x.ident))
            self.Clock[HOST] = max(self.Clock[HOST], n.Priority[HOST])
            self._remove_subtree(n, plan)
        return True

    # ---- Algorithm 1, EVICT_IN_GPU, with the swap-out-only-once bookkeeping
    def _evict_in_gpu(self, required_size: int, plan: Plan) -> None:
        freed = 0
        while freed < required_size:
            S = self._gpu_leaves()
            assert S, "begin() has checked that enough can be freed"
            n = min(S, key=lambda x: (x.Priority[GPU], x.ident))
            self.Clock[GPU] = max(self.Clock[GPU], n.Priority[GPU])
            plan.evicted_gpu.append(n.ident)
            freed += n.n_owned
            if n.host_valid:
                self.zero_copy_evictions += 1
            elif n.n_owned == 0:
                n.host_valid = True  # nothing to copy
            elif self._evict_in_host(n.n_owned, plan):
                n.host_slots = [self.free_host.pop() for _ in range(n.n_owned)]
                plan.swap_out.extend(zip(n.dev_blocks, n.host_slots))
                self.blocks_swapped_out += n.n_owned
                n.host_valid = True
            else:
                self._remove_subtree(n, plan)  # frees its device blocks as well
                continue
            self.free_dev.extend(n.dev_blocks)
            n.dev_blocks = []
            n.where = HOST

    # ---- a request arrives with its retrieved documents, in order
    def begin(self, doc_ids: Sequence[int], doc_lens: Sequence[int], question_len: int) -> Plan:
        docs_total = sum(doc_lens)
        total = docs_total + question_len
        plan = Plan(self.next_request, 0, 0, 0, [], [], [], [], [])
        # prefix matching: stop at the first document that is not a child -- or whose node belongs to a
        # request still in flight: its blocks are reserved but its K/V is not written yet, so it cannot
        # serve as a cached prefix
        path: List[Node] = []
        cur = self.root
        for d, l in zip(doc_ids, doc_lens):
            nxt = cur.children.get(d)
            if nxt is None or not nxt.computed:
                break
            assert nxt.length == l, "a document id has one length"
            path.append(nxt)
            cur = nxt
        m = len(path)
        # The next document has a node that is being computed elsewhere: this request computes the
        # document for itself in blocks of its own and adds nothing to the tree below that point.
        in_progress: List[Node] = []
        nxt = cur
        for d, l in zip(doc_ids[m:], doc_lens[m:]):
            nxt = nxt.children.get(d)
            if nxt is None:
                break
            assert nxt.length == l, "a document id has one length"
            in_progress.append(nxt)
        blocked = bool(in_progress)
        for n in path:
            n.pins += 1
        matched_end = path[-1].tok_end if path else 0
        alpha = matched_end // BLOCK * BLOCK
        beta = total - alpha
        blocks_total = (total + BLOCK - 1) // BLOCK
        cacheable = alpha // BLOCK if blocked else docs_total // BLOCK
        to_swap_in = [n for n in path if n.where == HOST]
        need = sum(n.n_owned for n in to_swap_in) + (blocks_total - alpha // BLOCK)
        if need > len(self.free_dev) + self._freeable(self.root)[1]:
            for n in path:
                n.pins -= 1
            raise NoRoom()  # nothing has been changed
        if need > len(self.free_dev):
            self._evict_in_gpu(need - len(self.free_dev), plan)
        # swap-in of matched nodes that live in host memory (their host copy stays valid)
        for n in to_swap_in:
            n.dev_blocks = [self.free_dev.pop() for _ in range(n.n_owned)]
            plan.swap_in.extend(zip(n.dev_blocks, n.host_slots))
            self.blocks_swapped_in += n.n_owned
            n.where = GPU
        # new nodes for the documents that were not matched
        new_nodes: List[Node] = []
        tok = matched_end
        for d, l in (() if blocked else zip(doc_ids[m:], doc_lens[m:])):
            n = Node(self.next_ident, d, l, tok, cur)
            self.next_ident += 1
            n.dev_blocks = [self.free_dev.pop() for _ in range(n.n_owned)]
            n.pins = 1
            cur.children[d] = n
            new_nodes.append(n)
            cur = n
            tok += l
        private = [self.free_dev.pop() for _ in range(blocks_total - cacheable)]
        for n in path + new_nodes:
            plan.block_table.extend(n.dev_blocks)
        plan.block_table.extend(private)
        assert len(plan.block_table) == blocks_total
        # retrieval updates every document's node
        for n in path:
            self._update_node(n, True, alpha, beta)
        for n in new_nodes + in_progress:  # the documents this request computes (Algorithm 1: is_cached false)
            self._update_node(n, False, alpha, beta)
        self.docs_requested += len(doc_ids)
        self.docs_hit += m
        plan.matched_docs, plan.alpha, plan.beta = m, alpha, beta
        self.requests[plan.request_id] = (path + new_nodes, private, new_nodes)
        self.next_request += 1
        return plan

    def peek(self, doc_ids: Sequence[int], doc_lens: Sequence[int], question_len: int) -> Tuple[int, int]:
        """(cached length alpha, computation length beta) the request would get now; nothing changes."""
        cur, matched_end = self.root, 0
        for d in doc_ids:
            cur = cur.children.get(d)
            if cur is None or not cur.computed:
                break
            matched_end = cur.tok_end
        alpha = matched_end // BLOCK * BLOCK
        return alpha, sum(doc_lens) + question_len - alpha

    def end(self, request_id: int) -> None:
        nodes, private, created = self.requests.pop(request_id)
        for n in nodes:
            n.pins -= 1
        for n in created:
            n.computed = True  # the request has run: the K/V of its new documents is in their blocks
        self.free_dev.extend(private)

    def reset_frequencies(self) -> None:
        """Frequency counts retrievals within a time window (Sec. 5.1): start a new window."""
        for n in self._all_nodes():
            n.Frequency = 0

    # ---- views for tests
    def find(self, doc_path: Sequence[int]) -> Optional[Node]:
        cur = self.root
        for d in doc_path:
            cur = cur.children.get(d)
            if cur is None:
                return None
        return cur

    def hit_rate(self) -> float:
        return self.docs_hit / self.docs_requested if self.docs_requested else 0.0

    def check_invariants(self) -> None:
        used_dev, used_host = [], []
        for n in self._all_nodes():
            if n is self.root:
                continue
            if n.where == GPU:
                # GPU nodes are parents of host nodes, never the other way round
                assert n.parent is self.root or n.parent.where == GPU
                assert len(n.dev_blocks) == n.n_owned
                used_dev += n.dev_blocks
            else:
                assert n.host_valid and not n.dev_blocks
            if n.host_valid:
                assert len(n.host_slots) == n.n_owned
                used_host += n.host_slots
            assert n.tok_begin == (0 if n.parent is self.root else n.parent.tok_end)
            assert n.parent is self.root or n.parent.computed or not n.computed  # K/V of a path is written parent first
        for _, private, _created in self.requests.values():
            used_dev += private
        assert len(set(used_dev)) == len(used_dev) and not set(used_dev) & set(self.free_dev)
        assert len(set(used_host)) == len(used_host) and not set(used_host) & set(self.free_host)


# ----------------------------------------------------------------------------- cache-aware reordering
class ReorderQueue:
    """Waiting requests, served by OrderPriority = cached length / computation length against the
    tree as it is at the moment of the choice (paper Sec. 5.2); equal priorities go to the request
    that arrived first.  Starvation window: a request that has seen `window` later arrivals served
    before it is served next, oldest first.  (The paper gives the priority and the existence of a
    window; how the window counts is this reading.)"""

    def __init__(self, window: int):
        self.window = window
        self.waiting: List[list] = []  # [tag, doc_ids, doc_lens, question_len, times passed over]

    def push(self, tag: int, doc_ids: Sequence[int], doc_lens: Sequence[int], question_len: int) -> None:
        self.waiting.append([tag, list(doc_ids), list(doc_lens), question_len, 0])

    def pop(self, tree: KnowledgeTree):
        """The next request to serve: (tag, doc_ids, doc_lens, question_len)."""
        assert self.waiting
        starved = [i for i, w in enumerate(self.waiting) if w[4] >= self.window]
        if starved:
            pick = starved[0]
        else:
            best = None
            for i, w in enumerate(self.waiting):
                alpha, beta = tree.peek(w[1], w[2], w[3])
                prio = alpha / beta if beta > 0 else float("inf")
                if best is None or prio > best:
                    best, pick = prio, i
        for w in self.waiting[:pick]:
            w[4] += 1  # served before a request that arrived earlier
        tag, ids, lens, q, _ = self.waiting.pop(pick)
        return tag, ids, lens, q
