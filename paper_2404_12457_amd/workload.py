"""Seeded synthetic RAG-shaped inputs for the prefix-cached prefill path.

This module only *draws and places* data: random Q/K/V values, document
sequences, block ids, residency.  It holds none of the method's arithmetic
(no scores, no softmax, no attention) and imports neither the HIP binding nor
the CPU oracle.  Both sides are fed from here:

  * the oracle sees the *logical* tensors (`prefix_kv`, `k_new`, `v_new`, `q`);
  * the HIP path sees the *paged* image (`used_block_ids`/`used_k`/`used_v`
    scattered into a pool, plus `block_table`, `prefix_len`, `new_len`).

Shapes follow the paper's workloads: a request is an ordered sequence of
retrieved documents whose K/V is cached (Sec. 4 "Cache retriever", Sec. 5.1
knowledge tree) followed by non-cached tokens (uncached documents first, the
question last, Sec. 5.1 cost estimation); head shapes are those of
Table "Models used in the evaluation"; document popularity is skewed
(Sec. 3.2, retrieval pattern) and is drawn here from a Zipf law.  The items of
the paper's datasets are not reproduced: every value is a seeded draw.

Values are rounded to the storage dtype (bf16 or fp32) exactly once, here, so
both sides start from identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BLOCK = 16  # tokens per paged KV block
BASE_SEED = 24041245700

# stream tags for the counter-based generator (one stream per tensor kind)
_T_Q, _T_KNEW, _T_VNEW, _T_NODE_K, _T_NODE_V, _T_PERM, _T_SHAPE, _T_HOST, _T_DOCLEN = range(9)


# ----------------------------------------------------------------------------
# storage-dtype helpers (bit manipulation only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(u: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(u, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Storage array (uint16 bf16 bits or float32) -> float64 values."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def storage_np_dtype(dtype: str):
    return np.uint16 if dtype == "bf16" else np.float32


def poison_value(dtype: str):
    """Bit pattern written to every pool slot that holds no valid token (NaN)."""
    if dtype == "bf16":
        return np.uint16(0x7FC0)
    return np.float32(np.nan)


def _gen(seed: int, tag: int, idx: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), ((tag & 0xFFFF) << 48) | (idx & (2**48 - 1))]))


def _path_hash(path: Sequence[int]) -> int:
    h = 0xCBF29CE484222325
    for d in path:
        for b in int(d).to_bytes(8, "little", signed=False):
            h = ((h ^ b) * 0x100000001B3) & (2**64 - 1)
    return h & (2**48 - 1)


def _draw(seed: int, tag: int, idx: int, shape, sigma: float, dtype: str) -> np.ndarray:
    x = _gen(seed, tag, idx).standard_normal(shape, dtype=np.float32) * np.float32(sigma)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    return x.astype(np.float32)


# ----------------------------------------------------------------------------
# request description
# ----------------------------------------------------------------------------
@dataclass
class RequestSpec:
    """One augmented request: cached documents (id, tokens) in retrieval order,
    then `n_uncached` tokens of documents that missed the cache, then
    `n_question` question tokens.  new_len = n_uncached + n_question."""
    docs: List[Tuple[int, int]]
    n_question: int
    n_uncached: int = 0

    @property
    def prefix_len(self) -> int:
        return int(sum(l for _, l in self.docs))

    @property
    def new_len(self) -> int:
        return int(self.n_question + self.n_uncached)


@dataclass
class Workload:
    name: str
    dtype: str  # "bf16" | "f32"
    q_heads: int
    kv_heads: int
    head_dim: int
    num_blocks: int
    seed: int
    sigma: float
    requests: List[RequestSpec]
    # per-request metadata
    prefix_len: np.ndarray = None  # int32 [R]
    new_len: np.ndarray = None  # int32 [R]
    new_start: np.ndarray = None  # int32 [R+1]
    block_table: np.ndarray = None  # int32 [R, table_stride]
    table_stride: int = 0
    poison_block: int = 0
    # logical tensors (storage dtype)
    q: np.ndarray = None  # [sumN, Hq, D]
    k_new: np.ndarray = None  # [sumN, Hkv, D]
    v_new: np.ndarray = None
    # paged image of the cached prefix: distinct blocks and their contents
    used_block_ids: np.ndarray = None  # int32 [U]
    used_k: np.ndarray = None  # [U, Hkv, 16, D]
    used_v: np.ndarray = None
    # host tier (only when some blocks are host-resident)
    host_dev_blocks: np.ndarray = None  # int32 [S] device block ids to fill
    host_slots: np.ndarray = None  # int32 [S] slot of each in the host pool
    num_host_slots: int = 0
    needs_swap: np.ndarray = None  # bool [R]: request reads a host-resident block
    _node_kv: Dict[Tuple[int, ...], Tuple[np.ndarray, np.ndarray]] = field(default_factory=dict, repr=False)

    # ---- sizes -------------------------------------------------------------
    @property
    def num_reqs(self) -> int:
        return len(self.requests)

    @property
    def total_new(self) -> int:
        return int(self.new_start[-1])

    @property
    def esize(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def softmax_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))

    def attn_flops(self) -> int:
        """2 GEMMs x 2 flop per visible (query, key) pair and head-dim element."""
        p = self.prefix_len.astype(np.int64)
        n = self.new_len.astype(np.int64)
        return int(4 * self.head_dim * self.q_heads * np.sum(n * p + n * (n + 1) // 2))

    def attn_min_bytes(self) -> int:
        """Each K/V element of the distinct cached blocks a batch reads once, fresh K/V once,
        Q and O once, one table entry per 16 tokens."""
        row = self.kv_heads * self.head_dim * self.esize
        kv = 2 * row * (int(self.used_block_ids.size) * BLOCK + self.total_new)
        qo = 2 * self.q_heads * self.head_dim * self.esize * self.total_new
        tbl = 4 * int(np.sum((self.prefix_len.astype(np.int64) + self.new_len + BLOCK - 1) // BLOCK))
        return int(kv + qo + tbl)

    def append_bytes(self) -> int:
        return int(2 * 2 * self.kv_heads * self.head_dim * self.esize * self.total_new)

    # ---- logical views -------------------------------------------------------
    def prefix_kv(self, r: int) -> Tuple[np.ndarray, np.ndarray]:
        """Cached prefix of request r as contiguous [P, Hkv, D] storage arrays."""
        ks, vs, path = [], [], []
        for doc, _ in self.requests[r].docs:
            path.append(doc)
            k, v = self._node_kv[tuple(path)]
            ks.append(k)
            vs.append(v)
        shape = (0, self.kv_heads, self.head_dim)
        if not ks:
            z = np.zeros(shape, dtype=storage_np_dtype(self.dtype))
            return z, z.copy()
        return np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)

    def new_slice(self, r: int) -> slice:
        return slice(int(self.new_start[r]), int(self.new_start[r + 1]))

    def full_kv(self, r: int) -> Tuple[np.ndarray, np.ndarray]:
        """[P+N, Hkv, D]: cached prefix followed by the request's fresh K/V."""
        kp, vp = self.prefix_kv(r)
        s = self.new_slice(r)
        return np.concatenate([kp, self.k_new[s]], axis=0), np.concatenate([vp, self.v_new[s]], axis=0)

    # ---- paged views ---------------------------------------------------------
    def pool_shape(self) -> Tuple[int, int, int, int]:
        return (self.num_blocks, self.kv_heads, BLOCK, self.head_dim)

    def pool_image(self) -> Tuple[np.ndarray, np.ndarray]:
        """Whole pool before the call: cached blocks in place, everything else poison."""
        dt = storage_np_dtype(self.dtype)
        k = np.full(self.pool_shape(), poison_value(self.dtype), dtype=dt)
        v = np.full(self.pool_shape(), poison_value(self.dtype), dtype=dt)
        if self.used_block_ids.size:
            k[self.used_block_ids] = self.used_k
            v[self.used_block_ids] = self.used_v
        return k, v

    def appended_blocks(self) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """Blocks that receive fresh tokens and their expected contents after the
        append: (ids [A], k [A,Hkv,16,D], v [...]).  Slots past P+N stay poison."""
        dt = storage_np_dtype(self.dtype)
        where = {int(b): i for i, b in enumerate(self.used_block_ids)}
        ids: List[int] = []
        imgs_k, imgs_v = [], []
        index: Dict[int, int] = {}
        for r in range(self.num_reqs):
            p, n = int(self.prefix_len[r]), int(self.new_len[r])
            s0 = int(self.new_start[r])
            for i in range(n):
                pos = p + i
                blk = int(self.block_table[r, pos // BLOCK])
                if blk not in index:
                    index[blk] = len(ids)
                    ids.append(blk)
                    if blk in where:
                        imgs_k.append(self.used_k[where[blk]].copy())
                        imgs_v.append(self.used_v[where[blk]].copy())
                    else:
                        shp = (self.kv_heads, BLOCK, self.head_dim)
                        imgs_k.append(np.full(shp, poison_value(self.dtype), dtype=dt))
                        imgs_v.append(np.full(shp, poison_value(self.dtype), dtype=dt))
                j = index[blk]
                imgs_k[j][:, pos % BLOCK, :] = self.k_new[s0 + i]
                imgs_v[j][:, pos % BLOCK, :] = self.v_new[s0 + i]
        shp = (0, self.kv_heads, BLOCK, self.head_dim)
        if not ids:
            return np.zeros(0, np.int32), np.zeros(shp, dt), np.zeros(shp, dt)
        return np.asarray(ids, np.int32), np.stack(imgs_k), np.stack(imgs_v)


# ----------------------------------------------------------------------------
# builder
# ----------------------------------------------------------------------------
def build_workload(
    name: str,
    dtype: str,
    q_heads: int,
    kv_heads: int,
    head_dim: int,
    num_blocks: int,
    requests: List[RequestSpec],
    seed: int,
    sigma: float = 1.0,
    q_gain: float = 1.0,
    host_fraction: float = 0.0,
    table_stride: Optional[int] = None,
    placement_seed: Optional[int] = None,
    placement_skip: int = 0,
) -> Workload:
    """Draw tensors and place the cached prefix into paged blocks.

    Block ids are taken in order from a seeded permutation of the pool; `placement_skip`
    drops that many leading entries, so that several workloads can live in disjoint blocks
    of one pool.

    Sharing rule (flat logical addressing, full-block granularity): logical block b
    of a request may be shared with every request whose document path is identical
    through token 16(b+1)-1, provided the block lies entirely inside the cached
    prefix.  The block that contains the prefix/new boundary and all later blocks
    are private to the request (they receive appended tokens).
    """
    assert dtype in ("bf16", "f32")
    w = Workload(name, dtype, q_heads, kv_heads, head_dim, num_blocks, seed, sigma, requests)
    R = len(requests)
    w.prefix_len = np.asarray([rq.prefix_len for rq in requests], np.int32).reshape(R)
    w.new_len = np.asarray([rq.new_len for rq in requests], np.int32).reshape(R)
    w.new_start = np.zeros(R + 1, np.int32)
    if R:
        w.new_start[1:] = np.cumsum(w.new_len)
    total_new = int(w.new_start[-1])

    # fresh tensors
    w.q = _draw(seed, _T_Q, 0, (total_new, q_heads, head_dim), sigma * q_gain, dtype)
    w.k_new = _draw(seed, _T_KNEW, 0, (total_new, kv_heads, head_dim), sigma, dtype)
    w.v_new = _draw(seed, _T_VNEW, 0, (total_new, kv_heads, head_dim), sigma, dtype)

    # cached documents: K/V of a document depends on the whole path before it
    # (order sensitivity, Sec. 5.1), so data is keyed by the path, not the document
    for rq in requests:
        path: List[int] = []
        for doc, length in rq.docs:
            path.append(doc)
            key = tuple(path)
            if key not in w._node_kv:
                h = _path_hash(key)
                k = _draw(seed, _T_NODE_K, h, (length, kv_heads, head_dim), sigma, dtype)
                v = _draw(seed, _T_NODE_V, h, (length, kv_heads, head_dim), sigma, dtype)
                w._node_kv[key] = (k, v)
            else:
                assert w._node_kv[key][0].shape[0] == length, "same path, different length"

    # block assignment
    perm = _gen(seed if placement_seed is None else placement_seed, _T_PERM).permutation(num_blocks).astype(np.int32)
    nxt = int(placement_skip)
    max_blocks = max([1] + [(int(p) + int(n) + BLOCK - 1) // BLOCK for p, n in zip(w.prefix_len, w.new_len)])
    w.table_stride = int(table_stride) if table_stride is not None else max_blocks
    assert w.table_stride >= max_blocks
    w.poison_block = int(perm[nxt]); nxt += 1
    w.block_table = np.full((R, w.table_stride), w.poison_block, np.int32)
    shared: Dict[Tuple[Tuple[int, ...], int], int] = {}
    used_ids: List[int] = []
    used_src: List[Tuple[int, int]] = []  # (request, logical block) that defines the content
    block_nodes: Dict[int, Tuple[int, ...]] = {}  # block id -> path that owns it
    for ri, rq in enumerate(requests):
        p, n = rq.prefix_len, rq.new_len
        nblk = (p + n + BLOCK - 1) // BLOCK
        ends = np.cumsum([l for _, l in rq.docs]) if rq.docs else np.zeros(0, np.int64)
        for b in range(nblk):
            full_in_prefix = BLOCK * (b + 1) <= p
            if full_in_prefix:
                ndocs = int(np.searchsorted(ends, BLOCK * (b + 1), side="left")) + 1
                key = (tuple(d for d, _ in rq.docs[:ndocs]), b)
                if key in shared:
                    w.block_table[ri, b] = shared[key]
                    continue
            assert nxt < num_blocks, "pool too small for this workload"
            blk = int(perm[nxt]); nxt += 1
            w.block_table[ri, b] = blk
            if full_in_prefix:
                shared[key] = blk
                block_nodes[blk] = key[0]
            if BLOCK * b < p:  # holds at least one cached token
                used_ids.append(blk)
                used_src.append((ri, b))
                if not full_in_prefix:
                    block_nodes[blk] = tuple(d for d, _ in rq.docs)

    # contents of the cached blocks
    dt = storage_np_dtype(dtype)
    U = len(used_ids)
    w.used_block_ids = np.asarray(used_ids, np.int32)
    w.used_k = np.full((U, kv_heads, BLOCK, head_dim), poison_value(dtype), dtype=dt)
    w.used_v = np.full((U, kv_heads, BLOCK, head_dim), poison_value(dtype), dtype=dt)
    cache_r, cache_kv = -1, None
    for u, (ri, b) in enumerate(used_src):
        if ri != cache_r:
            cache_r, cache_kv = ri, w.prefix_kv(ri)
        kp, vp = cache_kv
        lo, hi = BLOCK * b, min(BLOCK * (b + 1), kp.shape[0])
        w.used_k[u, :, : hi - lo, :] = np.transpose(kp[lo:hi], (1, 0, 2))
        w.used_v[u, :, : hi - lo, :] = np.transpose(vp[lo:hi], (1, 0, 2))

    # host tier: host-resident nodes are a suffix of each path (GPU nodes are parents
    # of host nodes, Sec. 5.1 node placement); mark deepest documents first
    w.needs_swap = np.zeros(R, bool)
    w.host_dev_blocks = np.zeros(0, np.int32)
    w.host_slots = np.zeros(0, np.int32)
    if host_fraction > 0 and U:
        # owner path of each used block -> depth; a block is host-resident when its
        # owning path is marked
        marked: set = set()
        order = _gen(seed, _T_HOST).permutation(R)
        target = host_fraction * U

        def count_marked() -> int:
            return sum(1 for b in used_ids if _is_marked(block_nodes[b], marked))

        # request by request (random order): everything below the first document goes to
        # the host (a lone document goes whole), until the target share is reached; cold
        # paths are evicted as a whole while hot ones stay resident
        for ri in order:
            docs = [d for d, _ in requests[ri].docs]
            if not docs:
                continue
            marked.add(tuple(docs[:2]) if len(docs) > 1 else tuple(docs))
            if count_marked() >= target:
                break
        host_blocks = [b for b in used_ids if _is_marked(block_nodes[b], marked)]
        S = len(host_blocks)
        w.num_host_slots = max(1, int(np.ceil(S * 1.25)))
        slots = _gen(seed, _T_HOST, 1).permutation(w.num_host_slots)[:S].astype(np.int32)
        w.host_dev_blocks = np.asarray(host_blocks, np.int32)
        w.host_slots = slots
        hb = set(host_blocks)
        for ri in range(R):
            nb = (int(w.prefix_len[ri]) + BLOCK - 1) // BLOCK
            w.needs_swap[ri] = any(int(x) in hb for x in w.block_table[ri, :nb])
    return w


def _is_marked(path: Tuple[int, ...], marked: set) -> bool:
    """A block is host-resident when its owning path or any ancestor path is marked
    (children of host nodes are host nodes)."""
    for i in range(1, len(path) + 1):
        if path[:i] in marked:
            return True
    return False


# ----------------------------------------------------------------------------
# the five named configurations
# ----------------------------------------------------------------------------
CONFIG_NAMES = {
    1: "C1-f32-mha4-d64-P256-N32",
    2: "C2-llama2-7b-mha32-d128-R8-P1024-N100",
    3: "C3-mistral-7b-gqa32/8-d128-R16-ragged",
    4: "C4-llama2-70b-gqa64/8-d128-R4-P4096-N128",
    5: "C5-mistral-7b-gqa32/8-d128-R32-zipf-hosttier",
}


def _ragged_requests(seed: int, R: int, share_first: float, zipf: bool) -> List[RequestSpec]:
    g = _gen(seed, _T_SHAPE)
    reqs: List[RequestSpec] = []
    if zipf:
        ranks = np.arange(1, 10001, dtype=np.float64)
        pz = ranks ** -1.1
        pz /= pz.sum()
    next_doc = 1
    for _ in range(R):
        nd = int(g.integers(1, 6))
        docs: List[Tuple[int, int]] = []
        if zipf:
            ids: List[int] = []
            while len(ids) < nd:
                d = int(g.choice(10000, p=pz)) + 1
                if d not in ids:
                    ids.append(d)
            for d in ids:
                docs.append((d, int(_gen(seed, _T_DOCLEN, d).integers(256, 1025))))
        else:
            for _ in range(nd):
                docs.append((next_doc, int(g.integers(256, 1025))))
                next_doc += 1
        nq = int(g.integers(64, 257))
        nu = 512 if int(g.integers(0, 2)) else 0
        reqs.append(RequestSpec(docs, nq, nu))
    if share_first > 0 and R > 1:
        ns = max(2, int(round(share_first * R)))
        who = _gen(seed, _T_SHAPE, 1).permutation(R)[:ns]
        lead = reqs[int(who[0])].docs[0]
        for ri in who[1:]:
            reqs[int(ri)].docs[0] = lead
    return reqs


def make_config(index: int, seed: Optional[int] = None, peaked: bool = False, placement_skip: int = 0,
                placement_seed: Optional[int] = None) -> Workload:
    """The five synthetic configurations.  `peaked` multiplies Q by 8 so that the
    softmax is sharp and |O| is of the order of |V| (a tolerance of 2e-2 is then a
    meaningful fraction of the signal)."""
    seed = BASE_SEED + index if seed is None else seed
    gain = 8.0 if peaked else 1.0
    nm = CONFIG_NAMES[index] + ("-peaked" if peaked else "")
    place = dict(placement_skip=placement_skip, placement_seed=placement_seed)
    if index == 1:
        reqs = [RequestSpec([(1, 256)], 32)]
        return build_workload(nm, "f32", 4, 4, 64, 64, reqs, seed, 1.0, gain, **place)
    if index == 2:
        reqs = [RequestSpec([(2 * r + 1, 512), (2 * r + 2, 512)], 100) for r in range(8)]
        return build_workload(nm, "bf16", 32, 32, 128, 8192, reqs, seed, 0.5, gain, **place)
    if index == 3:
        reqs = _ragged_requests(seed, 16, 0.2, zipf=False)
        return build_workload(nm, "bf16", 32, 8, 128, 16384, reqs, seed, 1.0, gain, **place)
    if index == 4:
        reqs = [RequestSpec([(8 * r + d + 1, 512) for d in range(8)], 128) for r in range(4)]
        return build_workload(nm, "bf16", 64, 8, 128, 32768, reqs, seed, 1.0, gain, **place)
    if index == 5:
        reqs = _ragged_requests(seed, 32, 0.0, zipf=True)
        return build_workload(nm, "bf16", 32, 8, 128, 16384, reqs, seed, 1.0, gain, host_fraction=0.30, **place)
    raise ValueError(f"no such config: {index}")


def make_small(
    dtype: str,
    q_heads: int,
    kv_heads: int,
    head_dim: int,
    lens: Sequence[Tuple[int, int]],
    seed: int,
    num_blocks: Optional[int] = None,
    sigma: float = 1.0,
    q_gain: float = 1.0,
    shared_first_doc: int = 0,
    table_stride: Optional[int] = None,
    placement_seed: Optional[int] = None,
    docs: Optional[List[List[Tuple[int, int]]]] = None,
) -> Workload:
    """Ad-hoc case for tests: `lens` is a list of (prefix_len, new_len); every
    request gets one private cached document of prefix_len tokens, optionally
    preceded by a common first document of `shared_first_doc` tokens; `docs` gives
    the document sequences explicitly instead."""
    reqs = []
    for i, (p, n) in enumerate(lens):
        docs_i: List[Tuple[int, int]] = []
        if docs is not None:
            docs_i = list(docs[i])
            assert sum(l for _, l in docs_i) == p
        elif shared_first_doc and p > shared_first_doc:
            docs_i.append((1, shared_first_doc))
            docs_i.append((100 + i, p - shared_first_doc))
        elif p > 0:
            docs_i.append((100 + i, p))
        reqs.append(RequestSpec(docs_i, n, 0))
    need = 2 + sum((p + n + BLOCK - 1) // BLOCK for p, n in lens)
    nb = num_blocks if num_blocks is not None else max(8, 2 * need)
    return build_workload(f"small-{dtype}-{q_heads}/{kv_heads}-d{head_dim}", dtype, q_heads, kv_heads, head_dim,
                          nb, reqs, seed, sigma, q_gain, table_stride=table_stride, placement_seed=placement_seed)
