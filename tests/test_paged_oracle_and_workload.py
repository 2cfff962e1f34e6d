"""Pins of the byte-moving oracle (gather / append / swap) and checks of the
seeded input generator.  No GPU."""
import os

import numpy as np
import pytest
import torch

from oracle import paged as OP
from paper_2404_12457_amd import workload as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_bf16_rounding_matches_library_conversion():
    x = np.random.Generator(np.random.Philox(key=[5, 5])).standard_normal(100000).astype(np.float32)
    x[:4] = [0.0, -0.0, 1.0 + 2.0**-8, 1.0 + 3 * 2.0**-8]  # ties: to even
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = W.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_append_literal_positions():
    # table [3, 1], P=14, N=4: tokens land in block 3 slots 14,15 then block 1 slots 0,1
    pool_k = np.zeros((4, 2, 16, 4), np.float32)
    pool_v = np.zeros((4, 2, 16, 4), np.float32)
    k_new = np.arange(4 * 2 * 4, dtype=np.float32).reshape(4, 2, 4) + 1
    v_new = -k_new
    OP.append(pool_k, pool_v, np.array([[3, 1]], np.int32), [14], [4], [0, 4], k_new, v_new)
    want = np.zeros_like(pool_k)
    want[3, :, 14, :], want[3, :, 15, :], want[1, :, 0, :], want[1, :, 1, :] = k_new[0], k_new[1], k_new[2], k_new[3]
    assert np.array_equal(pool_k, want) and np.array_equal(pool_v, -want)


def test_gather_literal_positions():
    pool = np.arange(5 * 1 * 16 * 2, dtype=np.float32).reshape(5, 1, 16, 2)
    got = OP.gather(pool, np.array([4, 0, 2], np.int32), 35)
    assert np.array_equal(got[0, 0], pool[4, 0, 0]) and np.array_equal(got[15, 0], pool[4, 0, 15])
    assert np.array_equal(got[16, 0], pool[0, 0, 0]) and np.array_equal(got[34, 0], pool[2, 0, 2])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_gather_of_generated_pool_is_the_logical_prefix(dtype):
    w = W.make_small(dtype, 4, 2, 64, [(0, 5), (37, 20), (64, 1), (100, 33)], seed=11, shared_first_doc=32)
    pk, pv = w.pool_image()
    for r in range(w.num_reqs):
        kp, vp = w.prefix_kv(r)
        P = int(w.prefix_len[r])
        assert np.array_equal(OP.gather(pk, w.block_table[r], P).view(np.uint8), kp.view(np.uint8))
        assert np.array_equal(OP.gather(pv, w.block_table[r], P).view(np.uint8), vp.view(np.uint8))


def test_append_then_gather_is_the_full_sequence():
    w = W.make_small("bf16", 4, 2, 64, [(0, 5), (37, 20), (64, 1), (100, 33), (15, 0)], seed=12)
    pk, pv = w.pool_image()
    OP.append(pk, pv, w.block_table, w.prefix_len, w.new_len, w.new_start, w.k_new, w.v_new)
    for r in range(w.num_reqs):
        kf, vf = w.full_kv(r)
        L = kf.shape[0]
        assert np.array_equal(OP.gather(pk, w.block_table[r], L), kf)
        assert np.array_equal(OP.gather(pv, w.block_table[r], L), vf)
    # nothing but the slots of new tokens changed
    pk0, _ = w.pool_image()
    changed = (pk != pk0) & ~((pk != pk) & (pk0 != pk0))
    assert changed.sum() <= w.total_new * w.kv_heads * w.head_dim


def test_swap_round_trip():
    g = np.random.Generator(np.random.Philox(key=[9, 9]))
    pool_k = g.standard_normal((8, 2, 16, 4)).astype(np.float32)
    pool_v = g.standard_normal((8, 2, 16, 4)).astype(np.float32)
    keep_k, keep_v = pool_k.copy(), pool_v.copy()
    host_k, host_v = np.zeros((5, 2, 16, 4), np.float32), np.zeros((5, 2, 16, 4), np.float32)
    dev, slots = [6, 0, 3], [4, 1, 2]
    OP.swap(pool_k, pool_v, host_k, host_v, dev, slots, to_device=False)
    assert np.array_equal(host_k[4], keep_k[6]) and np.array_equal(host_v[2], keep_v[3]) and not host_k[0].any()
    pool_k[dev] = 0
    pool_v[dev] = 0
    OP.swap(pool_k, pool_v, host_k, host_v, dev, slots, to_device=True)
    assert np.array_equal(pool_k, keep_k) and np.array_equal(pool_v, keep_v)


def test_config_shapes():
    w1 = W.make_config(1)
    assert (w1.dtype, w1.q_heads, w1.kv_heads, w1.head_dim, w1.num_blocks) == ("f32", 4, 4, 64, 64)
    assert w1.prefix_len.tolist() == [256] and w1.new_len.tolist() == [32]
    assert len(set(w1.block_table[0, :18].tolist())) == 18
    w4 = W.make_config(4)
    assert (w4.q_heads, w4.kv_heads, w4.head_dim, w4.num_blocks) == (64, 8, 128, 32768)
    assert w4.prefix_len.tolist() == [4096] * 4 and w4.new_len.tolist() == [128] * 4
    assert w4.attn_flops() == 4 * 128 * 64 * 4 * (128 * 4096 + 128 * 129 // 2)


def test_config3_shares_a_first_document_chain():
    w = W.make_config(3)
    assert w.num_reqs == 16 and w.kv_heads == 8 and w.q_heads == 32
    firsts = {}
    for r, rq in enumerate(w.requests):
        firsts.setdefault(rq.docs[0], []).append(r)
        assert 1 <= len(rq.docs) <= 5 and all(256 <= l <= 1024 for _, l in rq.docs)
        assert 64 <= rq.n_question <= 256 and rq.n_uncached in (0, 512)
    sharers = max(firsts.values(), key=len)
    assert len(sharers) == 3  # 20 % of 16
    nfull = w.requests[sharers[0]].docs[0][1] // 16
    if len(w.requests[sharers[0]].docs) == 1:  # tail of the chain may hold the boundary
        nfull = min(nfull, int(w.prefix_len[sharers[0]]) // 16)
    a = w.block_table[sharers[0], :nfull]
    for r in sharers[1:]:
        n = min(nfull, int(w.prefix_len[r]) // 16)
        assert np.array_equal(w.block_table[r, :n], a[:n])
    # blocks that receive appended tokens are private
    seen = {}
    for r in range(w.num_reqs):
        p, n = int(w.prefix_len[r]), int(w.new_len[r])
        for b in range(p // 16, (p + n + 15) // 16):
            blk = int(w.block_table[r, b])
            assert blk not in seen, "append target shared"
            seen[blk] = r
    # and no cached block is an append target of another request
    assert not (set(seen) & set(int(b) for r in range(w.num_reqs) for b in w.block_table[r, : int(w.prefix_len[r]) // 16]))


def test_config5_host_resident_blocks_form_path_suffixes():
    w = W.make_config(5)
    frac = w.host_dev_blocks.size / w.used_block_ids.size
    assert 0.28 <= frac <= 0.40
    host = set(w.host_dev_blocks.tolist())
    assert len(set(w.host_slots.tolist())) == w.host_slots.size and w.host_slots.max() < w.num_host_slots
    for r in range(w.num_reqs):
        nb = (int(w.prefix_len[r]) + 15) // 16
        flags = [int(b) in host for b in w.block_table[r, :nb]]
        # once a block of the chain is host-resident, all later ones are
        assert flags == sorted(flags)
        assert bool(w.needs_swap[r]) == any(flags)


def test_seeds_reproduce_and_differ():
    a, b, c = W.make_config(1), W.make_config(1), W.make_config(1, seed=5)
    assert np.array_equal(a.q, b.q) and np.array_equal(a.block_table, b.block_table)
    assert not np.array_equal(a.q, c.q)


def test_kv_bytes_table_closed_form():
    for line in open(os.path.join(GOLD, "kv_bytes_per_token.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, layers, hq, hkv, mib = line.split()
        assert 2 * int(layers) * int(hkv) * 128 * 2 == float(mib) * 2**20, name
