"""Oracle for the byte-moving steps: paged gather, K/V append, block swap.
Test infrastructure only.  Plain loops over tokens and blocks; every function
works on numpy arrays of the storage dtype and never converts a value, so a
comparison with the HIP path is a comparison of bytes.

Addressing (flat, over the whole request): logical position j of a request lives
in pool block `table[j // 16]`, slot `j % 16`; pool planes are
[num_blocks][kv_heads][16][head_dim].  The paper stores each document's K/V in
non-contiguous blocks referenced from its tree node (Sec. 5.1, knowledge tree)
and hands the K/V of the request's tokens back for caching after the first
token (Sec. 4, architecture overview); block swap keeps the exact tensors in
host memory (Sec. 5.1, swap out only once).
"""
from __future__ import annotations

import numpy as np

BLOCK = 16


def gather(pool: np.ndarray, table_row: np.ndarray, length: int) -> np.ndarray:
    """pool [NB,Hkv,16,D], one request's table row -> logical [length,Hkv,D]."""
    nb, hkv, blk, d = pool.shape
    assert blk == BLOCK
    out = np.empty((length, hkv, d), pool.dtype)
    for j in range(length):
        out[j] = pool[int(table_row[j // BLOCK]), :, j % BLOCK, :]
    return out


def append(pool_k: np.ndarray, pool_v: np.ndarray, block_table: np.ndarray, prefix_len, new_len, new_start,
           k_new: np.ndarray, v_new: np.ndarray) -> None:
    """In place: token i of request r goes to position prefix_len[r]+i."""
    for r in range(len(prefix_len)):
        p, n, s0 = int(prefix_len[r]), int(new_len[r]), int(new_start[r])
        for i in range(n):
            pos = p + i
            b = int(block_table[r, pos // BLOCK])
            pool_k[b, :, pos % BLOCK, :] = k_new[s0 + i]
            pool_v[b, :, pos % BLOCK, :] = v_new[s0 + i]


def swap(pool_k: np.ndarray, pool_v: np.ndarray, host_k: np.ndarray, host_v: np.ndarray, dev_blocks, host_slots,
         to_device: bool) -> None:
    """In place: whole blocks (all kv heads, K and V) between pool and host tier."""
    for b, s in zip(dev_blocks, host_slots):
        if to_device:
            pool_k[int(b)] = host_k[int(s)]
            pool_v[int(b)] = host_v[int(s)]
        else:
            host_k[int(s)] = pool_k[int(b)]
            host_v[int(s)] = pool_v[int(b)]
