"""Device-side plumbing shared by the GPU tests, the smoke check and the
benchmark: allocate a pool with PyTorch-ROCm, place a generated workload in it,
build the C structs.  Allocation and copies only -- no arithmetic of the method.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B
from .workload import Workload


def torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_device(a: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """Storage array (uint16 bf16 bits / float32) -> device tensor of that dtype."""
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> storage array (uint16 bits for bf16, float32 otherwise)."""
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


def workspace_for(pool, batch, q_heads: int, flags: int = 0, device="cuda", have=None):
    """(tensor or None, bytes) large enough for ragc_prefill_attn on this batch; `have` is reused if it suffices."""
    need = B.ragc_prefill_attn_workspace(pool, batch, q_heads, flags)
    if need == 0:
        return have, (have.numel() if have is not None else 0)
    if have is None or have.numel() < need:
        have = torch.empty(need, dtype=torch.uint8, device=device)
    return have, have.numel()


class DeviceWorkload:
    """A Workload resident on the GPU: pool planes (poison everywhere except the
    cached blocks), Q / fresh K,V, tables, and the ragc structs pointing at them."""

    def __init__(self, w: Workload, device="cuda", resident_host_blocks: bool = True, with_host_table: bool = True,
                 pool=None):
        """`pool` = (pool_k, pool_v) of another DeviceWorkload with the same shape: this workload's
        blocks are placed into it (the placements must be disjoint) instead of a fresh pool."""
        self.w = w
        self.device = device
        td = torch_dtype(w.dtype)
        if pool is None:
            self.pool_k = torch.full(w.pool_shape(), float("nan"), dtype=td, device=device)
            self.pool_v = torch.full(w.pool_shape(), float("nan"), dtype=td, device=device)
        else:
            self.pool_k, self.pool_v = pool
            assert tuple(self.pool_k.shape) == tuple(w.pool_shape())
        ids = w.used_block_ids
        uk, uv = w.used_k, w.used_v
        if not resident_host_blocks and w.host_dev_blocks.size:
            keep = ~np.isin(ids, w.host_dev_blocks)
            ids, uk, uv = ids[keep], uk[keep], uv[keep]
        if ids.size:
            idx = torch.from_numpy(ids.astype(np.int64)).to(device)
            self.pool_k[idx] = to_device(uk, w.dtype, device)
            self.pool_v[idx] = to_device(uv, w.dtype, device)
        self.q = to_device(w.q, w.dtype, device)
        self.k_new = to_device(w.k_new, w.dtype, device)
        self.v_new = to_device(w.v_new, w.dtype, device)
        self.out = torch.full(tuple(w.q.shape), float("nan"), dtype=td, device=device)
        self.h_prefix_len = np.ascontiguousarray(w.prefix_len, np.int32)
        self.h_new_len = np.ascontiguousarray(w.new_len, np.int32)
        self.h_new_start = np.ascontiguousarray(w.new_start, np.int32)
        self.h_block_table = np.ascontiguousarray(w.block_table, np.int32) if with_host_table else None
        self.d_prefix_len = torch.from_numpy(self.h_prefix_len).to(device)
        self.d_new_len = torch.from_numpy(self.h_new_len).to(device)
        self.d_new_start = torch.from_numpy(self.h_new_start).to(device)
        self.d_block_table = torch.from_numpy(np.ascontiguousarray(w.block_table, np.int32)).to(device)
        self.dtype_code = B.RAGC_DTYPE_BF16 if w.dtype == "bf16" else B.RAGC_DTYPE_F32
        self.pool = B.make_pool(self.pool_k, self.pool_v, w.num_blocks, w.kv_heads, w.head_dim, self.dtype_code)
        self.batch = B.make_batch(w.num_reqs, w.table_stride, self.d_prefix_len, self.d_new_len, self.d_new_start,
                                  self.d_block_table, self.h_prefix_len, self.h_new_len, self.h_new_start,
                                  self.h_block_table)
        self.workspace = None
        self.workspace_bytes = 0
        # host tier
        self.host_k = self.host_v = None
        if w.host_dev_blocks.size:
            shp = (w.num_host_slots, w.kv_heads, 16, w.head_dim)
            self.host_k = torch.zeros(shp, dtype=td).pin_memory()
            self.host_v = torch.zeros(shp, dtype=td).pin_memory()
            where = {int(b): i for i, b in enumerate(w.used_block_ids)}
            sel = np.asarray([where[int(b)] for b in w.host_dev_blocks])
            slots = torch.from_numpy(w.host_slots.astype(np.int64))
            self.host_k[slots] = to_device(w.used_k[sel], w.dtype, "cpu")
            self.host_v[slots] = to_device(w.used_v[sel], w.dtype, "cpu")

    def sub_batch(self, reqs):
        """A batch struct over a subset of the requests, addressing the same packed
        tensors.  Returns (struct, keepalive)."""
        idx = np.asarray(reqs, np.int64)
        w = self.w
        hp = np.ascontiguousarray(w.prefix_len[idx], np.int32)
        hn = np.ascontiguousarray(w.new_len[idx], np.int32)
        hs = np.ascontiguousarray(np.concatenate([w.new_start[idx], [0]]), np.int32)
        ht = np.ascontiguousarray(w.block_table[idx], np.int32)
        dev = [torch.from_numpy(a).to(self.device) for a in (hp, hn, hs, ht)]
        batch = B.make_batch(len(idx), w.table_stride, dev[0], dev[1], dev[2], dev[3], hp, hn, hs, ht)
        return batch, (hp, hn, hs, ht, dev)

    def attn_batch(self, batch, flags: int = 0, stream: Optional[int] = None):
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        self.workspace, self.workspace_bytes = workspace_for(self.pool, batch, self.w.q_heads, flags, self.device, self.workspace)
        B.ragc_prefill_attn(self.pool, batch, self.q, self.k_new, self.v_new, self.out, self.w.q_heads,
                            self.w.softmax_scale, flags, self.workspace, self.workspace_bytes, s)

    def ensure_workspace(self, flags: int = 0):
        self.workspace, self.workspace_bytes = workspace_for(self.pool, self.batch, self.w.q_heads, flags, self.device, self.workspace)

    def attn(self, flags: int = 0, stream: Optional[int] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        self.ensure_workspace(flags)
        out = self.out if out is None else out
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        B.ragc_prefill_attn(self.pool, self.batch, self.q, self.k_new, self.v_new, out, self.w.q_heads,
                            self.w.softmax_scale, flags, self.workspace, self.workspace_bytes, s)
        return out

    def append(self, stream: Optional[int] = None):
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        B.ragc_kv_append(self.pool, self.batch, self.k_new, self.v_new, s)

    def swap(self, dev_blocks: np.ndarray, host_slots: np.ndarray, direction: int, flags: int = 0,
             stream: Optional[int] = None):
        s = torch.cuda.current_stream().cuda_stream if stream is None else stream
        w = self.w
        B.ragc_kv_swap(self.pool, self.host_k, self.host_v, w.kv_heads * 16 * w.head_dim, w.num_host_slots, dev_blocks,
                       host_slots, direction, flags, s)


class LayeredCache:
    """One paged K/V pool per transformer layer plus a pinned host pool per layer, all addressed by
    the same block ids and host slots (the controller's plan applies to every layer), and the
    stream choreography around the C-ABI calls: with `prefetch` the copies of layer l+1 run on a
    side stream under the attention of layer l (the controller decides WHAT moves, the kernels
    move it; this class only orders the calls).  Test and benchmark plumbing, no arithmetic."""

    def __init__(self, layers: int, gpu_blocks: int, host_slots: int, kv_heads: int, head_dim: int, dtype: str = "bf16",
                 device="cuda"):
        self.layers, self.kv_heads, self.head_dim, self.dtype, self.device = layers, kv_heads, head_dim, dtype, device
        td = torch_dtype(dtype)
        shp = (gpu_blocks, kv_heads, 16, head_dim)
        self.pool_k = [torch.full(shp, float("nan"), dtype=td, device=device) for _ in range(layers)]
        self.pool_v = [torch.full(shp, float("nan"), dtype=td, device=device) for _ in range(layers)]
        hshp = (max(host_slots, 1), kv_heads, 16, head_dim)
        self.host_k = [torch.zeros(hshp, dtype=td).pin_memory() for _ in range(layers)]
        self.host_v = [torch.zeros(hshp, dtype=td).pin_memory() for _ in range(layers)]
        self.host_slots = max(host_slots, 1)
        code = B.RAGC_DTYPE_BF16 if dtype == "bf16" else B.RAGC_DTYPE_F32
        self.pools = [B.make_pool(self.pool_k[l], self.pool_v[l], gpu_blocks, kv_heads, head_dim, code) for l in range(layers)]
        self.side = torch.cuda.Stream(device=device)
        self.ready = [torch.cuda.Event() for _ in range(layers)]
        self.begun = torch.cuda.Event()
        self.workspace = None  # shared by the layers: their attention calls run one after the other on one stream

    def _swap(self, layer: int, dev, slots, direction: int, stream: int):
        if len(dev):
            B.ragc_kv_swap(self.pools[layer], self.host_k[layer], self.host_v[layer], self.kv_heads * 16 * self.head_dim,
                           self.host_slots, dev, slots, direction, B.RAGC_SWAP_KERNEL, stream)

    def execute(self, plan, q, k_new, v_new, q_heads: int, scale: float, prefetch: bool = True):
        """Run one request through every layer: the plan's swap-outs, then its swap-ins, then
        prefix-cached attention with the fused append.  q / k_new / v_new: one device tensor per
        layer ([beta, H, D]).  Returns the per-layer outputs."""
        main = torch.cuda.current_stream()
        alpha, beta = int(plan.alpha), int(plan.beta)
        hp, hn, hs = np.asarray([alpha], np.int32), np.asarray([beta], np.int32), np.asarray([0, beta], np.int32)
        ht = np.ascontiguousarray(plan.block_table, np.int32).reshape(1, -1)
        dev = [torch.from_numpy(a).to(self.device) for a in (hp, hn, hs, ht)]
        batch = B.make_batch(1, ht.shape[1], dev[0], dev[1], dev[2], dev[3], hp, hn, hs, ht)
        outs = [torch.empty_like(q[l]) for l in range(self.layers)]
        self.workspace, ws_bytes = workspace_for(self.pools[0], batch, q_heads, B.RAGC_ATTN_APPEND_FUSED, self.device, self.workspace)
        copies = prefetch and (len(plan.swap_out_dev) or len(plan.swap_in_dev))
        if copies:
            # the copies may touch blocks that earlier work on the main stream still reads or writes
            self.begun.record(main)
            self.side.wait_event(self.begun)
            for l in range(self.layers):
                self._swap(l, plan.swap_out_dev, plan.swap_out_slot, B.RAGC_SWAP_TO_HOST, self.side.cuda_stream)
                self._swap(l, plan.swap_in_dev, plan.swap_in_slot, B.RAGC_SWAP_TO_DEVICE, self.side.cuda_stream)
                self.ready[l].record(self.side)
        for l in range(self.layers):
            if copies:
                main.wait_event(self.ready[l])
            elif not prefetch:
                self._swap(l, plan.swap_out_dev, plan.swap_out_slot, B.RAGC_SWAP_TO_HOST, main.cuda_stream)
                self._swap(l, plan.swap_in_dev, plan.swap_in_slot, B.RAGC_SWAP_TO_DEVICE, main.cuda_stream)
            if beta > 0:
                B.ragc_prefill_attn(self.pools[l], batch, q[l], k_new[l], v_new[l], outs[l], q_heads, scale,
                                    B.RAGC_ATTN_APPEND_FUSED, self.workspace, ws_bytes, main.cuda_stream)
        if copies:
            # later work on the main stream may reuse what the side stream was given
            self.side.wait_stream(main)
        self._keep = (batch, dev, hp, hn, hs, ht)
        return outs
