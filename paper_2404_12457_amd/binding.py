"""ctypes binding of libragc.so: same names as the C ABI (include/ragc.h),
argument marshalling only.  Every step of the path runs in the HIP kernels; if
the library has not been built, loading raises -- there is no fallback.

Device arguments may be torch tensors (their data_ptr() is passed) or integer
addresses.  Host id arrays are numpy int32 arrays.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libragc.so")

RAGC_OK = 0
RAGC_ERR_NULL, RAGC_ERR_SHAPE, RAGC_ERR_RANGE, RAGC_ERR_ALIGN, RAGC_ERR_HIP, RAGC_ERR_WORKSPACE = -1, -2, -3, -4, -5, -6
RAGC_DTYPE_F32, RAGC_DTYPE_BF16 = 0, 1
RAGC_ATTN_APPEND_FUSED, RAGC_ATTN_NO_SPLIT, RAGC_ATTN_VALIDATE = 0x1, 0x2, 0x4
RAGC_SWAP_AUTO, RAGC_SWAP_MEMCPY, RAGC_SWAP_KERNEL = 0, 1, 2
RAGC_SWAP_TO_DEVICE, RAGC_SWAP_TO_HOST = 0, 1

EXPORTS = ["ragc_version", "ragc_last_error", "ragc_kv_bytes_per_token", "ragc_prefill_attn_workspace",
           "ragc_prefill_attn", "ragc_prefill_attn_static", "ragc_kv_append", "ragc_kv_swap", "ragc_kv_gather",
           "ragc_batch_validate", "ragc_debug_set_attn_plan"]


class ragc_kv_pool(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("num_blocks", ctypes.c_int32),
                ("block_size", ctypes.c_int32), ("kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("reserved", ctypes.c_int32), ("block_stride_elems", ctypes.c_int64)]


class ragc_batch(ctypes.Structure):
    _fields_ = [("num_reqs", ctypes.c_int32), ("table_stride", ctypes.c_int32), ("prefix_len", ctypes.c_void_p),
                ("new_len", ctypes.c_void_p), ("new_start", ctypes.c_void_p), ("block_table", ctypes.c_void_p),
                ("h_prefix_len", ctypes.c_void_p), ("h_new_len", ctypes.c_void_p), ("h_new_start", ctypes.c_void_p),
                ("h_block_table", ctypes.c_void_p)]


class RagcError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"ragc error {code}: {msg}")
        self.code = code


_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2404_12457_amd.build` "
                               "(the HIP library is the only implementation; there is no fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        P, I32, I64, U32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32
        lib.ragc_version.restype = ctypes.c_int
        lib.ragc_last_error.restype = ctypes.c_char_p
        lib.ragc_kv_bytes_per_token.restype = I64
        lib.ragc_kv_bytes_per_token.argtypes = [I32, I32, I32, I32]
        lib.ragc_prefill_attn_workspace.restype = I64
        lib.ragc_prefill_attn_workspace.argtypes = [P, P, I32, U32]
        lib.ragc_prefill_attn.restype = ctypes.c_int
        lib.ragc_prefill_attn.argtypes = [P, P, P, P, P, P, I32, ctypes.c_float, U32, P, ctypes.c_size_t, P]
        lib.ragc_prefill_attn_static.restype = ctypes.c_int
        lib.ragc_prefill_attn_static.argtypes = [P, P, P, P, P, P, I32, ctypes.c_float, U32, P]
        lib.ragc_batch_validate.restype = ctypes.c_int
        lib.ragc_batch_validate.argtypes = [P, P, I32]
        lib.ragc_debug_set_attn_plan.restype = ctypes.c_int
        lib.ragc_debug_set_attn_plan.argtypes = [I32, I32]
        lib.ragc_kv_append.restype = ctypes.c_int
        lib.ragc_kv_append.argtypes = [P, P, P, P, P]
        lib.ragc_kv_swap.restype = ctypes.c_int
        lib.ragc_kv_swap.argtypes = [P, P, P, I64, I32, P, P, I32, I32, U32, P]
        lib.ragc_kv_gather.restype = ctypes.c_int
        lib.ragc_kv_gather.argtypes = [P, P, I32, I32, P, P, P]
        _lib = lib
    return _lib


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return int(x.data_ptr())  # torch tensor


def _ref(s):
    return None if s is None else ctypes.cast(ctypes.byref(s), ctypes.c_void_p)


def _check(rc: int) -> int:
    if rc < 0:
        raise RagcError(rc, load().ragc_last_error().decode())
    return rc


def make_pool(k, v, num_blocks: int, kv_heads: int, head_dim: int, dtype: int, block_stride_elems: Optional[int] = None,
              block_size: int = 16) -> ragc_kv_pool:
    if block_stride_elems is None:
        block_stride_elems = kv_heads * block_size * head_dim
    return ragc_kv_pool(_ptr(k), _ptr(v), num_blocks, block_size, kv_heads, head_dim, dtype, 0, block_stride_elems)


def make_batch(num_reqs: int, table_stride: int, prefix_len, new_len, new_start, block_table, h_prefix_len: np.ndarray,
               h_new_len: np.ndarray, h_new_start: np.ndarray, h_block_table: Optional[np.ndarray] = None) -> ragc_batch:
    """Device arrays + host copies.  The caller keeps every array alive while the struct is used."""
    return ragc_batch(num_reqs, table_stride, _ptr(prefix_len), _ptr(new_len), _ptr(new_start), _ptr(block_table),
                      _ptr(h_prefix_len), _ptr(h_new_len), _ptr(h_new_start), _ptr(h_block_table))


def ragc_version() -> int:
    return load().ragc_version()


def ragc_last_error() -> str:
    return load().ragc_last_error().decode()


def ragc_kv_bytes_per_token(layers: int, kv_heads: int, head_dim: int, dtype: int) -> int:
    return int(load().ragc_kv_bytes_per_token(layers, kv_heads, head_dim, dtype))


def ragc_prefill_attn_workspace(pool: ragc_kv_pool, batch: ragc_batch, q_heads: int, flags: int = 0) -> int:
    return _check(int(load().ragc_prefill_attn_workspace(_ref(pool), _ref(batch), q_heads, flags)))


def ragc_prefill_attn(pool, batch, q, k_new, v_new, out, q_heads: int, softmax_scale: float, flags: int = 0,
                      workspace=None, workspace_bytes: int = 0, stream: int = 0) -> int:
    return _check(load().ragc_prefill_attn(_ref(pool), _ref(batch), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), q_heads,
                                           softmax_scale, flags, _ptr(workspace), workspace_bytes, stream or None))


def ragc_prefill_attn_static(pool, batch, q, k_new, v_new, out, q_heads: int, softmax_scale: float, flags: int = 0,
                             stream: int = 0) -> int:
    return _check(load().ragc_prefill_attn_static(_ref(pool), _ref(batch), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                                  q_heads, softmax_scale, flags, stream or None))


def ragc_batch_validate(pool, batch, writes_new_tokens: bool = True) -> int:
    return _check(load().ragc_batch_validate(_ref(pool), _ref(batch), 1 if writes_new_tokens else 0))


def ragc_debug_set_attn_plan(variant: int = -1, splits: int = 0) -> int:
    return _check(load().ragc_debug_set_attn_plan(variant, splits))


def ragc_kv_append(pool, batch, k_new, v_new, stream: int = 0) -> int:
    return _check(load().ragc_kv_append(_ref(pool), _ref(batch), _ptr(k_new), _ptr(v_new), stream or None))


def ragc_kv_swap(pool, host_k, host_v, host_block_stride_elems: int, num_host_slots: int, dev_block_ids: np.ndarray,
                 host_slots: np.ndarray, direction: int, flags: int = 0, stream: int = 0) -> int:
    dev_block_ids = np.ascontiguousarray(dev_block_ids, np.int32)
    host_slots = np.ascontiguousarray(host_slots, np.int32)
    assert dev_block_ids.size == host_slots.size
    return _check(load().ragc_kv_swap(_ref(pool), _ptr(host_k), _ptr(host_v), host_block_stride_elems, num_host_slots,
                                      _ptr(dev_block_ids), _ptr(host_slots), int(dev_block_ids.size), direction, flags,
                                      stream or None))


def ragc_kv_gather(pool, batch, req: int, length: int, k_out, v_out, stream: int = 0) -> int:
    return _check(load().ragc_kv_gather(_ref(pool), _ref(batch), req, length, _ptr(k_out), _ptr(v_out), stream or None))
