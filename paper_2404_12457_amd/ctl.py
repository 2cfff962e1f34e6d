"""ctypes binding of the controller half of libragc.so (include/ragc_ctl.h): same names as the
C ABI, argument marshalling only.  `Tree` is a thin handle around ragc_tree_* that turns the
plan's arrays into numpy arrays; every decision is taken in the C++ library.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from typing import Sequence

import numpy as np

import os

from . import binding as B

# T(alpha, beta) measured with ragc_prefill_attn on one MI355X (see CostGrid.save / bench.py --write-cost-grid)
MEASURED_GRID = os.path.join(os.path.dirname(os.path.abspath(__file__)), "data", "cost_grid_mi355x_llama2_7b.json")

EXPORTS = ["ragc_cost_interp", "ragc_tree_create", "ragc_tree_destroy", "ragc_tree_begin", "ragc_tree_plan_read",
           "ragc_tree_end", "ragc_tree_get_stats", "ragc_tree_find", "ragc_tree_reset_frequencies", "ragc_tree_peek",
           "ragc_queue_create", "ragc_queue_destroy", "ragc_queue_push", "ragc_queue_pop", "ragc_queue_size"]

_D, _I32, _I64, _P = ctypes.c_double, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p


class ragc_cost_grid(ctypes.Structure):
    _fields_ = [("n_alpha", _I32), ("n_beta", _I32), ("alpha", _P), ("beta", _P), ("t", _P)]


class ragc_plan(ctypes.Structure):
    _fields_ = [("request_id", _I64), ("matched_docs", _I32), ("alpha", _I32), ("beta", _I32), ("n_blocks", _I32),
                ("n_swap_out", _I32), ("n_swap_in", _I32), ("n_evicted_gpu", _I32), ("n_evicted_host", _I32)]


class ragc_plan_buffers(ctypes.Structure):
    _fields_ = [("block_table", _P), ("table_cap", _I32), ("swap_out_dev", _P), ("swap_out_slot", _P),
                ("swap_in_dev", _P), ("swap_in_slot", _P), ("swap_cap", _I32), ("evicted_gpu", _P),
                ("evicted_host", _P), ("evicted_cap", _I32)]


class ragc_tree_stats(ctypes.Structure):
    _fields_ = [("clock_gpu", _D), ("clock_host", _D), ("nodes", _I64), ("nodes_in_gpu", _I64),
                ("free_gpu_blocks", _I64), ("free_host_slots", _I64), ("docs_requested", _I64), ("docs_hit", _I64),
                ("blocks_swapped_out", _I64), ("blocks_swapped_in", _I64), ("zero_copy_evictions", _I64)]


class ragc_node_info(ctypes.Structure):
    _fields_ = [("id", _I64), ("in_gpu", _I32), ("host_valid", _I32), ("length", _I32), ("n_owned", _I32),
                ("pins", _I32), ("computed", _I32), ("frequency", _I64), ("num_computed", _I64), ("avg_cost", _D),
                ("priority_gpu", _D), ("priority_host", _D)]


_ready = False


def _lib():
    global _ready
    lib = B.load()
    if not _ready:
        lib.ragc_cost_interp.restype = ctypes.c_int
        lib.ragc_cost_interp.argtypes = [_P, _D, _D, _P]
        lib.ragc_tree_create.restype = _P
        lib.ragc_tree_create.argtypes = [_I32, _I32, _P]
        lib.ragc_tree_destroy.restype = None
        lib.ragc_tree_destroy.argtypes = [_P]
        lib.ragc_tree_begin.restype = ctypes.c_int
        lib.ragc_tree_begin.argtypes = [_P, _P, _P, _I32, _I32, _P]
        lib.ragc_tree_plan_read.restype = ctypes.c_int
        lib.ragc_tree_plan_read.argtypes = [_P, _I64, _P]
        lib.ragc_tree_end.restype = ctypes.c_int
        lib.ragc_tree_end.argtypes = [_P, _I64]
        lib.ragc_tree_get_stats.restype = ctypes.c_int
        lib.ragc_tree_get_stats.argtypes = [_P, _P]
        lib.ragc_tree_find.restype = ctypes.c_int
        lib.ragc_tree_find.argtypes = [_P, _P, _I32, _P]
        lib.ragc_tree_reset_frequencies.restype = ctypes.c_int
        lib.ragc_tree_reset_frequencies.argtypes = [_P]
        lib.ragc_tree_peek.restype = ctypes.c_int
        lib.ragc_tree_peek.argtypes = [_P, _P, _P, _I32, _I32, _P, _P]
        lib.ragc_queue_create.restype = _P
        lib.ragc_queue_create.argtypes = [_I32]
        lib.ragc_queue_destroy.restype = None
        lib.ragc_queue_destroy.argtypes = [_P]
        lib.ragc_queue_push.restype = ctypes.c_int
        lib.ragc_queue_push.argtypes = [_P, _I64, _P, _P, _I32, _I32]
        lib.ragc_queue_pop.restype = ctypes.c_int
        lib.ragc_queue_pop.argtypes = [_P, _P, _P]
        lib.ragc_queue_size.restype = _I32
        lib.ragc_queue_size.argtypes = [_P]
        _ready = True
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise B.RagcError(rc, B.load().ragc_last_error().decode())


class CostGrid:
    """Host arrays of a profiled T(alpha, beta) table plus the C struct that points at them."""

    def __init__(self, alphas: Sequence[float], betas: Sequence[float], t):
        self.alpha = np.ascontiguousarray(alphas, np.float64)
        self.beta = np.ascontiguousarray(betas, np.float64)
        self.t = np.ascontiguousarray(t, np.float64)
        assert self.t.shape == (self.alpha.size, self.beta.size)
        self.c = ragc_cost_grid(self.alpha.size, self.beta.size, self.alpha.ctypes.data, self.beta.ctypes.data,
                                self.t.ctypes.data)
        self.meta: dict = {}

    # A profiled table travels as a small JSON file: {"alpha": [...], "beta": [...], "t": [[...]], ...};
    # any other key (unit, shape, device, noise) is kept in `meta`.  `bench.py --write-cost-grid PATH`
    # writes one from measurements with the attention kernel; MEASURED_GRID is the copy in this package.
    def save(self, path: str, **meta) -> None:
        import json

        doc = dict(self.meta)
        doc.update(meta)
        doc.update({"alpha": self.alpha.tolist(), "beta": self.beta.tolist(), "t": self.t.tolist()})
        with open(path, "w") as f:
            json.dump(doc, f, indent=1)
            f.write("\n")

    @classmethod
    def load(cls, path: str) -> "CostGrid":
        import json

        with open(path) as f:
            doc = json.load(f)
        grid = cls(doc["alpha"], doc["beta"], doc["t"])
        grid.meta = {k: v for k, v in doc.items() if k not in ("alpha", "beta", "t")}
        return grid


def ragc_cost_interp(grid: CostGrid, alpha: float, beta: float) -> float:
    out = _D()
    _check(_lib().ragc_cost_interp(ctypes.byref(grid.c), alpha, beta, ctypes.byref(out)))
    return out.value


@dataclass
class Plan:
    request_id: int
    matched_docs: int
    alpha: int
    beta: int
    block_table: np.ndarray
    swap_out_dev: np.ndarray
    swap_out_slot: np.ndarray
    swap_in_dev: np.ndarray
    swap_in_slot: np.ndarray
    evicted_gpu: np.ndarray
    evicted_host: np.ndarray


class Tree:
    def __init__(self, gpu_blocks: int, host_slots: int, grid: CostGrid):
        self._h = _lib().ragc_tree_create(gpu_blocks, host_slots, ctypes.byref(grid.c))
        if not self._h:
            raise B.RagcError(-1, B.load().ragc_last_error().decode())

    def close(self) -> None:
        if self._h:
            _lib().ragc_tree_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def begin(self, doc_ids: Sequence[int], doc_lens: Sequence[int], question_len: int) -> Plan:
        ids = np.ascontiguousarray(doc_ids, np.int64)
        lens = np.ascontiguousarray(doc_lens, np.int32)
        p = ragc_plan()
        _check(_lib().ragc_tree_begin(self._h, ids.ctypes.data, lens.ctypes.data, ids.size, question_len, ctypes.byref(p)))
        table = np.empty(p.n_blocks, np.int32)
        n_swap = max(p.n_swap_out, p.n_swap_in)
        n_ev = max(p.n_evicted_gpu, p.n_evicted_host)
        so_d, so_s, si_d, si_s = (np.empty(n_swap, np.int32) for _ in range(4))
        eg, eh = np.empty(n_ev, np.int64), np.empty(n_ev, np.int64)
        buf = ragc_plan_buffers(table.ctypes.data, table.size, so_d.ctypes.data, so_s.ctypes.data, si_d.ctypes.data,
                                si_s.ctypes.data, n_swap, eg.ctypes.data, eh.ctypes.data, n_ev)
        _check(_lib().ragc_tree_plan_read(self._h, p.request_id, ctypes.byref(buf)))
        return Plan(p.request_id, p.matched_docs, p.alpha, p.beta, table, so_d[:p.n_swap_out], so_s[:p.n_swap_out],
                    si_d[:p.n_swap_in], si_s[:p.n_swap_in], eg[:p.n_evicted_gpu], eh[:p.n_evicted_host])

    def end(self, request_id: int) -> None:
        _check(_lib().ragc_tree_end(self._h, request_id))

    def stats(self) -> ragc_tree_stats:
        s = ragc_tree_stats()
        _check(_lib().ragc_tree_get_stats(self._h, ctypes.byref(s)))
        return s

    def find(self, doc_path: Sequence[int]):
        """ragc_node_info of the node at the end of the path, or None if the path is not cached."""
        ids = np.ascontiguousarray(doc_path, np.int64)
        info = ragc_node_info()
        rc = _lib().ragc_tree_find(self._h, ids.ctypes.data, ids.size, ctypes.byref(info))
        if rc == B.RAGC_ERR_RANGE:
            return None
        _check(rc)
        return info

    def reset_frequencies(self) -> None:
        _check(_lib().ragc_tree_reset_frequencies(self._h))

    def peek(self, doc_ids: Sequence[int], doc_lens: Sequence[int], question_len: int):
        ids = np.ascontiguousarray(doc_ids, np.int64)
        lens = np.ascontiguousarray(doc_lens, np.int32)
        a, b = _I32(), _I32()
        _check(_lib().ragc_tree_peek(self._h, ids.ctypes.data, lens.ctypes.data, ids.size, question_len, ctypes.byref(a), ctypes.byref(b)))
        return a.value, b.value


class Queue:
    """ragc_queue_*: cache-aware reordering of waiting requests."""

    def __init__(self, window: int):
        self._h = _lib().ragc_queue_create(window)
        if not self._h:
            raise B.RagcError(-3, B.load().ragc_last_error().decode())

    def close(self) -> None:
        if self._h:
            _lib().ragc_queue_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def push(self, tag: int, doc_ids: Sequence[int], doc_lens: Sequence[int], question_len: int) -> None:
        ids = np.ascontiguousarray(doc_ids, np.int64)
        lens = np.ascontiguousarray(doc_lens, np.int32)
        _check(_lib().ragc_queue_push(self._h, tag, ids.ctypes.data, lens.ctypes.data, ids.size, question_len))

    def pop(self, tree: Tree) -> int:
        tag = _I64()
        _check(_lib().ragc_queue_pop(self._h, tree._h, ctypes.byref(tag)))
        return tag.value

    def __len__(self) -> int:
        return int(_lib().ragc_queue_size(self._h))
