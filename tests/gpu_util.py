"""Helpers of the GPU parity tests: run the oracle on a generated workload and
compare it with what the HIP path left in device memory."""
from __future__ import annotations

from typing import List, Optional, Tuple

import numpy as np

from oracle import attention as OA
from paper_2404_12457_amd import workload as W

# tolerances of the parity bar (max abs error against the fp64 oracle)
TOL = {"bf16": 2e-2, "f32": 1e-4}


def oracle_all(w: W.Workload) -> np.ndarray:
    """[sumN, Hq, D] float64 for the whole batch."""
    out = np.zeros((w.total_new, w.q_heads, w.head_dim), np.float64)
    for r in range(w.num_reqs):
        if int(w.new_len[r]) == 0:
            continue
        kf, vf = w.full_kv(r)
        s = w.new_slice(r)
        out[s] = OA.prefill_attn(W.to_f64(w.q[s], w.dtype), W.to_f64(kf, w.dtype), W.to_f64(vf, w.dtype),
                                 int(w.prefix_len[r]), w.softmax_scale)
    return out


def oracle_rows(w: W.Workload, r: int, rows: List[Tuple[int, int]]) -> np.ndarray:
    kf, vf = w.full_kv(r)
    s = w.new_slice(r)
    return OA.prefill_attn(W.to_f64(w.q[s], w.dtype), W.to_f64(kf, w.dtype), W.to_f64(vf, w.dtype),
                           int(w.prefix_len[r]), w.softmax_scale, rows=rows)


def sample_rows(w: W.Workload, r: int, count: int, seed: int) -> List[Tuple[int, int]]:
    """Rows (token, head) of request r: first, last, tile edges, and random ones."""
    n = int(w.new_len[r])
    g = np.random.Generator(np.random.Philox(key=[seed, r]))
    rows = {(0, 0), (n - 1, w.q_heads - 1), (n - 1, 0), (0, w.q_heads - 1)}
    G = w.q_heads // w.kv_heads
    for edge in (31, 32, 127, 128):  # wave and workgroup tile edges in packed rows
        tok = edge // G
        if tok < n:
            rows.add((tok, (edge % G)))
    while len(rows) < min(count, n * w.q_heads):
        rows.add((int(g.integers(0, n)), int(g.integers(0, w.q_heads))))
    return sorted(rows)


def out_to_f64(out_storage: np.ndarray, dtype: str) -> np.ndarray:
    return W.to_f64(out_storage, dtype)


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))
