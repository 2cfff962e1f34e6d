#!/usr/bin/env python3
"""Benchmark of the prefix-cached paged prefill path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 4] [--no-extras]

One step = one pass of the hot path over one batch of synthetic RAG-shaped input:
ragc_prefill_attn with the fused K/V append (block-table gather, QK^T, causal mask,
online softmax, PV, GQA grouping, new-token part, append, normalise + store).  The
headline workload is configuration 4 (LLaMA2-70B-shaped GQA layer, batch 4, 4096-token
cached prefix, 128 new tokens): the long-prefix, matrix-core-bound case on which the
metric "% of MFMA peak" is quoted.  Inputs are resident in HBM before the timed region;
several placements are rotated so that consecutive steps do not hit the same lines of
the 256 MB last-level cache.  Every other configuration is timed with the same number
of steps and gets its own roofline object under `other_workloads`.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
PCIE5_X16_GBS = 63.0


def _time_steps(fn, steps, warmup, torch):
    """Wall clock and HIP-event time of `steps` calls on the current stream."""
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def _rotating(index, copies, harness, W, one_pool):
    """`copies` instances of the configuration.  one_pool: the same data placed at disjoint
    blocks of ONE pool (cold data, warm address translations: what a long-running server
    sees); otherwise every instance has a pool of its own."""
    w0 = W.make_config(index)
    if copies == 1:
        return w0, [harness.DeviceWorkload(w0)]
    if not one_pool:
        return w0, [harness.DeviceWorkload(w0) for _ in range(copies)]
    per = int(sum((int(p) + int(n) + 15) // 16 for p, n in zip(w0.prefix_len, w0.new_len))) + 2  # blocks one placement can take
    dws = [harness.DeviceWorkload(w0)]
    for c in range(1, copies):
        wc = W.make_config(index, placement_skip=c * per)
        dws.append(harness.DeviceWorkload(wc, pool=(dws[0].pool_k, dws[0].pool_v)))
    return w0, dws


def bench_attention(index, steps, warmup, torch, harness, B, W, flags, copies=4, one_pool=True):
    w, dws = _rotating(index, copies, harness, W, one_pool)
    for d in dws:
        d.ensure_workspace(flags)
    wall_ms, ev_ms = _time_steps(lambda i: dws[i % copies].attn(flags), steps, warmup, torch)
    del dws
    torch.cuda.empty_cache()
    return w, wall_ms, ev_ms


def attn_bytes(w, fused):
    return w.attn_min_bytes() + (w.append_bytes() // 2 if fused else 0)  # fused append adds only the writes


def cpu_baseline(w, target_s=12.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the workload: whole
    requests on all threads, cycling through the batch until the time target (the rate of the
    best pass is also given), then a single-thread figure on a slice of rows of one request."""
    from oracle import attention as OA
    from paper_2404_12457_amd import workload as W

    threads = OA.max_threads()
    flops_done, t_used, reqs, toks, best = 0.0, 0.0, 0, 0, 0.0
    live = [r for r in range(w.num_reqs) if int(w.new_len[r]) > 0]
    for it in range(100000):
        r = live[it % len(live)]
        n, p = int(w.new_len[r]), int(w.prefix_len[r])
        kf, vf = w.full_kv(r)
        s = w.new_slice(r)
        q, k, v = W.to_f64(w.q[s], w.dtype), W.to_f64(kf, w.dtype), W.to_f64(vf, w.dtype)
        t0 = time.perf_counter()
        OA.prefill_attn(q, k, v, p, w.softmax_scale, threads=threads)
        dt = time.perf_counter() - t0
        fl = 4.0 * w.head_dim * w.q_heads * (n * p + n * (n + 1) // 2)
        t_used += dt
        flops_done += fl
        best = max(best, fl / dt)
        reqs += 1
        toks += n
        if t_used > target_s and reqs >= 3:
            break
    # one thread: the first 8 tokens (all heads) of the first request, best of 3
    r = live[0]
    n, p = int(w.new_len[r]), int(w.prefix_len[r])
    kf, vf = w.full_kv(r)
    s = w.new_slice(r)
    q, k, v = W.to_f64(w.q[s], w.dtype), W.to_f64(kf, w.dtype), W.to_f64(vf, w.dtype)
    ntok = min(8, n)
    rows = [(i, h) for i in range(ntok) for h in range(w.q_heads)]
    fl1 = 4.0 * w.head_dim * w.q_heads * sum(p + i + 1 for i in range(ntok))
    t1 = []
    for _ in range(3):
        t0 = time.perf_counter()
        OA.prefill_attn(q, k, v, p, w.softmax_scale, rows=rows, threads=1)
        t1.append(time.perf_counter() - t0)
    return {"value": flops_done / t_used / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"{reqs} request passes (cycling the {len(live)} requests of {w.name}), all rows, fp64, {t_used:.1f} s",
            "best_pass_tflops": best / 1e12, "new_tokens_per_s": float(toks / t_used),
            "single_thread": {"value": fl1 / min(t1) / 1e12, "unit": "TFLOP/s", "cores": 1,
                              "sample": f"first {ntok} tokens x {w.q_heads} heads of request {r}, best of 3, {min(t1):.2f} s"}}


def read_traffic(kernel_tag):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if present."""
    path = os.path.join(ROOT, "profiles", f"{kernel_tag}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split()[1])
    except OSError:
        pass
    return None


def roofline_of(w, ev_ms, tag):
    """The roofline object of one attention launch: bound by whichever of the two published
    peaks gives the longer time for the algorithmic work of this batch."""
    flops, nbytes = w.attn_flops(), attn_bytes(w, True)
    ach_gbs = nbytes / (ev_ms * 1e-3) / 1e9
    ach_tfl = flops / (ev_ms * 1e-3) / 1e12
    hbm_bound = (nbytes / (HBM_PEAK_GBS * 1e9)) > (flops / (MFMA_BF16_PEAK_TFLOPS * 1e12))
    if w.dtype != "bf16":
        roof = {"bound": "latency", "achieved": ach_tfl, "peak": None, "unit": "TFLOP/s", "frac": None}
    elif hbm_bound:
        roof = {"bound": "hbm", "achieved": ach_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach_gbs / HBM_PEAK_GBS}
    else:
        roof = {"bound": "mfma", "achieved": ach_tfl, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach_tfl / MFMA_BF16_PEAK_TFLOPS}
    roof.update({"kernel": "attn_bf16_kernel<128>" if w.dtype == "bf16" else "attn_f32_kernel<64>", "kernel_ms": ev_ms,
                 "algorithmic_bytes": nbytes, "flops": flops, "mfma_frac": ach_tfl / MFMA_BF16_PEAK_TFLOPS,
                 "hbm_frac": ach_gbs / HBM_PEAK_GBS, "traffic": read_traffic(tag)})
    return roof


def calibrate(torch):
    """What this machine sustains on plain kernels (libragc_calib.so): a register-only bf16 MFMA loop
    on random operands with the whole chip busy, a streaming device copy, pinned-memory copies
    over the host link.  The shader clock under that MFMA load follows from the loop's rate: a
    32x32x16 MFMA occupies a SIMD's matrix core for 32 cycles."""
    import ctypes

    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2404_12457_amd", "libragc_calib.so"))
    P, I32, I64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.ragc_calib_mfma.argtypes = [P, P, P, I32, I32, P]
    lib.ragc_calib_copy.argtypes = [P, P, I64, I32, P]
    props = torch.cuda.get_device_properties(0)
    cus = props.multi_processor_count
    st = torch.cuda.current_stream().cuda_stream
    out = {"compute_units": cus}
    # matrix cores: two 4-wave workgroups per CU, 2 waves per SIMD
    wgs, iters = 2 * cus, 20000
    waves = wgs * 4
    sink = torch.empty(waves * 64, dtype=torch.float32, device="cuda")
    clocks = torch.zeros(waves * 2, dtype=torch.int64, device="cuda")
    for name, fill in (("random", lambda n: torch.randn(n, device="cuda").mul_(0.5)), ("constant", lambda n: torch.ones(n, device="cuda"))):
        ops = fill(64 * 2048).to(torch.bfloat16)

        def run(i):
            rc = lib.ragc_calib_mfma(ops.data_ptr(), sink.data_ptr(), clocks.data_ptr(), wgs, iters, st)
            assert rc == 0, rc

        _, em = _time_steps(run, 5, 2, torch)
        tfl = waves * iters * 8 * 32768 / (em * 1e-3) / 1e12
        out[f"mfma_tflops_{name}_operands"] = tfl
        out[f"sclk_mhz_under_mfma_load_{name}"] = tfl * 1e12 / (cus * 4 * 1024) / 1e6
        c = clocks.view(-1, 2).double()
        if float(c[:, 1].min()) > 0:  # shader-clock ticks per 100 MHz tick, as the kernel itself read them
            out[f"s_memtime_ticks_per_us_{name}"] = float((c[:, 0] / c[:, 1]).median()) * 100.0
    out["mfma_tflops"] = out["mfma_tflops_random_operands"]
    out["sclk_mhz_under_load"] = out["sclk_mhz_under_mfma_load_random"]
    # streaming copy, 1 GiB each way per call (far above the 256 MB last-level cache)
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    best = 0.0
    for wg in (cus * 4, cus * 8, cus * 16, cus * 32):
        def run(i):
            rc = lib.ragc_calib_copy(dst.data_ptr(), src.data_ptr(), n, wg, st)
            assert rc == 0, rc

        _, em = _time_steps(run, 5, 2, torch)
        best = max(best, 2 * n / (em * 1e-3) / 1e9)
    out["copy_gbs"] = best  # bytes read + bytes written per second
    _, em = _time_steps(lambda i: dst.copy_(src), 5, 2, torch)
    out["runtime_d2d_copy_gbs"] = 2 * n / (em * 1e-3) / 1e9
    del dst
    # host link: pinned memory, 256 MiB per copy
    m = 256 << 20
    pin = torch.empty(m, dtype=torch.uint8).pin_memory()
    _, em = _time_steps(lambda i: src[:m].copy_(pin, non_blocking=True), 5, 2, torch)
    out["h2d_gbs"] = m / (em * 1e-3) / 1e9
    _, em = _time_steps(lambda i: pin.copy_(src[:m], non_blocking=True), 5, 2, torch)
    out["d2h_gbs"] = m / (em * 1e-3) / 1e9
    del src, pin, sink, clocks
    torch.cuda.empty_cache()
    return out


GRID_ALPHAS = [0, 256, 512, 768, 1024, 1280, 1536, 2048, 2560, 3072, 4096, 5120, 6144, 8192]
# T steps with the number of 128-row tiles of a request (beta rows per head here), so the grid has a
# point on either side of every step: linear interpolation between them then follows the staircase
GRID_BETAS = [1] + [x for k in range(1, 9) for x in (128 * k, 128 * k + 1)][:-1]
GRID_BATCH = 8


def measure_cost_grid(harness, W, B, torch, write_path=None, quick=False):
    """T(alpha, beta) of the paper's cost model (Sec. 5.1, Algorithm 1), measured with this kernel:
    the time of one layer's attention with the fused append for a batch of GRID_BATCH requests with
    alpha cached and beta non-cached tokens each, LLaMA2-7B head shape, divided by GRID_BATCH.  A
    batch (Sec. 7: the system batches several requests per prefill iteration) fills the chip, so T
    is the cost a request adds under load and is smooth in alpha and beta; a lone request would be
    split along its keys in steps.  The grid is measured twice (the spread is the run-to-run noise
    the policy has to tolerate); off-grid points are then measured as well and compared with what
    ragc_cost_interp returns for them."""
    from paper_2404_12457_amd import ctl

    probes = [(768, 96), (1280, 48), (1792, 192), (2560, 384), (3584, 700), (300, 700), (5000, 40), (7000, 200), (640, 600), (4500, 900)]

    # Timing only: random K/V written on the device, every request on blocks of its own (no sharing,
    # so every request's prefix comes from HBM), no oracle-consistent generator in the loop.
    hq = hkv = 32
    d = 128
    per_req = (max(GRID_ALPHAS) + max(GRID_BETAS) + 15) // 16
    nblk = GRID_BATCH * per_req
    pool_k = torch.randn(nblk, hkv, 16, d, device="cuda").mul_(0.5).to(torch.bfloat16)
    pool_v = torch.randn(nblk, hkv, 16, d, device="cuda").mul_(0.5).to(torch.bfloat16)
    pool = B.make_pool(pool_k, pool_v, nblk, hkv, d, B.RAGC_DTYPE_BF16)
    h_table = np.arange(nblk, dtype=np.int32).reshape(GRID_BATCH, per_req)
    d_table = torch.from_numpy(h_table).cuda()
    nmax = GRID_BATCH * max(GRID_BETAS)
    q = torch.randn(nmax, hq, d, device="cuda").mul_(0.5).to(torch.bfloat16)
    kn = torch.randn(nmax, hkv, d, device="cuda").mul_(0.5).to(torch.bfloat16)
    vn = torch.randn(nmax, hkv, d, device="cuda").mul_(0.5).to(torch.bfloat16)
    out = torch.empty_like(q)
    scale = 1.0 / float(np.sqrt(d))
    st = torch.cuda.current_stream().cuda_stream

    def one(a, b):
        hp, hn = np.full(GRID_BATCH, a, np.int32), np.full(GRID_BATCH, b, np.int32)
        hs = (np.arange(GRID_BATCH + 1) * b).astype(np.int32)
        dev = [torch.from_numpy(x).cuda() for x in (hp, hn, hs)]
        batch = B.make_batch(GRID_BATCH, per_req, dev[0], dev[1], dev[2], d_table, hp, hn, hs, h_table)
        ws, nb = harness.workspace_for(pool, batch, hq, B.RAGC_ATTN_APPEND_FUSED)
        call = lambda i: B.ragc_prefill_attn(pool, batch, q, kn, vn, out, hq, scale, B.RAGC_ATTN_APPEND_FUSED, ws, nb, st)
        em = sorted(_time_steps(call, 12 if quick else 40, 10 if seg == 0 else 0, torch)[1] for seg in range(3))[1]  # median of three segments
        return em * 1e3 / GRID_BATCH  # microseconds per request

    runs = []
    for rep in range(1 if quick else 2):  # quick: one pass with short segments (the default benchmark run)
        rows = []
        for a in GRID_ALPHAS:
            rows.append([one(a, b) for b in GRID_BETAS])
            print(f"cost grid run {rep}: alpha {a} done", file=sys.stderr, flush=True)
        runs.append(np.asarray(rows))
    t = sum(runs) / len(runs)
    noise = float(np.max(np.abs(runs[0] - runs[-1]) / t)) if len(runs) > 1 else None
    grid = ctl.CostGrid(GRID_ALPHAS, GRID_BETAS, t)
    check = []
    for a, b in probes:
        m, e = one(a, b), ctl.ragc_cost_interp(grid, a, b)
        check.append({"alpha": a, "beta": b, "measured_us": m, "interpolated_us": e, "rel_err": abs(e - m) / m})
    torch.cuda.empty_cache()
    shape = f"batch of {GRID_BATCH} equal requests, 32 heads MHA, head_dim 128, bf16, one layer, fused append; per request"
    res = {"shape": shape, "alpha": GRID_ALPHAS, "beta": GRID_BETAS, "t_us": t.tolist(), "run_to_run_rel_noise": noise,
           "off_grid": check, "max_rel_err": max(c["rel_err"] for c in check)}
    if write_path:
        grid.save(write_path, unit="us", shape=shape, device=torch.cuda.get_device_name(0), run_to_run_rel_noise=noise,
                  off_grid_max_rel_err=res["max_rel_err"], written_by="python bench.py --write-cost-grid")
    return res


DECODE_SHAPES = (("R64_P1024_gqa32/8", 64, 1024, 32, 8), ("R128_P2048_gqa32/8", 128, 2048, 32, 8),
                 ("R8_P1024_mha32", 8, 1024, 32, 32), ("R4_P4096_gqa64/8", 4, 4096, 64, 8))


def measure_decode(harness, W, B, torch, only=None):
    """Decode steps (one new token per request) on the same pool and kernel: the K/V of every
    request is read once, so the figure of merit is K/V bytes per second against the HBM peak.
    The same data is read every step (warm in the last-level cache when it fits)."""
    out = {}
    for name, R, P, hq, hkv in DECODE_SHAPES:
        if only is not None and name != only:
            continue
        w = W.make_small("bf16", hq, hkv, 128, [(P, 1)] * R, seed=3, sigma=0.5)
        dw = harness.DeviceWorkload(w)
        _, em = _time_steps(lambda i: dw.attn(B.RAGC_ATTN_APPEND_FUSED), 30, 5, torch)
        kv = R * (P + 1) * hkv * 128 * 2 * 2
        out[name] = {"us": em * 1e3, "kv_bytes": kv, "gbs": kv / em / 1e6, "hbm_frac": kv / em / 1e6 / HBM_PEAK_GBS,
                     "split_workspace_bytes": int(dw.workspace_bytes)}
        del dw
    torch.cuda.empty_cache()
    return out


def measure_layer_prefetch(harness, B, torch):
    """One request through 8 layers, each with its own pool: 4096 cached tokens that live in
    pinned host memory (256 blocks per layer to bring in) and 512 new tokens, Mistral-7B head
    shape.  Serial: copy then attention, layer after layer, on one stream.  Prefetch: the copies
    of layer l+1 run on a side stream under the attention of layer l."""
    from paper_2404_12457_amd import ctl

    layers, hq, hkv, d, alpha, beta = 8, 32, 8, 128, 4096, 512
    nblk = (alpha + beta) // 16
    cache = harness.LayeredCache(layers, 1024, 512, hkv, d)
    for l in range(layers):
        cache.host_k[l].normal_(0, 0.5)
        cache.host_v[l].normal_(0, 0.5)
    i32 = lambda n: np.arange(n, dtype=np.int32)
    e32, e64 = np.empty(0, np.int32), np.empty(0, np.int64)
    plan = ctl.Plan(1, 1, alpha, beta, i32(nblk), e32, e32, i32(alpha // 16), i32(alpha // 16), e64, e64)
    q = [torch.randn(beta, hq, d, device="cuda").mul_(0.5).to(torch.bfloat16) for _ in range(layers)]
    kn = [torch.randn(beta, hkv, d, device="cuda").mul_(0.5).to(torch.bfloat16) for _ in range(layers)]
    vn = [torch.randn(beta, hkv, d, device="cuda").mul_(0.5).to(torch.bfloat16) for _ in range(layers)]
    scale = 1.0 / float(np.sqrt(d))
    res = {}
    for name, pf in (("serial_ms", False), ("prefetch_ms", True)):
        _, em = _time_steps(lambda i: cache.execute(plan, q, kn, vn, hq, scale, prefetch=pf), 10, 2, torch)
        cache.side.synchronize()
        res[name] = em
    noswap = ctl.Plan(1, 1, alpha, beta, i32(nblk), e32, e32, e32, e32, e64, e64)
    _, em = _time_steps(lambda i: cache.execute(noswap, q, kn, vn, hq, scale, prefetch=False), 10, 2, torch)
    res["attention_only_ms"] = em
    res.update({"layers": layers, "blocks_swapped_in_per_layer": alpha // 16, "bytes_swapped_in": layers * (alpha // 16) * 2 * hkv * 16 * d * 2,
                "shape": "1 request, 32/8 heads, head_dim 128, bf16, alpha 4096 (host-resident), beta 512"})
    del cache
    torch.cuda.empty_cache()
    return res


def measure_controller():
    """The C++ knowledge tree on a Zipf(1.1) trace over 10,000 documents of 256-1024 tokens, top-2
    retrieval, through the Python binding (begin + plan_read + end per request)."""
    from paper_2404_12457_amd import ctl

    rng = np.random.Generator(np.random.Philox(key=[7, 7]))
    ndocs, nreq = 10000, 20000
    lens = rng.integers(256, 1025, ndocs)
    ranks = np.minimum(rng.zipf(1.1, (nreq, 2)) - 1, ndocs - 1)
    grid = ctl.CostGrid.load(ctl.MEASURED_GRID)  # T(alpha, beta) as measured with the attention kernel on an MI355X
    tree = ctl.Tree(8192, 65536, grid)
    t0 = time.perf_counter()
    for i in range(nreq):
        docs = [int(ranks[i, 0])] + ([int(ranks[i, 1])] if ranks[i, 1] != ranks[i, 0] else [])
        p = tree.begin(docs, [int(lens[d]) for d in docs], 100)
        tree.end(p.request_id)
    dt = time.perf_counter() - t0
    s = tree.stats()
    return {"requests": nreq, "requests_per_s": nreq / dt, "hit_rate": s.docs_hit / s.docs_requested, "nodes": int(s.nodes),
            "blocks_swapped_out": int(s.blocks_swapped_out), "blocks_swapped_in": int(s.blocks_swapped_in),
            "zero_copy_evictions": int(s.zero_copy_evictions), "gpu_blocks": 8192, "host_slots": 65536,
            "cost_grid": os.path.relpath(ctl.MEASURED_GRID, ROOT)}



def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=4, help="configuration index for the headline line (2, 3 or 4)")
    ap.add_argument("--no-extras", action="store_true", help="skip the other configurations, append and swap figures")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-calibration", action="store_true", help="skip the MFMA / copy / host-link calibration kernels")
    ap.add_argument("--pool-copies", type=int, default=4,
                    help="pool copies rotated between steps (1 = every step re-reads the same, cache-warm buffers)")
    ap.add_argument("--separate-pools", action="store_true",
                    help="give every rotated copy a pool of its own instead of disjoint blocks of one pool")
    ap.add_argument("--force-variant", type=int, default=-1, help="debug: kernel variant for every bf16 attention call (-1 = library's choice)")
    ap.add_argument("--force-splits", type=int, default=0, help="debug: copies of every work item along the keys (0 = library's choice)")
    ap.add_argument("--write-cost-grid", metavar="PATH", default=None,
                    help="measure T(alpha, beta) and write it as a JSON file that ctl.CostGrid.load reads; nothing else runs")
    ap.add_argument("--decode-only", metavar="SHAPE", default=None,
                    help="time one decode shape only (%s) and print its figures: the run to put under rocprofv3" % ", ".join(n for n, *_ in DECODE_SHAPES))
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run a plain 512 MiB device copy three times (scale for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; the path issues no collective and --gpus > 1 is not supported")

    import torch

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    from paper_2404_12457_amd import binding as B
    from paper_2404_12457_amd import harness
    from paper_2404_12457_amd import workload as W

    B.load()  # fails loudly if libragc.so is missing
    if args.force_variant >= 0 or args.force_splits > 0:
        B.ragc_debug_set_attn_plan(args.force_variant, args.force_splits)
    if args.write_cost_grid:
        res = measure_cost_grid(harness, W, B, torch, write_path=args.write_cost_grid)
        print(json.dumps({k: res[k] for k in ("run_to_run_rel_noise", "max_rel_err", "off_grid")}))
        return
    if args.decode_only:
        print(json.dumps(measure_decode(harness, W, B, torch, only=args.decode_only)))
        return
    if args.calibrate_copy:
        src = torch.ones(512 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)  # reads 512 MiB, writes 512 MiB
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    FUSED = B.RAGC_ATTN_APPEND_FUSED
    w, wall_ms, ev_ms = bench_attention(args.workload, args.steps, args.warmup, torch, harness, B, W, FUSED,
                                        copies=args.pool_copies, one_pool=not args.separate_pools)
    flops = w.attn_flops()
    tflops = flops / (wall_ms * 1e-3) / 1e12
    roof = roofline_of(w, ev_ms, f"attn_bf16_C{args.workload}")

    result = {
        "metric": "prefix-cached prefill attention TFLOP/s + new-tokens/s; % of MFMA peak",
        "value": tflops, "unit": "TFLOP/s", "new_tokens_per_s": w.total_new / (wall_ms * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "requests": w.num_reqs, "q_heads": w.q_heads, "kv_heads": w.kv_heads,
                   "head_dim": w.head_dim, "prefix_tokens": int(w.prefix_len.sum()), "new_tokens": w.total_new,
                   "block_size": 16, "pool_blocks": w.num_blocks, "fused_append": True, "placements_rotated": args.pool_copies, "one_pool": not args.separate_pools},
        "roofline": roof,
    }

    if not args.no_extras:
        extras = {}
        steps2, warm2 = max(20, args.steps // 4), max(5, args.warmup // 2)
        for idx in (1, 2, 3, 4):
            if idx == args.workload:
                continue
            # same number of steps as the headline, so that these figures and the profiler's agree
            wx, wm, em = bench_attention(idx, args.steps, args.warmup, torch, harness, B, W, FUSED, copies=4 if idx != 1 else 1,
                                         one_pool=not args.separate_pools)
            extras[f"C{idx}"] = {"workload": wx.name, "ms_per_step": wm, "tflops": wx.attn_flops() / wm / 1e9,
                                 "new_tokens_per_s": wx.total_new / (wm * 1e-3),
                                 "roofline": roofline_of(wx, em, f"attn_bf16_C{idx}" if idx != 1 else "attn_f32_C1")}
        # standalone append: at the workload's size and on a scaled sweep of the same row shape
        for idx in (2, 3):
            wa = W.make_config(idx)
            dw = harness.DeviceWorkload(wa)
            _, em = _time_steps(lambda i: dw.append(), steps2, warm2, torch)
            extras[f"append_C{idx}"] = {"bytes": wa.append_bytes(), "kernel_ms": em, "gbs": wa.append_bytes() / em / 1e6,
                                        "hbm_frac": wa.append_bytes() / em / 1e6 / HBM_PEAK_GBS}
            del dw
        big = W.build_workload("append-sweep", "bf16", 8, 8, 128, 1 << 17,
                               [W.RequestSpec([], 65536) for _ in range(16)], seed=7)
        dwb = harness.DeviceWorkload(big)
        _, em = _time_steps(lambda i: dwb.append(), 20, 3, torch)
        extras["append_sweep"] = {"bytes": big.append_bytes(), "kernel_ms": em, "gbs": big.append_bytes() / em / 1e6,
                                  "hbm_frac": big.append_bytes() / em / 1e6 / HBM_PEAK_GBS}
        del dwb, big
        torch.cuda.empty_cache()
        # host tier: swap-in of the host-resident blocks of configuration 5, both mechanisms
        w5 = W.make_config(5)
        d5 = harness.DeviceWorkload(w5, resident_host_blocks=False)
        sw_bytes = int(w5.host_dev_blocks.size) * 2 * w5.kv_heads * 16 * w5.head_dim * 2
        side = torch.cuda.Stream()
        for name, mode in (("kernel", B.RAGC_SWAP_KERNEL), ("memcpy", B.RAGC_SWAP_MEMCPY)):
            with torch.cuda.stream(side):
                _, em = _time_steps(lambda i: d5.swap(w5.host_dev_blocks, w5.host_slots, B.RAGC_SWAP_TO_DEVICE, mode,
                                                      stream=side.cuda_stream), 10, 2, torch)
            extras[f"swap_in_{name}"] = {"blocks": int(w5.host_dev_blocks.size), "bytes": sw_bytes, "ms": em,
                                         "gbs": sw_bytes / em / 1e6, "pcie5_x16_frac": sw_bytes / em / 1e6 / PCIE5_X16_GBS}
        with torch.cuda.stream(side):
            _, em = _time_steps(lambda i: d5.swap(w5.host_dev_blocks, w5.host_slots, B.RAGC_SWAP_TO_HOST, B.RAGC_SWAP_KERNEL,
                                                  stream=side.cuda_stream), 10, 2, torch)
        extras["swap_out_kernel"] = {"bytes": sw_bytes, "ms": em, "gbs": sw_bytes / em / 1e6,
                                     "pcie5_x16_frac": sw_bytes / em / 1e6 / PCIE5_X16_GBS}
        # whole batch resident; then the real flow: swap-in on the side stream while the
        # requests that are already resident run, the others wait on the event
        _, em_alone = _time_steps(lambda i: d5.attn(FUSED), 20, 3, torch)
        res_idx = [r for r in range(w5.num_reqs) if not w5.needs_swap[r]]
        swp_idx = [r for r in range(w5.num_reqs) if w5.needs_swap[r]]
        b_res, keep1 = d5.sub_batch(res_idx)
        b_swp, keep2 = d5.sub_batch(swp_idx)
        ev = torch.cuda.Event()

        def serial(i):
            d5.swap(w5.host_dev_blocks, w5.host_slots, B.RAGC_SWAP_TO_DEVICE, 0)
            d5.attn(FUSED)

        def overlapped(i):
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                d5.swap(w5.host_dev_blocks, w5.host_slots, B.RAGC_SWAP_TO_DEVICE, 0, stream=side.cuda_stream)
                ev.record(side)
            d5.attn_batch(b_res, FUSED)
            torch.cuda.current_stream().wait_event(ev)
            d5.attn_batch(b_swp, FUSED)

        _, em_ser = _time_steps(serial, 10, 2, torch)
        _, em_ovl = _time_steps(overlapped, 10, 2, torch)
        side.synchronize()
        extras["C5"] = {"workload": w5.name, "requests_resident": len(res_idx), "requests_waiting_for_swap": len(swp_idx),
                        "attn_ms_all_resident": em_alone, "swap_then_attn_ms": em_ser, "swap_overlapped_with_attn_ms": em_ovl,
                        "tflops_all_resident": w5.attn_flops() / em_alone / 1e9,
                        "roofline_all_resident": roofline_of(w5, em_alone, "attn_bf16_C5")}
        del d5
        torch.cuda.empty_cache()
        # the controller side: measured cost model, layer-ahead copies over per-layer pools, tree throughput
        extras["cost_grid"] = measure_cost_grid(harness, W, B, torch, quick=True)
        extras["decode"] = measure_decode(harness, W, B, torch)
        extras["layer_prefetch"] = measure_layer_prefetch(harness, B, torch)
        extras["controller"] = measure_controller()
        result["other_workloads"] = extras

    if not args.no_calibration:
        result["calibration"] = calibrate(torch)
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
