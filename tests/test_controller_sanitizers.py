"""The controller (csrc/ragc_ctl.cpp: raw node pointers, ordered-set erases, free lists) built for
the CPU with AddressSanitizer and UndefinedBehaviorSanitizer and driven through its C ABI on seeded
traces: no report may appear, and every decision must equal what the shipped library (and, through
tests/test_controller_parity.py, the oracle) gives for the same trace.  CPU only."""
import os
import random
import shutil
import subprocess

import numpy as np
import pytest

from paper_2404_12457_amd import binding as B
from paper_2404_12457_amd import ctl as C

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ALPHAS = [0.0, 256.0, 1024.0, 4096.0]
BETAS = [1.0, 64.0, 256.0, 1024.0, 4096.0]


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    out = str(tmp_path_factory.mktemp("san") / "ctl_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-I/opt/rocm/include", "-D__HIP_PLATFORM_AMD__",
           os.path.join(ROOT, "tests", "ctl_sanitizer_driver.cpp"),
           os.path.join(ROOT, "paper_2404_12457_amd", "csrc", "ragc_ctl.cpp"), "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    return out


def _docs(ids, lens):
    return " ".join(f"{i} {l}" for i, l in zip(ids, lens))


def _trace(gpu_blocks, host_slots, ndocs, seed, steps):
    """Operations as text lines plus what the shipped library answers to each."""
    rng = random.Random(seed)
    f = lambda a, b: 3.0 + 0.004 * a + 0.11 * b + 2.5e-5 * a * b
    t = [[f(a, b) for b in BETAS] for a in ALPHAS]
    tree = C.Tree(gpu_blocks, host_slots, C.CostGrid(ALPHAS, BETAS, t))
    head = f"{gpu_blocks} {host_slots} {len(ALPHAS)} {len(BETAS)} " + " ".join(map(repr, ALPHAS + BETAS + [x for row in t for x in row]))
    ops, want, live = [], [], []
    lens = {d: rng.choice([rng.randrange(1, 16), rng.randrange(16, 200), 16 * rng.randrange(1, 9)]) for d in range(ndocs)}
    for step in range(steps):
        if live and (len(live) >= 3 or rng.random() < 0.5):
            k = rng.randrange(len(live))
            tree.end(live.pop(k))
            ops.append(f"E {k}")
            want.append("E 0")
        docs = list(dict.fromkeys(min(int(rng.paretovariate(1.05)) - 1, ndocs - 1) for _ in range(rng.randrange(0, 5))))
        q = rng.randrange(0 if docs else 1, 50)
        dl = [lens[d] for d in docs]
        if step % 7 == 3:
            ops.append(f"P {len(docs)} {q} {_docs(docs, dl)}")
            a, b = tree.peek(docs, dl, q)
            want.append(f"P 0 {a} {b}")
        ops.append(f"B {len(docs)} {q} {_docs(docs, dl)}")
        try:
            p = tree.begin(docs, dl, q)
        except B.RagcError as e:
            want.append(f"B {e.code}")
            continue
        live.append(p.request_id)
        pairs = lambda d, s: "".join(f" {x}:{y}" for x, y in zip(d.tolist(), s.tolist()))
        want.append(f"B 0 {p.request_id} {p.matched_docs} {p.alpha} {p.beta} T" + "".join(f" {x}" for x in p.block_table.tolist()) +
                    " O" + pairs(p.swap_out_dev, p.swap_out_slot) + " I" + pairs(p.swap_in_dev, p.swap_in_slot) +
                    " G" + "".join(f" {x}" for x in p.evicted_gpu.tolist()) + " H" + "".join(f" {x}" for x in p.evicted_host.tolist()))
        if step == steps // 2:
            tree.reset_frequencies()
            ops.append("R")
            want.append("R 0")
        if step % 97 == 50:  # a reorder queue against the tree as it is now
            waiting = []
            for tag in range(6):
                wd = list(dict.fromkeys(min(int(rng.paretovariate(1.05)) - 1, ndocs - 1) for _ in range(rng.randrange(1, 4))))
                waiting.append((tag, wd, [lens[d] for d in wd], rng.randrange(1, 40)))
            qu = C.Queue(3)
            for tag, wd, wl, wq in waiting:
                qu.push(tag, wd, wl, wq)
            order = [qu.pop(tree) for _ in range(len(waiting))]
            qu.close()
            ops.append(f"Q 3 {len(waiting)} " + " ".join(f"{tag} {len(wd)} {wq} {_docs(wd, wl)}" for tag, wd, wl, wq in waiting))
            want.append("Q" + "".join(f" {x}" for x in order))
    s = tree.stats()
    want.append(f"S {s.nodes} {s.nodes_in_gpu} {s.free_gpu_blocks} {s.free_host_slots} {s.docs_requested} {s.docs_hit} "
                f"{s.blocks_swapped_out} {s.blocks_swapped_in} {s.zero_copy_evictions}")
    return head + "\n" + "\n".join(ops) + "\n", want


@pytest.mark.parametrize("gpu_blocks,host_slots,ndocs,seed", [(48, 96, 40, 1), (24, 12, 25, 2), (400, 0, 60, 3), (64, 4096, 200, 4)])
def test_controller_under_asan_and_ubsan_matches_the_shipped_library(driver, tmp_path, gpu_blocks, host_slots, ndocs, seed):
    text, want = _trace(gpu_blocks, host_slots, ndocs, seed, 800)
    path = tmp_path / "trace.txt"
    path.write_text(text)
    # verify_asan_link_order=0: whatever the environment preloads stays in place; the runtime then does not insist on being first
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([driver, str(path)], capture_output=True, text=True, env=env, timeout=300)
    assert "AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr and "LeakSanitizer" not in res.stderr, res.stderr[-4000:]
    assert res.returncode == 0, (res.returncode, res.stderr[-2000:])
    got = res.stdout.strip().split("\n")
    assert len(got) == len(want)
    for i, (g, w) in enumerate(zip(got, want)):
        assert g == w, f"operation {i}: sanitized build says {g!r}, shipped library {w!r}"
    assert sum(w.startswith("B 0") for w in want) > 300
