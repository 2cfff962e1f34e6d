"""The entry point for callers that cannot allocate (ragc_prefill_attn_static): its partial
results live in an array that is part of the library's device image.  It must give what
ragc_prefill_attn gives with a caller-owned workspace -- same kernels, same plan, so the same
bits -- on two calls in a row, the second with a smaller input (the array keeps the first
call's contents), and the oracle's answer within the usual tolerance."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2404_12457_amd import binding as B
from paper_2404_12457_amd import workload as W

import gpu_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2404_12457_amd import harness

    B.load()
    return harness


def _both(H, w, flags):
    """(static-scratch output, workspace output, pools after each) for one workload."""
    a, b = H.DeviceWorkload(w), H.DeviceWorkload(w)
    st = torch.cuda.current_stream().cuda_stream
    assert B.ragc_prefill_attn_workspace(a.pool, a.batch, w.q_heads, flags) > 0, "the case must be split along its keys"
    B.ragc_prefill_attn_static(a.pool, a.batch, a.q, a.k_new, a.v_new, a.out, w.q_heads, w.softmax_scale, flags, st)
    b.attn(flags)
    torch.cuda.synchronize()
    return a, b


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row(H):
    flags = B.RAGC_ATTN_APPEND_FUSED
    first = W.make_small("bf16", 32, 8, 128, [(4096, 48), (3000, 1), (2500, 70)], seed=8801, q_gain=4.0)
    second = W.make_small("bf16", 8, 2, 128, [(1500, 17)], seed=8802, q_gain=4.0)  # smaller: fewer and shorter partial results
    for w in (first, second):
        a, b = _both(H, w, flags)
        assert torch.equal(a.out.view(torch.int16), b.out.view(torch.int16))
        assert torch.equal(a.pool_k.view(torch.int16), b.pool_k.view(torch.int16))
        assert torch.equal(a.pool_v.view(torch.int16), b.pool_v.view(torch.int16))
        got = U.out_to_f64(H.to_host(a.out), "bf16")
        want = U.oracle_all(w)
        assert np.all(np.isfinite(got))
        assert float(np.max(np.abs(got - want))) <= U.TOL["bf16"]
        assert U.rel_l2(got, want) <= 1e-2


def test_static_scratch_entry_point_without_a_split_and_in_fp32(H):
    """Batches that need no partial results take the same path as ragc_prefill_attn."""
    for w in (W.make_config(1), W.make_small("bf16", 8, 2, 128, [(100, 70), (37, 5), (0, 130)] * 40, seed=8803)):
        a, b = H.DeviceWorkload(w), H.DeviceWorkload(w)
        st = torch.cuda.current_stream().cuda_stream
        B.ragc_prefill_attn_static(a.pool, a.batch, a.q, a.k_new, a.v_new, a.out, w.q_heads, w.softmax_scale, 0, st)
        b.attn(0)
        torch.cuda.synchronize()
        bits = torch.int16 if w.dtype == "bf16" else torch.int32
        assert torch.equal(a.out.view(bits), b.out.view(bits))


def test_static_scratch_entry_point_rejects_what_does_not_fit(H):
    """Forced to 16 copies of each of 24 work items x 2 kv heads the partial results need 51 MB."""
    w = W.make_small("bf16", 8, 2, 128, [(2000, 40)] * 24, seed=8804)
    dw = H.DeviceWorkload(w)
    try:
        B.ragc_debug_set_attn_plan(-1, 16)
        with pytest.raises(B.RagcError) as e:
            B.ragc_prefill_attn_static(dw.pool, dw.batch, dw.q, dw.k_new, dw.v_new, dw.out, w.q_heads, w.softmax_scale, 0,
                                       torch.cuda.current_stream().cuda_stream)
        assert e.value.code == B.RAGC_ERR_WORKSPACE
    finally:
        B.ragc_debug_set_attn_plan(-1, 0)
