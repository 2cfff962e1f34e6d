"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before touching the
device."""
import os
import re

import numpy as np
import pytest

from paper_2404_12457_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2404_12457_amd import build

        build.build()
    return B.load()


@pytest.mark.parametrize("header_name,exports", [("ragc.h", "binding"), ("ragc_ctl.h", "ctl")])
def test_every_declared_symbol_is_exported(lib, header_name, exports):
    from paper_2404_12457_amd import ctl

    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(ragc_[a-z_0-9]+)\s*\(", header))
    assert names == set(B.EXPORTS if exports == "binding" else ctl.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_kv_bytes_per_token_match_the_model_table(lib):
    assert B.ragc_version() >= 100
    for line in open(os.path.join(ROOT, "tests", "golden", "kv_bytes_per_token.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, layers, hq, hkv, mib = line.split()
        assert B.ragc_kv_bytes_per_token(int(layers), int(hkv), 128, B.RAGC_DTYPE_BF16) == float(mib) * 2**20, name
    assert B.ragc_kv_bytes_per_token(0, 8, 128, 1) == 0 and B.ragc_kv_bytes_per_token(32, 8, 128, 7) == 0


A = 0x10000  # a fake, aligned, non-NULL address: validation never dereferences device pointers


def _pool(**kw):
    args = dict(k=A, v=A, num_blocks=64, kv_heads=2, head_dim=128, dtype=B.RAGC_DTYPE_BF16)
    args.update(kw)
    return B.make_pool(**args)


def _batch(p=(10,), n=(5,), stride=4, table=None, dev=A):
    hp, hn = np.asarray(p, np.int32), np.asarray(n, np.int32)
    hs = np.concatenate([[0], np.cumsum(np.maximum(hn, 0))]).astype(np.int32)
    b = B.make_batch(len(p), stride, dev, dev, dev, dev, hp, hn, hs, table)
    return b, (hp, hn, hs, table)


def _attn_code(pool, batch, q=A, k=A, v=A, o=A, hq=8, scale=0.1, flags=0):
    with pytest.raises(B.RagcError) as e:
        B.ragc_prefill_attn(pool, batch, q, k, v, o, hq, scale, flags)
    return e.value.code


def test_attention_argument_errors(lib):
    b, keep = _batch()
    assert _attn_code(_pool(k=None), b) == B.RAGC_ERR_NULL
    assert _attn_code(_pool(block_size=32), b) == B.RAGC_ERR_SHAPE
    assert _attn_code(_pool(head_dim=96), b) == B.RAGC_ERR_SHAPE
    assert _attn_code(_pool(dtype=3), b) == B.RAGC_ERR_SHAPE
    assert _attn_code(_pool(block_stride_elems=100), b) == B.RAGC_ERR_SHAPE
    assert _attn_code(_pool(k=A + 2), b) == B.RAGC_ERR_ALIGN
    assert _attn_code(_pool(), b, hq=3) == B.RAGC_ERR_SHAPE
    assert _attn_code(_pool(), b, scale=0.0) == B.RAGC_ERR_SHAPE
    assert _attn_code(_pool(), b, scale=float("nan")) == B.RAGC_ERR_SHAPE
    assert _attn_code(_pool(), b, flags=0x80) == B.RAGC_ERR_SHAPE
    assert _attn_code(_pool(), b, q=None) == B.RAGC_ERR_NULL
    assert _attn_code(_pool(), b, o=A + 4) == B.RAGC_ERR_ALIGN
    b2, keep2 = _batch(dev=None)
    assert _attn_code(_pool(), b2) == B.RAGC_ERR_NULL
    b3, keep3 = _batch(p=(60,), n=(10,), stride=4)  # 70 tokens need 5 entries
    assert _attn_code(_pool(), b3) == B.RAGC_ERR_RANGE
    b4, keep4 = _batch(p=(-1,))
    assert _attn_code(_pool(), b4) == B.RAGC_ERR_RANGE
    tbl = np.array([[1, 64, 0, 0]], np.int32)  # block 64 does not exist
    b5, keep5 = _batch(p=(20,), n=(5,), table=tbl)
    assert _attn_code(_pool(), b5) == B.RAGC_ERR_RANGE
    assert "block_table[1] = 64" in B.ragc_last_error()
    hp = np.asarray([1], np.int32)
    b6 = B.make_batch(1, 4, None, None, None, None, None, hp, hp, None)  # no host copy and no device array to read it from
    with pytest.raises(B.RagcError) as e:
        B.ragc_prefill_attn_workspace(_pool(), b6, 8)
    assert e.value.code == B.RAGC_ERR_NULL and "prefix_len" in B.ragc_last_error()
    with pytest.raises(B.RagcError) as e:  # the entry point that may not read anything back wants all three host copies
        B.ragc_prefill_attn_static(_pool(), B.make_batch(1, 4, A, A, A, A, None, hp, hp, None), A, A, A, A, 8, 0.1)
    assert e.value.code == B.RAGC_ERR_NULL
    with pytest.raises(B.RagcError) as e:
        B.ragc_prefill_attn_static(_pool(), b, A, A, A, A, 8, 0.1, B.RAGC_ATTN_VALIDATE)
    assert e.value.code == B.RAGC_ERR_SHAPE


def test_append_wants_rows_packed_in_request_order(lib):
    """The append kernel finds a row's request by searching new_start, so the offsets must be the
    running sum of new_len; attention takes any offsets.  Both checks happen before any launch."""
    hp, hn = np.asarray([10, 20, 5], np.int32), np.asarray([5, 0, 7], np.int32)
    for hs, ok in ((np.asarray([0, 5, 5, 12], np.int32), True), (np.asarray([3, 8, 8, 15], np.int32), True),
                   (np.asarray([0, 6, 6, 13], np.int32), False), (np.asarray([7, 0, 0, 0], np.int32), False)):
        b = B.make_batch(3, 4, A, A, A, A, hp, hn, hs, None)
        if ok:
            continue  # would launch: covered by the GPU tests
        with pytest.raises(B.RagcError) as e:
            B.ragc_kv_append(_pool(), b, A, A)
        assert e.value.code == B.RAGC_ERR_RANGE and "packed in request order" in B.ragc_last_error()


def test_debug_plan_override_changes_the_workspace_and_rejects_bad_values(lib):
    one, keep = _batch(p=(4096,), n=(16,), stride=300)
    pool = _pool(num_blocks=512)
    auto = B.ragc_prefill_attn_workspace(pool, one, 8)
    try:
        B.ragc_debug_set_attn_plan(-1, 3)
        assert B.ragc_prefill_attn_workspace(pool, one, 8) == 3 * 2 * 128 * (128 + 2) * 4
        B.ragc_debug_set_attn_plan(0, 1)
        assert B.ragc_prefill_attn_workspace(pool, one, 8) == 0
        for bad in ((2, 0), (-2, 0), (0, 17), (0, -1)):
            with pytest.raises(B.RagcError) as e:
                B.ragc_debug_set_attn_plan(*bad)
            assert e.value.code == B.RAGC_ERR_SHAPE
        assert B.ragc_prefill_attn_workspace(pool, one, 8) == 0  # a rejected call leaves the setting alone
    finally:
        B.ragc_debug_set_attn_plan(-1, 0)
    assert B.ragc_prefill_attn_workspace(pool, one, 8) == auto


def test_key_split_rule_as_seen_through_the_workspace_size(lib):
    """S = min(CUs / workgroups, key tiles of the longest item / 3, 16), 256 CUs when no GPU is visible
    (an MI355X has as many); the workspace is one partial result per (item, copy, kv head)."""
    part = 128 * (128 + 2) * 4

    def copies(p, n, hq, hkv, stride=1200):
        b, keep = _batch(p=p, n=n, stride=stride)
        items = sum(-(-(x * (hq // hkv)) // 128) for x in n)
        ws = B.ragc_prefill_attn_workspace(_pool(num_blocks=4096, kv_heads=hkv), b, hq)
        assert ws % (items * hkv * part) == 0
        return ws // (items * hkv * part)  # 0: not split

    assert copies((4096,) * 4, (1,) * 4, 64, 8) == 8       # 32 workgroups, 65 tiles: every CU gets one
    assert copies((1024,), (100,), 32, 32) == 6            # 32 workgroups, 18 tiles: three tiles per copy
    assert copies((2048,) * 2, (1,) * 2, 32, 8) == 11      # 16 workgroups, 33 tiles
    assert copies((16384,), (1,), 32, 8) == 16             # capped
    assert copies((1024,) * 8, (1,) * 8, 32, 32) == 0      # 256 workgroups already
    assert copies((100,), (20,), 8, 8) == 0                # two tiles: nothing to split
    assert copies((256,) * 8, (100,) * 8, 32, 32) == 0


def test_size_limits_and_workspace_errors(lib):
    many, keep = _batch(p=(0,) * 65536, n=(1,) * 65536, stride=1)
    assert _attn_code(_pool(), many) == B.RAGC_ERR_SHAPE  # more requests than a work item can name
    huge, keep2 = _batch(p=(0,), n=(2_000_000,), stride=125_000)
    assert _attn_code(_pool(), huge, hq=16) == B.RAGC_ERR_RANGE  # 16 M rows: more than 65535 row tiles
    assert "too large" in B.ragc_last_error()
    # one request with a long prefix is split along its keys: the workspace is then mandatory
    one, keep3 = _batch(p=(4096,), n=(16,), stride=300)
    need = B.ragc_prefill_attn_workspace(_pool(num_blocks=512), one, 8)
    assert need > 0 and need % (128 * (128 + 2) * 4) == 0
    assert B.ragc_prefill_attn_workspace(_pool(num_blocks=512), one, 8, B.RAGC_ATTN_NO_SPLIT) == 0
    assert B.ragc_prefill_attn_workspace(_pool(num_blocks=512, dtype=B.RAGC_DTYPE_F32), one, 8) == 0
    for ws, nbytes, code in ((None, 0, B.RAGC_ERR_WORKSPACE), (A, need - 1, B.RAGC_ERR_WORKSPACE), (A + 16, need, B.RAGC_ERR_ALIGN)):
        with pytest.raises(B.RagcError) as e:
            B.ragc_prefill_attn(_pool(num_blocks=512), one, A, A, A, A, 8, 0.1, 0, ws, nbytes)
        assert e.value.code == code
    with pytest.raises(B.RagcError) as e:
        B.ragc_prefill_attn_workspace(_pool(num_blocks=512), one, 3)
    assert e.value.code == B.RAGC_ERR_SHAPE


def test_empty_work_returns_ok_without_a_device(lib):
    b, keep = _batch(p=(10, 3), n=(0, 0))
    assert B.ragc_prefill_attn(_pool(), b, None, None, None, None, 8, 0.1) == 0
    assert B.ragc_kv_append(_pool(), b, None, None) == 0
    b0 = B.make_batch(0, 0, None, None, None, None, None, None, None, None)
    assert B.ragc_prefill_attn(_pool(), b0, None, None, None, None, 8, 0.1) == 0
    ids = np.zeros(0, np.int32)
    assert B.ragc_kv_swap(_pool(), A, A, 2 * 16 * 128, 4, ids, ids, B.RAGC_SWAP_TO_DEVICE) == 0
    assert B.ragc_kv_gather(_pool(), b, 0, 0, None, None) == 0


def _swap_code(pool, hk=A, hv=A, stride=2 * 16 * 128, slots_n=4, dev=(1,), slots=(0,), direction=0, flags=0):
    with pytest.raises(B.RagcError) as e:
        B.ragc_kv_swap(pool, hk, hv, stride, slots_n, np.asarray(dev, np.int32), np.asarray(slots, np.int32), direction, flags)
    return e.value.code


def test_swap_and_gather_argument_errors(lib):
    assert _swap_code(_pool(), hk=None) == B.RAGC_ERR_NULL
    assert _swap_code(_pool(), stride=100) == B.RAGC_ERR_SHAPE
    assert _swap_code(_pool(), direction=2) == B.RAGC_ERR_SHAPE
    assert _swap_code(_pool(), flags=9) == B.RAGC_ERR_SHAPE
    assert _swap_code(_pool(), dev=(64,)) == B.RAGC_ERR_RANGE
    assert _swap_code(_pool(), slots=(4,)) == B.RAGC_ERR_RANGE
    assert _swap_code(_pool(), dev=(1, 1), slots=(0, 1), direction=0) == B.RAGC_ERR_RANGE  # two writes to block 1
    assert _swap_code(_pool(), dev=(1, 2), slots=(3, 3), direction=1) == B.RAGC_ERR_RANGE  # two writes to slot 3
    assert _swap_code(_pool(), hv=A + 8) == B.RAGC_ERR_ALIGN
    b, keep = _batch()
    with pytest.raises(B.RagcError) as e:
        B.ragc_kv_gather(_pool(), b, 1, 4, A, A)
    assert e.value.code == B.RAGC_ERR_RANGE
    with pytest.raises(B.RagcError) as e:
        B.ragc_kv_gather(_pool(), b, 0, 65, A, A)
    assert e.value.code == B.RAGC_ERR_RANGE


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.ragc_version()
