"""Pins of the CPU oracle against things other than itself: hand-worked values,
closed forms, invariants, a library routine, brute force.  No GPU."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import attention as OA

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.Generator(np.random.Philox(key=[777, seed])).standard_normal(shape)


def _cases():
    cases, cur = [], None
    for line in open(os.path.join(GOLD, "hand_worked_attention.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        if key == "case":
            cur = {"name": vals[0]}
            cases.append(cur)
        elif key == "dims":
            cur["dims"] = [int(x) for x in vals[:5]] + [float(vals[5])]
        else:
            cur[key] = np.asarray([float(x) for x in vals], np.float64)
    return cases


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_hand_worked_cases(case):
    P, N, Hq, Hkv, D, scale = case["dims"]
    q = case["q"].reshape(N, Hq, D)
    k = case["k"].reshape(P + N, Hkv, D)
    v = case["v"].reshape(P + N, Hkv, D)
    out = OA.prefill_attn(q, k, v, P, scale)
    np.testing.assert_allclose(out.ravel(), case["out"], rtol=0, atol=1e-13)
    out2 = OA.prefill_attn_full_recompute(q, k, v, P, scale)
    np.testing.assert_allclose(out2.ravel(), case["out"], rtol=0, atol=1e-13)


def test_single_key_returns_v_exactly():
    q = _rand((1, 4, 8), 1)
    k = _rand((1, 2, 8), 2)
    v = _rand((1, 2, 8), 3)
    out = OA.prefill_attn(q, k, v, 0, 0.37)
    for h in range(4):
        assert np.array_equal(out[0, h], v[0, h // 2])


def test_zero_query_gives_running_mean():
    P, N, Hq, Hkv, D = 37, 9, 4, 2, 16
    k = _rand((P + N, Hkv, D), 4)
    v = _rand((P + N, Hkv, D), 5)
    out = OA.prefill_attn(np.zeros((N, Hq, D)), k, v, P, 1.0)
    for i in range(N):
        for h in range(Hq):
            np.testing.assert_allclose(out[i, h], v[: P + i + 1, h // 2].mean(axis=0), rtol=0, atol=1e-14)


def test_weights_sum_to_one():
    P, N, Hq, Hkv, D = 300, 40, 4, 4, 32
    q, k, v = _rand((N, Hq, D), 6) * 3, _rand((P + N, Hkv, D), 7), _rand((P + N, Hkv, D), 8)
    _, ws = OA.prefill_attn(q, k, v, P, 0.5, return_weight_sums=True)
    assert np.max(np.abs(ws - 1.0)) < 1e-12


@pytest.mark.parametrize("hot", [0, 17, 63, 70])
def test_dominant_key_returns_its_value(hot):
    P, N, Hq, Hkv, D = 64, 8, 2, 1, 8
    q = np.ones((N, Hq, D))
    k = np.zeros((P + N, Hkv, D))
    v = _rand((P + N, Hkv, D), 9)
    k[hot] = 10.0  # score 80 against 0 for everyone else
    out = OA.prefill_attn(q, k, v, P, 1.0)
    for i in range(N):
        if hot <= P + i:
            np.testing.assert_allclose(out[i, 0], v[hot, 0], atol=1e-30 + 1e-12)
        else:  # the hot key is in this token's future: plain mean
            np.testing.assert_allclose(out[i, 0], v[: P + i + 1, 0].mean(axis=0), atol=1e-13)


@pytest.mark.parametrize("P,N,Hq,Hkv,D", [(0, 19, 2, 2, 8), (33, 21, 4, 2, 16), (130, 5, 8, 2, 32), (16, 16, 1, 1, 64)])
def test_row_definition_equals_full_recomputation(P, N, Hq, Hkv, D):
    q, k, v = _rand((N, Hq, D), 10), _rand((P + N, Hkv, D), 11), _rand((P + N, Hkv, D), 12)
    a = OA.prefill_attn(q, k, v, P, 1 / math.sqrt(D))
    b = OA.prefill_attn_full_recompute(q, k, v, P, 1 / math.sqrt(D), q_prefix=_rand((P, Hq, D), 13))
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)


def test_no_prefix_equals_library_causal_attention():
    N, H, D = 50, 3, 16
    q, k, v = _rand((N, H, D), 14), _rand((N, H, D), 15), _rand((N, H, D), 16)
    a = OA.prefill_attn(q, k, v, 0, 1 / math.sqrt(D))
    tq, tk, tv = (torch.from_numpy(x).permute(1, 0, 2).unsqueeze(0) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    np.testing.assert_allclose(a, ref[0].permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)


def test_prefix_equals_library_attention_with_explicit_mask():
    P, N, H, D = 45, 11, 2, 8
    q, k, v = _rand((N, H, D), 17), _rand((P + N, H, D), 18), _rand((P + N, H, D), 19)
    a = OA.prefill_attn(q, k, v, P, 0.3)
    mask = torch.zeros(N, P + N, dtype=torch.bool)
    for i in range(N):
        mask[i, : P + i + 1] = True
    tq = torch.from_numpy(q).permute(1, 0, 2).unsqueeze(0)
    tk, tv = (torch.from_numpy(x).permute(1, 0, 2).unsqueeze(0) for x in (k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=0.3)
    np.testing.assert_allclose(a, ref[0].permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)


def test_brute_force_python_floats():
    P, N, Hq, Hkv, D = 3, 4, 2, 1, 3
    q, k, v = _rand((N, Hq, D), 20), _rand((P + N, Hkv, D), 21), _rand((P + N, Hkv, D), 22)
    scale = 0.7
    out = OA.prefill_attn(q, k, v, P, scale)
    for i in range(N):
        for h in range(Hq):
            e = [math.exp(scale * sum(q[i, h, d] * k[j, 0, d] for d in range(D))) for j in range(P + i + 1)]
            z = sum(e)
            for d in range(D):
                want = sum(e[j] / z * v[j, 0, d] for j in range(P + i + 1))
                assert abs(out[i, h, d] - want) < 1e-13


def test_future_tokens_do_not_matter():
    P, N, Hq, Hkv, D = 20, 10, 2, 2, 8
    q, k, v = _rand((N, Hq, D), 23), _rand((P + N, Hkv, D), 24), _rand((P + N, Hkv, D), 25)
    base = OA.prefill_attn(q, k, v, P, 0.4)
    for i in range(N - 1):
        k2, v2 = k.copy(), v.copy()
        k2[P + i + 1 :] += 100.0
        v2[P + i + 1 :] -= 50.0
        pert = OA.prefill_attn(q, k2, v2, P, 0.4)
        assert np.array_equal(pert[: i + 1], base[: i + 1])
        assert not np.array_equal(pert[i + 1 :], base[i + 1 :])


def test_last_visible_key_is_the_token_itself():
    # perturbing key P+i must change row i (inclusive mask), key P+i+1 must not
    P, N, D = 5, 3, 4
    q, k, v = _rand((N, 1, D), 26), _rand((P + N, 1, D), 27), _rand((P + N, 1, D), 28)
    base = OA.prefill_attn(q, k, v, P, 1.0)
    for i in range(N):
        v2 = v.copy()
        v2[P + i] += 1.0
        assert not np.array_equal(OA.prefill_attn(q, k, v2, P, 1.0)[i], base[i])


def test_gqa_equals_mha_with_repeated_kv_heads():
    P, N, Hq, Hkv, D = 40, 12, 8, 2, 16
    q, k, v = _rand((N, Hq, D), 29), _rand((P + N, Hkv, D), 30), _rand((P + N, Hkv, D), 31)
    a = OA.prefill_attn(q, k, v, P, 0.25)
    G = Hq // Hkv
    b = OA.prefill_attn(q, np.repeat(k, G, axis=1), np.repeat(v, G, axis=1), P, 0.25)
    assert np.array_equal(a, b)
    # and head h really reads kv head h // G: change kv head 1, heads 0..3 unchanged
    k2 = k.copy()
    k2[:, 1] += 1.0
    c = OA.prefill_attn(q, k2, v, P, 0.25)
    assert np.array_equal(c[:, :G], a[:, :G]) and not np.array_equal(c[:, G:], a[:, G:])


def test_prefix_order_of_keys_is_irrelevant_when_moved_with_values():
    P, N, Hq, Hkv, D = 64, 6, 2, 1, 8
    q, k, v = _rand((N, Hq, D), 32), _rand((P + N, Hkv, D), 33), _rand((P + N, Hkv, D), 34)
    perm = np.random.Generator(np.random.Philox(key=[1, 2])).permutation(P)
    k2, v2 = k.copy(), v.copy()
    k2[:P], v2[:P] = k[perm], v[perm]
    np.testing.assert_allclose(OA.prefill_attn(q, k2, v2, P, 0.35), OA.prefill_attn(q, k, v, P, 0.35), rtol=0, atol=1e-13)


def test_linear_in_values_and_shift():
    P, N, Hq, Hkv, D = 30, 7, 2, 2, 8
    q, k = _rand((N, Hq, D), 35), _rand((P + N, Hkv, D), 36)
    v1, v2 = _rand((P + N, Hkv, D), 37), _rand((P + N, Hkv, D), 38)
    o1, o2 = OA.prefill_attn(q, k, v1, P, 0.3), OA.prefill_attn(q, k, v2, P, 0.3)
    np.testing.assert_allclose(OA.prefill_attn(q, k, 2 * v1 - v2, P, 0.3), 2 * o1 - o2, rtol=0, atol=1e-13)
    np.testing.assert_allclose(OA.prefill_attn(q, k, v1 + 3.0, P, 0.3), o1 + 3.0, rtol=0, atol=1e-13)


def test_rows_subset_matches_full_and_threads_do_not_matter():
    P, N, Hq, Hkv, D = 50, 20, 4, 2, 16
    q, k, v = _rand((N, Hq, D), 39), _rand((P + N, Hkv, D), 40), _rand((P + N, Hkv, D), 41)
    full = OA.prefill_attn(q, k, v, P, 0.25, threads=1)
    assert np.array_equal(full, OA.prefill_attn(q, k, v, P, 0.25, threads=4))
    rows = [(0, 0), (19, 3), (7, 2)]
    sub = OA.prefill_attn(q, k, v, P, 0.25, rows=rows)
    for n, (i, h) in enumerate(rows):
        assert np.array_equal(sub[n], full[i, h])


def test_large_scores_do_not_overflow():
    q = np.full((2, 1, 4), 50.0)
    k = np.full((3, 1, 4), 50.0)
    k[0] = -50.0
    v = _rand((3, 1, 4), 42)
    out = OA.prefill_attn(q, k, v, 1, 1.0)
    assert np.all(np.isfinite(out))
    np.testing.assert_allclose(out[0, 0], v[1, 0], atol=1e-12)
    np.testing.assert_allclose(out[1, 0], 0.5 * (v[1, 0] + v[2, 0]), atol=1e-12)
