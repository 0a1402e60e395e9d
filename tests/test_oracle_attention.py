"""Pins for the fp64 attention oracle: brute force, closed forms, invariants, a worked example.

None of these re-types the oracle's loop: the brute force builds the full masked score
matrix and uses library matmul / exp; the closed forms fix values without any softmax code.
"""
import math
import os

import numpy as np
import pytest

from oracle import attention

GOLD = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(20241001)


def bf16_round(x):
    """Round float32 -> bf16 (nearest even) -> float32, in numpy."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)


def dense_causal(q_all, k, v, scale):
    """Textbook one-shot causal attention over n tokens: q_all [n, Hq, D], k/v [n, Hkv, D].
    Full n x n score matrix per head, masked above the diagonal."""
    n, Hq, D = q_all.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    out = np.zeros((n, Hq, D))
    mask = np.triu(np.ones((n, n), dtype=bool), 1)
    for h in range(Hq):
        S = scale * (q_all[:, h, :].astype(np.float64) @ k[:, h // G, :].astype(np.float64).T)
        S[mask] = -np.inf
        E = np.exp(S - S.max(axis=1, keepdims=True))
        W = E / E.sum(axis=1, keepdims=True)
        out[:, h, :] = W @ v[:, h // G, :].astype(np.float64)
    return out


def rand(*shape):
    return bf16_round(RNG.standard_normal(shape).astype(np.float32))


@pytest.mark.parametrize("Hq,Hkv,D", [(4, 2, 64), (7, 1, 16), (5, 5, 8), (8, 1, 128)])
def test_chunk_equals_rows_of_dense_causal(Hq, Hkv, D):
    # chunk of 32 new tokens on 48 prior == rows 48..79 of dense causal attention over 80
    n, C = 80, 48
    q_all, k, v = rand(n, Hq, D), rand(n, Hkv, D), rand(n, Hkv, D)
    scale = 1 / math.sqrt(D)
    dense = dense_causal(q_all, k, v, scale)
    got = attention.attention_chunk(q_all[C:], k, v, C, scale)
    np.testing.assert_allclose(got, dense[C:], rtol=0, atol=1e-12)
    # first chunk (no prior context): rows 0..31; row 0 sees only itself -> exactly v0
    got0 = attention.attention_chunk(q_all[:32], k[:32], v[:32], 0, scale)
    np.testing.assert_allclose(got0, dense[:32], rtol=0, atol=1e-12)
    G = Hq // Hkv
    for h in range(Hq):
        np.testing.assert_array_equal(got0[0, h], v[0, h // G].astype(np.float64))


@pytest.mark.parametrize("ctx", [0, 1, 15, 16, 17, 40, 63, 100])
def test_decode_is_last_row_of_dense(ctx):
    Hq, Hkv, D = 4, 2, 64
    n = ctx + 1
    q_all, k, v = rand(n, Hq, D), rand(n, Hkv, D), rand(n, Hkv, D)
    dense = dense_causal(q_all, k, v, 0.125)
    got = attention.attention_chunk(q_all[-1:], k, v, ctx, 0.125)
    np.testing.assert_allclose(got[0], dense[-1], rtol=0, atol=1e-12)


def test_extra_rows_beyond_position_are_ignored():
    # keys after a row's position (e.g. later tokens of its own chunk) must not be seen
    Hq, Hkv, D = 4, 2, 16
    q, k, v = rand(3, Hq, D), rand(20, Hkv, D), rand(20, Hkv, D)
    a = attention.attention_rows(q, np.array([4, 9, 9]), k, v, 0.3)
    k2, v2 = k.copy(), v.copy()
    k2[10:] = 1e4
    v2[10:] = -1e4
    b = attention.attention_rows(q, np.array([4, 9, 9]), k2, v2, 0.3)
    np.testing.assert_array_equal(a, b)
    c = attention.attention_rows(q[:1], np.array([4]), k[:5], v[:5], 0.3)
    np.testing.assert_array_equal(a[:1], c)


def test_weights_sum_to_one():
    q, k, v = rand(9, 6, 32), rand(300, 3, 32), rand(300, 3, 32)
    _, w = attention.attention_chunk(q, k, v, 291, 1 / math.sqrt(32), return_weight_sums=True)
    assert np.max(np.abs(w - 1.0)) < 1e-12


def test_closed_forms():
    Hq, Hkv, D, n = 4, 2, 16, 37
    q, k, v = rand(5, Hq, D), rand(n, Hkv, D), rand(n, Hkv, D)
    pos = np.array([0, 3, 16, 31, 36])
    # V == 1 -> out == 1
    out = attention.attention_rows(q, pos, k, np.ones_like(v), 0.25)
    np.testing.assert_allclose(out, 1.0, rtol=0, atol=1e-14)
    # all keys identical -> uniform weights -> running mean of V
    kk = np.broadcast_to(k[:1], k.shape).copy()
    out = attention.attention_rows(q, pos, kk, v, 0.25)
    for i, p in enumerate(pos):
        mean = v[:p + 1].astype(np.float64).mean(axis=0)          # [Hkv, D]
        for h in range(Hq):
            np.testing.assert_allclose(out[i, h], mean[h // 2], rtol=0, atol=1e-13)
    # scale 0 -> uniform as well
    out0 = attention.attention_rows(q, pos, k, v, 0.0)
    np.testing.assert_allclose(out0, out, rtol=0, atol=1e-13)
    # adding the same vector to every key shifts every score of a row by one constant
    base = attention.attention_rows(q, pos, k, v, 0.25)
    shifted = attention.attention_rows(q, pos, k + np.float32(2.0), v, 0.25)
    np.testing.assert_allclose(shifted, base, rtol=0, atol=1e-9)
    # output lies in the convex hull of the visible V rows
    for i, p in enumerate(pos):
        for h in range(Hq):
            vv = v[:p + 1, h // 2].astype(np.float64)
            assert np.all(base[i, h] <= vv.max(axis=0) + 1e-12)
            assert np.all(base[i, h] >= vv.min(axis=0) - 1e-12)


def test_planted_key_dominates():
    # one key equal to 64*q makes its weight ~1: the output is that key's value row
    Hq, Hkv, D, n = 2, 1, 32, 200
    q, k, v = rand(1, Hq, D), rand(n, Hkv, D), rand(n, Hkv, D)
    q[0, 1] = q[0, 0]
    k[123, 0] = bf16_round(64 * q[0, 0])
    out = attention.attention_rows(q, np.array([199]), k, v, 1.0)
    np.testing.assert_allclose(out[0, 0], v[123, 0], rtol=0, atol=1e-6)
    # ... and is invisible to a row positioned before it
    out2 = attention.attention_rows(q, np.array([122]), k, v, 1.0)
    assert np.max(np.abs(out2[0, 0] - v[123, 0])) > 0.1


def test_gqa_head_mapping():
    # query head h reads kv head h // G (contiguous groups): compare with single-head runs
    Hq, Hkv, D, n = 6, 3, 8, 21
    q, k, v = rand(2, Hq, D), rand(n, Hkv, D), rand(n, Hkv, D)
    out = attention.attention_rows(q, np.array([20, 7]), k, v, 0.5)
    for h in range(Hq):
        g = h // 2
        one = attention.attention_rows(q[:, h:h + 1], np.array([20, 7]), k[:, g:g + 1], v[:, g:g + 1], 0.5)
        np.testing.assert_array_equal(out[:, h], one[:, 0])


def test_worked_example_from_fixture():
    vals = {}
    for line in open(os.path.join(GOLD, "softmax_two_keys.txt")):
        if line.strip() and not line.startswith("#"):
            name, *nums = line.split()
            vals[name] = [float(x) for x in nums]
    q = np.array([[[1.0, 0.0]]], dtype=np.float32)
    k = np.array([[[0.0, 0.0]], [[math.log(3), 0.0]], [[math.log(4), 5.0]]], dtype=np.float32)
    v = np.array([[[4.0, -8.0]], [[0.0, 8.0]], [[2.0, 2.0]]], dtype=np.float32)
    two = attention.attention_rows(q, np.array([1]), k, v, 1.0)[0, 0]
    three = attention.attention_rows(q, np.array([2]), k, v, 1.0)[0, 0]
    np.testing.assert_allclose(two, vals["out_two"], rtol=0, atol=1e-6)
    np.testing.assert_allclose(three, vals["out_three"], rtol=0, atol=1e-6)


def test_fp32_evaluation_agrees():
    # the fp64 result is converged far inside the 1e-2 parity tolerance
    Hq, Hkv, D, n = 4, 2, 64, 500
    q, k, v = rand(2, Hq, D), rand(n, Hkv, D), rand(n, Hkv, D)
    ref = attention.attention_rows(q, np.array([499, 250]), k, v, 0.125)
    for i, p in enumerate([499, 250]):
        for h in range(Hq):
            s = (k[:p + 1, h // 2] @ q[i, h]) * np.float32(0.125)
            e = np.exp(s - s.max(), dtype=np.float32)
            o = (e / e.sum(dtype=np.float32)) @ v[:p + 1, h // 2]
            assert np.max(np.abs(o - ref[i, h])) < 1e-5


def test_batch_composition_independence():
    # rows of the online requests do not change when offline requests leave the batch
    Hq, Hkv, D = 4, 2, 16
    ctx, ql = [5, 30, 0, 12], [1, 1, 8, 4]
    ks = [rand(c + n, Hkv, D) for c, n in zip(ctx, ql)]
    vs = [rand(c + n, Hkv, D) for c, n in zip(ctx, ql)]
    q = rand(sum(ql), Hq, D)
    full = attention.attention_batch(q, ks, vs, ctx, ql, 0.25)
    online = attention.attention_batch(q[:2], ks[:2], vs[:2], ctx[:2], ql[:2], 0.25)
    np.testing.assert_array_equal(full[:2], online)


def test_bad_arguments_rejected():
    q, k, v = rand(1, 4, 8), rand(3, 3, 8), rand(3, 3, 8)
    with pytest.raises(ValueError):
        attention.attention_rows(q, np.array([0]), k, v, 1.0)       # 4 % 3 != 0
    q, k, v = rand(1, 4, 8), rand(3, 2, 8), rand(3, 2, 8)
    with pytest.raises(ValueError):
        attention.attention_rows(q, np.array([3]), k, v, 1.0)       # position past the keys
