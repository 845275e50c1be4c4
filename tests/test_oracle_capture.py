"""Pins of the oracle's pattern capture (Sec. 4.2.1 / 4.2.2: attention probabilities of a captured
sequence summed into A, validity counts into C) against what the mathematics fixes: closed forms,
a library softmax, invariances and hand-built cases. None re-types the oracle's loop."""
import numpy as np
import pytest
import torch

import oracle


def rnd(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


def test_zero_queries_give_uniform_rows_closed_form():
    # q = 0 makes every logit 0: row i attends its i + 1 causal keys equally, whatever K is.
    rng = np.random.default_rng(0)
    A, C = oracle.capture(np.zeros((3, 9, 8), np.float32), rnd(rng, 3, 9, 8), 9)
    for i in range(9):
        np.testing.assert_array_equal(A[:, i, :i + 1], np.float32(1.0 / (i + 1)))
        assert not A[:, i, i + 1:].any()
    np.testing.assert_array_equal(C[0], np.tril(np.ones((9, 9), np.float32)))


def test_matches_library_softmax_and_rows_sum_to_one():
    rng = np.random.default_rng(1)
    Q, K = rnd(rng, 4, 33, 16), rnd(rng, 4, 33, 16)
    A, _ = oracle.capture(Q, K, 33)
    s = torch.from_numpy(Q).double() @ torch.from_numpy(K).double().transpose(1, 2) / 4.0
    s = s.masked_fill(~torch.tril(torch.ones(33, 33, dtype=torch.bool)), float("-inf"))
    ref = torch.softmax(s, -1).numpy()
    np.testing.assert_allclose(A, ref, rtol=0, atol=6e-8)   # half an ulp of fp32 at 1
    np.testing.assert_allclose(A.astype(np.float64).sum(-1), 1.0, atol=1e-6)


def test_a_dominant_key_takes_the_whole_row():
    # key 2 is aligned with every query and 60 logit units above the rest: probability 1 in fp32
    # for rows >= 2 (exp(-60) is far below half an ulp), untouched rows before it.
    d = 4
    Q = np.zeros((1, 6, d), np.float32)
    Q[..., 0] = 1.0
    K = np.zeros((1, 6, d), np.float32)
    K[0, 2, 0] = 60.0
    A, _ = oracle.capture(Q, K, 6, scale=1.0)
    assert (A[0, 2:, 2] == 1.0).all() and A[0, 1, 2] == 0.0
    np.testing.assert_array_equal(A[0, 1, :2], np.float32(0.5))


def test_scale_and_shift_invariances():
    rng = np.random.default_rng(2)
    Q, K = rnd(rng, 2, 12, 8), rnd(rng, 2, 12, 8)
    A0, _ = oracle.capture(Q, K, 12)
    A1, _ = oracle.capture(2 * Q, K, 12, scale=0.5 / np.sqrt(8.0))          # exact power-of-two rescaling
    np.testing.assert_array_equal(A0, A1)
    # adding one vector to every key shifts all logits of a row by the same amount
    A2, _ = oracle.capture(Q, K + rnd(rng, 1, 1, 8), 12)
    np.testing.assert_allclose(A0, A2, atol=3e-7)


def test_grouped_query_heads_read_their_kv_head():
    rng = np.random.default_rng(3)
    Q, K = rnd(rng, 4, 10, 8), rnd(rng, 2, 10, 8)
    A, _ = oracle.capture(Q, K, 10)
    A_rep, _ = oracle.capture(Q, np.repeat(K, 2, axis=0), 10)   # MHA with each KV head repeated
    np.testing.assert_array_equal(A, A_rep)
    A_swapped, _ = oracle.capture(Q, K[::-1].copy(), 10)
    assert not np.array_equal(A, A_swapped)


def test_accumulation_over_sequences_of_different_length():
    # Two captures, the second shorter than L: sums add, counts say how often a pair was valid, and
    # the mean A / C of a pair seen twice is the average of the two probabilities.
    rng = np.random.default_rng(4)
    L = 8
    Q1, K1 = rnd(rng, 2, 8, 4), rnd(rng, 2, 8, 4)
    Q2, K2 = rnd(rng, 2, 5, 4), rnd(rng, 2, 5, 4)
    A1, _ = oracle.capture(Q1, K1, L)
    A2, _ = oracle.capture(Q2, K2, L)
    A, C = oracle.capture(Q1, K1, L)
    A, C = oracle.capture(Q2, K2, L, attn_sum=A, attn_cnt=C)
    np.testing.assert_array_equal(A, A1 + A2)
    tri = np.tril(np.ones((L, L), np.float32))
    expect = tri.copy()
    expect[:5, :5] += tri[:5, :5]
    np.testing.assert_array_equal(C[1], expect)
    assert not A2[:, 5:].any() and not A2[:, :, 5:].any()
    # prefix property of causal attention: the first 5 rows of a longer capture equal the capture
    # of its first 5 tokens
    A_pre, _ = oracle.capture(Q1[:, :5].copy(), K1[:, :5].copy(), L)
    np.testing.assert_array_equal(A_pre[:, :5], A1[:, :5])


def test_brute_force_tiny():
    rng = np.random.default_rng(5)
    Q, K = rnd(rng, 1, 4, 3), rnd(rng, 1, 4, 3)
    A, _ = oracle.capture(Q, K, 4)
    for i in range(4):
        logits = [sum(float(Q[0, i, t]) * float(K[0, j, t]) for t in range(3)) / 3 ** 0.5 for j in range(i + 1)]
        z = sum(np.exp(x) for x in logits)
        for j in range(i + 1):
            assert abs(float(A[0, i, j]) - np.exp(logits[j]) / z) < 1e-7
