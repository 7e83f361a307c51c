"""Pins for the CPU oracle's attention function (Table 5 of the paper: Self Attention, named
only; the standard definition softmax(scale * Q K^T) V is used).

Closed forms, invariants and special cases that reduce to library routines; each is chosen so
that one plausible mistake (dropped scale, softmax over the wrong axis, Q and K swapped, wrong
row pitch or batch stride, missing max subtraction) fails it.
"""
import math

import numpy as np
import pytest
from scipy.special import expit, softmax

from paper_2505_02146_amd import inputs


def _rand(shape, tid, seed=11):
    return inputs.normal(shape, seed, tid).astype(np.float32)


def test_single_key_returns_its_value_row(oracle):
    b, Lq, d, dv = 3, 5, 4, 6
    Q, K, V = _rand((b, Lq, d), 1), _rand((b, 1, d), 2), _rand((b, 1, dv), 3)
    out = oracle.attention(Q, K, V, batch=b, Lq=Lq, Lk=1, d=d, dv=dv, scale=0.7)
    for i in range(Lq):
        assert np.array_equal(out[:, i, :], V[:, 0, :].astype(np.float64))


def test_zero_queries_average_the_values(oracle):
    b, Lq, Lk, d, dv = 2, 3, 9, 5, 4
    Q = np.zeros((b, Lq, d), np.float32)
    K, V = _rand((b, Lk, d), 2), _rand((b, Lk, dv), 3)
    out = oracle.attention(Q, K, V, batch=b, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=3.0)
    mean = V.astype(np.float64).mean(axis=1)
    for i in range(Lq):
        np.testing.assert_allclose(out[:, i, :], mean, rtol=1e-14, atol=1e-15)


def test_zero_scale_averages_the_values(oracle):
    b, Lq, Lk, d, dv = 1, 4, 6, 3, 2
    Q, K, V = _rand((b, Lq, d), 1), _rand((b, Lk, d), 2), _rand((b, Lk, dv), 3)
    out = oracle.attention(Q, K, V, batch=b, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=0.0)
    np.testing.assert_allclose(out[0], np.tile(V[0].astype(np.float64).mean(axis=0), (Lq, 1)), rtol=1e-14)


def test_weights_one_two_three(oracle):
    # d = 1, query 1, keys 0, ln 2, ln 3 in fp32: the weights are exp(key) / sum, i.e. (1, 2, 3) / 6
    # up to the fp32 rounding of the logarithms, which the expectation carries along
    Q = np.array([[[1.0]]], np.float32)
    K = np.array([[[0.0], [math.log(2.0)], [math.log(3.0)]]], np.float32)
    V = np.array([[[6.0, -6.0], [12.0, 0.0], [-6.0, 18.0]]], np.float32)
    out = oracle.attention(Q, K, V, batch=1, Lq=1, Lk=3, d=1, dv=2, scale=1.0)
    w = np.array([1.0, math.exp(float(K[0, 1, 0])), math.exp(float(K[0, 2, 0]))])
    expect = (w[:, None] * V[0].astype(np.float64)).sum(axis=0) / w.sum()
    np.testing.assert_allclose(out[0, 0], expect, rtol=1e-14)
    np.testing.assert_allclose(out[0, 0], [(6 + 24 - 18) / 6.0, (-6 + 54) / 6.0], rtol=1e-6)


def test_two_keys_is_the_logistic_function(oracle):
    b, Lq, d, dv = 1, 7, 3, 2
    Q, K, V = _rand((b, Lq, d), 1), _rand((b, 2, d), 2), _rand((b, 2, dv), 3)
    scale = 1.3
    out = oracle.attention(Q, K, V, batch=b, Lq=Lq, Lk=2, d=d, dv=dv, scale=scale)
    q, k, v = Q[0].astype(np.float64), K[0].astype(np.float64), V[0].astype(np.float64)
    gap = scale * (q @ (k[0] - k[1]))              # s(i,0) - s(i,1)
    p0 = expit(gap)
    expect = p0[:, None] * v[0] + (1.0 - p0)[:, None] * v[1]
    np.testing.assert_allclose(out[0], expect, rtol=1e-13, atol=1e-15)


def test_identity_values_return_the_weights(oracle):
    # V = I: the output rows are the softmax weights themselves: positive, summing to 1, with
    # ratios exp(s(i,j) - s(i,j'))
    b, Lq, Lk, d = 1, 4, 6, 5
    Q, K = _rand((b, Lq, d), 1), _rand((b, Lk, d), 2)
    V = np.eye(Lk, dtype=np.float32)[None]
    scale = 0.9
    out = oracle.attention(Q, K, V, batch=b, Lq=Lq, Lk=Lk, d=d, dv=Lk, scale=scale)[0]
    assert (out > 0).all()
    np.testing.assert_allclose(out.sum(axis=1), 1.0, rtol=1e-14)
    s = scale * (Q[0].astype(np.float64) @ K[0].astype(np.float64).T)
    np.testing.assert_allclose(np.log(out[:, 1:] / out[:, :1]), s[:, 1:] - s[:, :1], rtol=1e-11, atol=1e-12)


def test_matches_library_softmax_and_matmul_with_padding_and_bf16(oracle):
    b, Lq, Lk, d, dv = 3, 10, 13, 8, 5
    ldq, ldk, ldv = d + 3, d + 1, dv + 2
    sq, sk, sv = Lq * ldq + 7, Lk * ldk + 5, Lk * ldv + 11
    Qm = inputs.to_bf16_bits(_rand((b, Lq, d), 1))
    Km = inputs.to_bf16_bits(_rand((b, Lk, d), 2))
    Vm = _rand((b, Lk, dv), 3)

    def pack(m, ld, stride, dtype, fill):
        buf = np.full(b * stride, fill, dtype=dtype)
        for x in range(b):
            for r in range(m.shape[1]):
                buf[x * stride + r * ld: x * stride + r * ld + m.shape[2]] = m[x, r]
        return buf
    Qb, Kb = pack(Qm, ldq, sq, np.uint16, 0x7FC0), pack(Km, ldk, sk, np.uint16, 0x7FC0)   # NaN padding
    Vb = pack(Vm, ldv, sv, np.float32, np.nan)
    scale = 1.0 / math.sqrt(d)
    out = oracle.attention(Qb, Kb, Vb, batch=b, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=scale,
                           ldq=ldq, ldk=ldk, ldv=ldv, strideQ=sq, strideK=sk, strideV=sv)
    q = inputs.bf16_bits_to_f32(Qm).astype(np.float64)
    k = inputs.bf16_bits_to_f32(Km).astype(np.float64)
    expect = softmax(scale * np.einsum("bic,bjc->bij", q, k), axis=-1) @ Vm.astype(np.float64)
    assert np.isfinite(out).all()
    np.testing.assert_allclose(out, expect, rtol=1e-12, atol=1e-14)


def test_permuting_keys_with_their_values_changes_nothing(oracle):
    b, Lq, Lk, d, dv = 2, 5, 11, 4, 3
    Q, K, V = _rand((b, Lq, d), 1), _rand((b, Lk, d), 2), _rand((b, Lk, dv), 3)
    perm = np.random.default_rng(5).permutation(Lk)
    a = oracle.attention(Q, K, V, batch=b, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=0.6)
    c = oracle.attention(Q, np.ascontiguousarray(K[:, perm]), np.ascontiguousarray(V[:, perm]),
                         batch=b, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=0.6)
    np.testing.assert_allclose(a, c, rtol=1e-13, atol=1e-15)


def test_adding_one_vector_to_every_key_changes_nothing(oracle):
    # s(i,j) moves by scale * q_i . c for every j alike, which a softmax over j ignores
    b, Lq, Lk, d, dv = 1, 6, 8, 4, 3
    Q, K, V = _rand((b, Lq, d), 1), _rand((b, Lk, d), 2), _rand((b, Lk, dv), 3)
    shift = np.array([0.5, -1.25, 2.0, 0.75], np.float32)     # exactly representable sums are not needed
    a = oracle.attention(Q, K, V, batch=b, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=0.8)
    c = oracle.attention(Q, (K + shift).astype(np.float32), V, batch=b, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=0.8)
    np.testing.assert_allclose(a, c, rtol=1e-5, atol=1e-6)    # K + shift is rounded to fp32


def test_huge_scores_do_not_overflow_and_pick_the_best_key(oracle):
    b, Lq, Lk, d, dv = 1, 3, 5, 2, 4
    Q = np.array([[[1.0, 0.0], [0.0, 1.0], [-1.0, 0.0]]], np.float32)
    K = np.array([[[3.0, 0.0], [0.0, 2.0], [-5.0, 0.0], [1.0, 1.0], [0.0, -1.0]]], np.float32)
    V = _rand((b, Lk, dv), 3)
    out = oracle.attention(Q, K, V, batch=b, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=1000.0)
    assert np.isfinite(out).all()
    # the best key wins by a score gap of at least 1000: every other weight is below exp(-1000) = 0
    np.testing.assert_array_equal(out[0], V[0, [0, 1, 2]].astype(np.float64))


def test_queries_and_keys_are_not_interchangeable(oracle):
    # Lq != Lk and asymmetric data: swapping the roles of Q and K gives another shape altogether,
    # and the softmax axis matters: weights sum to 1 over keys, not over queries
    b, Lq, Lk, d = 1, 3, 5, 2
    Q, K = _rand((b, Lq, d), 1), _rand((b, Lk, d), 2)
    V = np.ones((b, Lk, 1), np.float32)
    out = oracle.attention(Q, K, V, batch=b, Lq=Lq, Lk=Lk, d=d, dv=1, scale=1.0)
    assert out.shape == (1, Lq, 1)
    np.testing.assert_allclose(out, 1.0, rtol=1e-14)           # sum_j p(i,j) = 1 for every query


def test_batches_are_independent_problems(oracle):
    b, Lq, Lk, d, dv = 4, 3, 6, 4, 2
    Q, K, V = _rand((b, Lq, d), 1), _rand((b, Lk, d), 2), _rand((b, Lk, dv), 3)
    whole = oracle.attention(Q, K, V, batch=b, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=0.5)
    for x in range(b):
        one = oracle.attention(Q[x:x + 1].copy(), K[x:x + 1].copy(), V[x:x + 1].copy(),
                               batch=1, Lq=Lq, Lk=Lk, d=d, dv=dv, scale=0.5)
        assert np.array_equal(whole[x], one[0])


def test_rejects_empty_key_set_and_short_pitch(oracle):
    Q = np.zeros((1, 2, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.attention(Q, Q, Q, batch=1, Lq=2, Lk=0, d=4, dv=4, scale=1.0)
    with pytest.raises(ValueError):
        oracle.attention(Q, Q, Q, batch=1, Lq=2, Lk=2, d=4, dv=4, scale=1.0, ldq=3)


def test_empty_outputs_are_fine(oracle):
    Q = np.zeros((1, 2, 4), np.float32)
    assert oracle.attention(Q, Q, Q, batch=0, Lq=2, Lk=2, d=4, dv=4, scale=1.0).shape == (0, 2, 4)
    assert oracle.attention(Q, Q, Q, batch=1, Lq=0, Lk=2, d=4, dv=4, scale=1.0).shape == (1, 0, 4)
