"""Pins of the sampling oracle (CPU only): its fixed integer arithmetic is tied to the plain
definitions (exponential weights, softmax draw, top-k / top-p sets, argmax) it stands for."""
import math

import numpy as np
import pytest

import oracle


def _params(t=1.0, p=1.0, r=1.0, k=0, n=1):
    return oracle.sampling_params(t, p, r, k, n)


def test_weight_is_the_exponential():
    rng = np.random.default_rng(0)
    ds = np.concatenate([[0.0, 1e-8, 1e-3, 0.5, 1.0, 10.0, 27.0, 30.0, 44.0, 45.0, 1e30],
                         rng.uniform(0, 30, 2000), rng.uniform(0, 1, 500)]).astype(np.float32)
    assert oracle.sample_weight(0.0) == 1 << 40
    for d in ds:
        w = oracle.sample_weight(float(d))
        exact = 2.0 ** 40 * math.exp(-float(d))
        assert abs(w - exact) <= exact * (3e-7 + 1e-7 * float(d)) + 1.0, d
    assert oracle.sample_weight(50.0) == 0 and oracle.sample_weight(float("inf")) == 0
    # monotone: a larger distance never weighs more
    grid = np.sort(rng.uniform(0, 28, 5000).astype(np.float32))
    ws = [oracle.sample_weight(float(d)) for d in grid]
    assert all(a >= b for a, b in zip(ws, ws[1:]))


def test_draws_follow_the_softmax():
    z = np.array([[1.5, -0.25, 3.0, 0.0, 2.0, 2.9]], dtype=np.float32)
    for temp in (1.0, 0.7):
        prob = np.exp(z[0].astype(np.float64) / np.float32(temp))
        prob /= prob.sum()
        n = 20001
        us = ((np.arange(n) + 0.5) / n).astype(np.float32)
        toks, kept = oracle.sample(np.repeat(z, n, 0), _params(t=temp, n=n), us)
        assert (kept == 6).all()
        freq = np.bincount(toks, minlength=6) / n
        assert np.abs(freq - prob).max() <= 2.0 / n + 1e-6
        # the order of the cumulative walk is descending probability: small u gives the mode
        assert toks[0] == 2 and toks[-1] == 1


def test_top_k_and_top_p_sets_match_numpy():
    rng = np.random.default_rng(3)
    v = 1000
    z = (rng.standard_normal((1, v)) * 2.5).astype(np.float32)
    y = z[0].astype(np.float64) / np.float32(0.8)
    order = np.lexsort((np.arange(v), -y))
    n = 4001
    us = ((np.arange(n) + 0.5) / n).astype(np.float32)
    # top-k alone
    toks, kept = oracle.sample(np.repeat(z, n, 0), _params(t=0.8, k=50, n=n), us)
    assert (kept == 50).all() and set(toks) <= set(order[:50])
    p50 = np.exp(y[order[:50]] - y[order[0]])
    p50 /= p50.sum()
    assert set(order[:50][p50 > 2e-3]) <= set(toks)
    # top-p alone and after top-k: the shortest prefix reaching top_p
    for k, top_p in ((0, 0.9), (0, 0.5), (50, 0.95), (7, 0.3)):
        m = v if k == 0 else k
        pk = np.exp(y[order[:m]] - y[order[0]])
        cum = np.cumsum(pk) / pk.sum()
        size = int(np.searchsorted(cum, top_p, side="left") + 1)
        assert abs(cum[size - 1] - top_p) > 1e-5  # clear margin for this pin
        toks, kept = oracle.sample(np.repeat(z, n, 0), _params(t=0.8, p=top_p, k=k, n=n), us)
        assert (kept == size).all() and set(toks) <= set(order[:size])
        pn = pk[:size] / pk[:size].sum()
        freq = np.bincount(toks, minlength=v)[order[:size]] / n
        assert np.abs(freq - pn).max() <= 2.0 / n + 1e-5


def test_greedy_penalty_ties_and_window():
    z = np.array([[2.0, 1.9, -1.0, 1.9]], dtype=np.float32)
    tok, kept = oracle.sample(z, _params(t=0.0), [0.7])
    assert tok[0] == 0 and kept[0] == 1
    # penalty divides positive logits: 2.0 / 1.3 < 1.9, and the first of the tied 1.9s wins
    hist = np.array([[0, 0, -1, 99]], dtype=np.int32)  # repeated, empty and out-of-range slots
    tok, _ = oracle.sample(z, _params(t=0.0, r=1.3), [0.7], history=hist)
    assert tok[0] == 1
    # a token that occurs twice in the window is penalised once: 2.0 / 1.3 > 1.4 > 2.0 / 1.69
    tok, _ = oracle.sample(np.array([[2.0, 1.4]], np.float32), _params(t=0.0, r=1.3), [0.7],
                           history=np.array([[0, 0]], np.int32))
    assert tok[0] == 0
    # negative logits are multiplied: -1.0 * 1.3 stays last; penalising 1 and 3 restores 0
    tok, _ = oracle.sample(z, _params(t=0.0, r=1.3), [0.7], history=np.array([[1, 3, 2]], np.int32))
    assert tok[0] == 0
    z2 = np.array([[-1.0, -1.2]], dtype=np.float32)
    tok, _ = oracle.sample(z2, _params(t=0.0, r=1.3), [0.1], history=np.array([[0]], np.int32))
    assert tok[0] == 1  # -1.0 * 1.3 = -1.3 < -1.2
    # equal logits: equal weights, cumulative walk in ascending id
    eq = np.ones((4, 4), dtype=np.float32)
    toks, _ = oracle.sample(eq, _params(n=4), np.array([0.0, 0.3, 0.5, 0.99], np.float32))
    assert list(toks) == [0, 1, 2, 3]


def test_extreme_uniforms_and_tiny_top_p():
    rng = np.random.default_rng(5)
    z = rng.standard_normal((3, 64)).astype(np.float32)
    order0 = np.lexsort((np.arange(64), -z[0].astype(np.float64)))
    toks, kept = oracle.sample(z, _params(p=np.float32([1.0, 1e-9, 1.0]), k=[5, 0, 5], n=3),
                               np.float32([0.0, 0.9, np.nextafter(np.float32(1), np.float32(0))]))
    assert toks[0] == order0[0]
    assert kept[1] == 1 and toks[1] == int(np.argmax(z[1]))
    order2 = np.lexsort((np.arange(64), -z[2].astype(np.float64)))
    assert toks[2] == order2[4] and kept[2] == 5


def test_bad_arguments():
    z = np.zeros((1, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.sample(z, _params(n=2), [0.5])
