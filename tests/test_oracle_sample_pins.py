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


def test_sample_weights_rows_follow_the_stated_arithmetic():
    # d and w of every token, recomputed here in numpy with the same single fp32 operations
    # (penalty on the window's tokens, one division for 1/T, one product, max, one difference):
    # a wrong sign of d, a penalty applied the wrong way round, to the wrong tokens or twice, or
    # a temperature that is divided instead of multiplied by its inverse changes bits of d.
    rng = np.random.default_rng(11)
    s, v, window = 5, 777, 40
    z = (rng.standard_normal((s, v)) * 3.0).astype(np.float32)
    hist = rng.integers(-3, v + 3, size=(s, window)).astype(np.int32)  # some ids out of range
    hist[:, 5] = hist[:, 4]  # a token that occurs twice is penalised once
    temps = np.float32([0.8, 0.6, 1.0, 0.0, 2.5])  # stream 3 is greedy: y = z'
    pens = np.float32([1.1, 1.3, 1.0, 1.05, 2.0])
    for r in np.unique(pens):
        prm = oracle.sampling_params(temps, 1.0, np.float32(r), 0, s)
        d, w = oracle.sample_weights(z, prm, history=hist)
        for i in range(s):
            seen = np.zeros(v, dtype=bool)
            ids = hist[i][(hist[i] >= 0) & (hist[i] < v)]
            seen[ids] = True
            zp = z[i].copy()
            pos = seen & (zp > 0)
            neg = seen & ~(zp > 0)
            zp[pos] = zp[pos] / np.float32(r)
            zp[neg] = zp[neg] * np.float32(r)
            inv_t = np.float32(1.0) / temps[i] if temps[i] > 0 else np.float32(1.0)
            y = (zp * inv_t).astype(np.float32)
            want = (y.max() - y).astype(np.float32)
            assert want.dtype == np.float32
            assert np.array_equal(d[i].view(np.uint32), want.view(np.uint32)), (r, i)
            assert (d[i] >= 0).all() and d[i][int(np.argmax(y))] == 0
            # the weight of each token is the scalar weight function of its own distance
            # (pinned to exp above), and stays within that function's error of 2^40 exp(-d)
            assert all(int(w[i, t]) == oracle.sample_weight(float(d[i, t])) for t in range(0, v, 7))
            exact = 2.0 ** 40 * np.exp(-d[i].astype(np.float64))
            assert np.all(np.abs(w[i].astype(np.float64) - exact)
                          <= exact * (3e-7 + 1e-7 * d[i]) + 1.0)
            assert int(w[i].max()) == 1 << 40
    # without a window nothing is penalised, whatever the penalty says
    prm = oracle.sampling_params(0.7, 1.0, 1.3, 0, s)
    d0, _ = oracle.sample_weights(z, prm)
    y = (z * (np.float32(1.0) / np.float32(0.7))).astype(np.float32)
    assert np.array_equal(d0, (y.max(axis=1, keepdims=True) - y).astype(np.float32))


def test_sample_weights_add_up_to_what_the_sampler_keeps():
    # the kept count of a top-p draw is the shortest prefix, in the order (d, id), of exactly
    # these integer weights that reaches trunc(top_p * total): the rows of sample_weights and the
    # totals inside sample are the same numbers
    rng = np.random.default_rng(12)
    s, v = 6, 500
    z = (rng.standard_normal((s, v)) * 2.0).astype(np.float32)
    hist = rng.integers(0, v, size=(s, 16)).astype(np.int32)
    for top_p, k in ((0.9, 0), (0.5, 0), (0.95, 50)):
        prm = oracle.sampling_params(0.8, np.float32(top_p), 1.1, k, s)
        d, w = oracle.sample_weights(z, prm, history=hist)
        u = rng.random(s).astype(np.float32)
        toks, kept = oracle.sample(z, prm, u, history=hist)
        for i in range(s):
            order = np.lexsort((np.arange(v), d[i].view(np.uint32)))
            n = v if k == 0 else k
            ws = [int(x) for x in w[i][order[:n]]]
            total = sum(ws)
            thr = max(1, int(float(np.float32(top_p)) * float(total)))
            cum, size = 0, 0
            while size < n:
                cum += ws[size]
                size += 1
                if cum >= thr:
                    break
            assert kept[i] == size, (top_p, k, i)
            target = int(float(u[i]) * float(cum))
            run, pick = 0, size - 1
            for j in range(size):
                run += ws[j]
                if run > target:
                    pick = j
                    break
            assert toks[i] == order[pick], (top_p, k, i)


def test_weight_polynomial_is_the_taylor_series_of_the_exponential():
    # the ten constants of the weight function, read from the oracle's source, are the Taylor
    # coefficients (-ln 2)^k / k! of 2^-f rounded to fp32, highest degree first (Horner form):
    # nothing fitted or tuned hides in them
    import os
    import re

    src = open(os.path.join(os.path.dirname(oracle.__file__), "vox_oracle_sample.c")).read()
    body = src[src.index("uint64_t vox_oracle_sample_weight(float d)"):]
    body = body[:body.index("\n}\n")]
    consts = [float.fromhex(c) for c in re.findall(r"(-?0x1\.[0-9a-f]+p[+-]\d+)f", body)]
    assert np.float32(consts[0]) == np.float32(1.4426950408889634)  # log2(e), scales d
    coeffs = consts[1:]
    assert len(coeffs) == 9 and body.count("fmaf(p, f,") == 9 and "fmaf(p, f, 1.0f)" in body
    ln2 = math.log(2.0)
    for i, c in enumerate(coeffs):
        k = 9 - i
        want = (-ln2) ** k / math.factorial(k)
        # rounded to fp32, give or take the last bits (the series may have been rounded after a
        # final adjustment of the truncated tail): well inside 1e-6 relative of the series term
        assert abs(c - want) <= abs(want) * 2e-6, (k, c, want)
    # degree 9 on [0, 1): the first neglected term bounds the truncation error far below 2^-24
    assert ln2 ** 10 / math.factorial(10) < 2.0 ** -25
