"""Pins for the oracle's multi-token step (causal prefill / chunk attention and multi-append)."""

import math

import numpy as np
import pytest

import oracle
from helpers import (B, deal_tables, dense_attention_numpy, from_bits, pack_pools, random_rows,
                     to_bits)


def _problem(seed, lens, nq, hq, hkv, d, slack=4):
    rng = np.random.default_rng(seed)
    lens = np.asarray(lens, dtype=np.int32)
    nq = np.asarray(nq, dtype=np.int32)
    assert (nq <= lens).all()
    p = int(sum((int(L) + B - 1) // B for L in lens)) + slack
    tables, _ = deal_tables(rng, lens, p)
    k_rows, v_rows = random_rows(rng, lens, hkv, d)
    kp, vp = pack_pools(k_rows, v_rows, tables, p, hkv, d)
    qo = np.zeros(lens.size + 1, dtype=np.int32)
    qo[1:] = np.cumsum(nq)
    q = to_bits(rng.standard_normal((int(qo[-1]), hq, d)))
    return dict(q=q, k_rows=k_rows, v_rows=v_rows, kp=kp, vp=vp, tables=tables, lens=lens, nq=nq,
                qo=qo, hkv=hkv, d=d, p=p, scale=np.float32(1.0 / math.sqrt(d)))


def _prefill(pr, **over):
    a = dict(pr)
    a.update(over)
    return oracle.paged_prefill(a["q"], a["kp"], a["vp"], a["tables"], a["lens"], a["qo"],
                                a["scale"], num_kv_heads=a["hkv"])


def test_one_new_token_per_stream_is_decode():
    lens = [1, 16, 17, 40, 129]
    pr = _problem(1, lens, [1] * 5, 8, 2, 64)
    out, lse = _prefill(pr)
    dout, dlse = oracle.paged_decode(pr["q"], pr["kp"], pr["vp"], pr["tables"], pr["lens"],
                                     pr["scale"], num_kv_heads=2)
    assert np.array_equal(out, dout) and np.array_equal(lse, dlse)


@pytest.mark.parametrize("hq,hkv,d", [(8, 2, 64), (6, 2, 128), (4, 4, 64)])
def test_matches_dense_causal_attention(hq, hkv, d):
    lens, nq = [37, 16, 5, 64, 9], [37, 3, 0, 17, 9]  # whole prompt, a chunk, nothing, ...
    pr = _problem(2, lens, nq, hq, hkv, d)
    out, lse = _prefill(pr)
    for s, (L, n) in enumerate(zip(lens, nq)):
        for j in range(n):
            ctx = L - n + j + 1
            row = int(pr["qo"][s]) + j
            ref, ref_lse = dense_attention_numpy(pr["q"][row:row + 1],
                                                 [pr["k_rows"][s][:ctx]], [pr["v_rows"][s][:ctx]],
                                                 pr["scale"], hkv)
            assert np.abs(out[row] - ref[0]).max() <= 1e-12
            assert np.abs(lse[row] - ref_lse[0]).max() <= 1e-12


def test_each_row_equals_a_decode_over_the_truncated_context():
    lens, nq = [50, 33], [7, 33]
    pr = _problem(3, lens, nq, 8, 2, 64)
    out, lse = _prefill(pr)
    for s, (L, n) in enumerate(zip(lens, nq)):
        for j in range(n):
            row = int(pr["qo"][s]) + j
            cut = np.array([L - n + j + 1 if x == s else 0 for x in range(len(lens))],
                           dtype=np.int32)
            qd = np.zeros((len(lens),) + pr["q"].shape[1:], dtype=np.uint16)
            qd[s] = pr["q"][row]
            dout, dlse = oracle.paged_decode(qd, pr["kp"], pr["vp"], pr["tables"], cut,
                                             pr["scale"], num_kv_heads=2)
            assert np.array_equal(out[row], dout[s]) and np.array_equal(lse[row], dlse[s])


def test_later_tokens_do_not_influence_earlier_queries():
    lens, nq = [48], [20]
    pr = _problem(4, lens, nq, 8, 2, 64)
    out, _ = _prefill(pr)
    rng = np.random.default_rng(5)
    j_cut = 11  # rewrite the keys/values of the new tokens after query j_cut
    k2 = [kr.copy() for kr in pr["k_rows"]]
    v2 = [vr.copy() for vr in pr["v_rows"]]
    first_changed = lens[0] - nq[0] + j_cut + 1
    k2[0][first_changed:] = to_bits(rng.standard_normal(k2[0][first_changed:].shape) * 5)
    v2[0][first_changed:] = 0x7FC0  # NaN
    kp2, vp2 = pack_pools(k2, v2, pr["tables"], pr["p"], 2, 64)
    out2 = _prefill(pr, kp=kp2, vp=vp2)[0]
    assert np.array_equal(out[:j_cut + 1], out2[:j_cut + 1])
    assert not np.array_equal(out[j_cut + 1:], out2[j_cut + 1:])


def test_multi_append_equals_repeated_single_appends():
    hkv, d = 2, 64
    lens = np.array([20, 16, 7, 33], dtype=np.int32)
    nq = np.array([5, 16, 0, 1], dtype=np.int32)
    pr = _problem(6, lens, nq, 4, hkv, d)
    rng = np.random.default_rng(7)
    tq = int(pr["qo"][-1])
    k_new = to_bits(rng.standard_normal((tq, hkv, d)))
    v_new = to_bits(rng.standard_normal((tq, hkv, d)))
    kp, vp = pr["kp"].copy(), pr["vp"].copy()
    oracle.kv_append_multi(k_new, v_new, kp, vp, pr["tables"], lens, pr["qo"], head_dim=d)
    kp2, vp2 = pr["kp"].copy(), pr["vp"].copy()
    for j in range(int(nq.max())):  # token j of every stream that has one, as a decode-style append
        cur = np.where(j < nq, lens - nq + j + 1, 0).astype(np.int32)
        kn = np.zeros((lens.size, hkv, d), dtype=np.uint16)
        vn = np.zeros((lens.size, hkv, d), dtype=np.uint16)
        for s in range(lens.size):
            if j < nq[s]:
                kn[s], vn[s] = k_new[pr["qo"][s] + j], v_new[pr["qo"][s] + j]
        oracle.kv_append(kn, vn, kp2, vp2, pr["tables"], cur, head_dim=d)
    assert np.array_equal(kp, kp2) and np.array_equal(vp, vp2)
    assert (kp != pr["kp"]).any()


def test_bad_offsets_are_rejected():
    pr = _problem(8, [10, 10], [3, 3], 4, 2, 64)
    bad = pr["qo"].copy()
    bad[1] = 12  # stream 0 would bring 12 > L_0 tokens
    bad[2] = 15
    q = np.zeros((15, 4, 64), dtype=np.uint16)
    with pytest.raises(RuntimeError):
        oracle.paged_prefill(q, pr["kp"], pr["vp"], pr["tables"], pr["lens"], bad, pr["scale"],
                             num_kv_heads=2)
