"""Pins for the CPU oracle: each test checks it against something other than itself.

The paper prints no value for the decode step (it names only the attention backend of the LLM
Forward stage, Section 3.1.1), so the pins are brute force, closed forms and exact invariants.
"""

import math

import numpy as np
import pytest

import oracle
from helpers import (B, deal_tables, dense_attention_loops, dense_attention_numpy, from_bits,
                     k_view, pack_pools, random_rows, to_bits, unpack_rows, v_view)


def _problem(seed, lens, hq, hkv, d, slack=5, std=1.0):
    rng = np.random.default_rng(seed)
    lens = np.asarray(lens, dtype=np.int32)
    need = int(sum((int(L) + B - 1) // B for L in lens))
    p = need + slack
    tables, unused = deal_tables(rng, lens, p)
    k_rows, v_rows = random_rows(rng, lens, hkv, d, std)
    kp, vp = pack_pools(k_rows, v_rows, tables, p, hkv, d)
    q = to_bits(rng.standard_normal((lens.size, hq, d)))
    return dict(q=q, k_rows=k_rows, v_rows=v_rows, kp=kp, vp=vp, tables=tables, lens=lens,
                hkv=hkv, d=d, p=p, unused=unused, scale=np.float32(1.0 / math.sqrt(d)))


def _run(pr, **over):
    a = dict(pr)
    a.update(over)
    return oracle.paged_decode(a["q"], a["kp"], a["vp"], a["tables"], a["lens"], a["scale"],
                               num_kv_heads=a["hkv"])


@pytest.mark.parametrize("hq,hkv,d,lens", [
    (8, 2, 64, [1, 15, 16, 17, 40]),
    (24, 8, 128, [33, 5, 64]),
    (14, 2, 64, [31, 32, 47]),
    (4, 4, 64, [3, 18]),
    (6, 1, 128, [20]),
])
def test_matches_dense_numpy(hq, hkv, d, lens):
    pr = _problem(11, lens, hq, hkv, d)
    out, lse = _run(pr)
    ref, ref_lse = dense_attention_numpy(pr["q"], pr["k_rows"], pr["v_rows"], pr["scale"], hkv)
    assert np.abs(out - ref).max() <= 1e-12
    assert np.abs(lse - ref_lse).max() <= 1e-12


def test_matches_pure_python_loops():
    pr = _problem(5, [1, 7, 19], 6, 2, 64)
    out, _ = _run(pr)
    ref = dense_attention_loops(pr["q"], pr["k_rows"], pr["v_rows"], pr["scale"], 2)
    assert np.abs(out - ref).max() <= 1e-12


def test_distinct_heads_and_dims_are_not_mixed():
    # Structured values: K row of (t, h) is the indicator of dim (t + 3h) % D, V(t, h, d) =
    # (7t + 3h + d) % 128 (exact in bf16).  With q head i = one-hot on
    # dim c_i scaled by 64 the softmax is essentially one-hot at t = (c_i - 3h) % D, so a wrong
    # head mapping, a transposed granule or a shifted token index changes the answer by >= 1.
    hq, hkv, d, L = 4, 2, 64, 48
    lens = np.array([L], dtype=np.int32)
    rng = np.random.default_rng(3)
    tables, _ = deal_tables(rng, lens, 7)
    k = np.zeros((L, hkv, d), dtype=np.float32)
    v = np.zeros((L, hkv, d), dtype=np.float32)
    for t in range(L):
        for h in range(hkv):
            k[t, h, (t + 3 * h) % d] = 1.0
            v[t, h] = (7 * t + 3 * h + np.arange(d)) % 128  # small integers, exact in bf16
    assert np.array_equal(from_bits(to_bits(v)), v.astype(np.float64))
    kp, vp = pack_pools([to_bits(k)], [to_bits(v)], tables, 7, hkv, d)
    cols = [5, 40, 9, 33]
    q = np.zeros((1, hq, d), dtype=np.float32)
    for i, c in enumerate(cols):
        q[0, i, c] = 64.0
    out, _ = oracle.paged_decode(to_bits(q), kp, vp, tables, lens, np.float32(1.0),
                                 num_kv_heads=hkv)
    for i, c in enumerate(cols):
        h = i // 2
        t = (c - 3 * h) % d
        assert t < L
        assert np.abs(out[0, i] - v[t, h]).max() < 1e-9


def test_single_key_returns_that_v_row_exactly():
    pr = _problem(2, [1, 1, 1], 8, 2, 64)
    out, lse = _run(pr)
    for s in range(3):
        for i in range(8):
            assert np.array_equal(out[s, i], from_bits(pr["v_rows"][s][0, i // 4]))
    # lse of a single score is the score itself
    ref, ref_lse = dense_attention_numpy(pr["q"], pr["k_rows"], pr["v_rows"], pr["scale"], 2)
    assert np.abs(lse - ref_lse).max() <= 1e-13


def test_equal_scores_return_mean_of_v():
    pr = _problem(4, [37, 16], 8, 2, 64)
    k_rows = [np.repeat(kr[:1], kr.shape[0], axis=0) for kr in pr["k_rows"]]  # all keys identical
    kp, vp = pack_pools(k_rows, pr["v_rows"], pr["tables"], pr["p"], 2, 64)
    out, _ = _run(pr, kp=kp, vp=vp)
    for s, L in enumerate(pr["lens"]):
        mean = from_bits(pr["v_rows"][s]).mean(axis=0)  # [Hkv, D]
        for i in range(8):
            assert np.abs(out[s, i] - mean[i // 4]).max() <= 1e-13
    # a zero query gives equal scores too, and lse = log L
    out0, lse0 = _run(pr, q=np.zeros_like(pr["q"]))
    for s, L in enumerate(pr["lens"]):
        mean = from_bits(pr["v_rows"][s]).mean(axis=0)
        assert np.abs(out0[s, 0] - mean[0]).max() <= 1e-13
        assert abs(lse0[s, 0] - math.log(int(L))) <= 1e-13


def test_physical_block_permutation_is_bit_identical():
    pr = _problem(6, [50, 3, 129], 8, 2, 64)
    out, lse = _run(pr)
    rng = np.random.default_rng(99)
    sigma = rng.permutation(pr["p"])  # new id of old block b is sigma[b]
    kp2, vp2 = np.empty_like(pr["kp"]), np.empty_like(pr["vp"])
    kp2[sigma] = pr["kp"]
    vp2[sigma] = pr["vp"]
    t2 = pr["tables"].copy()
    t2[t2 >= 0] = sigma[t2[t2 >= 0]]
    out2, lse2 = _run(pr, kp=kp2, vp=vp2, tables=t2)
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)


def test_unread_slots_may_hold_nan_or_inf():
    pr = _problem(7, [21, 16, 1], 8, 2, 64)
    out, _ = _run(pr)
    kp, vp, tables = pr["kp"].copy(), pr["vp"].copy(), pr["tables"].copy()
    kv, vv = k_view(kp, 2, 64), v_view(vp, 2, 64)
    for s, L in enumerate(pr["lens"]):
        last = int(tables[s, (int(L) - 1) // B])
        for t in range(int(L) % B or B, B):  # tail slots of the last block
            kv[last, :, :, t, :] = 0x7F80  # +inf
            vv[last, :, t // 4, :, t % 4] = 0xFFC1  # NaN
        tables[s, (int(L) + B - 1) // B:] = -7  # entries past the last block
    kp[pr["unused"]] = 0x7FFF
    vp[pr["unused"]] = 0xFF80  # -inf
    out2, _ = _run(pr, kp=kp, vp=vp, tables=tables)
    assert np.isfinite(out2).all()
    assert np.array_equal(out, out2)


def test_power_of_two_rescale_is_bit_identical():
    pr = _problem(8, [77, 9], 8, 2, 64)
    out, _ = _run(pr)
    k2 = [to_bits(from_bits(kr) * 2.0) for kr in pr["k_rows"]]
    kp2, vp2 = pack_pools(k2, pr["v_rows"], pr["tables"], pr["p"], 2, 64)
    out2, _ = _run(pr, kp=kp2, vp=vp2, scale=np.float32(pr["scale"] / 2))
    assert np.array_equal(out, out2)


def test_score_shift_leaves_output_unchanged():
    # dim 63 carries q = c and K = 1 for every key: all scores move by c * scale
    pr = _problem(9, [45, 17], 8, 2, 64)
    for kr in pr["k_rows"]:
        kr[:, :, 63] = to_bits(np.float32(1.0))
    q0 = pr["q"].copy()
    q0[:, :, 63] = 0
    q1 = pr["q"].copy()
    q1[:, :, 63] = to_bits(np.float32(48.0))
    kp, vp = pack_pools(pr["k_rows"], pr["v_rows"], pr["tables"], pr["p"], 2, 64)
    o0, l0 = _run(pr, q=q0, kp=kp, vp=vp)
    o1, l1 = _run(pr, q=q1, kp=kp, vp=vp)
    assert np.abs(o0 - o1).max() <= 1e-12
    assert np.abs((l1 - l0) - 48.0 * float(pr["scale"])).max() <= 1e-12


def test_gqa_equals_mha_with_duplicated_kv_heads():
    hq, hkv, d = 12, 4, 64
    pr = _problem(10, [40, 23], hq, hkv, d)
    out, lse = _run(pr)
    g = hq // hkv
    k_rep = [np.repeat(kr, g, axis=1) for kr in pr["k_rows"]]
    v_rep = [np.repeat(vr, g, axis=1) for vr in pr["v_rows"]]
    kp, vp = pack_pools(k_rep, v_rep, pr["tables"], pr["p"], hq, d)
    out2, lse2 = oracle.paged_decode(pr["q"], kp, vp, pr["tables"], pr["lens"], pr["scale"],
                                     num_kv_heads=hq)
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)


def test_output_is_a_convex_combination():
    pr = _problem(12, [90, 2, 31], 8, 2, 64, std=3.0)
    out, _ = _run(pr)
    for s in range(3):
        vf = from_bits(pr["v_rows"][s])
        for i in range(8):
            lo, hi = vf[:, i // 4].min(axis=0), vf[:, i // 4].max(axis=0)
            assert (out[s, i] >= lo - 1e-12).all() and (out[s, i] <= hi + 1e-12).all()


@pytest.mark.parametrize("L", [1, 15, 16, 17, 511, 512, 513])
def test_split_merge_identity(L):
    # Attention over [0, L) equals the lse-weighted merge of attention over any block-aligned
    # partition: o = sum_c exp(lse_c - lse) o_c, lse = log sum_c exp(lse_c).
    hq, hkv, d = 4, 2, 64
    pr = _problem(100 + L, [L], hq, hkv, d)
    out, lse = _run(pr)
    nb = (L + B - 1) // B
    for cut_blocks in sorted({1, nb // 2, nb - 1} - {0, nb}):
        cuts = [0, cut_blocks * B, L]
        parts = []
        for a, b in zip(cuts[:-1], cuts[1:]):
            if b <= a:
                continue
            sub_tables = pr["tables"][:, a // B:].copy()
            o, l = oracle.paged_decode(pr["q"], pr["kp"], pr["vp"], sub_tables,
                                       np.array([b - a], dtype=np.int32), pr["scale"],
                                       num_kv_heads=hkv)
            parts.append((o[0], l[0]))
        m = np.max([l for _, l in parts], axis=0)
        tot = sum(np.exp(l - m) for _, l in parts)
        merged = sum(np.exp(l - m)[:, None] * o for o, l in parts) / tot[:, None]
        assert np.abs(merged - out[0]).max() <= 1e-12
        assert np.abs(m + np.log(tot) - lse[0]).max() <= 1e-12


def test_inactive_stream_gives_zero_and_minus_inf():
    pr = _problem(13, [0, 20, 0], 8, 2, 64)
    out, lse = _run(pr)
    assert (out[0] == 0).all() and (out[2] == 0).all()
    assert np.isneginf(lse[0]).all() and np.isneginf(lse[2]).all()
    assert np.isfinite(lse[1]).all()


def test_stream_subset_matches_full_run():
    pr = _problem(14, [30, 8, 65, 17], 8, 2, 64)
    out, lse = _run(pr)
    o2, l2 = oracle.paged_decode(pr["q"], pr["kp"], pr["vp"], pr["tables"], pr["lens"],
                                 pr["scale"], num_kv_heads=2, streams=(1, 3))
    assert np.array_equal(out[1:3], o2) and np.array_equal(lse[1:3], l2)


def test_bad_block_id_is_an_error():
    pr = _problem(15, [20], 8, 2, 64)
    t = pr["tables"].copy()
    t[0, 1] = pr["p"]  # out of range and needed (20 tokens span two blocks)
    with pytest.raises(RuntimeError):
        _run(pr, tables=t)


# ---------------------------------------------------------------- append / gather


def test_append_writes_exactly_position_L_minus_1():
    hkv, d = 2, 64
    lens = np.array([1, 16, 17, 0, 40], dtype=np.int32)
    pr = _problem(20, lens, 8, hkv, d)
    rng = np.random.default_rng(21)
    k_new = to_bits(rng.standard_normal((lens.size, hkv, d)))
    v_new = to_bits(rng.standard_normal((lens.size, hkv, d)))
    kp, vp = pr["kp"].copy(), pr["vp"].copy()
    oracle.kv_append(k_new, v_new, kp, vp, pr["tables"], lens, head_dim=d)
    # expected pool: repack the logical rows with the last row replaced
    k_rows = [kr.copy() for kr in pr["k_rows"]]
    v_rows = [vr.copy() for vr in pr["v_rows"]]
    for s, L in enumerate(lens):
        if L > 0:
            k_rows[s][L - 1] = k_new[s]
            v_rows[s][L - 1] = v_new[s]
    kp_ref, vp_ref = pack_pools(k_rows, v_rows, pr["tables"], pr["p"], hkv, d)
    assert np.array_equal(kp, kp_ref) and np.array_equal(vp, vp_ref)  # every block, bit for bit
    changed = (kp != pr["kp"]).sum() + (vp != pr["vp"]).sum()
    assert 0 < changed <= 2 * 4 * hkv * d
    # idempotent
    kp2, vp2 = kp.copy(), vp.copy()
    oracle.kv_append(k_new, v_new, kp2, vp2, pr["tables"], lens, head_dim=d)
    assert np.array_equal(kp, kp2) and np.array_equal(vp, vp2)


def test_append_then_decode_sees_the_new_token():
    hkv, d = 2, 64
    lens = np.array([33], dtype=np.int32)
    pr = _problem(22, lens, 4, hkv, d)
    k_new = to_bits(np.zeros((1, hkv, d), dtype=np.float32))
    k_new[0, :, 0] = to_bits(np.float32(64.0))
    v_new = to_bits(np.full((1, hkv, d), 7.0, dtype=np.float32))
    q = np.zeros((1, 4, d), dtype=np.float32)
    q[0, :, 0] = 64.0  # score of the new token dominates every other one by construction
    for kr in pr["k_rows"]:
        kr[:, :, 0] = 0
    kp, vp = pack_pools(pr["k_rows"], pr["v_rows"], pr["tables"], pr["p"], hkv, d)
    oracle.kv_append(k_new, v_new, kp, vp, pr["tables"], lens, head_dim=d)
    out, _ = oracle.paged_decode(to_bits(q), kp, vp, pr["tables"], lens, np.float32(1.0),
                                 num_kv_heads=hkv)
    assert np.abs(out - 7.0).max() < 1e-9


def test_gather_is_bit_exact():
    hkv, d = 2, 128
    lens = np.array([5, 0, 48, 17], dtype=np.int32)
    pr = _problem(23, lens, 4, hkv, d)
    k, v, offs = oracle.kv_gather(pr["kp"], pr["vp"], pr["tables"], lens, num_kv_heads=hkv,
                                  head_dim=d)
    ks, vs = unpack_rows(pr["kp"], pr["vp"], pr["tables"], lens, hkv, d)
    for s, L in enumerate(lens):
        assert np.array_equal(k[offs[s]:offs[s] + L], pr["k_rows"][s])
        assert np.array_equal(v[offs[s]:offs[s] + L], pr["v_rows"][s])
        assert np.array_equal(ks[s], pr["k_rows"][s]) and np.array_equal(vs[s], pr["v_rows"][s])
