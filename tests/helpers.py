"""Test-side statements of the cache layout and brute-force references.

These are written independently of both the oracle's C index arithmetic and the HIP
kernels: pools are viewed through numpy reshapes that spell the layout the header documents,
  K granule (blk, h) = [D/32][B][32]   V granule (blk, h) = [B/4][D][4]
"""

import math

import numpy as np
import torch

B = 16


def to_bits(x) -> np.ndarray:
    """float array -> bf16 bit patterns (round to nearest even) as uint16."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bits_of(t: torch.Tensor) -> np.ndarray:
    """bf16 torch tensor (any device) -> uint16 numpy bit patterns."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16).copy()


def from_bits(b) -> np.ndarray:
    """bf16 bit patterns -> exact float64 values."""
    b = np.asarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def k_view(pool: np.ndarray, hkv: int, d: int) -> np.ndarray:
    """[P, Hkv, B*D] -> view indexed [blk, h, d // 32, t, d % 32]."""
    return pool.reshape(pool.shape[0], hkv, d // 32, B, 32)


def v_view(pool: np.ndarray, hkv: int, d: int) -> np.ndarray:
    """[P, Hkv, B*D] -> view indexed [blk, h, t // 4, d, t % 4]."""
    return pool.reshape(pool.shape[0], hkv, B // 4, d, 4)


def pack_pools(k_rows, v_rows, tables, num_blocks, hkv, d, fill=0x7FC0):
    """k_rows[s]: uint16 [L_s, Hkv, D] logical rows -> (k_pool, v_pool) uint16 [P, Hkv, B*D]."""
    kp = np.full((num_blocks, hkv, B * d), fill, dtype=np.uint16)
    vp = np.full((num_blocks, hkv, B * d), fill, dtype=np.uint16)
    kv, vv = k_view(kp, hkv, d), v_view(vp, hkv, d)
    for s, (kr, vr) in enumerate(zip(k_rows, v_rows)):
        for t in range(kr.shape[0]):
            blk = int(tables[s, t // B])
            assert 0 <= blk < num_blocks
            for h in range(hkv):
                kv[blk, h, :, t % B, :] = kr[t, h].reshape(d // 32, 32)
                vv[blk, h, (t % B) // 4, :, t % 4] = vr[t, h]
    return kp, vp


def unpack_rows(k_pool, v_pool, tables, lens, hkv, d):
    """Inverse of pack_pools through the same numpy views: lists of uint16 [L_s, Hkv, D]."""
    kv, vv = k_view(k_pool, hkv, d), v_view(v_pool, hkv, d)
    ks, vs = [], []
    for s, L in enumerate(lens):
        kr = np.zeros((int(L), hkv, d), dtype=np.uint16)
        vr = np.zeros((int(L), hkv, d), dtype=np.uint16)
        for t in range(int(L)):
            blk = int(tables[s, t // B])
            for h in range(hkv):
                kr[t, h] = kv[blk, h, :, t % B, :].reshape(d)
                vr[t, h] = vv[blk, h, (t % B) // 4, :, t % 4]
        ks.append(kr)
        vs.append(vr)
    return ks, vs


def dense_attention_numpy(q_bits, k_rows, v_rows, scale, hkv):
    """softmax(q K^T * scale) V with numpy matmuls on contiguous rows; fp64.  Returns out, lse."""
    s, hq, d = q_bits.shape
    g = hq // hkv
    out = np.zeros((s, hq, d))
    lse = np.full((s, hq), -np.inf)
    qf = from_bits(q_bits)
    sc = float(np.float32(scale))
    for si in range(s):
        if k_rows[si].shape[0] == 0:
            continue
        kf, vf = from_bits(k_rows[si]), from_bits(v_rows[si])
        for i in range(hq):
            z = sc * (kf[:, i // g, :] @ qf[si, i])
            m = z.max()
            e = np.exp(z - m)
            out[si, i] = (e / e.sum()) @ vf[:, i // g, :]
            lse[si, i] = m + math.log(e.sum())
    return out, lse


def dense_attention_loops(q_bits, k_rows, v_rows, scale, hkv):
    """The same definition as nested pure-Python loops with math.fsum (tiny inputs only)."""
    s, hq, d = q_bits.shape
    g = hq // hkv
    qf = from_bits(q_bits).tolist()
    sc = float(np.float32(scale))
    out = np.zeros((s, hq, d))
    for si in range(s):
        kf, vf = from_bits(k_rows[si]).tolist(), from_bits(v_rows[si]).tolist()
        n = len(kf)
        if n == 0:
            continue
        for i in range(hq):
            h = i // g
            z = [sc * math.fsum(qf[si][i][x] * kf[t][h][x] for x in range(d)) for t in range(n)]
            m = max(z)
            e = [math.exp(v - m) for v in z]
            tot = math.fsum(e)
            for x in range(d):
                out[si, i, x] = math.fsum(e[t] * vf[t][h][x] for t in range(n)) / tot
    return out


def random_rows(rng, lens, hkv, d, std=1.0):
    k_rows = [to_bits(rng.standard_normal((int(L), hkv, d)) * std) for L in lens]
    v_rows = [to_bits(rng.standard_normal((int(L), hkv, d)) * std) for L in lens]
    return k_rows, v_rows


def deal_tables(rng, lens, num_blocks):
    nb = [(int(L) + B - 1) // B for L in lens]
    width = max(1, max(nb) if nb else 1)
    perm = rng.permutation(num_blocks)
    tables = np.full((len(lens), width), -1, dtype=np.int32)
    pos = 0
    for s, n in enumerate(nb):
        tables[s, :n] = perm[pos:pos + n]
        pos += n
    return tables, perm[pos:]
