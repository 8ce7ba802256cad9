"""Writes tests/golden/oracle_decode_samples.json by calling ONLY the CPU oracle.

The paper prints no value for the decode step, so this fixture does not pin the oracle to the
paper; it freezes the oracle's own answers on a platform-independent integer-pattern input so
that (a) an accidental change to the oracle shows up on the CPU and (b) the GPU library can be
checked against stored values without running the oracle.  Inputs come from
`golden_problem()` below (pure integer arithmetic, values exact in bf16).

Run from the repository root:  python tests/golden/make_golden.py
"""

import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

OUT = os.path.join(HERE, "oracle_decode_samples.json")


def _bits(x):
    """float32 array whose values are exact in bf16 -> uint16 bit patterns."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32)
    assert (u & 0xFFFF).max() == 0, "pattern values must be exact in bf16"
    return (u >> 16).astype(np.uint16)


def golden_problem():
    """4 streams, 8 q heads, 2 kv heads, head_dim 64; pools filled by an integer pattern."""
    s, hq, hkv, d, p = 4, 8, 2, 64, 40
    lens = np.array([1, 37, 0, 200], dtype=np.int32)
    nb = (lens + 15) // 16
    tables = np.full((s, int(nb.max())), -1, dtype=np.int32)
    ids = [(7 * i + 3) % p for i in range(p)]  # a fixed permutation of the pool
    pos = 0
    for i in range(s):
        tables[i, :nb[i]] = ids[pos:pos + nb[i]]
        pos += int(nb[i])
    n = p * hkv * 16 * d
    idx = np.arange(n, dtype=np.int64)
    k_pool = _bits(((idx * 37 + 11) % 61 - 30) / 16.0).reshape(p, hkv, 16 * d)
    v_pool = _bits(((idx * 53 + 5) % 127 - 63) / 32.0).reshape(p, hkv, 16 * d)
    qi = np.arange(s * hq * d, dtype=np.int64)
    q = _bits(((qi * 29 + 7) % 31 - 15) / 8.0).reshape(s, hq, d)
    return dict(q=q, k_pool=k_pool, v_pool=v_pool, tables=tables, lens=lens, hkv=hkv,
                scale=np.float32(0.125))


def main():
    import oracle

    pr = golden_problem()
    out, lse = oracle.paged_decode(pr["q"], pr["k_pool"], pr["v_pool"], pr["tables"], pr["lens"],
                                   pr["scale"], num_kv_heads=pr["hkv"])
    samples = []
    for s in range(out.shape[0]):
        for i in (0, 3, 7):
            for d in (0, 1, 31, 63):
                samples.append([s, i, d, float(out[s, i, d])])
    doc = {
        "comment": "fp64 oracle outputs on tests/golden/make_golden.py:golden_problem(); the "
                   "paper (Section 3.1.1 names only the attention backend) prints no values",
        "out_samples": samples,
        "lse": [[float(x) if np.isfinite(x) else None for x in row] for row in lse],
    }
    with open(OUT, "w") as f:
        json.dump(doc, f, indent=1)
    print("wrote", OUT)


if __name__ == "__main__":
    main()
