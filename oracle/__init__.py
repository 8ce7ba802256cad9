"""CPU fp64 oracle for the paged decode step (test infrastructure, not product code).

Thin ctypes wrapper over ``vox_oracle.c``; arrays are numpy, bf16 values travel as
uint16 bit patterns.  Importing this package never touches the HIP library.
"""

import ctypes

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        i, f, p = ctypes.c_int, ctypes.c_float, ctypes.c_void_p
        lib.vox_oracle_kv_append.argtypes = [i] * 6 + [p] * 6
        lib.vox_oracle_kv_append.restype = i
        lib.vox_oracle_kv_gather.argtypes = [i] * 6 + [p] * 7
        lib.vox_oracle_kv_gather.restype = i
        lib.vox_oracle_paged_decode.argtypes = [i] * 7 + [f] + [p] * 5 + [i, i, p, p]
        lib.vox_oracle_paged_decode.restype = i
        lib.vox_oracle_kv_append_multi.argtypes = [i] * 6 + [p] * 7
        lib.vox_oracle_kv_append_multi.restype = i
        lib.vox_oracle_paged_prefill.argtypes = [i] * 7 + [f] + [p] * 8
        lib.vox_oracle_paged_prefill.restype = i
        lib.vox_oracle_rope_append.argtypes = [i] * 7 + [p] * 3 + [i] + [p] * 5
        lib.vox_oracle_rope_append.restype = i
        lib.vox_oracle_sample.argtypes = [i, i, p, p, p, i, p, p, p]
        lib.vox_oracle_sample.restype = i
        lib.vox_oracle_sample_weights.argtypes = [i, i, p, p, p, i, p, p]
        lib.vox_oracle_sample_weights.restype = i
        lib.vox_oracle_sample_weight.argtypes = [f]
        lib.vox_oracle_sample_weight.restype = ctypes.c_uint64
        lib.vox_oracle_num_threads.restype = i
        lib.vox_oracle_set_num_threads.argtypes = [i]
        lib.vox_oracle_set_num_threads.restype = None
        _lib = lib
    return _lib


def _u16(a, shape=None):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 data must be passed as uint16 bit patterns")
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"{what} failed with oracle status {rc}")


def num_threads() -> int:
    return int(_load().vox_oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the C oracle may use from now on (0: all processors)."""
    _load().vox_oracle_set_num_threads(int(n))


def kv_append(k_new, v_new, k_pool, v_pool, block_tables, context_lens, *, head_dim, block_size=16):
    """In-place append on uint16 pools shaped [P, Hkv, B*D]."""
    k_new, v_new = _u16(k_new), _u16(v_new)
    bt, lens = _i32(block_tables), _i32(context_lens)
    for pool in (k_pool, v_pool):
        if pool.dtype != np.uint16 or not pool.flags.c_contiguous or not pool.flags.writeable:
            raise TypeError("pools must be writable C-contiguous uint16 arrays")
    s, hkv = k_new.shape[0], k_new.shape[1]
    rc = _load().vox_oracle_kv_append(s, hkv, head_dim, block_size, k_pool.shape[0], bt.shape[1],
                                      _ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool),
                                      _ptr(bt), _ptr(lens))
    _check(rc, "kv_append")


def kv_gather(k_pool, v_pool, block_tables, context_lens, *, num_kv_heads, head_dim, block_size=16):
    """Return (k, v, row_offsets): packed [T, Hkv, D] uint16 rows, stream s at row_offsets[s]."""
    k_pool, v_pool = _u16(k_pool), _u16(v_pool)
    bt, lens = _i32(block_tables), _i32(context_lens)
    offs = np.zeros(lens.size, dtype=np.int64)
    offs[1:] = np.cumsum(lens.astype(np.int64))[:-1]
    total = int(lens.astype(np.int64).sum())
    k = np.zeros((total, num_kv_heads, head_dim), dtype=np.uint16)
    v = np.zeros_like(k)
    rc = _load().vox_oracle_kv_gather(lens.size, num_kv_heads, head_dim, block_size,
                                      k_pool.shape[0], bt.shape[1], _ptr(k_pool), _ptr(v_pool),
                                      _ptr(bt), _ptr(lens), _ptr(offs), _ptr(k), _ptr(v))
    _check(rc, "kv_gather")
    return k, v, offs


def paged_decode(q, k_pool, v_pool, block_tables, context_lens, scale, *, num_kv_heads,
                 block_size=16, streams=None):
    """fp64 (out [n, Hq, D], lse [n, Hq]) for streams ``range(*streams)`` (default: all)."""
    q, k_pool, v_pool = _u16(q), _u16(k_pool), _u16(v_pool)
    bt, lens = _i32(block_tables), _i32(context_lens)
    s, hq, d = q.shape
    s0, s1 = (0, s) if streams is None else streams
    out = np.zeros((s1 - s0, hq, d), dtype=np.float64)
    lse = np.zeros((s1 - s0, hq), dtype=np.float64)
    rc = _load().vox_oracle_paged_decode(s, hq, num_kv_heads, d, block_size, k_pool.shape[0],
                                         bt.shape[1], np.float32(scale), _ptr(q), _ptr(k_pool),
                                         _ptr(v_pool), _ptr(bt), _ptr(lens), s0, s1 - s0,
                                         _ptr(out), _ptr(lse))
    _check(rc, "paged_decode")
    return out, lse


def kv_append_multi(k_new, v_new, k_pool, v_pool, block_tables, context_lens, q_offsets, *,
                    head_dim, block_size=16):
    """In-place append of packed rows [Tq, Hkv, D]; stream s owns rows q_offsets[s]:q_offsets[s+1]."""
    k_new, v_new = _u16(k_new), _u16(v_new)
    bt, lens, qo = _i32(block_tables), _i32(context_lens), _i32(q_offsets)
    for pool in (k_pool, v_pool):
        if pool.dtype != np.uint16 or not pool.flags.c_contiguous or not pool.flags.writeable:
            raise TypeError("pools must be writable C-contiguous uint16 arrays")
    rc = _load().vox_oracle_kv_append_multi(lens.size, k_new.shape[1], head_dim, block_size,
                                            k_pool.shape[0], bt.shape[1], _ptr(k_new),
                                            _ptr(v_new), _ptr(k_pool), _ptr(v_pool), _ptr(bt),
                                            _ptr(lens), _ptr(qo))
    _check(rc, "kv_append_multi")


def paged_prefill(q, k_pool, v_pool, block_tables, context_lens, q_offsets, scale, *,
                  num_kv_heads, block_size=16):
    """Causal multi-token attention: fp64 (out [Tq, Hq, D], lse [Tq, Hq])."""
    q, k_pool, v_pool = _u16(q), _u16(k_pool), _u16(v_pool)
    bt, lens, qo = _i32(block_tables), _i32(context_lens), _i32(q_offsets)
    tq, hq, d = q.shape
    if int(qo[-1]) != tq:
        raise ValueError("q_offsets[-1] must equal the number of query rows")
    out = np.zeros((tq, hq, d), dtype=np.float64)
    lse = np.zeros((tq, hq), dtype=np.float64)
    rc = _load().vox_oracle_paged_prefill(lens.size, hq, num_kv_heads, d, block_size,
                                          k_pool.shape[0], bt.shape[1], np.float32(scale),
                                          _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(bt),
                                          _ptr(lens), _ptr(qo), _ptr(out), _ptr(lse))
    _check(rc, "paged_prefill")
    return out, lse


def rope_append(qkv, rope_cos, rope_sin, k_pool, v_pool, block_tables, context_lens, *,
                num_q_heads, num_kv_heads, block_size=16, q_out=None):
    """Rotate q and k heads of packed rows [S, Hq + 2*Hkv, D] at position L_s - 1, append k / v
    in place, return the rotated q [S, Hq, D] (uint16; rows of empty streams keep ``q_out``)."""
    qkv = _u16(qkv)
    bt, lens = _i32(block_tables), _i32(context_lens)
    cos = np.ascontiguousarray(rope_cos, dtype=np.float32)
    sin = np.ascontiguousarray(rope_sin, dtype=np.float32)
    s, heads, d = qkv.shape
    if heads != num_q_heads + 2 * num_kv_heads or cos.shape != sin.shape or cos.shape[1] != d // 2:
        raise ValueError("qkv / table shapes do not match the head counts")
    for pool in (k_pool, v_pool):
        if pool.dtype != np.uint16 or not pool.flags.c_contiguous or not pool.flags.writeable:
            raise TypeError("pools must be writable C-contiguous uint16 arrays")
    if q_out is None:
        q_out = np.zeros((s, num_q_heads, d), dtype=np.uint16)
    rc = _load().vox_oracle_rope_append(s, num_q_heads, num_kv_heads, d, block_size,
                                        k_pool.shape[0], bt.shape[1], _ptr(qkv), _ptr(cos),
                                        _ptr(sin), cos.shape[0], _ptr(q_out), _ptr(k_pool),
                                        _ptr(v_pool), _ptr(bt), _ptr(lens))
    _check(rc, "rope_append")
    return q_out


SAMPLING_DTYPE = np.dtype([("temperature", np.float32), ("top_p", np.float32),
                           ("repetition_penalty", np.float32), ("top_k", np.int32)])


def sampling_params(temperature, top_p, repetition_penalty, top_k, n=None):
    """Structured array of per-stream sampling parameters (scalars broadcast to ``n``)."""
    cols = [np.atleast_1d(np.asarray(c)) for c in (temperature, top_p, repetition_penalty, top_k)]
    n = max(c.size for c in cols) if n is None else n
    out = np.zeros(n, dtype=SAMPLING_DTYPE)
    for name, c in zip(("temperature", "top_p", "repetition_penalty", "top_k"), cols):
        out[name] = np.broadcast_to(c, (n,))
    return out


def sample(logits, params, uniforms, history=None):
    """(tokens [S] int32, kept [S] int32) for fp32 logits [S, V] and ``sampling_params``."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    s, v = logits.shape
    params = np.ascontiguousarray(params, dtype=SAMPLING_DTYPE)
    u = np.ascontiguousarray(uniforms, dtype=np.float32)
    if params.shape != (s,) or u.shape != (s,):
        raise ValueError("params and uniforms must have one entry per stream")
    window = 0
    hist_ptr = None
    if history is not None:
        history = np.ascontiguousarray(history, dtype=np.int32)
        if history.ndim != 2 or history.shape[0] != s:
            raise ValueError("history must be [S, window]")
        window = history.shape[1]
        hist_ptr = _ptr(history)
    tokens = np.zeros(s, dtype=np.int32)
    kept = np.zeros(s, dtype=np.int32)
    rc = _load().vox_oracle_sample(s, v, _ptr(logits), _ptr(params), hist_ptr, window, _ptr(u),
                                   _ptr(tokens), _ptr(kept))
    _check(rc, "sample")
    return tokens, kept


def sample_weight(d: float) -> int:
    """The integer softmax weight 2^40 * exp(-d) of the fixed sampling arithmetic."""
    return int(_load().vox_oracle_sample_weight(np.float32(d)))


def sample_weights(logits, params, history=None):
    """(d [S, V] float32, w [S, V] uint64): distance to the maximum and integer weight per token."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    s, v = logits.shape
    params = np.ascontiguousarray(params, dtype=SAMPLING_DTYPE)
    window, hist_ptr = 0, None
    if history is not None:
        history = np.ascontiguousarray(history, dtype=np.int32)
        window, hist_ptr = history.shape[1], _ptr(history)
    d = np.zeros((s, v), dtype=np.float32)
    w = np.zeros((s, v), dtype=np.uint64)
    rc = _load().vox_oracle_sample_weights(s, v, _ptr(logits), _ptr(params), hist_ptr, window,
                                           _ptr(d), _ptr(w))
    _check(rc, "sample_weights")
    return d, w
