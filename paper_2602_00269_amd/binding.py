"""ctypes binding to libvox.so: argument marshalling only.

Tensors are torch CUDA tensors (device memory owner); every step of the decode path runs in
the HIP kernels behind the C ABI declared in ``include/vox.h``.  There is no fallback: if the
library is missing, loading raises.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvox.so")

PATH_AUTO, PATH_MFMA, PATH_VALU = 0, 1, 2


class VoxShape(ctypes.Structure):
    _fields_ = [
        ("num_streams", ctypes.c_int32),
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("block_size", ctypes.c_int32),
        ("num_blocks", ctypes.c_int32),
        ("max_blocks_per_stream", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("decode_path", ctypes.c_int32),
        ("split_waves", ctypes.c_int32),
    ]


class VoxError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


_lib = None


def load() -> ctypes.CDLL:
    """Load libvox.so from the package directory; raise if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} not found: build it with `python -m paper_2602_00269_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    sp = ctypes.POINTER(VoxShape)
    lib.vox_kv_append.argtypes = [sp] + [vp] * 7
    lib.vox_kv_append.restype = ctypes.c_int
    lib.vox_kv_gather.argtypes = [sp] + [vp] * 8
    lib.vox_kv_gather.restype = ctypes.c_int
    lib.vox_paged_decode_workspace_bytes.argtypes = [sp]
    lib.vox_paged_decode_workspace_bytes.restype = ctypes.c_size_t
    lib.vox_paged_decode.argtypes = [sp] + [vp] * 9 + [ctypes.c_size_t, vp]
    lib.vox_paged_decode.restype = ctypes.c_int
    lib.vox_paged_decode_profiled.argtypes = [sp] + [vp] * 9 + [ctypes.c_size_t, vp, vp, vp, vp]
    lib.vox_paged_decode_profiled.restype = ctypes.c_int
    lib.vox_paged_decode_static.argtypes = [sp] + [vp] * 9
    lib.vox_paged_decode_static.restype = ctypes.c_int
    lib.vox_decode_step.argtypes = [sp, i32] + [vp] * 10 + [ctypes.c_size_t, vp]
    lib.vox_decode_step.restype = ctypes.c_int
    lib.vox_decode_plan.argtypes = [sp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.vox_decode_plan.restype = ctypes.c_int
    lib.vox_decode_layer.argtypes = [sp, i32] + [vp] * 11 + [ctypes.c_size_t, vp]
    lib.vox_decode_layer.restype = ctypes.c_int
    lib.vox_rope_append.argtypes = [sp, vp, vp, vp, i32] + [vp] * 6
    lib.vox_rope_append.restype = ctypes.c_int
    lib.vox_decode_step_rope.argtypes = [sp, i32, vp, vp, vp, i32] + [vp] * 8 + [ctypes.c_size_t, vp]
    lib.vox_decode_step_rope.restype = ctypes.c_int
    lib.vox_paged_prefill_workspace_bytes.argtypes = [sp, i32]
    lib.vox_paged_prefill_workspace_bytes.restype = ctypes.c_size_t
    lib.vox_kv_append_multi.argtypes = [sp] + [vp] * 7 + [i32, vp]
    lib.vox_kv_append_multi.restype = ctypes.c_int
    lib.vox_paged_prefill.argtypes = [sp] + [vp] * 11 + [ctypes.c_size_t, vp]
    lib.vox_paged_prefill.restype = ctypes.c_int
    lib.vox_paged_prefill_profiled.argtypes = [sp] + [vp] * 11 + [ctypes.c_size_t, vp, vp, vp]
    lib.vox_paged_prefill_profiled.restype = ctypes.c_int
    lib.vox_prefill_plan.argtypes = [sp] + [vp] * 6 + [ctypes.c_size_t, vp]
    lib.vox_prefill_plan.restype = ctypes.c_int
    lib.vox_prefill_layer.argtypes = [sp, i32] + [vp] * 13 + [ctypes.c_size_t, vp]
    lib.vox_prefill_layer.restype = ctypes.c_int
    lib.vox_sample.argtypes = [i32, i32, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.vox_sample.restype = ctypes.c_int
    lib.vox_sample_weights.argtypes = [i32, i32, vp, vp, vp, i32, vp, vp, vp]
    lib.vox_sample_weights.restype = ctypes.c_int
    lib.vox_read_probe.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.vox_read_probe.restype = ctypes.c_int
    lib.vox_strerror.argtypes = [ctypes.c_int]
    lib.vox_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load().vox_strerror(code).decode()


def make_shape(num_streams, num_q_heads, num_kv_heads, head_dim, num_blocks,
               max_blocks_per_stream, scale, block_size=16, decode_path=PATH_AUTO,
               split_waves=0) -> VoxShape:
    return VoxShape(num_streams, num_q_heads, num_kv_heads, head_dim, block_size, num_blocks,
                    max_blocks_per_stream, float(scale), decode_path, split_waves)


def shape_of(w, decode_path=PATH_AUTO, split_waves=0) -> VoxShape:
    """VoxShape of a ``synth.Workload``."""
    return make_shape(w.num_streams, w.num_q_heads, w.num_kv_heads, w.head_dim, w.num_blocks,
                      w.max_blocks_per_stream, w.scale, w.block_size, decode_path, split_waves)


def _dev(t: Optional[torch.Tensor], dtype, what: str, optional=False):
    if t is None:
        if optional:
            return None
        raise TypeError(f"{what} is required")
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{what} must be a contiguous CUDA tensor of dtype {dtype}")
    return ctypes.c_void_p(t.data_ptr())  # NULL for an empty tensor


def _host_lens(a):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(ctypes.c_void_p)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(rc, what):
    if rc != 0:
        raise VoxError(rc, what)


def kv_append(shape, k_new, v_new, k_pool, v_pool, block_tables, context_lens, stream=None):
    bf, i32 = torch.bfloat16, torch.int32
    rc = load().vox_kv_append(ctypes.byref(shape), _dev(k_new, bf, "k_new"),
                              _dev(v_new, bf, "v_new"), _dev(k_pool, bf, "k_pool"),
                              _dev(v_pool, bf, "v_pool"), _dev(block_tables, i32, "block_tables"),
                              _dev(context_lens, i32, "context_lens"), _stream(stream))
    _check(rc, "vox_kv_append")


def kv_gather(shape, k_pool, v_pool, block_tables, context_lens, row_offsets, k_out, v_out,
              stream=None):
    bf, i32 = torch.bfloat16, torch.int32
    rc = load().vox_kv_gather(ctypes.byref(shape), _dev(k_pool, bf, "k_pool"),
                              _dev(v_pool, bf, "v_pool"), _dev(block_tables, i32, "block_tables"),
                              _dev(context_lens, i32, "context_lens"),
                              _dev(row_offsets, torch.int64, "row_offsets"),
                              _dev(k_out, bf, "k_out"), _dev(v_out, bf, "v_out"), _stream(stream))
    _check(rc, "vox_kv_gather")


def paged_decode_workspace_bytes(shape) -> int:
    n = load().vox_paged_decode_workspace_bytes(ctypes.byref(shape))
    if n == 0:
        raise VoxError(-2, "vox_paged_decode_workspace_bytes")
    return int(n)


def alloc_workspace(shape, device="cuda", nbytes: Optional[int] = None) -> torch.Tensor:
    n = paged_decode_workspace_bytes(shape) if nbytes is None else nbytes
    return torch.empty(n, dtype=torch.uint8, device=device)  # torch allocations are 256-B aligned


def paged_decode(shape, q, k_pool, v_pool, block_tables, context_lens, out, workspace, lse=None,
                 context_lens_host=None, stream=None, events=None, wave_clock=None):
    """``events``: optional pair of recorded-once ``torch.cuda.Event(enable_timing=True)``;
    the library re-records them around the attention kernel.  ``wave_clock``: optional int64
    tensor [2 * waves] receiving every wave's start and end clock (100 MHz)."""
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    keep, host = _host_lens(context_lens_host)
    ev0 = ev1 = None
    if events is not None:
        ev0, ev1 = (ctypes.c_void_p(e.cuda_event) for e in events)
    rc = load().vox_paged_decode_profiled(
        ctypes.byref(shape), _dev(q, bf, "q"), _dev(k_pool, bf, "k_pool"),
        _dev(v_pool, bf, "v_pool"), _dev(block_tables, i32, "block_tables"),
        _dev(context_lens, i32, "context_lens"), host, _dev(out, f32, "out"),
        _dev(lse, f32, "lse", optional=True), _dev(workspace, torch.uint8, "workspace"),
        workspace.numel(), _stream(stream), ev0, ev1,
        _dev(wave_clock, torch.int64, "wave_clock", optional=True))
    del keep
    _check(rc, "vox_paged_decode")


def paged_decode_static(shape, q, k_pool, v_pool, block_tables, context_lens, out, lse=None,
                        context_lens_host=None, stream=None):
    """``paged_decode`` on the library's built-in scratch memory: no workspace, no allocation."""
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    keep, host = _host_lens(context_lens_host)
    rc = load().vox_paged_decode_static(
        ctypes.byref(shape), _dev(q, bf, "q"), _dev(k_pool, bf, "k_pool"),
        _dev(v_pool, bf, "v_pool"), _dev(block_tables, i32, "block_tables"),
        _dev(context_lens, i32, "context_lens"), host, _dev(out, f32, "out"),
        _dev(lse, f32, "lse", optional=True), _stream(stream))
    del keep
    _check(rc, "vox_paged_decode_static")


class StepArgs:
    """Host arrays of per-layer device pointers for ``decode_step``, built once and reused."""

    def __init__(self, q: Sequence[torch.Tensor], k_new, v_new, k_pool, v_pool, out):
        bf, f32 = torch.bfloat16, torch.float32
        n = len(q)
        if not all(len(x) == n for x in (k_new, v_new, k_pool, v_pool, out)):
            raise ValueError("per-layer lists must have the same length")
        self.num_layers = n
        self._keep = (q, k_new, v_new, k_pool, v_pool, out)

        def arr(ts, dtype, what):
            a = (ctypes.c_void_p * n)()
            for i, t in enumerate(ts):
                a[i] = _dev(t, dtype, f"{what}[{i}]").value
            return a

        self.q = arr(q, bf, "q")
        self.k_new = arr(k_new, bf, "k_new")
        self.v_new = arr(v_new, bf, "v_new")
        self.k_pool = arr(k_pool, bf, "k_pool")
        self.v_pool = arr(v_pool, bf, "v_pool")
        self.out = arr(out, f32, "out")


def decode_step(shape, args: StepArgs, block_tables, context_lens, workspace,
                context_lens_host=None, stream=None):
    i32 = torch.int32
    keep, host = _host_lens(context_lens_host)
    rc = load().vox_decode_step(ctypes.byref(shape), args.num_layers, args.q, args.k_new,
                                args.v_new, args.k_pool, args.v_pool,
                                _dev(block_tables, i32, "block_tables"),
                                _dev(context_lens, i32, "context_lens"), host, args.out,
                                _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                _stream(stream))
    del keep
    _check(rc, "vox_decode_step")


def decode_plan(shape, block_tables, context_lens, workspace, context_lens_host=None, stream=None):
    """Split-K descriptors of one step, shared by the ``decode_layer`` calls that follow."""
    i32 = torch.int32
    keep, host = _host_lens(context_lens_host)
    rc = load().vox_decode_plan(ctypes.byref(shape), _dev(block_tables, i32, "block_tables"),
                                _dev(context_lens, i32, "context_lens"), host,
                                _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                _stream(stream))
    del keep
    _check(rc, "vox_decode_plan")


def decode_layer(shape, layer, q, k_new, v_new, k_pool, v_pool, block_tables, context_lens, out,
                 workspace, lse=None, context_lens_host=None, stream=None):
    """Append (unless ``k_new`` / ``v_new`` are None) and attention of one layer on the plan."""
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    keep, host = _host_lens(context_lens_host)
    rc = load().vox_decode_layer(
        ctypes.byref(shape), int(layer), _dev(q, bf, "q"), _dev(k_new, bf, "k_new", optional=True),
        _dev(v_new, bf, "v_new", optional=True), _dev(k_pool, bf, "k_pool"),
        _dev(v_pool, bf, "v_pool"), _dev(block_tables, i32, "block_tables"),
        _dev(context_lens, i32, "context_lens"), host, _dev(out, f32, "out"),
        _dev(lse, f32, "lse", optional=True), _dev(workspace, torch.uint8, "workspace"),
        workspace.numel(), _stream(stream))
    del keep
    _check(rc, "vox_decode_layer")


def rope_append(shape, qkv, rope_cos, rope_sin, q_out, k_pool, v_pool, block_tables,
                context_lens, stream=None):
    """Rotate q / k heads of packed rows at position L_s - 1, write q_out, append k / v."""
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    if rope_cos.shape != rope_sin.shape:
        raise ValueError("rope_cos and rope_sin must have the same shape")
    rc = load().vox_rope_append(ctypes.byref(shape), _dev(qkv, bf, "qkv"),
                                _dev(rope_cos, f32, "rope_cos"), _dev(rope_sin, f32, "rope_sin"),
                                int(rope_cos.shape[0]), _dev(q_out, bf, "q_out"),
                                _dev(k_pool, bf, "k_pool"), _dev(v_pool, bf, "v_pool"),
                                _dev(block_tables, i32, "block_tables"),
                                _dev(context_lens, i32, "context_lens"), _stream(stream))
    _check(rc, "vox_rope_append")


class RopeStepArgs:
    """Host arrays of per-layer device pointers for ``decode_step_rope``."""

    def __init__(self, qkv: Sequence[torch.Tensor], q_rot, k_pool, v_pool, out, rope_cos,
                 rope_sin):
        bf, f32 = torch.bfloat16, torch.float32
        n = len(qkv)
        if not all(len(x) == n for x in (q_rot, k_pool, v_pool, out)):
            raise ValueError("per-layer lists must have the same length")
        if rope_cos.shape != rope_sin.shape:
            raise ValueError("rope_cos and rope_sin must have the same shape")
        self.num_layers = n
        self._keep = (qkv, q_rot, k_pool, v_pool, out, rope_cos, rope_sin)

        def arr(ts, dtype, what):
            a = (ctypes.c_void_p * n)()
            for i, t in enumerate(ts):
                a[i] = _dev(t, dtype, f"{what}[{i}]").value
            return a

        self.qkv = arr(qkv, bf, "qkv")
        self.q_rot = arr(q_rot, bf, "q_rot")
        self.k_pool = arr(k_pool, bf, "k_pool")
        self.v_pool = arr(v_pool, bf, "v_pool")
        self.out = arr(out, f32, "out")
        self.rope_cos = _dev(rope_cos, f32, "rope_cos")
        self.rope_sin = _dev(rope_sin, f32, "rope_sin")
        self.rope_positions = int(rope_cos.shape[0])


def decode_step_rope(shape, args: RopeStepArgs, block_tables, context_lens, workspace,
                     context_lens_host=None, stream=None):
    i32 = torch.int32
    keep, host = _host_lens(context_lens_host)
    rc = load().vox_decode_step_rope(ctypes.byref(shape), args.num_layers, args.qkv,
                                     args.rope_cos, args.rope_sin, args.rope_positions,
                                     args.q_rot, args.k_pool, args.v_pool,
                                     _dev(block_tables, i32, "block_tables"),
                                     _dev(context_lens, i32, "context_lens"), host, args.out,
                                     _dev(workspace, torch.uint8, "workspace"),
                                     workspace.numel(), _stream(stream))
    del keep
    _check(rc, "vox_decode_step_rope")


def paged_prefill_workspace_bytes(shape, total_q: int) -> int:
    n = load().vox_paged_prefill_workspace_bytes(ctypes.byref(shape), int(total_q))
    if n == 0:
        raise VoxError(-2, "vox_paged_prefill_workspace_bytes")
    return int(n)


def kv_append_multi(shape, k_new, v_new, k_pool, v_pool, block_tables, context_lens, q_offsets,
                    stream=None):
    bf, i32 = torch.bfloat16, torch.int32
    rc = load().vox_kv_append_multi(ctypes.byref(shape), _dev(k_new, bf, "k_new"),
                                    _dev(v_new, bf, "v_new"), _dev(k_pool, bf, "k_pool"),
                                    _dev(v_pool, bf, "v_pool"),
                                    _dev(block_tables, i32, "block_tables"),
                                    _dev(context_lens, i32, "context_lens"),
                                    _dev(q_offsets, i32, "q_offsets"), int(k_new.shape[0]),
                                    _stream(stream))
    _check(rc, "vox_kv_append_multi")


def paged_prefill(shape, q, k_pool, v_pool, block_tables, context_lens, q_offsets,
                  context_lens_host, q_offsets_host, out, workspace, lse=None, stream=None,
                  events=None):
    """``events``: optional pair of events as in ``paged_decode``."""
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    keep1, lens_h = _host_lens(context_lens_host)
    keep2, qo_h = _host_lens(q_offsets_host)
    ev0 = ev1 = None
    if events is not None:
        ev0, ev1 = (ctypes.c_void_p(e.cuda_event) for e in events)
    rc = load().vox_paged_prefill_profiled(ctypes.byref(shape), _dev(q, bf, "q"),
                                  _dev(k_pool, bf, "k_pool"), _dev(v_pool, bf, "v_pool"),
                                  _dev(block_tables, i32, "block_tables"),
                                  _dev(context_lens, i32, "context_lens"),
                                  _dev(q_offsets, i32, "q_offsets"), lens_h, qo_h,
                                  _dev(out, f32, "out"), _dev(lse, f32, "lse", optional=True),
                                  _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                  _stream(stream), ev0, ev1)
    del keep1, keep2
    _check(rc, "vox_paged_prefill")


def prefill_plan(shape, block_tables, context_lens, q_offsets, context_lens_host, q_offsets_host,
                 workspace, stream=None):
    """Plan of one multi-token step, shared by the ``prefill_layer`` calls that follow."""
    i32 = torch.int32
    keep1, lens_h = _host_lens(context_lens_host)
    keep2, qo_h = _host_lens(q_offsets_host)
    rc = load().vox_prefill_plan(ctypes.byref(shape), _dev(block_tables, i32, "block_tables"),
                                 _dev(context_lens, i32, "context_lens"),
                                 _dev(q_offsets, i32, "q_offsets"), lens_h, qo_h,
                                 _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                 _stream(stream))
    del keep1, keep2
    _check(rc, "vox_prefill_plan")


def prefill_layer(shape, layer, q, k_new, v_new, k_pool, v_pool, block_tables, context_lens,
                  q_offsets, context_lens_host, q_offsets_host, out, workspace, lse=None,
                  stream=None):
    """One layer on the plan ``prefill_plan`` left in ``workspace``; ``k_new`` / ``v_new`` may
    both be None (attention over the cache as it is)."""
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    keep1, lens_h = _host_lens(context_lens_host)
    keep2, qo_h = _host_lens(q_offsets_host)
    rc = load().vox_prefill_layer(ctypes.byref(shape), int(layer), _dev(q, bf, "q"),
                                  _dev(k_new, bf, "k_new", optional=True),
                                  _dev(v_new, bf, "v_new", optional=True),
                                  _dev(k_pool, bf, "k_pool"), _dev(v_pool, bf, "v_pool"),
                                  _dev(block_tables, i32, "block_tables"),
                                  _dev(context_lens, i32, "context_lens"),
                                  _dev(q_offsets, i32, "q_offsets"), lens_h, qo_h,
                                  _dev(out, f32, "out"), _dev(lse, f32, "lse", optional=True),
                                  _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                  _stream(stream))
    del keep1, keep2
    _check(rc, "vox_prefill_layer")


def sampling_params(temperature, top_p, repetition_penalty, top_k, num_streams, device="cuda"):
    """Device array of ``vox_sampling_t`` (one per stream; scalars are broadcast), as an int32
    tensor [S, 4] holding the struct's bytes."""
    a = np.zeros((num_streams, 4), dtype=np.int32)
    f = a.view(np.float32)
    f[:, 0] = np.broadcast_to(np.asarray(temperature, dtype=np.float32), (num_streams,))
    f[:, 1] = np.broadcast_to(np.asarray(top_p, dtype=np.float32), (num_streams,))
    f[:, 2] = np.broadcast_to(np.asarray(repetition_penalty, dtype=np.float32), (num_streams,))
    a[:, 3] = np.broadcast_to(np.asarray(top_k, dtype=np.int32), (num_streams,))
    return torch.from_numpy(a).to(device)


def _sample_args(logits, params, history):
    f32, i32 = torch.float32, torch.int32
    if logits.dim() != 2:
        raise ValueError("logits must be [S, V]")
    s, v = logits.shape
    if tuple(params.shape) != (s, 4):
        raise ValueError("params must be the [S, 4] tensor made by sampling_params")
    window = 0
    hist = None
    if history is not None:
        if history.dim() != 2 or history.shape[0] != s:
            raise ValueError("history must be [S, window]")
        window = int(history.shape[1])
        hist = _dev(history, i32, "history") if window > 0 else None
    return s, v, _dev(logits, f32, "logits"), _dev(params, i32, "params"), hist, window


def sample(logits, params, uniforms, tokens, history=None, kept=None, stream=None):
    """Next token of every stream from fp32 logits [S, V]; writes ``tokens`` (and ``kept``)."""
    s, v, lp, pp, hist, window = _sample_args(logits, params, history)
    rc = load().vox_sample(s, v, lp, pp, hist, window,
                           _dev(uniforms, torch.float32, "uniforms"),
                           _dev(tokens, torch.int32, "tokens"),
                           _dev(kept, torch.int32, "kept", optional=True), _stream(stream))
    _check(rc, "vox_sample")


def sample_weights(logits, params, d_out, w_out, history=None, stream=None):
    """Verification aid: per-token distance to the maximum (fp32) and integer weight (int64 bits)."""
    s, v, lp, pp, hist, window = _sample_args(logits, params, history)
    rc = load().vox_sample_weights(s, v, lp, pp, hist, window,
                                   _dev(d_out, torch.float32, "d_out"),
                                   _dev(w_out, torch.int64, "w_out"), _stream(stream))
    _check(rc, "vox_sample_weights")


def read_probe(buf, sink, stream=None):
    """Stream ``buf`` (uint8 tensor, length a multiple of 16) once; ``sink``: int32 tensor [8192]."""
    rc = load().vox_read_probe(_dev(buf, torch.uint8, "buf"), buf.numel(),
                               _dev(sink, torch.int32, "sink"), _stream(stream))
    _check(rc, "vox_read_probe")
