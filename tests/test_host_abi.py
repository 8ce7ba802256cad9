"""Host-only checks of the C-ABI library: it loads, exports what the header declares, and its
argument validation and workspace planning answer without touching a GPU."""

import ctypes
import os
import re

import pytest

from paper_2602_00269_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2602_00269_amd import build
        build.build(verbose=False)
    return binding.load()


def _declared():
    text = open(os.path.join(ROOT, "include", "vox.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vox_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert {"vox_kv_append", "vox_kv_gather", "vox_paged_decode", "vox_decode_step",
            "vox_paged_decode_workspace_bytes", "vox_paged_decode_profiled", "vox_strerror",
            "vox_kv_append_multi", "vox_paged_prefill", "vox_paged_prefill_profiled",
            "vox_paged_prefill_workspace_bytes", "vox_rope_append", "vox_decode_step_rope", "vox_sample",
            "vox_sample_weights", "vox_paged_decode_static", "vox_decode_plan",
            "vox_decode_layer", "vox_prefill_plan", "vox_prefill_layer"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_struct_matches_header():
    assert ctypes.sizeof(binding.VoxShape) == 40
    text = open(os.path.join(ROOT, "include", "vox.h")).read()
    body = text[text.index("typedef struct {"):text.index("} vox_shape_t;")]
    fields = re.findall(r"(?:int32_t|float)\s+(\w+);", body)
    assert fields == [f[0] for f in binding.VoxShape._fields_]


def _shape(**kw):
    a = dict(num_streams=4, num_q_heads=8, num_kv_heads=2, head_dim=64, num_blocks=128,
             max_blocks_per_stream=16, scale=0.125)
    a.update(kw)
    return binding.make_shape(**a)


@pytest.mark.parametrize("kw", [dict(num_streams=0), dict(num_q_heads=7), dict(head_dim=96),
                                dict(block_size=32), dict(num_q_heads=18, num_kv_heads=2),
                                dict(num_blocks=0), dict(max_blocks_per_stream=0),
                                dict(num_streams=8193)])
def test_bad_shapes_are_rejected_before_any_launch(lib, kw):
    sh = _shape(**kw)
    one = ctypes.c_void_p(256)
    rc = lib.vox_kv_append(ctypes.byref(sh), one, one, one, one, one, one, None)
    assert rc == -2
    assert lib.vox_paged_decode_workspace_bytes(ctypes.byref(sh)) == 0
    rc = lib.vox_paged_decode(ctypes.byref(sh), one, one, one, one, one, None, one, None, one,
                              1 << 20, None)
    assert rc == -2


def test_null_pointers_and_bad_scalars(lib):
    sh = _shape()
    one = ctypes.c_void_p(256)
    assert lib.vox_kv_append(ctypes.byref(sh), None, one, one, one, one, one, None) == -1
    assert lib.vox_paged_decode(ctypes.byref(sh), one, one, one, one, one, None, None, None, one,
                                1 << 20, None) == -1
    assert lib.vox_kv_append(None, one, one, one, one, one, one, None) == -1
    assert lib.vox_kv_gather(ctypes.byref(sh), one, one, one, one, None, one, one, None) == -1
    assert lib.vox_decode_step(ctypes.byref(sh), 0, one, one, one, one, one, one, one, None, one,
                               one, 1 << 20, None) == -5
    for kw in (dict(split_waves=-1), dict(split_waves=1 << 21), dict(decode_path=9),
               dict(scale=float("nan"))):
        bad = _shape(**kw)
        assert lib.vox_kv_append(ctypes.byref(bad), one, one, one, one, one, one, None) == -5
    # misaligned workspace
    assert lib.vox_paged_decode(ctypes.byref(sh), one, one, one, one, one, None, one, None,
                                ctypes.c_void_p(257), 1 << 20, None) == -5
    # tensors are accessed 16 bytes at a time: a base address that is no multiple of 16 is refused
    odd = ctypes.c_void_p(264)
    assert lib.vox_kv_append(ctypes.byref(sh), odd, one, one, one, one, one, None) == -5
    assert lib.vox_kv_append(ctypes.byref(sh), one, one, one, odd, one, one, None) == -5
    assert lib.vox_paged_decode(ctypes.byref(sh), odd, one, one, one, one, None, one, None, one,
                                1 << 20, None) == -5
    assert lib.vox_paged_decode(ctypes.byref(sh), one, one, one, one, one, None, odd, None, one,
                                1 << 20, None) == -5
    assert lib.vox_kv_gather(ctypes.byref(sh), one, one, one, one, one, odd, one, None) == -5
    assert lib.vox_kv_append_multi(ctypes.byref(sh), one, odd, one, one, one, one, one, 3,
                                   None) == -5


def test_multi_token_calls_validate_on_the_host(lib):
    sh = _shape()
    one = ctypes.c_void_p(256)
    i32 = ctypes.c_int32
    lens = (i32 * 4)(40, 7, 0, 3)
    zeros = (i32 * 5)(0, 0, 0, 0, 0)
    # no rows: accepted with empty (NULL) row arrays, nothing is launched
    assert lib.vox_kv_append_multi(ctypes.byref(sh), None, None, one, one, one, one, one, 0,
                                   None) == 0
    assert lib.vox_paged_prefill(ctypes.byref(sh), None, one, one, one, one, one, lens, zeros,
                                 None, None, one, 1 << 20, None) == 0
    assert lib.vox_kv_append_multi(ctypes.byref(sh), one, one, one, one, one, one, one, -1,
                                   None) == -5
    # host copies are required
    assert lib.vox_paged_prefill(ctypes.byref(sh), one, one, one, one, one, one, None, zeros,
                                 one, None, one, 1 << 20, None) == -1
    # more new tokens than the stream holds, offsets that do not start at zero
    bad = (i32 * 5)(0, 41, 41, 41, 41)
    assert lib.vox_paged_prefill(ctypes.byref(sh), one, one, one, one, one, one, lens, bad, one,
                                 None, one, 1 << 20, None) == -5
    shifted = (i32 * 5)(1, 2, 2, 2, 2)
    assert lib.vox_paged_prefill(ctypes.byref(sh), one, one, one, one, one, one, lens, shifted,
                                 one, None, one, 1 << 20, None) == -5
    # workspace too small for one real row
    ok = (i32 * 5)(0, 1, 1, 1, 1)
    assert lib.vox_paged_prefill(ctypes.byref(sh), one, one, one, one, one, one, lens, ok, one,
                                 None, one, 64, None) == -3
    assert lib.vox_paged_prefill_workspace_bytes(ctypes.byref(sh), 5) > 0
    assert lib.vox_paged_prefill_workspace_bytes(ctypes.byref(sh), -1) == 0
    # it has room for the decode kernels' workspace too (mixed batches use both)
    assert (lib.vox_paged_prefill_workspace_bytes(ctypes.byref(sh), 5) >
            lib.vox_paged_decode_workspace_bytes(ctypes.byref(sh)))


def test_multi_token_plan_and_layer_calls_validate_on_the_host(lib):
    sh = _shape()
    one, odd = ctypes.c_void_p(256), ctypes.c_void_p(264)
    i32 = ctypes.c_int32
    lens = (i32 * 4)(40, 7, 0, 3)
    qo = (i32 * 5)(0, 5, 5, 5, 8)
    big = 1 << 22
    none = (i32 * 5)(0, 0, 0, 0, 0)
    # no rows: nothing to plan or run
    assert lib.vox_prefill_plan(ctypes.byref(sh), None, None, None, lens, none, None, 0, None) == 0
    # plan: host copies and device arrays are required, workspace aligned and large enough
    assert lib.vox_prefill_plan(ctypes.byref(sh), one, one, one, None, qo, one, big, None) == -1
    assert lib.vox_prefill_plan(ctypes.byref(sh), one, None, one, lens, qo, one, big, None) == -1
    assert lib.vox_prefill_plan(ctypes.byref(sh), one, one, one, lens, qo, ctypes.c_void_p(257),
                                big, None) == -5
    assert lib.vox_prefill_plan(ctypes.byref(sh), one, one, one, lens, qo, one, 64, None) == -3
    bad = (i32 * 5)(0, 41, 41, 41, 41)  # more new tokens than the stream holds
    assert lib.vox_prefill_plan(ctypes.byref(sh), one, one, one, lens, bad, one, big, None) == -5
    # layer: index range, k_new without v_new, missing and misaligned tensors
    # q k_new v_new k_pool v_pool bt lens qo | lens_host qo_host | out lse ws bytes stream
    args = [one, None, None, one, one, one, one, one, lens, qo, one, None, one, big, None]
    assert lib.vox_prefill_layer(ctypes.byref(sh), -1, *args) == -5
    assert lib.vox_prefill_layer(ctypes.byref(sh), 4096, *args) == -5
    a = list(args)
    a[1] = one
    assert lib.vox_prefill_layer(ctypes.byref(sh), 0, *a) == -1
    for missing in (0, 3, 4, 5, 6, 7, 10, 12):
        a = list(args)
        a[missing] = None
        assert lib.vox_prefill_layer(ctypes.byref(sh), 0, *a) == -1, missing
    for odd_at in (0, 3, 10):
        a = list(args)
        a[odd_at] = odd
        assert lib.vox_prefill_layer(ctypes.byref(sh), 0, *a) == -5, odd_at
    a = list(args)
    a[13] = 64
    assert lib.vox_prefill_layer(ctypes.byref(sh), 0, *a) == -3


def test_rope_calls_validate_on_the_host(lib):
    sh = _shape()  # 16 blocks per stream: positions 0..255
    one = ctypes.c_void_p(256)
    assert lib.vox_rope_append(ctypes.byref(sh), one, one, one, 255, one, one, one, one, one,
                               None) == -5  # table shorter than the positions the shape admits
    assert lib.vox_rope_append(ctypes.byref(sh), None, one, one, 256, one, one, one, one, one,
                               None) == -1
    assert lib.vox_decode_step_rope(ctypes.byref(sh), 0, one, one, one, 256, one, one, one, one,
                                    one, None, one, one, 1 << 20, None) == -5
    assert lib.vox_decode_step_rope(ctypes.byref(sh), 1, None, one, one, 256, one, one, one, one,
                                    one, None, one, one, 1 << 20, None) == -1


def test_sampling_call_validates_on_the_host(lib):
    one = ctypes.c_void_p(256)
    # streams, vocab, logits, params, history, window, uniforms, tokens, kept, stream
    assert lib.vox_sample(4, (1 << 18) + 1, one, one, None, 0, one, one, None, None) == -2
    assert lib.vox_sample(0, 100, one, one, None, 0, one, one, None, None) == -2
    assert lib.vox_sample(4, 100, one, one, None, -1, one, one, None, None) == -2
    assert lib.vox_sample(4, 100, None, one, None, 0, one, one, None, None) == -1
    assert lib.vox_sample(4, 100, one, one, None, 8, one, one, None, None) == -1  # window without history
    assert lib.vox_sample_weights(4, 100, one, one, None, 0, None, one, None) == -1
    assert ctypes.sizeof(ctypes.c_float) * 3 + 4 == 16  # vox_sampling_t: three floats and an int32


def test_layer_by_layer_and_static_calls_validate_on_the_host(lib):
    sh = _shape()
    one, odd = ctypes.c_void_p(256), ctypes.c_void_p(264)
    big = 1 << 20
    # plan: null pointers, misaligned or too small workspace, bad shape
    assert lib.vox_decode_plan(ctypes.byref(sh), None, one, None, one, big, None) == -1
    assert lib.vox_decode_plan(ctypes.byref(sh), one, one, None, None, big, None) == -1
    assert lib.vox_decode_plan(ctypes.byref(sh), one, one, None, ctypes.c_void_p(257), big, None) == -5
    assert lib.vox_decode_plan(ctypes.byref(sh), one, one, None, one, 64, None) == -3
    assert lib.vox_decode_plan(ctypes.byref(_shape(head_dim=96)), one, one, None, one, big, None) == -2
    # layer: index range, pointers, k_new without v_new, alignment, workspace
    args = [one] * 7 + [None, one, None, one, big, None]  # q k_new v_new k_pool v_pool bt lens | host out lse ws bytes stream
    assert lib.vox_decode_layer(ctypes.byref(sh), -1, *args) == -5
    assert lib.vox_decode_layer(ctypes.byref(sh), 4096, *args) == -5
    for missing in (0, 3, 4, 5, 6, 8, 10):
        a = list(args)
        a[missing] = None
        assert lib.vox_decode_layer(ctypes.byref(sh), 0, *a) == -1, missing
    a = list(args)
    a[2] = None  # v_new without k_new's partner
    assert lib.vox_decode_layer(ctypes.byref(sh), 0, *a) == -1
    for bad in (0, 1, 3, 8):
        a = list(args)
        a[bad] = odd
        assert lib.vox_decode_layer(ctypes.byref(sh), 0, *a) == -5, bad
    a = list(args)
    a[11] = 64
    assert lib.vox_decode_layer(ctypes.byref(sh), 0, *a) == -3
    # the static-scratch call checks its arguments before it looks for a device
    assert lib.vox_paged_decode_static(ctypes.byref(sh), None, one, one, one, one, None, one, None,
                                       None) == -1
    assert lib.vox_paged_decode_static(ctypes.byref(_shape(num_streams=0)), one, one, one, one, one,
                                       None, one, None, None) == -2
    assert binding.strerror(-6)


def test_workspace_too_small_is_reported(lib):
    sh = _shape()
    one = ctypes.c_void_p(256)
    assert binding.paged_decode_workspace_bytes(sh) > 0
    rc = lib.vox_paged_decode(ctypes.byref(sh), one, one, one, one, one, None, one, None, one, 64,
                              None)
    assert rc == -3


def test_workspace_sizes_for_the_presets(lib):
    # recommended sizes stay modest even when only the shape is known
    for s, hq, hkv, d, p, mnb in [(256, 24, 8, 128, 45000, 250), (512, 24, 8, 128, 55000, 512),
                                  (1024, 14, 2, 64, 170000, 256)]:
        sh = binding.make_shape(s, hq, hkv, d, p, mnb, 0.1)
        assert 0 < binding.paged_decode_workspace_bytes(sh) < (1 << 28)


def test_strerror_is_total(lib):
    for code in (0, -1, -2, -3, -4, -5, -99, 7):
        assert binding.strerror(code)
