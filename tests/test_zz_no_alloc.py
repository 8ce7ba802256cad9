"""The entry point that allocates nothing (built-in scratch memory) against the one that takes a
caller workspace: same kernels, so the outputs must agree bit for bit; and against the oracle."""

import numpy as np
import pytest
import torch

import oracle
from helpers import bits_of
from paper_2602_00269_amd import binding, synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X (torch.cuda.is_available() is False)")
    binding.load()
    return torch.device("cuda:0")


def _i32(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(dev)


def _both(w, dev, host_lens):
    sh = binding.shape_of(w)
    bt, lens = _i32(w.block_tables, dev), _i32(w.context_lens, dev)
    shape = (w.num_streams, w.num_q_heads, w.head_dim)
    host = w.context_lens if host_lens else None
    out_ws = torch.full(shape, float("nan"), device=dev)
    lse_ws = torch.full(shape[:2], float("nan"), device=dev)
    ws = binding.alloc_workspace(sh, dev)
    ws.fill_(0xFF)
    binding.paged_decode(sh, w.q[0], w.k_pool[0], w.v_pool[0], bt, lens, out_ws, ws, lse=lse_ws,
                         context_lens_host=host)
    out_st = torch.full(shape, float("nan"), device=dev)
    lse_st = torch.full(shape[:2], float("nan"), device=dev)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info(dev)[0]  # the driver's own count of free device memory
    binding.paged_decode_static(sh, w.q[0], w.k_pool[0], w.v_pool[0], bt, lens, out_st,
                                lse=lse_st, context_lens_host=host)
    torch.cuda.synchronize()
    if _both.warm:  # the first call on a device looks up the array's address; later ones do nothing
        assert torch.cuda.mem_get_info(dev)[0] == free_before, "the call changed free device memory"
    _both.warm = True
    return out_ws, lse_ws, out_st, lse_st


_both.warm = False


def test_static_scratch_decode_equals_workspace_decode_on_two_calls_in_a_row(dev):
    # first a large call (pool ranges active, thousands of records and descriptors left behind
    # in the scratch array), then a smaller one on the same GPU: nothing of the first may leak
    big = synth.make_custom(np.random.default_rng(430).integers(2900, 3100, size=160), 24, 8, 128,
                            seed=430, device=dev)
    small = synth.make_custom([33, 0, 700, 64, 1, 255, 17], 24, 8, 128, seed=431, device=dev)
    other = synth.make_custom([5, 1000, 0, 64], 14, 2, 64, seed=432, device=dev)  # another shape
    for w, host_lens in ((big, True), (small, True), (big, False), (other, False), (small, False)):
        out_ws, lse_ws, out_st, lse_st = _both(w, dev, host_lens)
        assert torch.equal(out_st, out_ws), f"{w.name} host_lens {host_lens}: outputs differ"
        assert torch.equal(lse_st, lse_ws), f"{w.name} host_lens {host_lens}: lse differs"
        sample = range(w.num_streams) if w.num_streams <= 8 else (0, 1, 80, 159)
        got = out_st.cpu().numpy()
        for s in sample:
            ref, _ = oracle.paged_decode(bits_of(w.q[0]), bits_of(w.k_pool[0]), bits_of(w.v_pool[0]),
                                         w.block_tables, w.context_lens, w.scale,
                                         num_kv_heads=w.num_kv_heads, streams=(s, s + 1))
            err = np.abs(got[s:s + 1].astype(np.float64) - ref)
            assert err.max() <= 5e-3 and err.mean() <= 5e-4, f"{w.name} stream {s}"


def test_static_scratch_decode_refuses_what_does_not_fit(dev):
    # 8192 streams of up to 8192 tokens need far more than 64 MiB of descriptors: refused on the
    # host, nothing launched, outputs untouched
    w = synth.make_custom([40, 7], 8, 2, 64, seed=433, device=dev)
    sh = binding.make_shape(8192, 8, 2, 64, w.num_blocks, 512, w.scale)
    bt = torch.zeros((8192, 512), dtype=torch.int32, device=dev)
    lens = torch.zeros(8192, dtype=torch.int32, device=dev)
    q = torch.zeros((8192, 8, 64), dtype=torch.bfloat16, device=dev)
    out = torch.full((8192, 8, 64), 7.0, device=dev)
    with pytest.raises(binding.VoxError) as e:
        binding.paged_decode_static(sh, q, w.k_pool[0], w.v_pool[0], bt, lens, out)
    assert e.value.code == -6
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    # with the host copy of the (all zero) lengths the same shape fits: every output row zero
    binding.paged_decode_static(sh, q, w.k_pool[0], w.v_pool[0], bt, lens, out,
                                context_lens_host=np.zeros(8192, dtype=np.int32))
    torch.cuda.synchronize()
    assert bool((out == 0).all())


def test_static_scratch_decode_replays_from_a_graph(dev):
    # the callers it is for include code under graph capture: captured after one eager call on
    # the device (which looks up the scratch array), replayed while the device lengths grow
    lens0 = np.array([33, 0, 700, 64, 1, 255, 17, 31], dtype=np.int32)
    w = synth.make_custom(np.where(lens0 > 0, lens0 + 3, 0), 24, 8, 128, seed=434, device=dev)
    sh = binding.shape_of(w)
    bt, lens_d = _i32(w.block_tables, dev), _i32(lens0, dev)
    out = torch.full((w.num_streams, w.num_q_heads, w.head_dim), float("nan"), device=dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        binding.paged_decode_static(sh, w.q[0], w.k_pool[0], w.v_pool[0], bt, lens_d, out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        binding.paged_decode_static(sh, w.q[0], w.k_pool[0], w.v_pool[0], bt, lens_d, out,
                                    context_lens_host=lens0)  # ignored under capture
    lens = lens0.copy()
    for rep in range(3):
        lens = np.where(lens > 0, lens + 1, 0).astype(np.int32)
        lens_d.copy_(torch.from_numpy(lens))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref, _ = oracle.paged_decode(bits_of(w.q[0]), bits_of(w.k_pool[0]), bits_of(w.v_pool[0]),
                                     w.block_tables, lens, w.scale, num_kv_heads=w.num_kv_heads)
        err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
        assert np.isfinite(out.cpu().numpy()).all() and err.max() <= 5e-3 and err.mean() <= 5e-4, rep
