"""Stored oracle answers on a platform-independent integer-pattern input."""

import importlib.util
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
_spec = importlib.util.spec_from_file_location("make_golden",
                                               os.path.join(HERE, "golden", "make_golden.py"))
make_golden = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(make_golden)

with open(os.path.join(HERE, "golden", "oracle_decode_samples.json")) as f:
    GOLD = json.load(f)


def test_oracle_reproduces_the_stored_samples():
    import oracle

    pr = make_golden.golden_problem()
    out, lse = oracle.paged_decode(pr["q"], pr["k_pool"], pr["v_pool"], pr["tables"], pr["lens"],
                                   pr["scale"], num_kv_heads=pr["hkv"])
    for s, i, d, val in GOLD["out_samples"]:
        assert abs(out[s, i, d] - val) <= 1e-13
    for s, row in enumerate(GOLD["lse"]):
        for i, val in enumerate(row):
            if val is None:
                assert np.isneginf(lse[s, i])
            else:
                assert abs(lse[s, i] - val) <= 1e-12


@pytest.mark.gpu
def test_gpu_matches_the_stored_samples_without_running_the_oracle():
    import torch

    from paper_2602_00269_amd import binding

    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a visible MI355X")
    dev = torch.device("cuda:0")
    pr = make_golden.golden_problem()

    def t(a):
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(dev)

    q, kp, vp = t(pr["q"]), t(pr["k_pool"]), t(pr["v_pool"])
    s, hq, d = pr["q"].shape
    sh = binding.make_shape(s, hq, pr["hkv"], d, kp.shape[0], pr["tables"].shape[1],
                            float(pr["scale"]))
    for path in (binding.PATH_MFMA, binding.PATH_VALU):
        sh.decode_path = path
        out = torch.full((s, hq, d), float("nan"), device=dev)
        lse = torch.full((s, hq), float("nan"), device=dev)
        ws = binding.alloc_workspace(sh, dev)
        binding.paged_decode(sh, q, kp, vp, torch.from_numpy(pr["tables"]).to(dev),
                             torch.from_numpy(pr["lens"]).to(dev), out, ws, lse=lse,
                             context_lens_host=pr["lens"])
        torch.cuda.synchronize()
        o, l = out.cpu().numpy(), lse.cpu().numpy()
        for si, i, di, val in GOLD["out_samples"]:
            assert abs(o[si, i, di] - val) <= 5e-3
        for si, row in enumerate(GOLD["lse"]):
            for i, val in enumerate(row):
                if val is None:
                    assert np.isneginf(l[si, i])
                else:
                    assert abs(l[si, i] - val) <= 2e-3
