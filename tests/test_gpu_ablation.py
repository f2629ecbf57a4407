"""Fusion ablation (Section 3.4, kernel versions 1-3): the unfused variants must compute the same
layer -- bit-identical packed activations / scale / zero / outlier block, output within the 5e-3
bar of the oracle."""
import numpy as np
import pytest

from paper_2310_09259_amd import synth
from tests.util import expected_xq, output_within_tolerance, upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2310_09259_amd import api as _api
    _api.load()
    return _api


SHAPES = [
    synth.CONFIGS["tiny"],
    synth.LayerShape("ragged", 150, 1024, 200, 64, 4, seed=51),
    synth.LayerShape("no_outliers", 70, 512, 136, 0, 4, seed=52),
    synth.LayerShape("w8a8", 130, 1032, 260, 64, 8, seed=53),
    synth.LayerShape("odd_pad", 33, 520, 72, 24, 4, seed=54),     # packed row 248 bytes -> padded to 256
]


@pytest.mark.parametrize("version", [1, 2, 3])
@pytest.mark.parametrize("shp", SHAPES, ids=lambda s: s.name)
def test_ablation_versions_match_oracle(api, oracle, shp, version):
    import torch
    inp = synth.make_inputs(shp)
    d = upload(inp)
    ref = oracle.linear(inp.x, inp.outlier_idx, shp.bits, inp.w_packed, inp.w_scale, inp.w_out)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, shp.bits)
    ws = torch.full((api.quik_ablation_workspace_bytes(shp.T, shp.K, shp.N, shp.n_out, shp.bits),), 0xAB,
                    dtype=torch.uint8, device="cuda")
    y, ws = api.quik_linear_ablation(version, d["x"], d["idx"], shp.bits, d["w_q"], d["w_scale"], w_red,
                                     d["w_out"], workspace=ws)
    torch.cuda.synchronize()
    xq, scale, zero, x_out = api.workspace_views(ws, shp.T, shp.K, shp.N, shp.n_out, shp.bits)
    assert np.array_equal(xq.cpu().numpy(), expected_xq(oracle, ref.q, shp.bits, xq.shape[1]))
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), ref.scale.view(np.uint32))
    assert np.array_equal(zero.cpu().numpy().view(np.uint32), ref.zero.view(np.uint32))
    if shp.n_out:
        assert np.array_equal(x_out.cpu().numpy().view(np.uint16), ref.x_out.view(np.uint16))
    ok, worst = output_within_tolerance(y.cpu().numpy(), ref.y)
    assert ok, f"version {version}: output outside 5e-3 ({worst:.2f}x)"


def test_ablation_full_size_sampled(api, oracle):
    import torch
    shp = synth.CONFIGS["llama7b_up"]
    inp = synth.make_inputs(shp)
    d = upload(inp)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    sel = np.array([0, 5, 777, 1024, 2047])
    ref = oracle.linear(inp.x[sel], inp.outlier_idx, 4, inp.w_packed, inp.w_scale, inp.w_out)
    for version in (1, 2):
        y, ws = api.quik_linear_ablation(version, d["x"], d["idx"], 4, d["w_q"], d["w_scale"], w_red,
                                         d["w_out"])
        torch.cuda.synchronize()
        xq, scale, zero, x_out = api.workspace_views(ws, shp.T, shp.K, shp.N, shp.n_out, 4)
        assert np.array_equal(xq.cpu().numpy()[sel], expected_xq(oracle, ref.q, 4, xq.shape[1]))
        ok, worst = output_within_tolerance(y.cpu().numpy()[sel], ref.y)
        assert ok, (version, worst)


def test_ablation_rejects_bad_arguments(api):
    import torch
    x = torch.zeros((4, 64), dtype=torch.float16, device="cuda")
    w = torch.zeros((8, 32), dtype=torch.uint8, device="cuda")
    sw = torch.ones(8, dtype=torch.float16, device="cuda")
    wr = torch.zeros(16, dtype=torch.float32, device="cuda")
    with pytest.raises(api.QuikError):
        api.quik_linear_ablation(4, x, None, 4, w, sw, wr, None)
    small = torch.zeros(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(api.QuikError):
        api.quik_linear_ablation(1, x, None, 4, w, sw, wr, None, workspace=small)
