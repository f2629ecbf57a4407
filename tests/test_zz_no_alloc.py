"""quik_linear_noalloc (the entry point for callers that cannot allocate: its workspace is a static
device array) against quik_linear, through the C ABI: bit-identical output on two calls in a row,
the second on a smaller input, and the size limit turns into an error code."""
import numpy as np
import pytest

from paper_2310_09259_amd import synth
from tests.util import output_within_tolerance, upload

pytestmark = pytest.mark.gpu


def test_noalloc_entry_point_matches_quik_linear(oracle):
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    from paper_2310_09259_amd import api
    api.load()
    # the larger call first (7B up-projection width at 600 tokens: several tiles, ragged), then a
    # smaller one with other sizes everywhere: the array keeps the first call's contents
    shapes = [synth.LayerShape("noalloc_a", 600, 4096, 1000, 256, 4, seed=81),
              synth.LayerShape("noalloc_b", 70, 1024, 333, 64, 4, seed=82),
              synth.LayerShape("noalloc_c_w8a8", 33, 520, 130, 24, 8, seed=83)]
    for shp in shapes:
        inp = synth.make_inputs(shp)
        d = upload(inp)
        w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, shp.bits)
        y_ref = api.quik_linear(d["x"], d["idx"], shp.bits, d["w_q"], d["w_scale"], w_red, d["w_out"])
        y = torch.full((shp.T, shp.N), 7.0, dtype=torch.float16, device="cuda")
        api.quik_linear_noalloc(d["x"], d["idx"], shp.bits, d["w_q"], d["w_scale"], w_red, d["w_out"], out=y)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy().view(np.uint16), y_ref.cpu().numpy().view(np.uint16)), shp.name
        ref = oracle.linear(inp.x, inp.outlier_idx, shp.bits, inp.w_packed, inp.w_scale, inp.w_out)
        ok, worst = output_within_tolerance(y.cpu().numpy(), ref.y)
        assert ok, (shp.name, worst)
    # beyond the array's size: an error code, nothing enqueued
    big = synth.LayerShape("noalloc_big", 4096, 8192, 64, 256, 4, seed=84)
    assert api.quik_workspace_bytes(big.T, big.K, big.N, big.n_out, 4) > (8 << 20)
    x = torch.zeros((big.T, big.K), dtype=torch.float16, device="cuda")
    idx = torch.arange(0, 256, dtype=torch.int32, device="cuda")
    w_q = torch.zeros((big.N, big.K_b // 2), dtype=torch.uint8, device="cuda")
    w_scale = torch.ones(big.N, dtype=torch.float16, device="cuda")
    w_out = torch.zeros((big.N, 256), dtype=torch.float16, device="cuda")
    w_red = api.quik_weight_reduce(w_q, w_scale, big.K_b, 4)
    y = torch.zeros((big.T, big.N), dtype=torch.float16, device="cuda")
    with pytest.raises(api.QuikError) as e:
        api.quik_linear_noalloc(x, idx, 4, w_q, w_scale, w_red, w_out, out=y)
    assert e.value.status == -5
