"""GPU-vs-oracle parity of the FP6 (E3M2) form of the 4-bit layer, through the C ABI.

Bars as for the integer path: FP6 panels of activations and weights (the oracle's integer codes,
mapped through the format's definition and the panel layout of include/quik.h), scale, zero, outlier
block and the INT32 accumulators are bit-exact; the fp16 output is within 5e-3 of the oracle's
binary32 result."""
import numpy as np
import pytest

from paper_2310_09259_amd import synth
from tests.util import fp6_panels, output_within_tolerance, to_dev, upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2310_09259_amd import api as _api
    _api.load()
    return _api


def _sync():
    import torch
    torch.cuda.synchronize()


# T, K, n_out: every row-caching variant of the quantization kernel up to 16384 columns, ragged
# group / stage ends (K_b not a multiple of 32 or 128), no outliers, several rows per workgroup
QUANT_SHAPES = [(16, 512, 32), (37, 520, 24), (5, 1024, 64), (33, 2048, 128), (64, 4096, 256), (19, 5120, 256),
                (9, 11008, 256), (3, 16384, 128), (16, 512, 0), (7, 64, 8), (1, 8, 0), (2100, 4096, 256),
                (1500, 11008, 256), (9001, 512, 32)]


@pytest.mark.parametrize("T,K,n_out", QUANT_SHAPES)
def test_quantize_fp6_is_bit_exact(api, oracle, T, K, n_out):
    shp = synth.LayerShape("q6", T, K, 8, n_out, 4, seed=2000 + T + K + n_out)
    inp = synth.make_inputs(shp)
    idxd = to_dev(inp.outlier_idx) if n_out else None
    xq6, scale, zero, x_out = api.quik_quantize_fp6(to_dev(inp.x), idxd)
    _sync()
    q, s, z, xo = oracle.quantize(inp.x, inp.outlier_idx, 4)
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32)), "scale"
    assert np.array_equal(zero.cpu().numpy().view(np.uint32), z.view(np.uint32)), "zero"
    got, want = xq6.cpu().numpy(), fp6_panels(q)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"FP6 panels differ at {len(bad)} bytes, first {bad[:5].tolist()}")
    if n_out:
        assert np.array_equal(x_out.cpu().numpy().view(np.uint16), xo.view(np.uint16)), "x_out"


@pytest.mark.parametrize("K", [4096, 6144, 8192, 11008, 16384])
def test_quantize_fp6_many_rows_per_workgroup_repeated(api, oracle, K):
    """As the integer form's test of the same name (tests/test_gpu_parity.py)."""
    T = 1500
    shp = synth.LayerShape("q6", T, K, 8, 256, 4, seed=77 + K)
    inp = synth.make_inputs(shp)
    q, s, z, xo = oracle.quantize(inp.x, inp.outlier_idx, 4)
    want = fp6_panels(q)
    xd, idxd = to_dev(inp.x), to_dev(inp.outlier_idx)
    for rep in range(3):
        xq6, scale, zero, x_out = api.quik_quantize_fp6(xd, idxd)
        _sync()
        got = xq6.cpu().numpy()
        assert np.array_equal(got, want), f"call {rep}: {int((got != want).sum())} bytes differ"


@pytest.mark.parametrize("N,K_b", [(8, 32), (33, 480), (100, 3840), (7, 130), (64, 10752)])
def test_weight_pack_fp6_is_bit_exact(api, oracle, N, K_b):
    rng = np.random.default_rng(N + K_b)
    wq = rng.integers(-8, 8, size=(N, K_b), dtype=np.int8)
    wp = oracle.pack(wq, 4)
    ld = (wp.shape[1] + 15) // 16 * 16
    buf = np.zeros((N, ld), np.uint8)
    buf[:, :wp.shape[1]] = wp
    w6 = api.quik_weight_pack_fp6(to_dev(buf), K_b)
    _sync()
    assert np.array_equal(w6.cpu().numpy(), fp6_panels(wq))


def _linear_case(api, oracle, shp, bias=False):
    inp = synth.make_inputs(shp)
    d = upload(inp)
    b = np.random.default_rng(1).standard_normal(shp.N).astype(np.float16) if bias else None
    ref = oracle.linear(inp.x, inp.outlier_idx, 4, inp.w_packed, inp.w_scale, inp.w_out, bias=b)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    w6 = api.quik_weight_pack_fp6(d["w_q"], shp.K_b)
    y = api.quik_linear_fp6(d["x"], d["idx"], w6, d["w_scale"], w_red, d["w_out"], bias=to_dev(b) if bias else None)
    _sync()
    ok, worst = output_within_tolerance(y.cpu().numpy(), ref.y)
    assert ok, f"fp16 output outside 5e-3 (worst error / tolerance = {worst:.2f})"
    assert worst > 0
    return inp, d, ref, w_red, w6, y


LINEAR_SHAPES = [
    synth.CONFIGS["tiny"],
    synth.LayerShape("ragged", 150, 1024, 200, 64, 4, seed=31),
    synth.LayerShape("multi_tile", 260, 2048, 390, 128, 4, seed=32),
    synth.LayerShape("no_outliers", 64, 512, 256, 0, 4, seed=33),
    synth.LayerShape("n_out_24", 40, 520, 136, 24, 4, seed=34),
    synth.LayerShape("one_token", 1, 4096, 512, 256, 4, seed=35),
    # eight-wave 256 x 192 tiles (>= 128 of them), ragged T and N, K_b not a multiple of 128
    synth.LayerShape("big_tiles_ragged", 520, 512, 11000, 32, 4, seed=38),
    synth.LayerShape("big_tiles_k", 700, 1320, 5000, 40, 4, seed=51),
    # 256 x 128 tiles (the 1.5x-area tile would not save a round here), ragged T and N
    synth.LayerShape("tiles_256x128", 1030, 256, 15300, 24, 4, seed=53),
]


@pytest.mark.parametrize("shp", LINEAR_SHAPES, ids=lambda s: s.name)
def test_linear_fp6_matches_oracle(api, oracle, shp):
    _linear_case(api, oracle, shp)


def test_linear_fp6_with_bias(api, oracle):
    _linear_case(api, oracle, synth.LayerShape("bias", 70, 512, 130, 32, 4, seed=41), bias=True)


@pytest.mark.parametrize("shp", [synth.LayerShape("acc_small", 100, 1024, 160, 64, 4, seed=42),
                                 synth.LayerShape("acc_big", 530, 2048, 5000, 128, 4, seed=52)],
                         ids=lambda s: s.name)
def test_fp6_accumulators_are_the_exact_integers_and_the_output_equals_the_int8_path(api, oracle, shp):
    inp, d, ref, w_red, w6, y = _linear_case(api, oracle, shp)
    xq6, scale, zero, x_out = api.quik_quantize_fp6(d["x"], d["idx"])
    acc = api.quik_int_gemm_fp6(xq6, w6, shp.K_b)
    y2 = api.quik_gemm_dequant_fp6(xq6, scale, zero, x_out, shp.K_b, w6, d["w_scale"], w_red, d["w_out"])
    _ = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    y_int = api.quik_linear(d["x"], d["idx"], 4, d["w_q"], d["w_scale"], w_red, d["w_out"])
    _sync()
    assert np.array_equal(acc.cpu().numpy(), ref.acc)
    assert np.array_equal(y.cpu().numpy().view(np.uint16), y2.cpu().numpy().view(np.uint16))
    # same integers, same dequantization arithmetic, same order of the outlier product
    assert np.array_equal(y.cpu().numpy().view(np.uint16), y_int.cpu().numpy().view(np.uint16))


def test_fp6_worst_case_magnitudes_stay_exact(api, oracle):
    """All codes -8 against all weights -8 over K_b = 10752 columns: the largest sum the format can
    produce at that length (688128 < 2^24) must come out exactly."""
    import torch
    T, N, K_b = 64, 64, 10752
    q = np.full((T, K_b), -8, np.int8)
    q[1::2, ::3] = 7
    w = np.full((N, K_b), -8, np.int8)
    w[::3, 1::2] = 7
    acc = api.quik_int_gemm_fp6(to_dev(fp6_panels(q)), to_dev(fp6_panels(w)), K_b)
    _sync()
    want = q.astype(np.int64) @ w.astype(np.int64).T
    assert want.max() == 64 * K_b
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), want)


FULL_SIZE = ["llama7b_up", "llama7b_down", "llama13b_qkv_t128", "llama13b_qkv_t1024", "llama13b_qkv_t4096",
             "llama70b_up"]


@pytest.mark.parametrize("name", FULL_SIZE)
def test_full_size_workloads_on_sampled_tokens_fp6(api, oracle, name):
    """The 4-bit benchmark workloads at full size on the FP6 path, in the launch configuration
    bench.py times: quantization checked in full (panels, scale, zero, outlier block), the output on
    sampled token rows, and the whole output against the int8-MFMA path's (bit-identical where that
    path runs its large-tile kernel, i.e. above 32 tokens)."""
    import torch
    shp = synth.CONFIGS[name]
    inp = synth.make_inputs(shp)
    d = upload(inp)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    w6 = api.quik_weight_pack_fp6(d["w_q"], shp.K_b)
    xq6, scale, zero, x_out = api.quik_quantize_fp6(d["x"], d["idx"])
    y = api.quik_linear_fp6(d["x"], d["idx"], w6, d["w_scale"], w_red, d["w_out"])
    _sync()
    q, s, z, xo = oracle.quantize(inp.x, inp.outlier_idx, 4)
    assert np.array_equal(xq6.cpu().numpy(), fp6_panels(q))
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32))
    assert np.array_equal(zero.cpu().numpy().view(np.uint32), z.view(np.uint32))
    assert np.array_equal(x_out.cpu().numpy().view(np.uint16), xo.view(np.uint16))
    T = shp.T
    sel = np.unique(np.array([0, 1, 31, 32, 127, 128, 255, 256, T // 2 - 1, T // 2, T - 2, T - 1]) % T)
    ref = oracle.linear(inp.x[sel], inp.outlier_idx, 4, inp.w_packed, inp.w_scale, inp.w_out)
    ok, worst = output_within_tolerance(y[torch.from_numpy(sel).cuda()].cpu().numpy(), ref.y)
    assert ok, worst
    y_int = api.quik_linear(d["x"], d["idx"], 4, d["w_q"], d["w_scale"], w_red, d["w_out"])
    _sync()
    assert torch.equal(y.view(torch.int16), y_int.view(torch.int16))
    del y, y_int
    # exact accumulators of the sampled rows (their panels are built by the test-side packer)
    acc = api.quik_int_gemm_fp6(to_dev(fp6_panels(ref.q)), w6, shp.K_b)
    _sync()
    assert np.array_equal(acc.cpu().numpy(), ref.acc)
