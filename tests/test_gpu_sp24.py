"""GPU-vs-oracle parity of the 2:4-sparse form of the 4-bit layer, through the C ABI.

The oracle knows nothing of sparsity: a 2:4 weight matrix is an ordinary matrix with zeros, and
Algorithm 1 on it is the reference.  Bars as for the integer path: the packed activations and weights
(the oracle's integer codes, laid out by the test-side packers written from include/quik.h), scale,
zero, outlier block and the INT32 accumulators are bit-exact; the fp16 output is within 5e-3 of the
oracle's binary32 result."""
import dataclasses

import numpy as np
import pytest

from paper_2310_09259_amd import synth
from tests.util import is_2of4, output_within_tolerance, sp24_act_panels, sp24_weight_panels, to_dev, upload

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


def _sparse(shp):
    return dataclasses.replace(shp, sparse24=True)


# T, K, n_out: every row-caching variant of the quantization kernel up to 16384 columns, ragged
# stage ends, no outliers, several rows per workgroup
QUANT_SHAPES = [(16, 512, 32), (37, 520, 24), (5, 1024, 64), (33, 2048, 128), (64, 4096, 256), (19, 5120, 256),
                (9, 11008, 256), (3, 16384, 128), (16, 512, 0), (7, 64, 8), (1, 8, 0), (2100, 4096, 256),
                (1500, 11008, 256), (9001, 512, 32)]


@pytest.mark.parametrize("T,K,n_out", QUANT_SHAPES)
def test_quantize_sp24_is_bit_exact(api, oracle, T, K, n_out):
    shp = synth.LayerShape("q24", T, K, 8, n_out, 4, seed=3000 + T + K + n_out)
    inp = synth.make_inputs(shp)
    idxd = to_dev(inp.outlier_idx) if n_out else None
    xq24, scale, zero, x_out = api.quik_quantize_sp24(to_dev(inp.x), idxd)
    _sync()
    q, s, z, xo = oracle.quantize(inp.x, inp.outlier_idx, 4)
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32)), "scale"
    assert np.array_equal(zero.cpu().numpy().view(np.uint32), z.view(np.uint32)), "zero"
    got, want = xq24.cpu().numpy(), sp24_act_panels(q)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"packed activations differ at {len(bad)} bytes, first {bad[:5].tolist()}")
    if n_out:
        assert np.array_equal(x_out.cpu().numpy().view(np.uint16), xo.view(np.uint16)), "x_out"


@pytest.mark.parametrize("K", [4096, 8192, 11008])
def test_quantize_sp24_many_rows_per_workgroup_repeated(api, oracle, K):
    """As the integer form's test of the same name (tests/test_gpu_parity.py)."""
    T = 1500
    shp = synth.LayerShape("q24", T, K, 8, 256, 4, seed=78 + K)
    inp = synth.make_inputs(shp)
    q, s, z, xo = oracle.quantize(inp.x, inp.outlier_idx, 4)
    want = sp24_act_panels(q)
    xd, idxd = to_dev(inp.x), to_dev(inp.outlier_idx)
    for rep in range(3):
        xq24, scale, zero, x_out = api.quik_quantize_sp24(xd, idxd)
        _sync()
        got = xq24.cpu().numpy()
        assert np.array_equal(got, want), f"call {rep}: {int((got != want).sum())} bytes differ"


def _random_2of4(rng, N, K_b):
    """Uniform signed nibbles with two random positions of every group of four cleared; now and then a
    third and a fourth one, so that groups with one and with no nonzero value occur."""
    w = rng.integers(-8, 8, size=(N, K_b // 4, 4), dtype=np.int8)
    order = np.argsort(rng.random((N, K_b // 4, 4)), axis=2)
    drop = 2 + (rng.random((N, K_b // 4)) < 0.2) + (rng.random((N, K_b // 4)) < 0.05)
    np.put_along_axis(w, order, np.where(np.arange(4) < drop[..., None], 0, np.take_along_axis(w, order, 2)), axis=2)
    return w.reshape(N, K_b)


def _pack_rows(oracle, wq):
    wp = oracle.pack(wq, 4)
    ld = (wp.shape[1] + 15) // 16 * 16
    buf = np.zeros((wq.shape[0], ld), np.uint8)
    buf[:, :wp.shape[1]] = wp
    return buf


@pytest.mark.parametrize("N,K_b", [(8, 32), (33, 480), (100, 3840), (7, 132), (64, 10752), (1, 4)])
def test_weight_pack_sp24_is_bit_exact(api, oracle, N, K_b):
    wq = _random_2of4(np.random.default_rng(N + K_b), N, K_b)
    assert is_2of4(wq).all()
    w24 = api.quik_weight_pack_sp24(to_dev(_pack_rows(oracle, wq)), K_b)
    _sync()
    assert np.array_equal(w24.cpu().numpy(), sp24_weight_panels(wq))


def test_weight_pack_sp24_counts_groups_that_are_not_2of4(api, oracle):
    import torch
    N, K_b = 50, 256
    wq = np.random.default_rng(5).integers(-8, 8, size=(N, K_b), dtype=np.int8)
    bad = int((~is_2of4(wq)).sum())
    assert bad > 0
    buf = to_dev(_pack_rows(oracle, wq))
    with pytest.raises(api.QuikError):
        api.quik_weight_pack_sp24(buf, K_b)
    # the raw entry point reports the count and leaves the decision to the caller
    w24 = torch.empty((K_b // 64, N, 32), dtype=torch.uint8, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    rc = api.load().quik_weight_pack_sp24(buf.data_ptr(), buf.stride(0), N, K_b, w24.data_ptr(), count.data_ptr(), None)
    _sync()
    assert rc == 0 and int(count.item()) == bad


def _linear_case(api, oracle, shp, bias=False):
    inp = synth.make_inputs(shp)
    assert is_2of4(oracle.unpack(inp.w_packed, shp.K_b, 4)).all(), "the generator's weights are not 2:4"
    d = upload(inp)
    b = np.random.default_rng(1).standard_normal(shp.N).astype(np.float16) if bias else None
    ref = oracle.linear(inp.x, inp.outlier_idx, 4, inp.w_packed, inp.w_scale, inp.w_out, bias=b)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    w24 = api.quik_weight_pack_sp24(d["w_q"], shp.K_b)
    y = api.quik_linear_sp24(d["x"], d["idx"], w24, d["w_scale"], w_red, d["w_out"], bias=to_dev(b) if bias else None)
    _sync()
    ok, worst = output_within_tolerance(y.cpu().numpy(), ref.y)
    assert ok, f"fp16 output outside 5e-3 (worst error / tolerance = {worst:.2f})"
    assert worst > 0
    return inp, d, ref, w_red, w24, y


LINEAR_SHAPES = [_sparse(s) for s in [
    synth.CONFIGS["tiny"],
    synth.LayerShape("ragged", 150, 1024, 200, 64, 4, seed=31),
    synth.LayerShape("multi_tile", 260, 2048, 390, 128, 4, seed=32),
    synth.LayerShape("no_outliers", 64, 512, 256, 0, 4, seed=33),
    synth.LayerShape("n_out_24", 40, 528, 136, 24, 4, seed=34),
    synth.LayerShape("odd_n", 70, 1024, 131, 64, 4, seed=36),
    synth.LayerShape("one_token", 1, 4096, 512, 256, 4, seed=35),
    # eight-wave 256 x 192 tiles (>= 128 of them), ragged T and N, K_b not a multiple of 64
    synth.LayerShape("big_tiles_ragged", 520, 512, 11000, 32, 4, seed=38),
    synth.LayerShape("big_tiles_k", 700, 1320, 5001, 40, 4, seed=51),
    # 256 x 128 tiles (the 1.5x-area tile would not save a round here), ragged T and N
    synth.LayerShape("tiles_256x128", 1030, 256, 15300, 24, 4, seed=53),
]]


LINEAR_SHAPES += [_sparse(s) for s in [
    # degenerate sizes: one token and one channel, two groups of four columns (K and the outlier count are
    # multiples of 8), one stage and a bit
    synth.LayerShape("one_by_one", 1, 16, 1, 8, 4, seed=61),
    synth.LayerShape("two_groups", 3, 24, 5, 16, 4, seed=62),
    synth.LayerShape("stage_plus_two_groups", 33, 80, 65, 8, 4, seed=63),
    # ring shorter than / equal to / one longer than the number of stages (eight buffers)
    synth.LayerShape("seven_stages", 130, 448 + 16, 200, 16, 4, seed=64),
    synth.LayerShape("eight_stages", 130, 512 + 16, 200, 16, 4, seed=65),
    synth.LayerShape("nine_stages", 300, 576 + 16, 400, 16, 4, seed=66),
    # 65 .. 128 tokens: 128 x 64 tiles (two matrix instructions per wave and stage), ragged T and N
    synth.LayerShape("tiles_128x64", 97, 1096, 150, 72, 4, seed=68),
    synth.LayerShape("tiles_128x64_full", 128, 2048 + 128, 192, 128, 4, seed=69),
    # odd number of integer stages followed by an odd number of outlier stages
    synth.LayerShape("odd_odd", 280, 64 * 21 + 48, 392, 48, 4, seed=67),
]]


@pytest.mark.parametrize("shp", LINEAR_SHAPES, ids=lambda s: s.name)
def test_linear_sp24_matches_oracle(api, oracle, shp):
    _linear_case(api, oracle, shp)


def test_linear_sp24_with_bias(api, oracle):
    _linear_case(api, oracle, _sparse(synth.LayerShape("bias", 70, 512, 130, 32, 4, seed=41)), bias=True)


@pytest.mark.parametrize("shp", [_sparse(synth.LayerShape("acc_small", 100, 1024, 160, 64, 4, seed=42)),
                                 # the K-split kernel for up to 32 tokens: ragged T and N, stage counts that do not
                                 # divide by four, fewer stages than waves, more than 256 outlier columns
                                 _sparse(synth.LayerShape("acc_skinny", 19, 1160, 75, 72, 4, seed=55)),
                                 _sparse(synth.LayerShape("acc_skinny_32", 32, 4096 + 320, 200, 320, 4, seed=56)),
                                 _sparse(synth.LayerShape("acc_skinny_short", 5, 136, 40, 8, 4, seed=57)),
                                 # its 64-token form: ragged second token fragment, N not a multiple of 32
                                 _sparse(synth.LayerShape("acc_skinny_64", 57, 2304 + 64, 101, 64, 4, seed=58)),
                                 _sparse(synth.LayerShape("acc_skinny_64_full", 64, 640 + 8, 64, 8, 4, seed=59)),
                                 _sparse(synth.LayerShape("acc_skinny_64_outliers", 40, 1024 + 264, 70, 264, 4, seed=60)),
                                 _sparse(synth.LayerShape("acc_big", 530, 2048, 5000, 128, 4, seed=52)),
                                 _sparse(synth.LayerShape("acc_odd_n", 300, 1088, 777, 64, 4, seed=54)),
                                 _sparse(synth.LayerShape("acc_128x64", 120, 1344 + 24, 333, 24, 4, seed=70))],
                         ids=lambda s: s.name)
def test_sp24_accumulators_are_the_exact_integers(api, oracle, shp):
    inp, d, ref, w_red, w24, y = _linear_case(api, oracle, shp)
    xq24, scale, zero, x_out = api.quik_quantize_sp24(d["x"], d["idx"])
    acc = api.quik_int_gemm_sp24(xq24, w24, shp.N, shp.K_b)
    y2 = api.quik_gemm_dequant_sp24(xq24, scale, zero, x_out, shp.K_b, w24, d["w_scale"], w_red, d["w_out"])
    _sync()
    assert np.array_equal(acc.cpu().numpy(), ref.acc)
    assert np.array_equal(y.cpu().numpy().view(np.uint16), y2.cpu().numpy().view(np.uint16))


def test_sp24_worst_case_magnitudes_stay_exact(api, oracle):
    """All codes -8 against weights -8 in two of every four columns over K_b = 10752 columns: the largest
    accumulator the format can produce at that length (256 * 64 * K_b / 2 < 2^31 before the scaling is
    removed) must come out exactly."""
    T, N, K_b = 64, 64, 10752
    q = np.full((T, K_b), -8, np.int8)
    q[1::2, ::3] = 7
    w = np.zeros((N, K_b), np.int8)
    w[:, 0::4] = -8
    w[:, 3::4] = -8
    w[::3, 3::4] = 7
    acc = api.quik_int_gemm_sp24(to_dev(sp24_act_panels(q)), to_dev(sp24_weight_panels(w)), N, K_b)
    _sync()
    want = q.astype(np.int64) @ w.astype(np.int64).T
    assert want.max() == 64 * K_b // 2
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), want)


FULL_SIZE = ["llama7b_up", "llama7b_down", "llama13b_qkv_t16", "llama13b_qkv_t128", "llama13b_qkv_t1024", "llama70b_up"]


@pytest.mark.parametrize("name", FULL_SIZE)
def test_full_size_workloads_on_sampled_tokens_sp24(api, oracle, name):
    """The 4-bit benchmark workloads at full size with 2:4-sparse weights, in the launch configuration
    bench.py times: quantization checked in full, the output on sampled token rows, the whole output
    against the dense int8-MFMA path's on the same matrices (within the output bar of each other's
    rounding: both are within 5e-3 of the oracle), and exact accumulators for the sampled rows."""
    import torch
    shp = _sparse(synth.CONFIGS[name])
    inp = synth.make_inputs(shp)
    d = upload(inp)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    w24 = api.quik_weight_pack_sp24(d["w_q"], shp.K_b)
    xq24, scale, zero, x_out = api.quik_quantize_sp24(d["x"], d["idx"])
    y = api.quik_linear_sp24(d["x"], d["idx"], w24, d["w_scale"], w_red, d["w_out"])
    _sync()
    q, s, z, xo = oracle.quantize(inp.x, inp.outlier_idx, 4)
    assert np.array_equal(xq24.cpu().numpy(), sp24_act_panels(q))
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
    diff = (y.float() - y_int.float()).abs()
    floor = 1e-3 * float(y_int.float().abs().max())
    assert bool((diff <= 1e-2 * torch.clamp(y_int.float().abs(), min=floor)).all())
    del y, y_int, diff
    acc = api.quik_int_gemm_sp24(to_dev(sp24_act_panels(ref.q)), w24, shp.N, shp.K_b)
    _sync()
    assert np.array_equal(acc.cpu().numpy(), ref.acc)
