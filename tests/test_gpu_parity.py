"""GPU-vs-oracle parity through the C ABI (run with -m gpu on an MI355X).

Bars: packed activations, scale, zero, outlier block, code sums and INT32 accumulators
are bit-exact; the fp16 output is within 5e-3 of the oracle's binary32 result
(|y - y_ref| <= 5e-3 * max(|y_ref|, 1e-3 * max|y_ref|) element by element).
"""
import numpy as np
import pytest

from paper_2310_09259_amd import synth
from tests.util import expected_xq, output_within_tolerance, to_dev, upload

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


def _quantize_case(api, oracle, x, idx, bits):
    import torch
    T, K = x.shape
    xd = to_dev(x)
    idxd = to_dev(idx) if idx.size else None
    xq, scale, zero, x_out, side = api.quik_quantize(xd, idxd, bits)
    _sync()
    q, s, z, xo = oracle.quantize(x, idx, bits)
    want = expected_xq(oracle, q, bits, xq.shape[1])
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32)), "scale"
    assert np.array_equal(zero.cpu().numpy().view(np.uint32), z.view(np.uint32)), "zero"
    got = xq.cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"xq differs at {len(bad)} bytes, first {bad[:5].tolist()}")
    if idx.size:
        assert np.array_equal(x_out.cpu().numpy().view(np.uint16), xo.view(np.uint16)), "x_out"


# T, K, n_out, bits: covers every row-caching variant of the kernel (K <= 512,
# 1024, 2048, 4096 with one wave per row; <= 8192, <= 16384 with a workgroup per
# row; the uncached form above), ragged T, n_out = 0, and a packed row length that
# is not a multiple of 16 bytes (K_b = 488 -> 244 bytes -> zero padding to 256), and
# row counts that make a workgroup loop over several rows.
QUANT_SHAPES = [
    (16, 512, 32, 4), (37, 512, 24, 4), (5, 1024, 64, 4), (33, 2048, 128, 4),
    (64, 4096, 256, 4), (19, 5120, 256, 4), (9, 11008, 256, 4), (3, 20480, 256, 4),
    (16, 512, 0, 4), (7, 64, 8, 4), (1, 8, 0, 4),
    (16, 512, 32, 8), (21, 4096, 256, 8), (6, 11008, 256, 8), (3, 20480, 128, 8), (11, 520, 24, 8),
    # more row blocks than workgroups: the software-pipelined row loop runs 2-3 times per workgroup
    (9001, 512, 32, 4), (5000, 5120, 256, 4), (2500, 8200, 64, 8), (3000, 4096, 256, 8),
]


@pytest.mark.parametrize("T,K,n_out,bits", QUANT_SHAPES)
def test_quantize_is_bit_exact(api, oracle, T, K, n_out, bits):
    shp = synth.LayerShape("q", T, K, 8, n_out, bits, seed=1000 + T + K + n_out + bits)
    inp = synth.make_inputs(shp)
    _quantize_case(api, oracle, inp.x, inp.outlier_idx, bits)


@pytest.mark.parametrize("K", [4096, 6144, 8192, 11008, 16384])
@pytest.mark.parametrize("bits", [4, 8])
def test_quantize_many_rows_per_workgroup_repeated(api, oracle, K, bits):
    """Every workgroup-per-row variant with several rows per workgroup and two or three workgroups per
    CU, three calls in a row: a misread register in the second workgroup of a CU once produced wrong
    packed bytes in some rows of some calls."""
    T = 1500
    shp = synth.LayerShape("q", T, K, 8, 256, bits, seed=77 + K)
    inp = synth.make_inputs(shp)
    q, s, z, xo = oracle.quantize(inp.x, inp.outlier_idx, bits)
    xd, idxd = to_dev(inp.x), to_dev(inp.outlier_idx)
    want = None
    for rep in range(3):
        xq, scale, zero, x_out, side = api.quik_quantize(xd, idxd, bits)
        _sync()
        if want is None:
            want = expected_xq(oracle, q, bits, xq.shape[1])
        got = xq.cpu().numpy()
        assert np.array_equal(got, want), f"call {rep}: {int((got != want).sum())} packed bytes differ"


def test_quantize_unsorted_indices_and_degenerate_rows(api, oracle):
    rng = np.random.default_rng(5)
    T, K = 12, 1024
    x = rng.standard_normal((T, K)).astype(np.float16)
    x[0, :] = np.float16(2.5)                   # constant row
    x[1, :] = np.float16(-0.0)                  # all minus zero
    x[2, :] = np.float16(0.0)
    x[2, 17] = np.float16(6.0e-8)               # smallest subnormal as the whole range
    x[3, :] = np.float16(65504.0)
    x[3, 5] = np.float16(-65504.0)              # full fp16 span
    idx = rng.permutation(K)[:40].astype(np.int32)          # unsorted
    _quantize_case(api, oracle, x, idx, 4)
    _quantize_case(api, oracle, x, idx, 8)
    # exact .5 ties: integer grid + halves, scale exactly 1
    xt = (rng.integers(0, 30, size=(4, 512)) / 2.0).astype(np.float16)
    xt[:, 0] = 0
    xt[:, 1] = 15
    xt = np.clip(xt, 0, 15)
    _quantize_case(api, oracle, xt, np.zeros(0, np.int32), 4)


# T, N, K_b, bits: several tiles in both directions with ragged edges, K tails that
# are not a multiple of the K stage, a single row/column, the deepest test K.
INT_GEMM_SHAPES = [
    (16, 512, 480, 4), (200, 300, 992, 4), (129, 257, 3840, 4), (1, 1, 32, 4), (130, 64, 96, 4),
    (16, 512, 480, 8), (150, 140, 1000, 8), (257, 129, 4864, 8),
    # enough 256 x 128 tiles to take the eight-wave configuration, ragged in T and N, K tail
    (520, 11000, 480, 4), (770, 5500, 224, 8),
    # the 1.5x-area tiles (256 x 192 for the shape above, 192 x 256 for this one): the accumulator hook
    # takes the tile choice of the fused call in every mode
    (576, 16640, 224, 4),
    # one round of 256 x 128 tiles: the 16 x 16 per-tile kernel, both widths, K tail
    (1000, 8190, 368, 4), (1000, 8190, 232, 8),
    # small-T paths: K-split kernel (T <= 32; K shorter than four stages, ragged N), 64 x 64 and
    # 128 x 64 tile configurations
    (32, 100, 160, 4), (7, 333, 2432, 4), (20, 95, 4864, 8), (50, 200, 992, 4), (64, 130, 480, 8),
    (100, 300, 480, 4), (128, 70, 1000, 8),
]


@pytest.mark.parametrize("widening", ["plain", "corrected"])
@pytest.mark.parametrize("T,N,K_b,bits", INT_GEMM_SHAPES)
def test_int32_accumulators_are_bit_exact(api, oracle, T, N, K_b, bits, widening):
    """Both operand widenings of the 4-bit K loop: the one that needs no correction, and the
    single-AND one of the fused kernel whose offset is removed with the two code-sum vectors."""
    import torch
    if widening == "corrected" and bits != 4:
        pytest.skip("the 8-bit path has one widening")
    rng = np.random.default_rng(T * 7 + N * 3 + K_b + bits)
    half = 1 << (bits - 1)
    q = rng.integers(-half, half, size=(T, K_b)).astype(np.int8)
    w = rng.integers(-half, half, size=(N, K_b)).astype(np.int8)
    q[0, :] = -half
    w[0, :] = -half                              # largest possible accumulator
    ld = api.quik_packed_row_bytes(K_b, bits)
    xq = to_dev(expected_xq(oracle, q, bits, ld))
    # weight pad bytes may hold anything: fill them with 0xFF to prove it
    wp = np.full((N, ld), 0xFF, np.uint8)
    wp[:, : K_b * bits // 8] = oracle.pack(w, bits)
    wpd = to_dev(wp)
    side = w_red = None
    if widening == "corrected":
        # side data as the library's own producers write it: quik_weight_reduce for the weights; for
        # the activations (given here as codes, not as fp16 input) the documented content of the
        # quantization workspace, one INT32 per token = sum of the codes at even k
        w_red = api.quik_weight_reduce(wpd, to_dev(np.ones(N, np.float16)), K_b, bits)
        side = to_dev(q[:, 0::2].astype(np.int32).sum(axis=1).astype(np.int32)).view(torch.uint8)
    acc = api.quik_debug_int_gemm(xq, wpd, K_b, bits, workspace=side, w_reduced=w_red)
    _sync()
    want = oracle.int_gemm(q, w, bits)
    got = acc.cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"{len(bad)} accumulators differ, first {bad[:5].tolist()}: "
                             f"{got[tuple(bad[0])]} vs {want[tuple(bad[0])]}")


@pytest.mark.parametrize("N,K_b,bits", [(37, 480, 4), (300, 3840, 4), (129, 1000, 8)])
def test_weight_reduce_is_bit_exact(api, oracle, N, K_b, bits):
    rng = np.random.default_rng(N + K_b)
    wp = rng.integers(0, 256, size=(N, K_b * bits // 8), dtype=np.uint8)
    sw = rng.uniform(0.005, 0.02, N).astype(np.float16)
    ld = api.quik_packed_row_bytes(K_b, bits)
    buf = np.full((N, ld), 0xFF, np.uint8)
    buf[:, : wp.shape[1]] = wp
    got = api.quik_weight_reduce(to_dev(buf), to_dev(sw), K_b, bits)
    _sync()
    wq = oracle.unpack(wp, K_b, bits)
    want = oracle.weight_reduce(wq, sw)
    assert got.numel() * 4 == api.quik_w_reduced_bytes(N, bits)
    assert np.array_equal(got[:N].cpu().numpy().view(np.uint32), want.view(np.uint32))
    if bits == 4:                                # side data: sum of the signed codes at odd positions
        assert np.array_equal(got[N:].cpu().numpy().view(np.int32), wq[:, 1::2].astype(np.int32).sum(axis=1))


def _linear_case(api, oracle, shp, bias=False, gain=40.0):
    inp = synth.make_inputs(shp, outlier_gain=gain)
    d = upload(inp)
    b = None
    if bias:
        b = np.random.default_rng(1).standard_normal(shp.N).astype(np.float16)
    ref = oracle.linear(inp.x, inp.outlier_idx, shp.bits, inp.w_packed, inp.w_scale, inp.w_out, bias=b)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, shp.bits)
    y = api.quik_linear(d["x"], d["idx"], shp.bits, d["w_q"], d["w_scale"], w_red, d["w_out"],
                        bias=to_dev(b) if bias else None)
    _sync()
    assert np.array_equal(w_red[: shp.N].cpu().numpy().view(np.uint32), ref.w_reduced.view(np.uint32))
    ok, worst = output_within_tolerance(y.cpu().numpy(), ref.y)
    assert ok, f"fp16 output outside 5e-3 (worst error / tolerance = {worst:.2f})"
    assert worst > 0                                   # not a trivially equal array
    return inp, d, ref, w_red


LINEAR_SHAPES = [
    synth.CONFIGS["tiny"],
    synth.LayerShape("ragged", 150, 1024, 200, 64, 4, seed=31),
    synth.LayerShape("multi_tile", 260, 2048, 390, 128, 4, seed=32),
    synth.LayerShape("no_outliers", 64, 512, 256, 0, 4, seed=33),
    synth.LayerShape("n_out_24", 40, 520, 136, 24, 4, seed=34),
    synth.LayerShape("one_token", 1, 4096, 512, 256, 4, seed=35),
    synth.LayerShape("w8a8", 130, 1024, 260, 64, 8, seed=36),
    synth.LayerShape("w8a8_tiny", 16, 512, 512, 32, 8, seed=37),
    # eight-wave 256 x 128 tile configuration (>= 256 such tiles), ragged T and N
    synth.LayerShape("big_tiles_ragged", 520, 512, 11000, 32, 4, seed=38),
    synth.LayerShape("big_tiles_w8a8", 770, 256, 5500, 24, 8, seed=39),
    # 1.5x-area tiles: 256 x 192 is picked for the two shapes above; 192 x 256 for these
    synth.LayerShape("tiles_192x256", 576, 256, 16640, 32, 4, seed=49),
    synth.LayerShape("tiles_192x256_w8a8_ragged", 570, 256, 16630, 24, 8, seed=50),
    # exactly one round of 256 x 128 tiles beats the larger tiles: the per-tile kernel on the 16 x 16 matrix
    # instructions (4-bit and 8-bit forms), ragged T, N and K
    synth.LayerShape("tiles16_256x128_ragged", 1000, 392, 8184, 24, 4, seed=55),
    synth.LayerShape("tiles16_256x128_w8a8_ragged", 1000, 280, 8184, 40, 8, seed=56),
    # small-T paths
    synth.LayerShape("t32_ragged_n", 32, 1024, 333, 64, 4, seed=40),
    synth.LayerShape("t5_w8a8", 5, 512, 200, 16, 8, seed=44),
    synth.LayerShape("t100", 100, 1024, 330, 64, 4, seed=45),
    synth.LayerShape("t60_w8a8", 60, 768, 190, 40, 8, seed=46),
]


@pytest.mark.parametrize("shp", LINEAR_SHAPES, ids=lambda s: s.name)
def test_linear_matches_oracle(api, oracle, shp):
    _linear_case(api, oracle, shp)


def test_linear_with_bias(api, oracle):
    _linear_case(api, oracle, synth.LayerShape("bias", 70, 512, 130, 32, 4, seed=41), bias=True)


def test_stages_called_separately_agree_with_the_fused_entry_point(api, oracle):
    shp = synth.LayerShape("stages", 100, 1024, 160, 64, 4, seed=42)
    inp, d, ref, w_red = _linear_case(api, oracle, shp)
    xq, scale, zero, x_out, side = api.quik_quantize(d["x"], d["idx"], 4)
    y2 = api.quik_gemm_dequant(xq, scale, zero, x_out, shp.K_b, 4, d["w_q"], d["w_scale"], w_red,
                               d["w_out"], workspace=side)
    acc = api.quik_debug_int_gemm(xq, d["w_q"], shp.K_b, 4)
    acc2 = api.quik_debug_int_gemm(xq, d["w_q"], shp.K_b, 4, workspace=side, w_reduced=w_red)
    y1 = api.quik_linear(d["x"], d["idx"], 4, d["w_q"], d["w_scale"], w_red, d["w_out"])
    _sync()
    assert np.array_equal(y1.cpu().numpy().view(np.uint16), y2.cpu().numpy().view(np.uint16))
    assert np.array_equal(acc.cpu().numpy(), ref.acc)
    assert np.array_equal(acc2.cpu().numpy(), ref.acc)


def test_strided_input_and_output(api, oracle):
    """Leading dimensions larger than the logical width (views into wider buffers)."""
    import torch
    shp = synth.LayerShape("strided", 50, 512, 72, 32, 4, seed=43)
    inp = synth.make_inputs(shp)
    d = upload(inp)
    ref = oracle.linear(inp.x, inp.outlier_idx, 4, inp.w_packed, inp.w_scale, inp.w_out)
    xbig = torch.full((shp.T, shp.K + 64), 777.0, dtype=torch.float16, device="cuda")
    xbig[:, : shp.K] = d["x"]
    ybig = torch.full((shp.T, shp.N + 24), -5.0, dtype=torch.float16, device="cuda")
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    api.quik_linear(xbig[:, : shp.K], d["idx"], 4, d["w_q"], d["w_scale"], w_red, d["w_out"],
                    out=ybig[:, : shp.N])
    _sync()
    yh = ybig.cpu().numpy()
    ok, worst = output_within_tolerance(yh[:, : shp.N], ref.y)
    assert ok, worst
    assert np.all(yh[:, shp.N:] == -5.0)               # nothing written outside the view


FULL_SIZE = ["llama7b_up", "llama7b_down", "llama7b_down_w8a8", "llama13b_qkv_t16",
             "llama13b_qkv_t128", "llama13b_qkv_t1024", "llama13b_qkv_t4096", "llama70b_up"]


def _sampled_rows(T, seed):
    """One seeded random row out of every block of 32 token rows, plus the first and the last row:
    every row block of every tile shape the library uses (32-row MFMA blocks inside 64 .. 256-row
    tiles) is compared."""
    rng = np.random.default_rng(seed)
    rows = np.arange(0, T, 32) + rng.integers(0, 32, size=(T + 31) // 32)
    return np.unique(np.concatenate([np.minimum(rows, T - 1), [0, T - 1]]))


@pytest.mark.parametrize("name", FULL_SIZE)
def test_full_size_workloads(api, oracle, name):
    """Every benchmark workload at full size, through the launches bench.py times (quik_linear on all
    T tokens; the accumulator hook on all T tokens, which picks the same kernel and tiles).
    Quantization is checked in full.  The fp16 output and the INT32 accumulators are compared with the
    oracle on the whole matrix for the headline workload (llama7b_up) and the small ones, else on one
    random row of every 32-row block (tokens are independent, so the oracle runs on those rows alone)."""
    import torch
    shp = synth.CONFIGS[name]
    bits = shp.bits
    inp = synth.make_inputs(shp)
    d = upload(inp)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, bits)
    xq, scale, zero, x_out, side = api.quik_quantize(d["x"], d["idx"], bits)
    y = api.quik_linear(d["x"], d["idx"], bits, d["w_q"], d["w_scale"], w_red, d["w_out"])
    _sync()
    q, s, z, xo = oracle.quantize(inp.x, inp.outlier_idx, bits)
    assert np.array_equal(xq.cpu().numpy(), expected_xq(oracle, q, bits, xq.shape[1]))
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32))
    assert np.array_equal(zero.cpu().numpy().view(np.uint32), z.view(np.uint32))
    assert np.array_equal(x_out.cpu().numpy().view(np.uint16), xo.view(np.uint16))
    T = shp.T
    whole = name == "llama7b_up" or T <= 128
    sel = np.arange(T) if whole else _sampled_rows(T, shp.seed)
    ref = oracle.linear(inp.x[sel], inp.outlier_idx, bits, inp.w_packed, inp.w_scale, inp.w_out)
    rows = torch.from_numpy(sel).cuda()
    ok, worst = output_within_tolerance(y[rows].cpu().numpy(), ref.y)
    assert ok, worst
    del y
    # raw accumulators: the hook runs on all T rows, the sampled ones are compared
    acc = api.quik_debug_int_gemm(xq, d["w_q"], shp.K_b, bits)
    _sync()
    got = acc[rows].cpu().numpy()
    del acc
    assert np.array_equal(got, ref.acc), f"{int((got != ref.acc).sum())} accumulators differ"
    if bits == 4:
        acc = api.quik_debug_int_gemm(xq, d["w_q"], shp.K_b, bits, workspace=side, w_reduced=w_red)
        _sync()
        got = acc[rows].cpu().numpy()
        del acc
        assert np.array_equal(got, ref.acc), f"{int((got != ref.acc).sum())} accumulators differ (side data)"


@pytest.fixture
def persistent_path(api):
    """Routes every 4-bit shape the persistent kernel can run to it (by itself the library picks it only
    where it is estimated to be faster, which leaves out the small shapes an oracle can check)."""
    api.quik_debug_set_gemm_path(1)
    yield
    api.quik_debug_set_gemm_path(0)


# Shapes the persistent 4-bit kernel can run (at least one 256-row tile per CU, K_b >= 1024): ragged in
# T and N, a packed row that is not a multiple of 16 bytes (the last 16-byte piece of a weight row ends
# in pad bytes), odd and even numbers of K stages, a last partial K stage, many narrow tiles.
STREAM_INT_SHAPES = [(1030, 9990, 1064), (2304, 5440, 2048), (600, 22016, 1320), (513, 16384, 1024)]


@pytest.mark.parametrize("widening", ["plain", "corrected"])
@pytest.mark.parametrize("T,N,K_b", STREAM_INT_SHAPES)
def test_persistent_kernel_accumulators_are_bit_exact(api, oracle, persistent_path, T, N, K_b, widening):
    """INT32 accumulators of the persistent kernel, both operand widenings, weight pad bytes 0xFF; the
    oracle runs on one random row of every 32-row block and on the first and last row."""
    import torch
    rng = np.random.default_rng(T + 3 * N + 5 * K_b)
    q = rng.integers(-8, 8, size=(T, K_b)).astype(np.int8)
    w = rng.integers(-8, 8, size=(N, K_b)).astype(np.int8)
    q[0, :] = -8
    w[0, :] = -8
    q[T - 1, :] = 7
    w[N - 1, :] = -8
    assert api.quik_debug_gemm_plan(T, N, K_b, 256) is not None
    ld = api.quik_packed_row_bytes(K_b, 4) + 16          # a stride larger than the padded row, too
    xq = to_dev(expected_xq(oracle, q, 4, ld))
    wp = np.full((N, ld), 0xFF, np.uint8)
    wp[:, : K_b // 2] = oracle.pack(w, 4)
    wpd = to_dev(wp)
    side = w_red = None
    if widening == "corrected":
        w_red = api.quik_weight_reduce(wpd, to_dev(np.ones(N, np.float16)), K_b, 4)
        side = to_dev(q[:, 0::2].astype(np.int32).sum(axis=1).astype(np.int32)).view(torch.uint8)
    acc = api.quik_debug_int_gemm(xq, wpd, K_b, 4, workspace=side, w_reduced=w_red)
    _sync()
    sel = _sampled_rows(T, N)
    got = acc[torch.from_numpy(sel).cuda()].cpu().numpy()
    want = oracle.int_gemm(q[sel], w, 4)
    assert np.array_equal(got, want), f"{int((got != want).sum())} accumulators differ"


STREAM_LINEAR_SHAPES = [
    # (shape, bias, extra columns of the output buffer's row stride)
    (synth.LayerShape("stream_ragged_partial_fp_stage", 1030, 1104, 9990, 40, 4, seed=81), False, 0),
    (synth.LayerShape("stream_no_outliers_bias", 2304, 2048, 5440, 0, 4, seed=82), True, 0),
    (synth.LayerShape("stream_scalar_stores", 600, 1448, 22016, 128, 4, seed=83), True, 3),
    (synth.LayerShape("stream_padded_rows", 520, 1288, 16390, 256, 4, seed=84), False, 10),
]


@pytest.mark.parametrize("shp,bias,ld_extra", STREAM_LINEAR_SHAPES, ids=lambda v: getattr(v, "name", str(v)))
def test_persistent_kernel_output_matches_oracle(api, oracle, persistent_path, shp, bias, ld_extra):
    """Fused output of the persistent kernel on shapes with ragged edges: with and without outlier
    columns and bias, 16-byte aligned output rows and rows that need element stores; nothing is written
    beyond column N.  Oracle on sampled rows (tokens are independent)."""
    import torch
    assert api.quik_debug_gemm_plan(shp.T, shp.N, shp.K_b, 256) is not None
    inp = synth.make_inputs(shp)
    d = upload(inp)
    b = np.random.default_rng(shp.seed).standard_normal(shp.N).astype(np.float16) if bias else None
    ybig = torch.full((shp.T, shp.N + ld_extra), -3.0, dtype=torch.float16, device="cuda")
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    api.quik_linear(d["x"], d["idx"], 4, d["w_q"], d["w_scale"], w_red, d["w_out"],
                    bias=to_dev(b) if bias else None, out=ybig[:, : shp.N])
    _sync()
    sel = _sampled_rows(shp.T, shp.seed)
    ref = oracle.linear(inp.x[sel], inp.outlier_idx, 4, inp.w_packed, inp.w_scale, inp.w_out, bias=b)
    yh = ybig[torch.from_numpy(sel).cuda()].cpu().numpy()
    ok, worst = output_within_tolerance(yh[:, : shp.N], ref.y)
    assert ok, f"fp16 output outside 5e-3 (worst error / tolerance = {worst:.2f})"
    assert worst > 0
    if ld_extra:
        assert bool((ybig[:, shp.N:] == -3.0).all())


CANARY_SHAPES = [
    synth.LayerShape("canary_small_t", 20, 1024, 200, 64, 4, seed=91),        # K-split kernel
    synth.LayerShape("canary_tiles", 300, 1096, 333, 32, 4, seed=92),         # per-tile kernel, ragged everything
    synth.LayerShape("canary_w8a8", 130, 1000, 140, 24, 8, seed=93),
    synth.LayerShape("canary_persistent", 1030, 1104, 9990, 40, 4, seed=94),  # persistent kernel
    synth.LayerShape("canary_tiles16", 1000, 392, 8190, 24, 4, seed=95),      # 16 x 16 per-tile kernel
    synth.LayerShape("canary_tiles16_w8a8", 1000, 280, 8190, 40, 8, seed=96),
]


@pytest.mark.parametrize("shp", CANARY_SHAPES, ids=lambda s: s.name)
def test_nothing_is_written_outside_the_documented_extents(api, oracle, persistent_path, shp):
    """Every output buffer sits inside a larger one filled with a canary byte: rows before the first and
    after the last, columns beyond the logical width (where the row stride is the caller's), the bytes
    behind scale / zero / the quantization workspace / the layer workspace must come back untouched.
    (Inside a row of xq the bytes up to the stride are documented to be written: zeros.)"""
    import torch
    CAN = 0xA5
    inp = synth.make_inputs(shp)
    d = upload(inp)
    T, K, N, n_out, bits = shp.T, shp.K, shp.N, shp.n_out, shp.bits
    ldq = api.quik_packed_row_bytes(shp.K_b, bits)

    def canary(nbytes):
        return torch.full((nbytes,), CAN, dtype=torch.uint8, device="cuda")

    def untouched(t):
        return bool((t == CAN).all())

    # ---- quik_quantize
    xq_buf = canary((T + 2) * (ldq + 16)).view(T + 2, ldq + 16)
    sc_buf, ze_buf = canary((T + 32) * 4), canary((T + 32) * 4)
    xo_buf = canary((T + 2) * (n_out + 8) * 2).view(torch.float16).view(T + 2, n_out + 8)
    qws = api.quik_quantize_workspace_bytes(T, bits)
    side_buf = canary(qws + 256)
    out = (xq_buf[1: T + 1], sc_buf[64: 64 + 4 * T].view(torch.float32), ze_buf[64: 64 + 4 * T].view(torch.float32),
           xo_buf[1: T + 1, :n_out], side_buf[:qws])
    xq, scale, zero, x_out, side = api.quik_quantize(d["x"], d["idx"], bits, out=out)
    _sync()
    q, s_, z_, xo = oracle.quantize(inp.x, inp.outlier_idx, bits)
    assert np.array_equal(xq[:, :ldq].cpu().numpy(), expected_xq(oracle, q, bits, ldq))
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), s_.view(np.uint32))
    assert np.array_equal(x_out.cpu().numpy().view(np.uint16), xo.view(np.uint16))
    assert untouched(xq_buf[0]) and untouched(xq_buf[T + 1]), "xq: rows outside [0, T)"
    assert untouched(sc_buf[:64]) and untouched(sc_buf[64 + 4 * T:]), "scale"
    assert untouched(ze_buf[:64]) and untouched(ze_buf[64 + 4 * T:]), "zero"
    xo_bytes = xo_buf.view(torch.uint8).view(T + 2, (n_out + 8) * 2)
    assert untouched(xo_bytes[0]) and untouched(xo_bytes[T + 1]) and untouched(xo_bytes[:, n_out * 2:]), "x_out"
    assert untouched(side_buf[qws:]), "quantization workspace"

    # ---- quik_gemm_dequant on those outputs, y inside a larger buffer
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, bits)
    y_buf = canary((T + 2) * (N + 8) * 2).view(torch.float16).view(T + 2, N + 8)
    api.quik_gemm_dequant(xq, scale, zero, x_out if n_out else None, shp.K_b, bits, d["w_q"], d["w_scale"], w_red,
                          d["w_out"], out=y_buf[1: T + 1, :N], workspace=side)
    _sync()
    ref = oracle.linear(inp.x, inp.outlier_idx, bits, inp.w_packed, inp.w_scale, inp.w_out)
    ok, worst = output_within_tolerance(y_buf[1: T + 1, :N].cpu().numpy(), ref.y)
    assert ok, worst
    y_bytes = y_buf.view(torch.uint8).view(T + 2, (N + 8) * 2)
    assert untouched(y_bytes[0]) and untouched(y_bytes[T + 1]) and untouched(y_bytes[:, N * 2:]), "y"

    # ---- quik_linear with a workspace of exactly the reported size
    need = api.quik_workspace_bytes(T, K, N, n_out, bits)
    ws_buf = canary(need + 512)
    y_buf = canary((T + 2) * (N + 8) * 2).view(torch.float16).view(T + 2, N + 8)
    api.quik_linear(d["x"], d["idx"], bits, d["w_q"], d["w_scale"], w_red, d["w_out"], out=y_buf[1: T + 1, :N],
                    workspace=ws_buf[:need])
    _sync()
    ok, worst = output_within_tolerance(y_buf[1: T + 1, :N].cpu().numpy(), ref.y)
    assert ok, worst
    y_bytes = y_buf.view(torch.uint8).view(T + 2, (N + 8) * 2)
    assert untouched(y_bytes[0]) and untouched(y_bytes[T + 1]) and untouched(y_bytes[:, N * 2:]), "y (quik_linear)"
    assert untouched(ws_buf[need:]), "layer workspace"


def test_prepared_call_matches_direct_call(api, oracle):
    """The marshal-once form of quik_linear enqueues exactly the same work."""
    shp = synth.LayerShape("prepared", 90, 1024, 200, 64, 4, seed=47)
    inp = synth.make_inputs(shp)
    d = upload(inp)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    y1 = api.quik_linear(d["x"], d["idx"], 4, d["w_q"], d["w_scale"], w_red, d["w_out"])
    call, y2 = api.prepare_linear(d["x"], d["idx"], 4, d["w_q"], d["w_scale"], w_red, d["w_out"])
    call()
    call()
    _sync()
    assert np.array_equal(y1.cpu().numpy().view(np.uint16), y2.cpu().numpy().view(np.uint16))


# ---- 4-bit weights under 8-bit activations

W4A8_INT_SHAPES = [(16, 512, 480), (200, 300, 992), (129, 257, 3840), (1, 1, 32), (40, 64, 96),
                   (520, 11000, 480), (100, 300, 1000), (300, 140, 4864)]


@pytest.mark.parametrize("T,N,K_b", W4A8_INT_SHAPES)
def test_w4a8_int32_accumulators_are_bit_exact(api, oracle, T, N, K_b):
    rng = np.random.default_rng(T * 5 + N * 3 + K_b)
    q = rng.integers(-128, 128, size=(T, K_b)).astype(np.int8)
    w = rng.integers(-8, 8, size=(N, K_b)).astype(np.int8)
    q[0, :] = -128
    w[0, :] = -8                                 # largest possible accumulator
    xq = to_dev(expected_xq(oracle, q, 8, api.quik_packed_row_bytes(K_b, 8)))
    ldw = api.quik_packed_row_bytes(K_b, 4)
    wp = np.full((N, ldw), 0xFF, np.uint8)       # weight pad bytes may hold anything
    wp[:, : K_b // 2] = oracle.pack(w, 4)
    acc = api.quik_int_gemm_w4a8(xq, to_dev(wp), K_b)
    _sync()
    want = oracle.int_gemm(q, w, 8)
    got = acc.cpu().numpy()
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"{len(bad)} accumulators differ, first {bad[:5].tolist()}: "
                             f"{got[tuple(bad[0])]} vs {want[tuple(bad[0])]}")


W4A8_LINEAR_SHAPES = [
    synth.LayerShape("w4a8_small", 16, 512, 512, 32, 8, seed=61, w_bits=4),
    synth.LayerShape("w4a8_ragged", 150, 1024, 200, 64, 8, seed=62, w_bits=4),
    synth.LayerShape("w4a8_multi_tile", 260, 2048, 390, 128, 8, seed=63, w_bits=4),
    synth.LayerShape("w4a8_no_outliers", 64, 512, 256, 0, 8, seed=64, w_bits=4),
    synth.LayerShape("w4a8_big_tiles", 520, 512, 11000, 32, 8, seed=65, w_bits=4),
    synth.LayerShape("w4a8_one_token", 1, 4096, 512, 256, 8, seed=66, w_bits=4),
]


@pytest.mark.parametrize("shp", W4A8_LINEAR_SHAPES, ids=lambda s: s.name)
def test_w4a8_linear_matches_oracle(api, oracle, shp):
    inp = synth.make_inputs(shp)
    d = upload(inp)
    ref = oracle.linear(inp.x, inp.outlier_idx, 8, inp.w_packed, inp.w_scale, inp.w_out, w_bits=4)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    y = api.quik_linear_w4a8(d["x"], d["idx"], d["w_q"], d["w_scale"], w_red, d["w_out"])
    _sync()
    assert np.array_equal(w_red[: shp.N].cpu().numpy().view(np.uint32), ref.w_reduced.view(np.uint32))
    ok, worst = output_within_tolerance(y.cpu().numpy(), ref.y)
    assert ok, f"fp16 output outside 5e-3 (worst error / tolerance = {worst:.2f})"
    assert worst > 0


def test_w4a8_full_size_on_sampled_tokens(api, oracle):
    import torch
    shp = synth.CONFIGS["llama7b_down_w4a8"]
    inp = synth.make_inputs(shp)
    d = upload(inp)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    xq, scale, zero, x_out, _ = api.quik_quantize(d["x"], d["idx"], 8)
    y = api.quik_linear_w4a8(d["x"], d["idx"], d["w_q"], d["w_scale"], w_red, d["w_out"])
    _sync()
    T = shp.T
    sel = np.unique(np.array([0, 1, 127, 128, 255, 256, T // 2, T - 2, T - 1]) % T)
    ref = oracle.linear(inp.x[sel], inp.outlier_idx, 8, inp.w_packed, inp.w_scale, inp.w_out, w_bits=4)
    rows = torch.from_numpy(sel).cuda()
    assert np.array_equal(xq[rows].cpu().numpy(), expected_xq(oracle, ref.q, 8, xq.shape[1]))
    ok, worst = output_within_tolerance(y[rows].cpu().numpy(), ref.y)
    assert ok, worst
    acc = api.quik_int_gemm_w4a8(xq[rows].contiguous(), d["w_q"], shp.K_b)
    _sync()
    assert np.array_equal(acc.cpu().numpy(), ref.acc)


def test_w8a8_with_the_papers_larger_outlier_counts(api, oracle):
    """8-bit layers keep more outlier columns in the paper (several hundred on the down-projection)."""
    for n_out, seed in ((688, 71), (896, 72)):
        shp = synth.LayerShape(f"w8a8_out{n_out}", 70, 2048, 136, n_out, 8, seed=seed)
        _linear_case(api, oracle, shp)


def test_vector_store_path_with_a_ragged_last_piece(api, oracle):
    """Output rows 16-byte aligned (ldy % 8 == 0) but N not a multiple of 8: the last 16-byte piece
    of a row is written element by element and nothing lands beyond column N."""
    import torch
    shp = synth.LayerShape("ragged_piece", 300, 512, 333, 32, 4, seed=48)
    inp = synth.make_inputs(shp)
    d = upload(inp)
    ref = oracle.linear(inp.x, inp.outlier_idx, 4, inp.w_packed, inp.w_scale, inp.w_out)
    ybig = torch.full((shp.T, 344), -7.0, dtype=torch.float16, device="cuda")
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, 4)
    api.quik_linear(d["x"], d["idx"], 4, d["w_q"], d["w_scale"], w_red, d["w_out"], out=ybig[:, : shp.N])
    _sync()
    yh = ybig.cpu().numpy()
    ok, worst = output_within_tolerance(yh[:, : shp.N], ref.y)
    assert ok, worst
    assert np.all(yh[:, shp.N:] == -7.0)


def _random_shape(seed):
    """A seeded random layer shape: ragged sizes, every tile configuration reachable."""
    rng = np.random.default_rng(9000 + seed)
    kind = seed % 4
    K = int(rng.integers(1, 160)) * 8 if kind != 3 else int(rng.integers(1, 40)) * 8
    n_out = int(rng.integers(0, max(1, min(K // 8, 40)))) * 8
    if n_out >= K:
        n_out = K - 8
    if kind == 0:      # few tokens: K-split kernel and small tiles
        T, N = int(rng.integers(1, 130)), int(rng.integers(1, 700))
    elif kind == 1:    # 128 x 128 tiles
        T, N = int(rng.integers(129, 700)), int(rng.integers(1, 900))
    elif kind == 2:    # mixed
        T, N = int(rng.integers(1, 400)), int(rng.integers(1, 2000))
    else:              # at least 256 tiles of 256 x 128: eight-wave configurations, shallow K
        T, N = int(rng.integers(513, 1100)), int(rng.integers(11000, 17000))
    mode = ("w4a4", "w8a8", "w4a8")[int(rng.integers(0, 3))]
    return T, K, N, n_out, mode


@pytest.mark.parametrize("seed", range(36))
def test_random_shapes_match_oracle(api, oracle, seed):
    T, K, N, n_out, mode = _random_shape(seed)
    bits = 4 if mode == "w4a4" else 8
    w_bits = 4 if mode != "w8a8" else 8
    shp = synth.LayerShape(f"rand{seed}", T, K, N, n_out, bits, seed=9100 + seed, w_bits=0 if w_bits == bits else w_bits)
    inp = synth.make_inputs(shp)
    d = upload(inp)
    ref = oracle.linear(inp.x, inp.outlier_idx, bits, inp.w_packed, inp.w_scale, inp.w_out,
                        w_bits=None if w_bits == bits else w_bits)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, w_bits)
    xq, scale, zero, x_out, side = api.quik_quantize(d["x"], d["idx"], bits)
    if mode == "w4a8":
        y = api.quik_linear_w4a8(d["x"], d["idx"], d["w_q"], d["w_scale"], w_red, d["w_out"])
        acc = api.quik_int_gemm_w4a8(xq, d["w_q"], shp.K_b)
    else:
        y = api.quik_linear(d["x"], d["idx"], bits, d["w_q"], d["w_scale"], w_red, d["w_out"])
        acc = api.quik_debug_int_gemm(xq, d["w_q"], shp.K_b, bits, workspace=side if bits == 4 else None,
                                      w_reduced=w_red if bits == 4 else None)
    _sync()
    what = f"T={T} K={K} N={N} n_out={n_out} {mode}"
    assert np.array_equal(xq.cpu().numpy(), expected_xq(oracle, ref.q, bits, xq.shape[1])), what
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), ref.scale.view(np.uint32)), what
    assert np.array_equal(zero.cpu().numpy().view(np.uint32), ref.zero.view(np.uint32)), what
    if n_out:
        assert np.array_equal(x_out.cpu().numpy().view(np.uint16), ref.x_out.view(np.uint16)), what
    assert np.array_equal(acc.cpu().numpy(), ref.acc), what
    ok, worst = output_within_tolerance(y.cpu().numpy(), ref.y)
    assert ok, f"{what}: output outside 5e-3 ({worst:.2f}x)"


# Kernel forms that run more than one workgroup per CU (the forms in which a register allocation that ends
# on a partial share of the SIMD's file has produced wrong bytes now and then): every one of them many times
# in a row on shapes with several workgroups per CU; the first result is checked against the oracle, every
# later one must equal it bit for bit.
REPEAT_SHAPES = [
    synth.LayerShape("rep_64x64", 60, 1024, 3000, 64, 4, seed=101),           # 64 x 64 tiles, deep ring
    synth.LayerShape("rep_128x64", 120, 1024, 3000, 64, 4, seed=102),         # 128 x 64 tiles
    synth.LayerShape("rep_128x128", 700, 1024, 2900, 64, 4, seed=103),        # 128 x 128 tiles, two per CU
    synth.LayerShape("rep_128x128_w8a8", 700, 1024, 2900, 64, 8, seed=104),
    synth.LayerShape("rep_ksplit", 24, 2048, 4000, 64, 4, seed=105),          # K-split kernel
]


@pytest.mark.parametrize("shp", REPEAT_SHAPES, ids=lambda s: s.name)
def test_repeated_calls_of_multi_workgroup_forms_are_bit_identical(api, oracle, shp):
    inp = synth.make_inputs(shp)
    d = upload(inp)
    ref = oracle.linear(inp.x, inp.outlier_idx, shp.bits, inp.w_packed, inp.w_scale, inp.w_out)
    w_red = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, shp.bits)
    first = {}
    for rep in range(8):
        got = {"layer": api.quik_linear(d["x"], d["idx"], shp.bits, d["w_q"], d["w_scale"], w_red, d["w_out"])}
        for version in (1, 2):                                     # the unfused kernels
            got[f"ablation_v{version}"], _ = api.quik_linear_ablation(version, d["x"], d["idx"], shp.bits, d["w_q"],
                                                                      d["w_scale"], w_red, d["w_out"])
        got["w_reduced"] = api.quik_weight_reduce(d["w_q"], d["w_scale"], shp.K_b, shp.bits)
        if shp.bits == 4:
            got["w6"] = api.quik_weight_pack_fp6(d["w_q"], shp.K_b)
            got["xq6"] = api.quik_quantize_fp6(d["x"], d["idx"])[0]
            got["xq24"] = api.quik_quantize_sp24(d["x"], d["idx"])[0]
        _sync()
        got = {k: v.cpu().numpy().view(np.uint8) for k, v in got.items()}
        if rep == 0:
            first = got
            for name in ("layer", "ablation_v1", "ablation_v2"):
                ok, worst = output_within_tolerance(got[name].view(np.float16), ref.y)
                assert ok, (name, worst)
        else:
            for k, v in got.items():
                assert np.array_equal(v, first[k]), f"{k}: call {rep} differs from call 0"


def test_measurement_probes_run(api):
    """The probes behind `measured_peaks` are not part of the layer, but bench.py depends on them: every
    instruction mix launches, finishes and reports its two clock counters."""
    import torch
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    src = torch.zeros(16 << 20, dtype=torch.uint8, device="cuda")
    clocks = torch.zeros(2, dtype=torch.int64, device="cuda")
    for mix in (0, 1, 7, 8, 16, 31, 33, 63, 97, 127):
        clocks.zero_()
        ops = api.quik_debug_mix_probe(mix, 64, 50, sink, src if mix & 8 else None, clocks)
        _sync()
        assert ops == 2.0 * 32 * 32 * 32 * 12 * 8 * 64 * 50
        c = clocks.cpu().numpy()
        assert c[0] > 0 and c[1] > 0, (mix, c)
    assert api.quik_debug_mfma_probe(64, 50, sink) > 0
    dst = torch.empty_like(src)
    api.quik_debug_copy_probe(src, dst)
    _sync()
    assert int(sink.item()) == 0 and bool((dst == 0).all())
