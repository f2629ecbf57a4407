"""Pins for the CPU oracle: closed forms, invariants, brute force, textbook cases.

None of these tests re-type the oracle's formulas to compare it with itself:
each expected value comes from a hand-worked example, a closed form, an
independent library routine (numpy), an invariant the method fixes, or a
pure-Python brute force on a tiny input.  CPU only.
"""
import os

import numpy as np
import pytest

from paper_2310_09259_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg1_worked_example.txt")


def _unpack_nibbles_py(packed_row):
    """Pure-Python nibble decoder used only to drive brute-force checks."""
    out = []
    for b in packed_row:
        for nib in (int(b) & 0xF, (int(b) >> 4) & 0xF):
            out.append(nib - 16 if nib >= 8 else nib)
    return out


def _read_golden():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, rhs = line.split("=", 1)
            toks = rhs.split()
            vals[key.strip()] = [int(t, 16) if t.startswith("0x") else float(t) for t in toks]
    return vals


# ---------------------------------------------------------------- fp16 decoding
def test_half_decoder_matches_numpy_on_every_bit_pattern(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    got = oracle.half_to_float(h)
    want = h.astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


# ---------------------------------------------------------------- worked example
def test_hand_worked_example_of_algorithm_1(oracle):
    g = _read_golden()
    x = np.array([g["x"]], np.float16)
    idx = np.array(g["idx"], np.int32)
    wq = np.array([g["wq_row0"], g["wq_row1"]], np.int8)
    w_scale = np.array(g["w_scale"], np.float16)
    w_out = np.array(g["w_out"], np.float16).reshape(2, 1)
    w_packed = oracle.pack(wq, 4)
    r = oracle.linear(x, idx, 4, w_packed, w_scale, w_out)
    assert r.scale.tolist() == g["scale"]
    assert r.zero.tolist() == g["zero"]
    assert r.q[0].tolist() == g["q"]
    assert oracle.pack(r.q, 4, activations=True)[0].tolist() == g["xq_bytes"]
    assert r.x_out[0].astype(np.float32).tolist() == g["x_out"]
    assert r.w_reduced.tolist() == g["w_reduced"]
    assert r.acc[0].tolist() == g["acc"]
    assert r.y[0].tolist() == g["y"]


# ---------------------------------------------------------------- evaluation order of the Quantization line
def _rn32(fr):
    """Positive exact fraction -> nearest IEEE binary32 value (normal range), ties to even, from the
    format's definition: 24 significant bits.  Returns an exact fraction."""
    import math
    from fractions import Fraction as F
    if fr == 0:
        return F(0)
    e = math.floor(math.log2(fr))
    while F(2) ** e > fr:
        e -= 1
    while F(2) ** (e + 1) <= fr:
        e += 1
    ulp = F(2) ** (e - 23)
    n = fr / ulp
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > F(1, 2) or (rem == F(1, 2) and fl % 2 == 1):
        fl += 1
    return fl * ulp


def _rne(fr):
    from fractions import Fraction as F
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    return fl + 1 if rem > F(1, 2) or (rem == F(1, 2) and fl % 2 == 1) else fl


def test_quantization_multiplies_by_a_once_per_token_reciprocal(oracle):
    """A row on which (x - zero) * (1 / scale) and (x - zero) / scale round to different codes in
    binary32 (tests/golden/reciprocal_reading_row.txt, worked by hand).  The file's numbers are first
    re-derived here in exact rational arithmetic with a rounding routine written from the IEEE
    definition; then the oracle must give the codes of the reciprocal reading."""
    from fractions import Fraction as F
    vals = {}
    with open(os.path.join(os.path.dirname(GOLDEN), "reciprocal_reading_row.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                key, rhs = line.split("=", 1)
                vals[key.strip()] = rhs.split()
    x = [F(v) for v in vals["x"]]
    q_want = [int(v) for v in vals["q"]]
    q_div = [int(v) for v in vals["q_if_divided"]]
    scale = _rn32((max(x) - min(x)) / 15)
    inv = _rn32(1 / scale)
    as_bits = lambda fr: int(np.float32(float(fr)).view(np.uint32))
    assert float(scale) == float(np.float32(float(scale)))        # exactly representable
    assert as_bits(scale) == int(vals["scale_bits"][0], 16) and as_bits(inv) == int(vals["inv_bits"][0], 16)
    assert [_rne(_rn32((v - min(x)) * inv)) - 8 for v in x] == q_want
    assert [_rne(_rn32((v - min(x)) / scale)) - 8 for v in x] == q_div
    assert q_want != q_div                                         # the row tells the two readings apart
    xh = np.array([[float(v) for v in x]], np.float16)
    q, s, z, _ = oracle.quantize(xh, np.zeros(0, np.int32), 4)
    assert int(s.view(np.uint32)[0]) == int(vals["scale_bits"][0], 16) and z[0] == float(vals["zero"][0])
    assert q[0].tolist() == q_want


# ---------------------------------------------------------------- split
def test_base_columns_brute_force(oracle):
    K = 11
    idx = np.array([7, 0, 4], np.int32)           # unsorted on purpose
    want = [k for k in range(K) if k not in (7, 0, 4)]
    assert oracle.base_columns(K, idx).tolist() == want
    assert oracle.base_columns(5, np.zeros(0, np.int32)).tolist() == [0, 1, 2, 3, 4]


def test_base_columns_rejects_bad_lists(oracle):
    with pytest.raises(ValueError):
        oracle.base_columns(8, np.array([1, 1], np.int32))
    with pytest.raises(ValueError):
        oracle.base_columns(8, np.array([8], np.int32))
    with pytest.raises(ValueError):
        oracle.base_columns(8, np.array([-1], np.int32))


def test_outlier_columns_are_bit_copies_in_index_order(oracle):
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 12)).astype(np.float16)
    x[0, 3] = np.float16(-0.0)
    idx = np.array([9, 3], np.int32)
    q, scale, zero, x_out = oracle.quantize(x, idx, 4)
    assert np.array_equal(x_out.view(np.uint16), x[:, [9, 3]].view(np.uint16))
    assert q.shape == (5, 10)


# ---------------------------------------------------------------- packing
def test_pack_known_bytes_and_round_trip(oracle):
    q = np.array([[-8, 7, -1, -1, 1, 2, 0, -8]], np.int8)
    assert oracle.pack(q, 4)[0].tolist() == [0x78, 0xFF, 0x21, 0x80]
    allbytes = np.arange(256, dtype=np.uint8).reshape(1, 256)
    unp = oracle.unpack(allbytes, 512, 4)
    assert unp.min() == -8 and unp.max() == 7
    assert unp[0].tolist() == _unpack_nibbles_py(allbytes[0])
    assert np.array_equal(oracle.pack(unp, 4), allbytes)
    # activation order: element 2p in the high nibble
    assert oracle.pack(q, 4, activations=True)[0].tolist() == [0x87, 0xFF, 0x12, 0x08]
    unp_a = oracle.unpack(allbytes, 512, 4, activations=True)
    assert unp_a[0, 0::2].tolist() == unp[0, 1::2].tolist() and unp_a[0, 1::2].tolist() == unp[0, 0::2].tolist()
    assert np.array_equal(oracle.pack(unp_a, 4, activations=True), allbytes)
    q8 = np.arange(-128, 128, dtype=np.int8).reshape(2, 128)
    assert np.array_equal(oracle.unpack(oracle.pack(q8, 8), 128, 8), q8)
    assert np.array_equal(oracle.pack(q8, 8).view(np.int8), q8)


# ---------------------------------------------------------------- findZeroScale + quantize
@pytest.mark.parametrize("bits", [4, 8])
def test_grid_rows_quantize_losslessly_with_closed_form_scale(oracle, bits):
    """Rows of the form min + j*s (s a power of two, j covering 0..L) must give
    scale == s, zero == min and q == j - halfRange exactly."""
    L = (1 << bits) - 1
    half = 1 << (bits - 1)
    rng = np.random.default_rng(1)
    T, K_b = 6, 64 if bits == 4 else 512
    s = np.array([2.0 ** e for e in (-6, -3, -1, 0, 1, 2)], np.float64)[:T]
    if bits == 8:
        s = s / 16                                   # keep min + 255*s inside fp16 exactly
    mins = np.array([-3.0, 0.0, 0.5, -8.0, 4.0, -16.0]) * s
    j = rng.integers(0, L + 1, size=(T, K_b))
    j[:, 0] = 0
    j[:, 1] = L
    xb = mins[:, None] + j * s[:, None]
    assert np.array_equal(xb.astype(np.float16).astype(np.float64), xb)   # exactly representable
    # interleave two outlier columns with huge values that must not affect the scale
    x = np.concatenate([xb[:, :10], np.full((T, 1), 6.0e4), xb[:, 10:], np.full((T, 1), -6.0e4)], 1)
    idx = np.array([10, K_b + 1], np.int32)
    q, scale, zero, x_out = oracle.quantize(x.astype(np.float16), idx, bits)
    assert np.array_equal(scale.astype(np.float64), s)
    assert np.array_equal(zero.astype(np.float64), mins)
    assert np.array_equal(q.astype(np.int64), j - half)


@pytest.mark.parametrize("bits", [4, 8])
def test_range_and_round_trip_invariants(oracle, bits):
    L = (1 << bits) - 1
    half = 1 << (bits - 1)
    shp = synth.LayerShape("t", 64, 1024, 8, 48, bits, seed=77)
    inp = synth.make_inputs(shp)
    q, scale, zero, x_out, mism = oracle.quantize(inp.x, inp.outlier_idx, bits, audit=True)
    assert q.min() == -half and q.max() == half - 1
    base = oracle.base_columns(shp.K, inp.outlier_idx)
    xb = inp.x[:, base].astype(np.float64)
    # row extremes land on the ends of the signed range
    rows = np.arange(shp.T)
    assert np.all(q[rows, xb.argmin(1)] == -half)
    assert np.all(q[rows, xb.argmax(1)] == half - 1)
    # closed form of scale/zero from the row extremes (binary32 arithmetic via numpy)
    mn32 = xb.min(1).astype(np.float32)
    mx32 = xb.max(1).astype(np.float32)
    assert np.array_equal(zero, mn32)
    assert np.array_equal(scale, (mx32 - mn32) / np.float32(L))
    # dequantization round trip error is at most scale/2 (plus binary32 slack)
    xhat = (q.astype(np.float64) + half) * scale[:, None].astype(np.float64) + zero[:, None]
    err = np.abs(xb - xhat)
    assert np.all(err <= 0.5 * scale[:, None] * (1 + 2.0 ** -10))
    # the reciprocal-multiply reading differs from exact division only at near-ties
    assert mism <= max(4, int(2e-4 * q.size))
    u = (xb - zero[:, None].astype(np.float64)) / scale[:, None].astype(np.float64)
    q_div = np.clip(np.rint(u), 0, L) - half
    diff = q_div != q
    assert int(diff.sum()) == mism
    assert np.all(np.abs(np.abs(u[diff] - np.floor(u[diff])) - 0.5) < 1e-5)


def test_outliers_do_not_influence_scale(oracle):
    shp = synth.LayerShape("t", 8, 256, 8, 16, 4, seed=5)
    a = synth.make_inputs(shp, outlier_gain=1.0)
    b = synth.make_inputs(shp, outlier_gain=1000.0)
    qa, sa, za, _ = oracle.quantize(a.x, a.outlier_idx, 4)
    qb, sb, zb, _ = oracle.quantize(b.x, b.outlier_idx, 4)
    assert np.array_equal(sa, sb) and np.array_equal(za, zb) and np.array_equal(qa, qb)


def test_constant_row_and_signed_zero(oracle):
    x = np.full((2, 16), 3.25, np.float16)
    x[1, :] = np.float16(-0.0)
    x[1, 5] = np.float16(0.0)
    q, scale, zero, _ = oracle.quantize(x, np.zeros(0, np.int32), 4)
    assert scale.tolist() == [1.0, 1.0]
    assert zero.tolist() == [3.25, 0.0] and not np.signbit(zero[1])
    assert np.all(q == -8)
    xhat = (q.astype(np.float64) + 8) * scale[:, None] + zero[:, None]
    assert np.array_equal(xhat, x.astype(np.float64))


def test_ties_round_to_even(oracle):
    # scale = 1 exactly (min 0, max 15); values j + 0.5 are exact ties
    x = np.array([[0, 15, 0.5, 1.5, 2.5, 3.5, 13.5, 14.5]], np.float16)
    q, scale, zero, _ = oracle.quantize(x, np.zeros(0, np.int32), 4)
    assert scale[0] == 1.0 and zero[0] == 0.0
    assert (q[0] + 8).tolist() == [0, 15, 0, 2, 2, 4, 14, 14]


# ---------------------------------------------------------------- integer GEMM
@pytest.mark.parametrize("bits,K_b", [(4, 6), (4, 30), (8, 7)])
def test_int_gemm_equals_pure_python_brute_force(oracle, bits, K_b):
    half = 1 << (bits - 1)
    rng = np.random.default_rng(3)
    T, N = 3, 4
    q = rng.integers(-half, half, size=(T, K_b)).astype(np.int8)
    w = rng.integers(-half, half, size=(N, K_b)).astype(np.int8)
    q[0, :] = -half
    w[0, :] = -half                      # extreme: (-h)*(-h) summed K_b times
    w[1, :] = half - 1
    acc = oracle.int_gemm(q, w, bits)
    for t in range(T):
        for n in range(N):
            s = 0
            for k in range(K_b):
                s += int(q[t, k]) * int(w[n, k])
            assert acc[t, n] == s
    assert acc[0, 0] == half * half * K_b
    assert acc[0, 1] == -half * (half - 1) * K_b


@pytest.mark.parametrize("bits", [4, 8])
def test_int_gemm_matches_numpy_int64_and_is_permutation_invariant(oracle, bits):
    half = 1 << (bits - 1)
    rng = np.random.default_rng(4)
    T, N, K_b = 17, 23, 250
    q = rng.integers(-half, half, size=(T, K_b)).astype(np.int8)
    w = rng.integers(-half, half, size=(N, K_b)).astype(np.int8)
    acc = oracle.int_gemm(q, w, bits)
    assert np.array_equal(acc.astype(np.int64), q.astype(np.int64) @ w.astype(np.int64).T)
    perm = rng.permutation(K_b)
    assert np.array_equal(oracle.int_gemm(q[:, perm], w[:, perm], bits), acc)


def test_int_gemm_refuses_depths_that_could_overflow(oracle):
    q = np.zeros((1, 1 << 17), np.int8)
    with pytest.raises(ValueError):
        oracle.int_gemm(q, q, 8)


# ---------------------------------------------------------------- wReduced
def test_weight_reduce_closed_forms(oracle):
    K_b = 40
    wq = np.ones((3, K_b), np.int8)
    wq[1] = -8
    wq[2, ::2] = -1                       # sums: 40, -320, 0
    sw = np.array([0.5, 0.0078125, 0.3], np.float16)
    got = oracle.weight_reduce(wq, sw)
    assert got.tolist() == [20.0, -2.5, 0.0]
    rng = np.random.default_rng(6)
    wq = rng.integers(-8, 8, size=(5, 33)).astype(np.int8)
    sw = rng.uniform(0.005, 0.02, 5).astype(np.float16)
    want = [np.float32(sw[n]) * np.float32(sum(int(v) for v in wq[n])) for n in range(5)]
    assert oracle.weight_reduce(wq, sw).tolist() == [float(v) for v in want]


# ---------------------------------------------------------------- whole layer
def _layer(oracle, T=24, K=320, N=40, n_out=24, bits=4, seed=9, gain=40.0):
    shp = synth.LayerShape("t", T, K, N, n_out, bits, seed=seed)
    inp = synth.make_inputs(shp, outlier_gain=gain)
    r = oracle.linear(inp.x, inp.outlier_idx, bits, inp.w_packed, inp.w_scale, inp.w_out)
    return shp, inp, r


@pytest.mark.parametrize("bits", [4, 8])
def test_layer_equals_plain_gemm_of_dequantized_operands(oracle, bits):
    """Eq. (1): the dequantization epilogue must reproduce X_hat W_hat^T exactly
    (up to rounding), X_hat = (q + halfRange) scale + zero, W_hat = wq * scaleWeight.
    The right-hand side is an ordinary float64 matmul done by numpy."""
    half = 1 << (bits - 1)
    shp, inp, r = _layer(oracle, bits=bits)
    wq = oracle.unpack(inp.w_packed, shp.K_b, bits).astype(np.float64)
    x_hat = (r.q.astype(np.float64) + half) * r.scale[:, None].astype(np.float64) + r.zero[:, None]
    w_hat = wq * inp.w_scale.astype(np.float64)[:, None]
    want = x_hat @ w_hat.T + inp.x[:, inp.outlier_idx].astype(np.float64) @ inp.w_out.astype(np.float64).T
    mag = np.abs(x_hat) @ np.abs(w_hat).T + 1.0
    assert np.all(np.abs(r.y - want) <= 2e-7 * mag)
    # and the pieces are consistent with each other
    assert np.array_equal(r.acc.astype(np.int64), r.q.astype(np.int64) @ wq.astype(np.int64).T)


def test_mixed_width_layer_equals_plain_gemm_of_dequantized_operands(oracle):
    """4-bit weights under 8-bit activations: the same Eq. (1) identity with halfRange = 128 for the
    activations and the weights unpacked as nibbles; the quantized activations and their scales
    are those of the plain 8-bit layer (they do not depend on the weights)."""
    shp = synth.LayerShape("mixed", 13, 160, 11, 16, 8, seed=23, w_bits=4)
    inp = synth.make_inputs(shp)
    assert inp.w_packed.shape == (11, 144 // 2)
    r = oracle.linear(inp.x, inp.outlier_idx, 8, inp.w_packed, inp.w_scale, inp.w_out, w_bits=4)
    wq = oracle.unpack(inp.w_packed, shp.K_b, 4).astype(np.float64)
    assert wq.min() >= -8 and wq.max() <= 7
    x_hat = (r.q.astype(np.float64) + 128) * r.scale[:, None].astype(np.float64) + r.zero[:, None]
    w_hat = wq * inp.w_scale.astype(np.float64)[:, None]
    want = x_hat @ w_hat.T + inp.x[:, inp.outlier_idx].astype(np.float64) @ inp.w_out.astype(np.float64).T
    mag = np.abs(x_hat) @ np.abs(w_hat).T + 1.0
    assert np.all(np.abs(r.y - want) <= 2e-7 * mag)
    assert np.array_equal(r.acc.astype(np.int64), r.q.astype(np.int64) @ wq.astype(np.int64).T)
    q8, s8, z8, _ = oracle.quantize(inp.x, inp.outlier_idx, 8)
    assert np.array_equal(q8, r.q) and np.array_equal(s8, r.scale) and np.array_equal(z8, r.zero)
    assert r.q.min() == -128 and r.q.max() == 127


def test_layer_is_within_the_quantization_error_bound_of_the_unquantized_layer(oracle):
    shp, inp, r = _layer(oracle)
    base = oracle.base_columns(shp.K, inp.outlier_idx)
    wq = oracle.unpack(inp.w_packed, shp.K_b, 4).astype(np.float64)
    w_hat = wq * inp.w_scale.astype(np.float64)[:, None]
    exact = inp.x[:, base].astype(np.float64) @ w_hat.T + \
        inp.x[:, inp.outlier_idx].astype(np.float64) @ inp.w_out.astype(np.float64).T
    bound = 0.5 * r.scale[:, None].astype(np.float64) * np.abs(w_hat).sum(1)[None, :]
    assert np.all(np.abs(r.y - exact) <= bound * (1 + 1e-3) + 1e-5)
    # and the bound is not vacuous: quantization error is really present
    assert np.abs(r.y - exact).max() > 1e-3


def test_zero_weights_reduce_to_the_outlier_matmul(oracle):
    shp = synth.LayerShape("t", 9, 96, 7, 16, 4, seed=11)
    inp = synth.make_inputs(shp)
    w0 = np.zeros_like(inp.w_packed)
    r = oracle.linear(inp.x, inp.outlier_idx, 4, w0, inp.w_scale, inp.w_out)
    want = inp.x[:, inp.outlier_idx].astype(np.float64) @ inp.w_out.astype(np.float64).T
    assert np.allclose(r.y, want, rtol=1e-6, atol=1e-6)
    assert not r.acc.any() and not r.w_reduced.any()


def test_no_outliers_and_integer_inputs_give_the_exact_integer_product(oracle):
    """x integer-valued in [0,15] with both ends present: zero = 0, scale = 1, so
    the layer is an exact integer matmul scaled by the weight scales."""
    rng = np.random.default_rng(12)
    T, K, N = 7, 64, 5
    xi = rng.integers(0, 16, size=(T, K))
    xi[:, 0] = 0
    xi[:, 1] = 15
    wq = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    sw = np.array([0.5, 0.25, 1.0, 2.0, 0.125], np.float16)
    r = oracle.linear(xi.astype(np.float16), np.zeros(0, np.int32), 4, oracle.pack(wq, 4), sw,
                      np.zeros((N, 0), np.float16))
    want = (xi @ wq.astype(np.int64).T) * sw.astype(np.float64)[None, :]
    assert np.array_equal(r.y.astype(np.float64), want)
    assert np.array_equal(r.q.astype(np.int64), xi - 8)


def test_bias_is_added_once(oracle):
    shp, inp, r = _layer(oracle, T=4, K=64, N=6, n_out=8)
    bias = np.arange(6, dtype=np.float16)
    rb = oracle.linear(inp.x, inp.outlier_idx, 4, inp.w_packed, inp.w_scale, inp.w_out, bias=bias)
    assert np.allclose(rb.y - r.y, bias.astype(np.float32)[None, :], atol=1e-4)


def test_tokens_are_independent(oracle):
    """Per-token quantization: a row's result does not depend on the other rows."""
    shp, inp, r = _layer(oracle, T=12)
    sel = [7, 2]
    r2 = oracle.linear(inp.x[sel], inp.outlier_idx, 4, inp.w_packed, inp.w_scale, inp.w_out)
    assert np.array_equal(r2.y, r.y[sel]) and np.array_equal(r2.q, r.q[sel])


# ---------------------------------------------------------------- input generator
def test_synthetic_inputs_have_the_stated_shapes_and_distributions():
    shp = synth.CONFIGS["tiny"]
    a = synth.make_inputs(shp)
    b = synth.make_inputs(shp)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.w_packed, b.w_packed)
    assert a.x.shape == (16, 512) and a.x.dtype == np.float16
    assert a.outlier_idx.shape == (32,) and len(set(a.outlier_idx.tolist())) == 32
    assert np.all(np.diff(a.outlier_idx) > 0)
    assert a.w_packed.shape == (512, 240) and a.w_out.shape == (512, 32)
    assert 0.005 <= a.w_scale.min() and a.w_scale.max() <= 0.02
    base = np.setdiff1d(np.arange(512), a.outlier_idx)
    assert np.abs(a.x[:, a.outlier_idx].astype(np.float32)).mean() > \
        10 * np.abs(a.x[:, base].astype(np.float32)).mean()
