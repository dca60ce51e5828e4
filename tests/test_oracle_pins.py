"""Pins for the CPU oracle: it is checked against what the paper and the
mathematics fix, never against itself or the GPU path."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle


def _read_table(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line.split())
    return rows


# --------------------------------------------------------------------------
# quantizer
# --------------------------------------------------------------------------

def test_tie_break_grid_from_paper_rules(golden_dir):
    """sgn(0)=+1 at x=m_i means half-way values go up (Sec. 3.1/3.2, Alg. 1)."""
    rows = _read_table(golden_dir + "/tie_break_grid.txt")
    assert len(rows) > 25
    for b, l, u, x, want in rows:
        got = oracle.quantize(np.array([float(x)], np.float32), float(l), float(u), int(b))
        assert int(got[0]) == int(want), (b, l, u, x, want, got)


@pytest.mark.parametrize("bits,l,u", [(2, 0.0, 2.5), (3, -0.7, 1.9), (4, 0.0, 3.0), (4, -0.0719, 0.0719)])
def test_level_set_and_half_interval_error(bits, l, u):
    """Dequantized values take exactly 2^b distinct values l + c*Delta; inside
    [l,u] the error is at most Delta/2; outside, the value is the bound."""
    l, u = float(np.float32(l)), float(np.float32(u))
    x = np.linspace(l - 1.0, u + 1.0, 200001).astype(np.float32)
    code = oracle.quantize(x, l, u, bits)
    assert code.min() == 0 and code.max() == 2 ** bits - 1
    assert len(np.unique(code)) == 2 ** bits
    val = oracle.dequantize(code, l, u, bits)
    d = (Fraction(u) - Fraction(l)) / (2 ** bits - 1)
    d32 = oracle.delta(l, u, bits)
    assert abs(Fraction(d32) - d) <= abs(d) * Fraction(1, 2 ** 23)
    levels = np.array([l + d32 * c for c in range(2 ** bits)])
    assert np.all(np.abs(val - levels[code]) == 0.0)
    inside = (x >= l) & (x <= u)
    err = np.abs(val[inside] - x[inside].astype(np.float64))
    assert err.max() <= 0.5 * float(d) * (1 + 1e-5)
    assert np.all(code[x <= l] == 0)
    assert np.all(code[x >= u] == 2 ** bits - 1)
    # monotone non-decreasing on a sorted sweep
    assert np.all(np.diff(code.astype(np.int32)) >= 0)


@pytest.mark.parametrize("bits,l,u", [(2, 0.0, 2.5), (3, -1.0, 2.0), (4, -0.3, 0.45)])
def test_codes_equal_exact_rational_nearest_level(bits, l, u):
    """Away from fp32-rounding distance of a midpoint, the code is the index of
    the nearest level computed in exact rational arithmetic."""
    rng = np.random.default_rng(7)
    l, u = float(np.float32(l)), float(np.float32(u))
    x = rng.uniform(l - 0.2, u + 0.2, 4000).astype(np.float32)
    code = oracle.quantize(x, l, u, bits)
    L = 2 ** bits - 1
    d = (Fraction(u) - Fraction(l)) / L
    checked = 0
    for xi, ci in zip(x, code):
        v = min(max(Fraction(float(xi)), Fraction(l)), Fraction(u))
        t = (v - Fraction(l)) / d
        if abs((t - math.floor(t)) - Fraction(1, 2)) < Fraction(1, 10 ** 5):
            continue
        want = min(max(math.floor(t + Fraction(1, 2)), 0), L)
        assert want == int(ci)
        checked += 1
    assert checked > 3900


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_soft_quantizer_route_gives_same_codes(bits):
    """Algorithm 1 steps 2-4 done literally in float64: find the interval i,
    evaluate phi = s*tanh(k(x-m_i)) with k from alpha (Sec. 3.3, alpha=0.2 as
    in Sec. 4.1), take sgn, code = i + (sgn+1)/2."""
    rng = np.random.default_rng(11)
    l, u = -0.8, 2.3
    l, u = float(np.float32(l)), float(np.float32(u))
    L = 2 ** bits - 1
    d = (u - l) / L
    alpha = 0.2
    k = math.log(2.0 / alpha - 1.0) / d
    s = 1.0 / (1.0 - alpha)
    # closed form of Sec. 3.3: tanh(0.5*k*Delta) = 1 - alpha
    assert abs(math.tanh(0.5 * k * d) - (1 - alpha)) < 1e-12
    x = rng.uniform(l, u, 5000).astype(np.float32)
    code = oracle.quantize(x, l, u, bits)
    n = 0
    for xi, ci in zip(x.astype(np.float64), code):
        i = min(int(math.floor((xi - l) / d)), L - 1)      # interval P_i, last one closed
        m = l + (i + 0.5) * d
        if abs(xi - m) < 1e-5 * d:
            continue
        phi = s * math.tanh(k * (xi - m))
        sgn = 1 if phi >= 0 else -1
        assert i + (sgn + 1) // 2 == int(ci)
        n += 1
    assert n > 4900


def test_numpy_affine_quantizer_special_case():
    """The recipe reduces to the textbook affine quantizer in float32."""
    rng = np.random.default_rng(3)
    for bits, l, u in [(2, 0.0, 2.5), (3, -0.11, 0.13), (4, 0.0, 3.0)]:
        l32, u32 = np.float32(l), np.float32(u)
        x = rng.normal(0.3, 1.5, 50000).astype(np.float32)
        d = (u32 - l32) / np.float32(2 ** bits - 1)
        want = np.floor((np.clip(x, l32, u32) - l32) / d + np.float32(0.5)).astype(np.int64)
        want = np.clip(want, 0, 2 ** bits - 1)
        got = oracle.quantize(x, float(l32), float(u32), bits)
        assert np.array_equal(got.astype(np.int64), want)


def test_special_values_and_bad_bounds():
    x = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0], np.float32)
    code = oracle.quantize(x, -1.0, 1.0, 4)
    assert code.tolist()[:3] == [0, 15, 0]
    assert code[3] == code[4]             # -0.0 and +0.0 are the same number
    # every NaN, quiet or signalling, of either sign, clips to l (code 0) whatever the range
    nans = np.array([0x7F800001, 0x7FBFFFFF, 0x7FC00000, 0x7FFFFFFF, 0xFF800001, 0xFFC00000, 0xFFFFFFFF],
                    np.uint32).view(np.float32)
    for bits in (1, 2, 3, 4):
        assert not oracle.quantize(nans, -1.0, 1.0, bits).any()
        assert not oracle.quantize(nans, 0.25, 2.0, bits).any()
    w = np.tile(nans, 2).reshape(2, 7, 1, 1)
    assert not oracle.quantize_weights(w, np.array([-1.0, 0.5], np.float32), np.array([1.0, 0.75], np.float32), 3).any()
    z = oracle.quantize(np.array([0.0, -0.0], np.float32), -1.5, 1.5, 2)
    assert z.tolist() == [2, 2]           # Delta = 1 exactly: t = 1.5 -> tie -> up
    for l, u in [(1.0, 1.0), (2.0, 1.0), (float("nan"), 1.0), (0.0, float("inf"))]:
        with pytest.raises(ValueError):
            oracle.quantize(x, l, u, 4)


def test_per_channel_weight_bounds():
    rng = np.random.default_rng(5)
    w = rng.normal(0, 0.1, (5, 3, 3, 3)).astype(np.float32)
    lw = np.array([-0.3, -0.2, -0.1, -0.25, -0.05], np.float32)
    uw = np.array([0.3, 0.1, 0.2, 0.25, 0.3], np.float32)
    code = oracle.quantize_weights(w, lw, uw, 3)
    for o in range(5):
        assert np.array_equal(code[o], oracle.quantize(w[o], float(lw[o]), float(uw[o]), 3))


# --------------------------------------------------------------------------
# convolution
# --------------------------------------------------------------------------

def _brute_conv(a, w, stride, pad):
    """Seven nested loops over python ints / Fractions."""
    N, C, H, W = a.shape
    O, _, R, S = w.shape
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
    out = np.empty((N, O, Ho, Wo), dtype=object)
    for n, o, y, x in itertools.product(range(N), range(O), range(Ho), range(Wo)):
        acc = 0
        for c, r, s in itertools.product(range(C), range(R), range(S)):
            iy, ix = y * stride - pad + r, x * stride - pad + s
            if 0 <= iy < H and 0 <= ix < W:
                acc += a[n, c, iy, ix] * w[o, c, r, s]
        out[n, o, y, x] = acc
    return out


GEOMS = [  # N, C_in, H, W, C_out, R, S, stride, pad  -- all asymmetric on purpose
    (2, 3, 5, 4, 4, 3, 3, 1, 1),
    (1, 2, 6, 7, 3, 3, 3, 2, 1),
    (1, 5, 4, 3, 2, 1, 1, 1, 0),
    (2, 2, 5, 6, 3, 1, 1, 2, 0),
    (1, 2, 5, 5, 3, 3, 3, 1, 0),
    (1, 3, 4, 6, 2, 3, 1, 1, 1),
]


@pytest.mark.parametrize("geom", GEOMS)
def test_conv_codes_vs_brute_force_and_torch(geom):
    N, C, H, W, O, R, S, stride, pad = geom
    rng = np.random.default_rng(sum(geom))
    a = rng.integers(0, 16, (N, C, H, W)).astype(np.uint8)
    w = rng.integers(0, 16, (O, C, R, S)).astype(np.uint8)
    got = oracle.conv_codes(a, w, stride, pad)
    want = _brute_conv(a.astype(object), w.astype(object), stride, pad)
    assert np.array_equal(got.astype(object), want)
    ref = F.conv2d(torch.from_numpy(a.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                   stride=stride, padding=pad).numpy()
    assert np.array_equal(got.astype(np.float64), ref)
    # cross-correlation, not flipped-kernel convolution: the flipped one must differ
    if R * S > 1:
        flipped = F.conv2d(torch.from_numpy(a.astype(np.float64)),
                           torch.from_numpy(w[:, :, ::-1, ::-1].astype(np.float64).copy()),
                           stride=stride, padding=pad).numpy()
        assert not np.array_equal(got.astype(np.float64), flipped)


def test_one_hot_places_the_tap_where_cross_correlation_says():
    a = np.zeros((1, 2, 5, 5), np.uint8)
    w = np.zeros((3, 2, 3, 3), np.uint8)
    a[0, 1, 2, 3] = 7
    w[2, 1, 0, 2] = 5          # tap r=0, s=2 of output channel 2
    acc = oracle.conv_codes(a, w, 1, 1)
    # out[y,x] reads in[y-1+r, x-1+s] -> y = 2+1-0 = 3, x = 3+1-2 = 2
    want = np.zeros((1, 3, 5, 5), np.int32)
    want[0, 2, 3, 2] = 35
    assert np.array_equal(acc, want)


@pytest.mark.parametrize("geom", GEOMS)
@pytest.mark.parametrize("bits", [2, 4])
def test_conv_real_vs_fractions_and_torch(geom, bits):
    """Step 5 on the dequantized tensors: exact rational brute force (rounded
    once) and torch's float64 conv2d."""
    N, C, H, W, O, R, S, stride, pad = geom
    rng = np.random.default_rng(100 + sum(geom) + bits)
    top = 2 ** bits - 1
    a = rng.integers(0, top + 1, (N, C, H, W)).astype(np.uint8)
    w = rng.integers(0, top + 1, (O, C, R, S)).astype(np.uint8)
    la, ua = float(np.float32(-0.37)), float(np.float32(2.11))
    lw = rng.uniform(-0.3, -0.1, O).astype(np.float32)
    uw = rng.uniform(0.1, 0.4, O).astype(np.float32)
    got = oracle.conv_real(a, la, ua, w, lw, uw, bits, stride, pad)

    da = Fraction(oracle.delta(la, ua, bits))
    ahat = np.vectorize(lambda c: Fraction(la) + da * int(c), otypes=[object])(a)
    what = np.empty(w.shape, dtype=object)
    for o in range(O):
        dw = Fraction(oracle.delta(float(lw[o]), float(uw[o]), bits))
        what[o] = np.vectorize(lambda c: Fraction(float(lw[o])) + dw * int(c), otypes=[object])(w[o])
    exact = _brute_conv(ahat, what, stride, pad)
    exact32 = np.vectorize(lambda q: np.float32(float(q)), otypes=[np.float32])(exact)
    # double accumulation then one rounding: within 1 ulp of the exactly rounded value
    assert np.all(np.abs(got.astype(np.float64) - exact32.astype(np.float64))
                  <= np.spacing(np.abs(exact32)).astype(np.float64))

    ah = oracle.dequantize(a, la, ua, bits)
    wh = np.stack([oracle.dequantize(w[o], float(lw[o]), float(uw[o]), bits) for o in range(O)])
    ref = F.conv2d(torch.from_numpy(ah), torch.from_numpy(wh), stride=stride, padding=pad).numpy()
    scale = np.abs(ref).max() + 1e-30
    assert np.abs(got.astype(np.float64) - ref).max() <= scale * 1e-7  # fp32 rounding of got
    assert np.abs(oracle.conv_dequantized(ah, wh, stride, pad).astype(np.float64) - ref).max() <= scale * 1e-7


@pytest.mark.parametrize("stride,pad,R", [(1, 1, 3), (2, 1, 3), (1, 0, 3), (1, 0, 1), (2, 0, 1)])
@pytest.mark.parametrize("la_int", [0, -2])
def test_integer_gemm_plus_corrections_is_the_float_conv(stride, pad, R, la_int):
    """With integer-valued levels (Delta = 1) the float convolution of the
    dequantized tensors is an integer and must equal, exactly,
        Da*Dw*ACC + la*Dw*SW + lw*Da*SA + KV*la*lw
    where SA / SW / KV only count taps that are not in the padding."""
    bits = 4
    rng = np.random.default_rng(17 + stride + 10 * pad + R)
    N, C, H, W, O = 2, 5, 6, 7, 4
    la, ua = float(la_int), float(la_int + 15)            # Delta_a = 1
    lw = np.array([-8, -7, 0, -15], np.float32)
    uw = lw + 15                                          # Delta_w = 1
    a = rng.integers(0, 16, (N, C, H, W)).astype(np.uint8)
    w = rng.integers(0, 16, (O, C, R, R)).astype(np.uint8)
    out = oracle.conv_real(a, la, ua, w, lw, uw, bits, stride, pad)
    acc = oracle.conv_codes(a, w, stride, pad).astype(np.int64)

    ones_a = np.ones_like(a)
    ones_w = np.ones_like(w)
    SA = oracle.conv_codes(a, ones_w, stride, pad).astype(np.int64)       # sum of act codes over valid taps
    SW = oracle.conv_codes(ones_a, w, stride, pad).astype(np.int64)       # sum of weight codes over valid taps
    KV = oracle.conv_codes(ones_a, ones_w, stride, pad).astype(np.int64)  # number of valid (tap, channel) pairs
    lw64 = lw.astype(np.int64).reshape(1, O, 1, 1)
    want = acc + la_int * SW + lw64 * SA + KV * la_int * lw64
    assert np.array_equal(out.astype(np.int64), want)
    assert np.all(out == np.round(out))


def test_conv_at_matches_full_tensors():
    rng = np.random.default_rng(23)
    a = rng.integers(0, 4, (2, 6, 7, 5)).astype(np.uint8)
    w = rng.integers(0, 4, (5, 6, 3, 3)).astype(np.uint8)
    lw = rng.uniform(-0.3, -0.1, 5).astype(np.float32)
    uw = rng.uniform(0.1, 0.4, 5).astype(np.float32)
    full = oracle.conv_real(a, 0.0, 2.5, w, lw, uw, 2, 2, 1)
    acc = oracle.conv_codes(a, w, 2, 1)
    idx = rng.permutation(full.size)[:50]
    v, c = oracle.conv_at(a, 0.0, 2.5, w, lw, uw, 2, 2, 1, idx)
    assert np.array_equal(v, full.reshape(-1)[idx])
    assert np.array_equal(c, acc.reshape(-1)[idx])


# --------------------------------------------------------------------------
# numbers the paper prints
# --------------------------------------------------------------------------

def test_accumulator_budget_matches_table1(golden_dir):
    """Sec. 3.5: b-bit signed codes allow floor((2^7-1)/(2^(b-1))^2) MLAs per
    SADDW.  The same argument with unsigned codes and 32-bit accumulators:
    (2^b-1)^2 * K stays far below 2^24 for the largest K used (3*3*512), so an
    int32 accumulator is exact and converts to binary32/64 without rounding."""
    for b, ratio in _read_table(golden_dir + "/table1_mla_per_saddw.txt"):
        b = int(b)
        assert (2 ** 7 - 1) // ((-2 ** (b - 1)) ** 2) == int(ratio)
    assert 15 * 15 * 3 * 3 * 512 == 1036800 < 2 ** 24


def test_table9_ratio_is_the_claimed_speedup(golden_dir):
    t = dict((k, float(v)) for k, v in _read_table(golden_dir + "/table9_resnet18_ms.txt"))
    assert round(t["ncnn_8bit_ms"] / t["dsq_2bit_ms"], 1) == t["claimed_speedup_upto"]


# ---------------------------------------------------------------------------
# layer-to-layer map (affine + ReLU + next layer's quantizer)
# ---------------------------------------------------------------------------

def test_affine_relu_hand_derived_roundings(golden_dir):
    for line in open(os.path.join(golden_dir, "affine_two_roundings.txt")):
        if line.startswith("#") or not line.strip():
            continue
        y, s, b, relu, want = line.split()
        got = oracle.affine_relu(np.full((1, 1, 1, 1), float.fromhex(y), np.float32),
                                 [float.fromhex(s)], [float.fromhex(b)], int(relu))
        assert got.reshape(()).item() == float.fromhex(want), line


def test_affine_relu_is_numpy_float32_arithmetic_per_channel():
    rng = np.random.default_rng(11)
    y = rng.standard_normal((3, 5, 4, 7)).astype(np.float32)     # H != W, N > 1
    s = rng.standard_normal(5).astype(np.float32)
    b = rng.standard_normal(5).astype(np.float32)
    want = y * s[None, :, None, None]          # numpy rounds each float32 operation
    want = want + b[None, :, None, None]
    assert np.array_equal(oracle.affine_relu(y, s, b, False), want)
    assert np.array_equal(oracle.affine_relu(y, s, b, True), np.maximum(want, np.float32(0)))
    # the channel index is axis 1: a one-hot scale leaves exactly that channel
    for c in range(5):
        e = np.zeros(5, np.float32)
        e[c] = 1
        z = oracle.affine_relu(y, e, np.zeros(5, np.float32), False)
        assert np.array_equal(z[:, c], y[:, c]) and not z[:, np.arange(5) != c].any()


def test_requantize_is_nearest_level_of_the_mapped_value():
    rng = np.random.default_rng(12)
    y = (rng.standard_normal((2, 3, 3, 4)) * 2).astype(np.float32)
    s = np.array([0.5, 1.25, 2.0], np.float32)
    b = np.array([0.1, -0.2, 0.3], np.float32)
    l, u, bits = 0.0, 3.0, 3
    got = oracle.requantize(y, s, b, True, l, u, bits)
    top = (1 << bits) - 1
    d = Fraction(float(np.float32(u) - np.float32(l))) / top
    for idx in np.ndindex(*y.shape):
        z = np.float32(y[idx] * s[idx[1]]) + b[idx[1]]          # float32 scalars: two roundings
        z = max(Fraction(float(z)), Fraction(0))
        z = min(max(z, Fraction(l)), Fraction(u))
        t = (z - Fraction(l)) / d
        if abs((t % 1) - Fraction(1, 2)) < Fraction(1, 1000):
            continue                                             # too close to a midpoint for this check
        assert got[idx] == int(t + Fraction(1, 2)), idx


# ---- weight-only quantized layers (quantized weights, real-valued activations) -----

def test_weight_only_layer_is_the_float_convolution_with_the_weight_levels():
    """oracle.conv_weight_only against torch's float64 conv2d on separately formed
    levels, asymmetric geometry, stride 2, padding."""
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(11)
    x = rng.standard_normal((2, 5, 7, 6)).astype(np.float32)
    w = (rng.standard_normal((4, 5, 3, 3)) * 0.2).astype(np.float32)
    lw = w.reshape(4, -1).min(axis=1) * np.float32(0.9)
    uw = w.reshape(4, -1).max(axis=1) * np.float32(0.8)
    for bits in (1, 2, 3):
        code = oracle.quantize_weights(w, lw, uw, bits)
        got, scale = oracle.conv_weight_only(x, code, lw, uw, bits, 2, 1)
        top = 2 ** bits - 1
        delta = ((uw.astype(np.float32) - lw.astype(np.float32)) / np.float32(top)).astype(np.float32)
        levels = lw.astype(np.float64)[:, None, None, None] + delta.astype(np.float64)[:, None, None, None] * code
        want = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(levels), stride=2, padding=1).numpy()
        assert np.abs(got - want).max() <= 1e-6 * np.abs(want).max()
        want_abs = F.conv2d(torch.from_numpy(np.abs(x)).double(), torch.from_numpy(np.abs(levels)), stride=2, padding=1).numpy()
        assert np.abs(scale - want_abs).max() <= 1e-6 * want_abs.max()
        assert (scale >= np.abs(got) * (1 - 1e-6)).all()


def test_binary_weights_with_symmetric_range_are_scaled_signs():
    """1-bit weights with (l, u) = (-alpha, +alpha): the layer is alpha times the
    convolution with sgn(w) (Sec. 3.1 binary quantizer, sgn(0) = +1)."""
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(12)
    x = rng.standard_normal((1, 6, 5, 5)).astype(np.float32)
    w = rng.standard_normal((3, 6, 3, 3)).astype(np.float32)
    w[0, 0, 0, 0] = 0.0
    alpha = np.array([0.5, 0.25, 2.0], np.float32)
    code = oracle.quantize_weights(w, -alpha, alpha, 1)
    got, _ = oracle.conv_weight_only(x, code, -alpha, alpha, 1, 1, 1)
    sgn = np.where(w >= 0, 1.0, -1.0)
    want = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(sgn), padding=1).numpy() * alpha[None, :, None, None]
    assert np.array_equal(got, want.astype(np.float32))
