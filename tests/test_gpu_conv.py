"""GPU parity of dsq_conv2d against the oracle: int32 accumulators bit-exact,
float output within 1e-5 (relative, with a floor of 1e-5 code products)."""
import numpy as np
import pytest
import torch

import oracle
from helpers import assert_out_close, oracle_layer, run_layer_gpu, unpack_act
from paper_1908_05033_amd import binding as B
from paper_1908_05033_amd import inputs

pytestmark = pytest.mark.gpu

KERNELS = [1, 3, 4, 5, 6]   # 1 = simple; 3..6 = LDS-patch kernel with each of its tiles


def _run(layer, inp, kernel, **kw):
    try:
        return run_layer_gpu(layer, inp, kernel=kernel, **kw)
    except B.DsqError as e:
        if kernel >= 2 and e.status == 5:
            pytest.skip("geometry not supported by the patch kernel")
        raise


@pytest.mark.parametrize("kernel", [3, 4, 5, 6])
@pytest.mark.parametrize("cfg", [1, 2])
def test_patch_kernel_takes_the_benchmark_shapes(cfg, kernel):
    """The tuned kernel (every tile) must accept configs 1 and 2 itself rather
    than hand them to the fallback: a planner regression would otherwise only
    show up as skipped tests."""
    layer, inp = inputs.make_config_layer(cfg)
    run_layer_gpu(layer, inp, kernel=kernel, with_acc=False)


def _check_full(layer, inp, kernel, w_codes=None, **kw):
    got = _run(layer, inp, kernel, w_codes=w_codes, **kw)
    a_code, w_code = oracle_layer(layer, inp, w_codes)
    acc = oracle.conv_codes(a_code, w_code, layer.stride, layer.pad)
    assert np.array_equal(got["acc"], acc)
    ref = oracle.conv_real(a_code, inp["l_a"], inp["u_a"], w_code, inp["l_w"], inp["u_w"],
                           layer.bits, layer.stride, layer.pad)
    da = oracle.delta(inp["l_a"], inp["u_a"], layer.bits)
    dw = [oracle.delta(float(a), float(b), layer.bits) for a, b in zip(inp["l_w"], inp["u_w"])]
    assert_out_close(got["out"], ref, da, dw)
    # without the raw-accumulator output the kernels may take a different
    # (faster) store path: check that one too
    got2 = _run(layer, inp, kernel, w_codes=w_codes, with_acc=False, **kw)
    assert_out_close(got2["out"], ref, da, dw)
    return got, ref


SMALL = [  # N, C_in, H, W, C_out, R, stride, pad
    (2, 64, 9, 7, 64, 3, 1, 1),
    (1, 24, 10, 11, 144, 1, 1, 0),
    (3, 144, 5, 6, 24, 1, 1, 0),
    (2, 96, 7, 9, 40, 3, 2, 1),
    (1, 128, 8, 8, 70, 3, 1, 0),
    (2, 64, 9, 9, 128, 1, 2, 0),
    (1, 192, 6, 5, 64, 3, 2, 0),
    (5, 70, 7, 7, 33, 3, 1, 1),
    (1, 320, 7, 7, 300, 1, 1, 0),
    (1, 64, 3, 3, 16, 3, 1, 2),
    (1, 64, 4, 150, 32, 3, 1, 1),      # wide rows: several column strips with a ragged last one
    (2, 64, 13, 37, 64, 3, 2, 1),      # stride 2 on odd sizes
    (3, 128, 1, 1, 48, 1, 1, 0),       # a single pixel per image
    (1, 3, 12, 12, 8, 3, 1, 1),        # fewer channels than one packed word
    (1, 64, 2, 300, 16, 1, 2, 0),      # 1x1 stride 2, very wide
]


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("bits", [1, 2, 3, 4])
@pytest.mark.parametrize("geom", SMALL)
def test_small_geometries_generic_bounds(geom, bits, kernel):
    """Ragged sizes, l_a != 0 (so the padding-dependent terms matter) and
    asymmetric per-channel weight ranges."""
    N, Ci, H, W, Co, R, stride, pad = geom
    layer, inp = inputs.small_random_case(sum(geom) + bits, N, Ci, H, W, Co, R, stride, pad, bits,
                                          l_a=-0.4, u_a=2.1)
    _check_full(layer, inp, kernel)


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("geom", SMALL[:4])
def test_nchw_in_and_out(geom, kernel):
    N, Ci, H, W, Co, R, stride, pad = geom
    layer, inp = inputs.small_random_case(sum(geom), N, Ci, H, W, Co, R, stride, pad, 4,
                                          l_a=0.0, u_a=2.5, asym_w=False)
    _check_full(layer, inp, kernel, x_layout=B.DSQ_NCHW, out_layout=B.DSQ_NCHW)


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("la_int", [0, -2])
def test_integer_levels_give_exact_integers(kernel, la_int):
    """Delta_a = Delta_w = 1 with integer bounds: the float output is an
    integer and must be reproduced exactly."""
    layer = inputs.ConvLayer("int", 2, 64, 6, 7, 20, 3, 3, 1, 1, 4)
    rng = np.random.default_rng(41)
    w_codes = rng.integers(0, 16, (20, 64, 3, 3)).astype(np.uint8)
    x = torch.from_numpy(rng.integers(la_int, la_int + 16, (2, 64, 6, 7)).astype(np.float32))
    lw = rng.integers(-15, 1, 20).astype(np.float32)
    inp = {"x": x, "w": None, "l_a": float(la_int), "u_a": float(la_int + 15), "l_w": lw, "u_w": lw + 15}
    got, ref = _check_full(layer, inp, kernel, w_codes=w_codes)
    assert np.array_equal(got["out"], ref)
    assert np.all(ref == np.round(ref))


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("cfg", [1, 2])
def test_config_1_and_2_full_tensors(cfg, kernel):
    layer, inp = inputs.make_config_layer(cfg)
    _check_full(layer, inp, kernel)


def _check_sampled(layer, inp, kernel, nsamples=4000):
    got = _run(layer, inp, kernel)
    fast = _run(layer, inp, kernel, with_acc=False)["out"]     # the store path bench.py times
    a_code, w_code = oracle_layer(layer, inp)
    total = got["out"].size
    rng = np.random.default_rng(layer.C_in + layer.H + layer.bits)
    idx = rng.integers(0, total, nsamples)
    # always include image corners / edges of first and last image and channel
    Ho, Wo, Co = layer.Ho, layer.Wo, layer.C_out
    corners = [((n * Co + o) * Ho + y) * Wo + x
               for n in (0, layer.N - 1) for o in (0, Co - 1)
               for y in (0, Ho - 1) for x in (0, Wo - 1)]
    idx = np.concatenate([idx, np.array(corners, np.int64)])
    vals, accs = oracle.conv_at(a_code, inp["l_a"], inp["u_a"], w_code, inp["l_w"], inp["u_w"],
                                layer.bits, layer.stride, layer.pad, idx)
    assert np.array_equal(got["acc"].reshape(-1)[idx], accs)
    o_of = (idx // (Ho * Wo)) % Co
    da = oracle.delta(inp["l_a"], inp["u_a"], layer.bits)
    dw = np.array([oracle.delta(float(inp["l_w"][o]), float(inp["u_w"][o]), layer.bits) for o in o_of])
    r = vals.astype(np.float64)
    for out in (got["out"], fast):
        g = out.reshape(-1)[idx].astype(np.float64)
        assert np.all(np.abs(g - r) <= 1e-5 * np.abs(r) + 1e-5 * da * dw)
    # both store paths evaluate the same expression: identical everywhere
    assert np.array_equal(got["out"], fast)
    # properties that hold at any size: finite everywhere, accumulators within
    # the closed-form bound (2^b-1)^2 * K
    assert np.isfinite(got["out"]).all()
    top = 2 ** layer.bits - 1
    assert got["acc"].min() >= 0 and got["acc"].max() <= top * top * layer.C_in * layer.R * layer.S
    # every code of the full tensor is still checked bit for bit
    from helpers import unpack_act
    codes = unpack_act(got["act_packed"], layer.N, layer.H, layer.W, layer.C_in, layer.bits)
    assert np.array_equal(codes[..., :layer.C_in], a_code.transpose(0, 2, 3, 1))


R18 = list(range(10))


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("li", R18)
def test_config_3_resnet18_full_size_sampled(li, bits):
    layer, inp = inputs.make_config_layer(3, li, bits=bits)
    _check_sampled(layer, inp, 0)


@pytest.mark.parametrize("li", range(5))
def test_config_4_mobilenetv2_pointwise_full_size_sampled(li):
    layer, inp = inputs.make_config_layer(4, li)
    _check_sampled(layer, inp, 0)


@pytest.mark.parametrize("li", range(8))
def test_config_5_vgg16_full_size_sampled(li):
    layer, inp = inputs.make_config_layer(5, li)
    _check_sampled(layer, inp, 0)


@pytest.mark.parametrize("kernel", [0, 1, 3, 4, 6])
@pytest.mark.parametrize("bits", [2, 4])
def test_largest_codes_at_the_largest_k(bits, kernel):
    """Every activation and weight code at its maximum over K = 9 * 512: the
    largest accumulator the benchmark shapes can produce (41 472 at 2-bit on
    the FP4 instruction's fp32 accumulators, 1 036 800 at 4-bit) must still be
    the exact integer."""
    top = (1 << bits) - 1
    layer, inp = inputs.small_random_case(3, 1, 512, 6, 7, 64, 3, 1, 1, bits, l_a=0.0, u_a=2.0, asym_w=False)
    inp["x"] = torch.full_like(inp["x"], 5.0)                       # clips to u_a: top code everywhere
    w_codes = np.full((64, 512, 3, 3), top, dtype=np.uint8)
    got = _run(layer, inp, kernel, w_codes=w_codes)
    a_code, _ = oracle_layer(layer, inp, w_codes)
    assert a_code.min() == top
    acc = oracle.conv_codes(a_code, w_codes, 1, 1)
    assert acc.max() == top * top * 9 * 512
    assert np.array_equal(got["acc"], acc)


@pytest.mark.parametrize("kernel", [0, 1])
@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_largest_codes_at_the_deepest_dot_product_the_library_accepts(bits, kernel):
    """K = 9 * 51 712 is the deepest the library takes (9 * K <= 2^22).  With every
    code at its maximum the accumulator of the centre pixel is top^2 * K: 4.19 M at
    2 bits, still an exact integer in the FP4 path's fp32 accumulators (quarter
    units below 2^24), 104.7 M at 4 bits in int32."""
    top = (1 << bits) - 1
    C_in = 51712
    layer, inp = inputs.small_random_case(5, 1, C_in, 3, 3, 32, 3, 1, 1, bits, l_a=0.0, u_a=2.0, asym_w=False)
    inp["x"] = torch.full_like(inp["x"], 5.0)
    w_codes = np.full((32, C_in, 3, 3), top, dtype=np.uint8)
    got = _run(layer, inp, kernel, w_codes=w_codes)
    a_code, _ = oracle_layer(layer, inp, w_codes)
    acc = oracle.conv_codes(a_code, w_codes, 1, 1)
    assert acc.max() == top * top * 9 * C_in
    assert np.array_equal(got["acc"], acc)


@pytest.mark.parametrize("kernel", [0, 1, 3, 6])
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("C_in", [51712, 4608])
def test_near_limit_accumulators_fed_by_small_odd_products(bits, kernel, C_in):
    """The 1/2-bit path sums quarter-unit products in the fp32 accumulators of the
    FP4 matrix instruction.  Here the accumulators climb to within a few percent
    of the deepest sum the library accepts (codes mostly at the top) while a
    scattered subset of activation and weight codes is 1 or 2, so that single
    quarter units (1 x 1), three (1 x 3) and six (2 x 3) keep arriving at an accumulator that is already
    large: any loss of low bits in the instruction's alignment or in the order of
    its partial sums would change the integer.  Codes differ from tap to tap, pixel
    to pixel and channel to channel."""
    top = (1 << bits) - 1
    rng = np.random.default_rng(1000 * bits + C_in)
    layer, inp = inputs.small_random_case(5, 1, C_in, 4, 5, 48, 3, 1, 1, bits, l_a=0.0, u_a=float(top), asym_w=False)
    a_codes = np.where(rng.random((1, C_in, 4, 5)) < 0.07, rng.integers(1, 3, (1, C_in, 4, 5)), top).astype(np.uint8)
    w_codes = np.where(rng.random((48, C_in, 3, 3)) < 0.05, rng.integers(1, 3, (48, C_in, 3, 3)), top).astype(np.uint8)
    inp["x"] = torch.from_numpy(a_codes.astype(np.float32))        # Delta_a = 1, l_a = 0: x is its own code
    got = _run(layer, inp, kernel, w_codes=w_codes)
    a_code, _ = oracle_layer(layer, inp, w_codes)
    assert np.array_equal(a_code, a_codes)
    acc = oracle.conv_codes(a_code, w_codes, 1, 1)
    assert acc.max() > 0.85 * top * top * 9 * C_in and len(np.unique(acc % 4)) == 4
    assert np.array_equal(got["acc"], acc)


@pytest.mark.parametrize("kernel", [0, 1, 3, 4, 6])
def test_binary_layer_is_the_convolution_of_signs(kernel):
    """bits = 1 with (l, u) = (-1, +1) is the binary quantizer of Sec. 3.1
    (sgn, with sgn(0) = +1): the layer output must be exactly the zero-padded
    cross-correlation of sgn(a) and sgn(w), an integer-valued tensor."""
    import torch.nn.functional as F
    layer, inp = inputs.small_random_case(9, 2, 192, 9, 8, 80, 3, 1, 1, 1, l_a=-1.0, u_a=1.0)
    inp["x"] = inp["x"] - inp["x"].mean()
    inp["x"][0, :, 0, 0] = 0.0                          # sgn(0) = +1
    inp["l_w"] = -np.ones(80, np.float32)
    inp["u_w"] = np.ones(80, np.float32)
    got = _run(layer, inp, kernel)
    sgn = lambda t: torch.where(t >= 0, 1.0, -1.0).double()
    want = F.conv2d(sgn(inp["x"]), sgn(inp["w"]), padding=1).numpy()
    assert np.array_equal(got["out"].astype(np.float64), want)


def _check_mixed_widths(bits_a, bits_w, kernel, geom):
    N, Ci, H, W, Co, R, stride, pad = geom
    layer, inp = inputs.small_random_case(31, N, Ci, H, W, Co, R, stride, pad, bits_a, l_a=0.0, u_a=2.2)
    L = layer
    buf = B.alloc_layer(L.N, L.C_in, L.H, L.W, L.C_out, R, R, stride, pad, bits_a, with_acc=True)
    xd = inp["x"].permute(0, 2, 3, 1).contiguous().cuda()
    B.dsq_quantize_act(xd, B.DSQ_NHWC, L.N, L.C_in, L.H, L.W, inp["l_a"], inp["u_a"], bits_a,
                       buf.act_packed, buf.pix_code_sum)
    B.dsq_pack_weights_for(inp["w"].contiguous().cuda(), torch.from_numpy(inp["l_w"]).cuda(),
                           torch.from_numpy(inp["u_w"]).cuda(), None, L.C_out, L.C_in, R, R, bits_w, bits_a,
                           buf.w_packed, buf.w_aux)
    buf.desc.flags = B.DSQ_CONV_KERNEL(kernel)
    B.dsq_conv2d(buf.desc, buf.act_packed, buf.pix_code_sum, inp["l_a"], inp["u_a"], buf.w_packed, buf.w_aux,
                 buf.out, B.DSQ_NHWC, buf.acc)
    torch.cuda.synchronize()
    a_code = oracle.quantize(inp["x"].numpy(), inp["l_a"], inp["u_a"], bits_a)
    w_code = oracle.quantize_weights(inp["w"].numpy(), inp["l_w"], inp["u_w"], bits_w)
    assert np.array_equal(buf.acc.cpu().numpy().transpose(0, 3, 1, 2), oracle.conv_codes(a_code, w_code, stride, pad))
    # the real-valued reference: dequantize each side with its own width
    a_hat = oracle.dequantize(a_code, inp["l_a"], inp["u_a"], bits_a)
    w_hat = np.stack([oracle.dequantize(w_code[o], float(inp["l_w"][o]), float(inp["u_w"][o]), bits_w)
                      for o in range(L.C_out)])
    ref = oracle.conv_dequantized(a_hat, w_hat, stride, pad)
    dw = [oracle.delta(float(a), float(b), bits_w) for a, b in zip(inp["l_w"], inp["u_w"])]
    assert_out_close(buf.out.cpu().numpy().transpose(0, 3, 1, 2), ref, oracle.delta(inp["l_a"], inp["u_a"], bits_a), dw)


@pytest.mark.parametrize("kernel", [0, 1, 3])
@pytest.mark.parametrize("bits_a,bits_w", [(4, 3), (3, 4), (2, 1), (1, 2), (4, 2), (4, 1), (3, 2), (3, 1)])
def test_mixed_widths(bits_a, bits_w, kernel):
    """Weights and activations of different widths: dsq_pack_weights_for is given
    both, dsq_quantize_act and the layer descriptor the activations'."""
    _check_mixed_widths(bits_a, bits_w, kernel, (2, 128, 7, 6, 72, 3, 1, 1))


@pytest.mark.parametrize("bits_a,bits_w", [(4, 3), (3, 4), (2, 1), (1, 2), (4, 1), (3, 2)])
def test_mixed_widths_through_the_split_k_kernel(bits_a, bits_w):
    _check_mixed_widths(bits_a, bits_w, 7, (37, 576, 1, 1, 40, 1, 1, 0))


@pytest.mark.parametrize("kernel", [0, 1])
def test_largest_tensors_the_library_accepts(kernel):
    """A 1x1 layer whose input and output both have just under 2^31 elements
    (33.5 M pixels of 64 channels, 8.6 GB of fp32 output, as much again of raw
    accumulators): addressing at the size limit.  Every pixel of a 1x1 layer
    stands alone, so the oracle checks a sample of them: the first and the last
    rows of the tensor and 4096 pixels in between."""
    bits = 4
    N, H, W, C = 1, 32768, 1023, 64
    P = N * H * W
    assert P * C < (1 << 31) <= N * H * (W + 1) * C
    g = torch.Generator(device="cuda").manual_seed(inputs.BASE_SEED + 77)
    x = torch.empty((P, C), dtype=torch.float32, device="cuda")
    for s in range(0, P, 1 << 21):
        x[s:s + (1 << 21)].normal_(0.4, 1.0, generator=g)
    l_a, u_a = 0.0, float(np.float32(2.75))
    gw = torch.Generator().manual_seed(inputs.BASE_SEED + 78)
    w = torch.randn((C, C, 1, 1), generator=gw) * 0.1
    uw = w.reshape(C, -1).abs().max(dim=1).values.numpy().astype(np.float32)
    lw = (-0.9 * uw).astype(np.float32)
    buf = B.alloc_layer(N, C, H, W, C, 1, 1, 1, 0, bits, with_acc=True)
    B.dsq_quantize_act(x, B.DSQ_NHWC, N, C, H, W, l_a, u_a, bits, buf.act_packed, buf.pix_code_sum)
    B.dsq_pack_weights(w.cuda(), torch.from_numpy(lw).cuda(), torch.from_numpy(uw).cuda(), None, C, C, 1, 1, bits,
                       buf.w_packed, buf.w_aux)
    buf.desc.flags = B.DSQ_CONV_KERNEL(kernel)
    B.dsq_conv2d(buf.desc, buf.act_packed, buf.pix_code_sum, l_a, u_a, buf.w_packed, buf.w_aux, buf.out,
                 B.DSQ_NHWC, buf.acc)
    torch.cuda.synchronize()
    rs = np.random.RandomState(5)
    sample = np.unique(np.concatenate([np.arange(2048), np.arange(P - 2048, P), rs.randint(0, P, 4096)]))
    idx = torch.from_numpy(sample).cuda()
    xs = x[idx].cpu().numpy().reshape(len(sample), C, 1, 1)             # each sampled pixel as a 1x1 image
    out = buf.out.reshape(P, C)[idx].cpu().numpy().reshape(len(sample), C, 1, 1)
    acc = buf.acc.reshape(P, C)[idx].cpu().numpy().reshape(len(sample), C, 1, 1)
    a_code = oracle.quantize(xs, l_a, u_a, bits)
    w_code = oracle.quantize_weights(w.numpy(), lw, uw, bits)
    assert np.array_equal(acc, oracle.conv_codes(a_code, w_code, 1, 0))
    ref = oracle.conv_real(a_code, l_a, u_a, w_code, lw, uw, bits, 1, 0)
    dw = [oracle.delta(float(a), float(b), bits) for a, b in zip(lw, uw)]
    assert_out_close(out, ref, oracle.delta(l_a, u_a, bits), dw)
    # the chained call on the same tensors: the next layer's codes and pixel sums of the sample
    scale = (0.5 + torch.rand(C, generator=gw)).numpy().astype(np.float32)
    shift = (torch.randn(C, generator=gw) * 0.3).numpy().astype(np.float32)
    l_n, u_n, bits_n = 0.0, float(np.float32(1.9)), 4
    codes_n = torch.empty((B.dsq_act_packed_bytes(N, H, W, C, bits_n),), dtype=torch.uint8, device="cuda")
    pix_n = torch.empty((P,), dtype=torch.int32, device="cuda")
    buf.desc.flags = B.DSQ_CONV_KERNEL(kernel)
    B.dsq_conv2d_requant(buf.desc, buf.act_packed, buf.pix_code_sum, l_a, u_a, buf.w_packed, buf.w_aux,
                         torch.from_numpy(scale).cuda(), torch.from_numpy(shift).cuda(), True, l_n, u_n, bits_n,
                         codes_n, pix_n)
    torch.cuda.synchronize()
    want_n = oracle.requantize(ref.astype(np.float32), scale, shift, True, l_n, u_n, bits_n).reshape(len(sample), C)
    got_rows = codes_n.reshape(P, -1)[idx].cpu().numpy()
    got_n = unpack_act(got_rows.reshape(-1), len(sample), 1, 1, C, bits_n).reshape(len(sample), -1)[:, :C]
    # (ref is the oracle's binary64 value; the layer's binary32 output may round to the other side of a
    # quantizer threshold once in a while: compare where the oracle's own two roundings agree)
    y32 = out.astype(np.float32)
    want_from_gpu_y = oracle.requantize(y32, scale, shift, True, l_n, u_n, bits_n).reshape(len(sample), C)
    assert np.array_equal(got_n, want_from_gpu_y)
    assert (got_n != want_n).mean() < 1e-3
    assert np.array_equal(pix_n[idx].cpu().numpy(), want_from_gpu_y.astype(np.int64).sum(axis=1))
    # nothing was written past the tensors' ends: the last pixel is the sample's last row, and a
    # pixel row more is refused
    d2 = B.dsq_conv_desc(N=N, C_in=C, H=H, W=W + 1, C_out=C, R=1, S=1, stride=1, pad=0, bits=bits)
    with pytest.raises(B.DsqError) as e:
        B.dsq_conv2d(d2, buf.act_packed, buf.pix_code_sum, l_a, u_a, buf.w_packed, buf.w_aux, buf.out, B.DSQ_NHWC, None)
    assert e.value.status == 5


@pytest.mark.parametrize("geom", [(2, 256, 14, 14, 256, 3, 1, 1), (1, 512, 7, 7, 512, 3, 1, 1), (2, 128, 9, 11, 96, 3, 2, 1),
                                  (1, 576, 6, 6, 96, 1, 1, 0)])
@pytest.mark.parametrize("bits", [2, 4])
def test_throughput_policy_gives_the_same_results(geom, bits):
    """DSQ_CONV_MANY_IN_FLIGHT only changes how a layer is spread over the chip
    (one wave group per workgroup where the default uses two): accumulators and
    outputs of layers that the default runs with two groups must not change."""
    N, Ci, H, W, Co, R, stride, pad = geom
    layer, inp = inputs.small_random_case(41 + bits, N, Ci, H, W, Co, R, stride, pad, bits, l_a=0.0, u_a=2.1)
    got, ref = _check_full(layer, inp, 0, many_in_flight=True)
    base = _run(layer, inp, 0)
    assert np.array_equal(got["acc"], base["acc"]) and np.array_equal(got["out"], base["out"])


FC_SHAPES = [  # N, C_in, H, W, C_out : 1x1 layers with few pixels and a deep dot product
    (64, 4096, 1, 1, 1000),
    (5, 520, 1, 1, 37),
    (2, 1024, 3, 2, 70),
    (256, 512, 1, 1, 96),
    (33, 2304, 1, 1, 128),
    (100, 640, 1, 1, 45),          # two pixel fragments per workgroup, the second one ragged
    (3, 576, 5, 9, 64),            # 135 pixels
    (1, 512, 40, 40, 544),         # 850 tiles: the split-K kernel takes it when forced, not by itself
]


@pytest.mark.parametrize("kernel", [0, 7])
@pytest.mark.parametrize("bits", [1, 2, 3, 4])
@pytest.mark.parametrize("shape", FC_SHAPES)
def test_fully_connected_shapes(shape, bits, kernel):
    """The split-K kernel (taken automatically for these shapes, and forced):
    accumulators bit-exact, outputs to tolerance, with and without the raw
    accumulator output."""
    N, Ci, H, W, Co = shape
    layer, inp = inputs.small_random_case(sum(shape) + bits, N, Ci, H, W, Co, 1, 1, 0, bits, l_a=0.0, u_a=2.3)
    _check_full(layer, inp, kernel)


@pytest.mark.parametrize("out_layout", [B.DSQ_NHWC, B.DSQ_NCHW])
@pytest.mark.parametrize("bits", [2, 4])
def test_fully_connected_general_epilogue(bits, out_layout):
    """l_a != 0 and NCHW output through the split-K kernel."""
    layer, inp = inputs.small_random_case(17 + bits, 9, 768, 2, 2, 50, 1, 1, 0, bits, l_a=-0.6, u_a=1.9)
    got = run_layer_gpu(layer, inp, kernel=7, out_layout=out_layout)
    a_code, w_code = oracle_layer(layer, inp)
    assert np.array_equal(got["acc"], oracle.conv_codes(a_code, w_code, 1, 0))
    ref = oracle.conv_real(a_code, inp["l_a"], inp["u_a"], w_code, inp["l_w"], inp["u_w"], bits, 1, 0)
    dw = [oracle.delta(float(a), float(b), bits) for a, b in zip(inp["l_w"], inp["u_w"])]
    assert_out_close(got["out"], ref, oracle.delta(inp["l_a"], inp["u_a"], bits), dw)


def test_split_k_kernel_refuses_other_layers():
    layer, inp = inputs.small_random_case(3, 2, 64, 5, 5, 32, 3, 1, 1, 4)
    with pytest.raises(B.DsqError) as e:
        run_layer_gpu(layer, inp, kernel=7)
    assert e.value.status == 5
