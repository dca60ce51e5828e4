"""Whole-tensor parity on the full benchmark shapes (Algorithm 1 steps 1, 3-5).

Every layer shape of config 3 (ResNet-18 stack, batch 64, at 2, 3 and 4 bits),
config 4 (MobileNetV2 pointwise pairs, batch 64) and config 5 (VGG-16 stack,
batch 32, 2 bits) goes through the C ABI at full size, in the automatic launch
configuration the benchmark times (kernel and tile chosen by the library) and
with both values of DSQ_CONV_MANY_IN_FLIGHT, and every element is compared
with the oracle:

  * activation codes and pixel code sums: bit-exact;
  * the int32 accumulators: bit-exact against the oracle's integer convolution;
  * the fp32 output: |gpu - ref| <= 1e-5 |ref| + 1e-5 Da Dw[o] per element and
    max|gpu - ref| <= 1e-5 max|ref| per tensor, against the oracle's direct
    convolution of the dequantized doubles;
  * the chained call's codes for the next layer: equal to the oracle's
    requantization of its own output except where that value lies within 1e-4
    of a quantizer midpoint (there: at most one code apart), and pixel sums
    equal to the sums of the codes written; and the codes equal those of the
    simple kernel bit for bit.

The launch plans chosen at these sizes (tile, wave groups, fetch units per
thread, strip width, ragged last tile, per-XCD tile ranges) are not reached by
the small-geometry tests, which is why the full tensors are compared here.
"""
import numpy as np
import pytest

import oracle
from helpers import assert_out_close, oracle_layer, run_layer_gpu, unpack_act
from paper_1908_05033_amd import inputs
from test_gpu_requant import assert_codes_match, run_requant_gpu

pytestmark = pytest.mark.gpu

CASES = [(3, li, bits) for bits in (2, 3, 4) for li in range(10)] + \
        [(4, li, 4) for li in range(5)] + [(5, li, 2) for li in range(8)]


@pytest.mark.parametrize("cfg,li,bits", CASES)
def test_every_element_of_the_layer_at_full_size(cfg, li, bits):
    layer, inp = inputs.make_config_layer(cfg, li, bits=bits if cfg == 3 else None)
    L = layer
    assert L.bits == bits
    a_code, w_code = oracle_layer(layer, inp)
    acc = oracle.conv_codes(a_code, w_code, L.stride, L.pad)
    ref = oracle.conv_real(a_code, inp["l_a"], inp["u_a"], w_code, inp["l_w"], inp["u_w"], bits, L.stride, L.pad)
    da = oracle.delta(inp["l_a"], inp["u_a"], bits)
    dw = [oracle.delta(float(a), float(b), bits) for a, b in zip(inp["l_w"], inp["u_w"])]

    # plain call, with the raw accumulators
    got = run_layer_gpu(layer, inp, kernel=0)
    codes = unpack_act(got["act_packed"], L.N, L.H, L.W, L.C_in, bits)
    assert np.array_equal(codes[..., :L.C_in], a_code.transpose(0, 2, 3, 1)), "activation codes differ"
    assert not codes[..., L.C_in:].any(), "padding channels must hold code 0"
    assert np.array_equal(got["pix_sum"].reshape(L.N, L.H, L.W), a_code.sum(axis=1, dtype=np.int32)), \
        "pixel code sums differ"
    del codes
    assert np.array_equal(got["acc"], acc), "accumulators differ"
    assert_out_close(got["out"], ref, da, dw)
    del acc
    # the store path the benchmark times (no accumulator output), under both policies:
    # the same expression everywhere, so bit-identical to the first run
    for many in (False, True):
        fast = run_layer_gpu(layer, inp, kernel=0, with_acc=False, many_in_flight=many)["out"]
        assert np.array_equal(fast, got["out"]), "outputs differ between store paths (many_in_flight=%s)" % many
        del fast
    del got

    # chained call: folded batch norm + ReLU + the next layer's quantizer
    scale, shift = inputs.affine_params(100 * cfg + li, L.C_out, shift_std=0.05)
    z = oracle.affine_relu(ref, scale, shift, True)
    l_n, u_n = 0.0, float(np.float32(max(np.quantile(z.reshape(-1)[::61], 0.98), 0.1)))
    want = oracle.quantize(z, l_n, u_n, bits)
    want_sum = want.sum(axis=1, dtype=np.int64)
    for many in (False, True):
        got_c, pix, *_ = run_requant_gpu(layer, inp, scale, shift, True, l_n, u_n, bits, many_in_flight=many)
        nbad = assert_codes_match(got_c, want, z, l_n, u_n, bits, L.C_out)
        assert np.array_equal(pix, got_c.sum(axis=3, dtype=np.int64)), "pixel sums are not the sums of the codes"
        if nbad == 0:
            assert np.array_equal(pix, want_sum)
        if not many:
            # the simple kernel runs the exact sequence (the recipe with its division) on every
            # output; the tuned kernels decide most codes from a cheaper evaluation: same bits
            ref_c, ref_pix, *_ = run_requant_gpu(layer, inp, scale, shift, True, l_n, u_n, bits, kernel=1)
            assert np.array_equal(got_c, ref_c), "codes differ from the simple kernel's"
            assert np.array_equal(pix, ref_pix)
            del ref_c, ref_pix
        del got_c, pix
