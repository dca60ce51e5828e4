"""CPU-only checks of the C ABI: the library loads, exports every symbol the
header declares, answers the size queries, and rejects bad arguments on the
host before anything is launched (no GPU is touched)."""
import ctypes as C
import os
import re

import pytest

from paper_1908_05033_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "dsqconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dsq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = B.load_library()
    names = _declared_functions()
    assert set(B.EXPORTS) == set(names)
    for n in names:
        assert getattr(lib, n) is not None


def test_size_queries():
    # 4-bit: C padded to 64, 2 codes per byte; 2-bit: 4 codes per byte
    assert B.dsq_act_packed_bytes(32, 14, 14, 256, 4) == 32 * 14 * 14 * 128
    assert B.dsq_act_packed_bytes(1, 2, 3, 24, 4) == 6 * 32
    assert B.dsq_act_packed_bytes(1, 2, 3, 24, 3) == 6 * 32       # 3-bit in 4-bit containers
    assert B.dsq_act_packed_bytes(1, 2, 3, 65, 2) == 6 * 32
    assert B.dsq_wgt_packed_bytes(256, 256, 3, 3, 4) == 256 * 9 * 128
    assert B.dsq_wgt_packed_bytes(24, 144, 1, 1, 4) == 256 * 96
    assert B.dsq_wgt_aux_bytes(64, 3, 3) == 256 * (3 + 9) * 4
    assert B.dsq_act_packed_bytes(0, 1, 1, 1, 4) == 0
    assert B.dsq_act_packed_bytes(1, 1, 1, 1, 5) == 0


def test_status_strings():
    lib = B.load_library()
    seen = set()
    for s in range(9):
        msg = lib.dsq_status_string(s).decode()
        assert msg and msg not in seen
        seen.add(msg)
    assert lib.dsq_status_string(99).decode() == "unknown status"


FAKE = 0x1000      # aligned, non-null; never dereferenced: validation fails first


def _q(x=FAKE, layout=0, N=1, Cc=8, H=2, W=2, l=0.0, u=1.0, bits=4, codes=FAKE, nbytes=1 << 20,
       pix=FAKE):
    return B.load_library().dsq_quantize_act(x, layout, N, Cc, H, W, l, u, bits, codes, nbytes, pix, None)


def test_quantize_act_rejects_bad_arguments():
    assert _q(x=None) == 1
    assert _q(codes=None) == 1
    assert _q(pix=None) == 1
    assert _q(bits=0) == 2 and _q(bits=5) == 2
    assert _q(l=1.0, u=1.0) == 3 and _q(l=2.0, u=1.0) == 3
    assert _q(l=float("nan")) == 3 and _q(u=float("inf")) == 3
    assert _q(l=0.0, u=1e-38) == 3 and _q(l=-3e38, u=3e38) == 3 and _q(l=0.0, u=9e-31) == 3
    assert _q(N=0) == 4 and _q(Cc=-1) == 4
    assert _q(layout=7) == 5
    assert _q(N=1 << 15, H=1 << 8, W=1 << 8, Cc=64, nbytes=1 << 62) == 5
    assert _q(x=FAKE + 4) == 6 and _q(codes=FAKE + 8) == 6
    assert _q(nbytes=2 * 2 * 32 - 1) == 7


def _p(w=FAKE, lw=FAKE, uw=FAKE, codes=None, Co=8, Ci=8, R=3, S=3, bits=4, wp=FAKE, wb=1 << 24,
       aux=FAKE, ab=1 << 20):
    return B.load_library().dsq_pack_weights(w, lw, uw, codes, Co, Ci, R, S, bits, wp, wb, aux, ab, None)


def test_pack_weights_rejects_bad_arguments():
    assert _p(w=None, codes=None) == 1
    assert _p(lw=None) == 1 and _p(wp=None) == 1 and _p(aux=None) == 1
    assert _p(bits=8) == 2
    assert _p(Co=0) == 4
    assert _p(R=3, S=1) == 5 and _p(R=5, S=5) == 5 and _p(R=2, S=2) == 5
    assert _p(wp=FAKE + 2) == 6
    assert _p(wb=100) == 7 and _p(ab=100) == 7


def test_pack_weights_for_rejects_bad_arguments():
    lib = B.load_library()
    f = lambda bw=2, ba=4, w=FAKE, wb=1 << 24: lib.dsq_pack_weights_for(w, FAKE, FAKE, None, 8, 8, 3, 3, bw, ba, FAKE, wb,
                                                                        FAKE, 1 << 20, None)
    assert f(bw=0) == 2 and f(ba=5) == 2
    assert f(bw=4, ba=2) == 5 and f(bw=3, ba=1) == 5          # wide weight codes, narrow fields
    assert f(w=None) == 1
    assert f(wb=100) == 7


def _c(desc=None, act=FAKE, pix=FAKE, la=0.0, ua=1.0, wp=FAKE, aux=FAKE, out=FAKE, layout=0, acc=None,
       **kw):
    d = dict(N=1, C_in=8, H=4, W=4, C_out=8, R=3, S=3, stride=1, pad=1, bits=4)
    d.update(kw)
    desc = B.dsq_conv_desc(**d) if desc is None else desc
    return B.load_library().dsq_conv2d(C.byref(desc), act, pix, la, ua, wp, aux, out, layout, acc, None)


def test_conv2d_rejects_bad_arguments():
    lib = B.load_library()
    assert lib.dsq_conv2d(None, FAKE, FAKE, 0.0, 1.0, FAKE, FAKE, FAKE, 0, None, None) == 1
    assert _c(act=None) == 1 and _c(out=None) == 1 and _c(aux=None) == 1
    assert _c(bits=7) == 2
    assert _c(la=1.0, ua=0.0) == 3 and _c(la=0.0, ua=1e-37) == 3 and _c(la=-2e38, ua=2e38) == 3
    assert _c(N=0) == 4 and _c(H=1, W=1, pad=0) == 4
    assert _c(R=3, S=1) == 5 and _c(R=5, S=5, pad=2) == 5
    assert _c(stride=3) == 5 and _c(pad=3) == 5 and _c(R=1, S=1, pad=1) == 5
    assert _c(layout=3) == 5
    assert _c(N=64, H=1024, W=1024, C_in=64) == 5
    assert _c(H=3, W=3, C_in=51840) == 5          # 9 * 9 * C_in above 2^22: dot products too deep
    assert _c(out=FAKE + 4) == 6 and _c(acc=FAKE + 4) == 6


def test_binding_raises_on_error_status():
    with pytest.raises(B.DsqError) as e:
        B._check(2)
    assert "bits" in str(e.value)


def test_conv_flags_are_validated_per_call():
    """Kernel choice and policy travel in the descriptor (the library keeps no
    state): unknown bits and kernel numbers above 7 are refused."""
    assert _c(flags=0x20) == 5 and _c(flags=0x100) == 5 and _c(flags=-1) == 5
    assert _c(flags=8) == 5 and _c(flags=15) == 5
    assert _r(flags=0x40) == 5 and _r(flags=9) == 5 and _r(flags=0x100) == 5
    # the chained call's own flags are refused by the plain call and pass the chained call's flag
    # check (which then fails on the misaligned output)
    assert _c(flags=B.DSQ_CONV_NEXT_SUMS_ZERO) == 5
    assert _r(flags=B.DSQ_CONV_NEXT_SUMS_ZERO, codes=FAKE + 4) == 6
    # valid flag values get past the flag check (and fail later, on the misaligned output)
    for flags in (0, 1, 7, B.DSQ_CONV_MANY_IN_FLIGHT, B.DSQ_CONV_MANY_IN_FLIGHT | B.DSQ_CONV_KERNEL(4)):
        assert _c(flags=flags, out=FAKE + 4) == 6


def test_library_exports_no_setters():
    lib = B.load_library()
    for name in ("dsq_set_conv_kernel", "dsq_set_conv_policy"):
        assert not hasattr(lib, name)


def _r(desc=None, act=FAKE, pix=FAKE, la=0.0, ua=1.0, wp=FAKE, aux=FAKE, scale=None, shift=None, relu=1,
       ln=0.0, un=1.0, bn=4, codes=FAKE, nbytes=1 << 20, pixn=FAKE, **kw):
    d = dict(N=1, C_in=8, H=4, W=4, C_out=8, R=3, S=3, stride=1, pad=1, bits=4)
    d.update(kw)
    desc = B.dsq_conv_desc(**d) if desc is None else desc
    return B.load_library().dsq_conv2d_requant(C.byref(desc), act, pix, la, ua, wp, aux, scale, shift, relu,
                                               ln, un, bn, codes, nbytes, pixn, None)


def test_conv2d_requant_rejects_bad_arguments():
    assert _r(codes=None) == 1 and _r(pixn=None) == 1 and _r(act=None) == 1
    assert _r(bn=0) == 2 and _r(bn=5) == 2 and _r(bits=9) == 2
    assert _r(ln=1.0, un=1.0) == 3 and _r(un=float("inf")) == 3 and _r(la=2.0, ua=1.0) == 3
    assert _r(ln=0.0, un=1e-36) == 3 and _r(ln=-3e38, un=3e38) == 3
    assert _r(C_out=0) == 4
    assert _r(stride=4) == 5
    assert _r(codes=FAKE + 8) == 6 and _r(scale=FAKE + 4) == 6 and _r(shift=FAKE + 12) == 6
    assert _r(nbytes=16 * 32 - 1) == 7            # 16 pixels x 64 padded channels x 4 bits


def test_soft_quantize_rejects_bad_arguments():
    lib = B.load_library()
    fwd = lambda x=FAKE, n=16, l=0.0, u=1.0, a=0.2, b=4, y=FAKE: lib.dsq_soft_quantize_fwd(x, n, l, u, a, b, y, None)
    bwd = lambda x=FAKE, g=FAKE, n=16, l=0.0, u=1.0, a=0.2, b=4, gx=FAKE, s=FAKE: \
        lib.dsq_soft_quantize_bwd(x, g, n, l, u, a, b, gx, s, None)
    assert fwd(x=None) == 1 and fwd(y=None) == 1
    assert fwd(b=0) == 2 and fwd(b=5) == 2
    assert fwd(a=0.0) == 3 and fwd(a=0.5) == 3 and fwd(a=float("nan")) == 3 and fwd(l=1.0, u=0.5) == 3
    assert fwd(n=0) == 4 and fwd(n=1 << 31) == 4
    assert fwd(x=FAKE + 4) == 6
    assert bwd(g=None) == 1 and bwd(s=None) == 1 and bwd(gx=None) == 1
    assert bwd(a=0.7) == 3 and bwd(b=7) == 2 and bwd(n=0) == 4
    assert bwd(s=FAKE + 8) == 6 and bwd(g=FAKE + 4) == 6


def test_dense_3bit_sizes_and_argument_checks():
    lib = B.load_library()
    assert B.dsq_act_packed_bytes_ex(2, 3, 5, 64, 3, B.DSQ_PACK_DENSE3) == 2 * 3 * 5 * 24
    assert B.dsq_act_packed_bytes_ex(1, 1, 1, 65, 3, B.DSQ_PACK_DENSE3) == 48          # channels padded to 128
    assert B.dsq_act_packed_bytes_ex(2, 3, 5, 64, 3, B.DSQ_PACK_CONTAINER) == B.dsq_act_packed_bytes(2, 3, 5, 64, 3)
    for bits in (1, 2, 4, 0, 9):
        assert B.dsq_act_packed_bytes_ex(2, 3, 5, 64, bits, B.DSQ_PACK_DENSE3) == 0
    assert B.dsq_act_packed_bytes_ex(2, 3, 5, 64, 3, 5) == 0
    q = lambda x=FAKE, bits=3, packing=1, C=64, codes=FAKE, nbytes=1 << 20, pix=FAKE, l=0.0, u=1.0: \
        lib.dsq_quantize_act_ex(x, 0, 1, C, 4, 4, l, u, bits, packing, codes, nbytes, pix, None)
    assert q(x=None) == 1 and q(codes=None) == 1 and q(pix=None) == 1
    assert q(bits=7) == 2 and q(bits=4) == 5 and q(packing=3) == 5
    assert q(l=1.0, u=0.0) == 3 and q(C=0) == 4 and q(C=8256) == 5
    assert q(x=FAKE + 4) == 6 and q(nbytes=16 * 24 - 1) == 7
    assert _c(bits=4, flags=B.DSQ_CONV_ACT_DENSE3) == 5 and _c(bits=3, flags=B.DSQ_CONV_NEXT_DENSE3) == 5
    assert _c(bits=3, flags=B.DSQ_CONV_ACT_DENSE3, out=FAKE + 4) == 6            # (valid flag: fails later)
    assert _r(bits=3, flags=B.DSQ_CONV_NEXT_DENSE3, bn=4) == 5
    assert _r(bits=3, flags=B.DSQ_CONV_NEXT_DENSE3, bn=3, nbytes=16 * 24 - 1) == 7


def test_dense_3bit_format_helpers_follow_the_documented_layout():
    """tests/helpers.py unpacks the dense format for the GPU tests; pin it here on a
    hand-made unit: channel 0 = 7, channel 5 = 4, channel 17 = 3, channel 31 = 6."""
    import numpy as np
    from helpers import pack_act_dense3, unpack_act_dense3
    codes = np.zeros((1, 1, 1, 64), np.uint8)          # (a pixel is padded to whole 64-channel blocks)
    codes[0, 0, 0, [0, 5, 17, 31]] = [7, 4, 3, 6]
    words = pack_act_dense3(codes).view(np.uint32)
    # low bits: ch 0 -> word 0 byte 0 bits 0-1 (3); ch 5 = 4 -> low 0; ch 17 -> word 1, k = 1: byte 1 bits 0-1 (3);
    # ch 31 -> word 1, k = 15: byte 3 bits 6-7 (2)
    assert words[0] == 0x00000003 and words[1] == (3 << 8) | (2 << 30)
    # high bits: bit 8j + g with g = ch // 4, j = ch % 4: ch 0 -> bit 0; ch 5 -> bit 9; ch 31 -> bit 31
    assert words[2] == (1 << 0) | (1 << 9) | (1 << 31)
    assert not words[3:].any()
    assert np.array_equal(unpack_act_dense3(words.view(np.uint8), 1, 1, 1, 64), codes)
