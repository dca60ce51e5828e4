"""CPU oracle for the DSQ low-bit convolution layer -- TEST INFRASTRUCTURE ONLY.

A ctypes view of ``dsq_oracle.c``: the hard uniform quantizer (paper Sec. 3.1,
with the tie rule that Algorithm 1 step 3 implies), the dequantization of
Algorithm 1 step 4 and the convolution of step 5, all written out plainly.
Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; the GPU library and its binding never do, and this
package imports nothing of theirs.

Layouts: activations NCHW, weights OIHW, outputs N x C_out x Ho x Wo, one code
per ``uint8``.
"""
import ctypes as C

import numpy as np

from .build import build_oracle

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build_oracle(force=False))
        f32p, u8p = C.POINTER(C.c_float), C.POINTER(C.c_uint8)
        i32p, i64p, f64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_double)
        geom = [C.c_int] * 9
        lib.dsq_oracle_threads.restype = C.c_int
        lib.dsq_oracle_delta.restype = C.c_float
        lib.dsq_oracle_delta.argtypes = [C.c_float, C.c_float, C.c_int]
        lib.dsq_oracle_quantize.argtypes = [f32p, C.c_size_t, C.c_float, C.c_float, C.c_int, u8p]
        lib.dsq_oracle_quantize_weights.argtypes = [f32p, f32p, f32p, C.c_int, C.c_size_t, C.c_int, u8p]
        lib.dsq_oracle_affine_relu.argtypes = [f32p, C.c_int, C.c_int, C.c_size_t, f32p, f32p, C.c_int, f32p]
        lib.dsq_oracle_dequantize.argtypes = [u8p, C.c_size_t, C.c_float, C.c_float, C.c_int, f64p]
        lib.dsq_oracle_conv_codes.argtypes = [u8p, u8p] + geom + [i32p]
        lib.dsq_oracle_conv_dequantized.argtypes = [f64p, f64p] + geom + [f32p]
        lib.dsq_oracle_conv_real.argtypes = [u8p, C.c_float, C.c_float, u8p, f32p, f32p, C.c_int] + geom + [f32p]
        lib.dsq_oracle_conv_at.argtypes = [u8p, C.c_float, C.c_float, u8p, f32p, f32p, C.c_int] + geom + \
            [i64p, C.c_size_t, f32p, i32p]
        _lib = lib
    return _lib


def _ptr(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s failed with status %d" % (what, rc))


def threads():
    """Number of host threads the convolution loops run on."""
    return int(_load().dsq_oracle_threads())


def delta(l, u, bits):
    """Interval length (u-l)/(2^b-1) in binary32 (Sec. 3.1)."""
    return float(_load().dsq_oracle_delta(l, u, bits))


def out_size(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def quantize(x, l, u, bits):
    """Codes of ``x`` (any shape, float32) for the range [l, u]."""
    x = _arr(x, np.float32)
    code = np.empty(x.shape, dtype=np.uint8)
    _check(_load().dsq_oracle_quantize(_ptr(x, C.c_float), x.size, l, u, bits,
                                       _ptr(code, C.c_uint8)), "quantize")
    return code


def quantize_weights(w, lw, uw, bits):
    """Codes of OIHW weights with one (l_w, u_w) pair per output channel."""
    w = _arr(w, np.float32)
    lw, uw = _arr(lw, np.float32), _arr(uw, np.float32)
    assert lw.shape == uw.shape == (w.shape[0],)
    code = np.empty(w.shape, dtype=np.uint8)
    per_ch = w.size // w.shape[0]
    _check(_load().dsq_oracle_quantize_weights(
        _ptr(w, C.c_float), _ptr(lw, C.c_float), _ptr(uw, C.c_float),
        w.shape[0], per_ch, bits, _ptr(code, C.c_uint8)), "quantize_weights")
    return code


def affine_relu(y, scale, shift, relu):
    """scale[c]*y + shift[c] (two binary32 roundings), then max(., 0) if relu;
    y is [N, C, H, W] float32."""
    y = _arr(y, np.float32)
    scale, shift = _arr(scale, np.float32), _arr(shift, np.float32)
    assert y.ndim == 4 and scale.shape == shift.shape == (y.shape[1],)
    z = np.empty(y.shape, dtype=np.float32)
    _check(_load().dsq_oracle_affine_relu(
        _ptr(y, C.c_float), y.shape[0], y.shape[1], y.shape[2] * y.shape[3],
        _ptr(scale, C.c_float), _ptr(shift, C.c_float), int(bool(relu)), _ptr(z, C.c_float)), "affine_relu")
    return z


def requantize(y, scale, shift, relu, l, u, bits):
    """Codes of the next layer's input: the layer output y [N, C, H, W] mapped
    by affine_relu and quantized for the next layer's range [l, u]
    (Algorithm 1 steps 1 and 3 of the next layer)."""
    return quantize(affine_relu(y, scale, shift, relu), l, u, bits)


def dequantize(code, l, u, bits):
    """l + Delta*code as float64 (Algorithm 1 step 4)."""
    code = _arr(code, np.uint8)
    val = np.empty(code.shape, dtype=np.float64)
    _check(_load().dsq_oracle_dequantize(_ptr(code, C.c_uint8), code.size, l, u,
                                         bits, _ptr(val, C.c_double)), "dequantize")
    return val


def _geom(a_shape, w_shape, stride, pad):
    N, Ci, H, W = a_shape
    Co, Ci2, R, S = w_shape
    assert Ci == Ci2, "channel mismatch"
    return (N, Ci, H, W, Co, R, S, stride, pad)


def conv_codes(a_code, w_code, stride, pad):
    """Integer cross-correlation of the codes -> int32 [N, C_out, Ho, Wo]."""
    a, w = _arr(a_code, np.uint8), _arr(w_code, np.uint8)
    g = _geom(a.shape, w.shape, stride, pad)
    Ho, Wo = out_size(g[2], g[3], g[5], g[6], stride, pad)
    acc = np.empty((g[0], g[4], Ho, Wo), dtype=np.int32)
    _check(_load().dsq_oracle_conv_codes(_ptr(a, C.c_uint8), _ptr(w, C.c_uint8),
                                         *g, _ptr(acc, C.c_int32)), "conv_codes")
    return acc


def conv_dequantized(a_hat, w_hat, stride, pad):
    """Step 5 on given float64 tensors -> float32 [N, C_out, Ho, Wo]."""
    a, w = _arr(a_hat, np.float64), _arr(w_hat, np.float64)
    g = _geom(a.shape, w.shape, stride, pad)
    Ho, Wo = out_size(g[2], g[3], g[5], g[6], stride, pad)
    out = np.empty((g[0], g[4], Ho, Wo), dtype=np.float32)
    _check(_load().dsq_oracle_conv_dequantized(_ptr(a, C.c_double), _ptr(w, C.c_double),
                                               *g, _ptr(out, C.c_float)), "conv_dequantized")
    return out


def conv_real(a_code, la, ua, w_code, lw, uw, bits, stride, pad):
    """Steps 4+5 from codes -> float32 [N, C_out, Ho, Wo]."""
    a, w = _arr(a_code, np.uint8), _arr(w_code, np.uint8)
    lw, uw = _arr(lw, np.float32), _arr(uw, np.float32)
    g = _geom(a.shape, w.shape, stride, pad)
    Ho, Wo = out_size(g[2], g[3], g[5], g[6], stride, pad)
    out = np.empty((g[0], g[4], Ho, Wo), dtype=np.float32)
    _check(_load().dsq_oracle_conv_real(
        _ptr(a, C.c_uint8), la, ua, _ptr(w, C.c_uint8), _ptr(lw, C.c_float),
        _ptr(uw, C.c_float), bits, *g, _ptr(out, C.c_float)), "conv_real")
    return out


def conv_weight_only(x, w_code, lw, uw, bits, stride, pad):
    """A layer whose weights are quantized and whose activations are not (the
    "b/32" rows of the paper's Tables 3, 6 and 7): Algorithm 1 with the
    activation quantizer left out.  Step 4 for the weights (levels in float64),
    step 5 with the float32 activations taken as they are (as float64), summed
    in float64 and rounded once -> float32 [N, C_out, Ho, Wo].  Also returns the
    same convolution of the absolute values (the scale a binary32 accumulation
    error is measured against), in float64 precision rounded to float32."""
    x = _arr(x, np.float32)
    w = _arr(w_code, np.uint8)
    lw, uw = _arr(lw, np.float32), _arr(uw, np.float32)
    w_hat = np.stack([dequantize(w[o], float(lw[o]), float(uw[o]), bits) for o in range(w.shape[0])])
    x64 = x.astype(np.float64)
    return conv_dequantized(x64, w_hat, stride, pad), conv_dequantized(np.abs(x64), np.abs(w_hat), stride, pad)


def conv_at(a_code, la, ua, w_code, lw, uw, bits, stride, pad, flat_idx):
    """Sampled outputs: (float32 values, int32 accumulators) at flat indices
    into the N x C_out x Ho x Wo output."""
    a, w = _arr(a_code, np.uint8), _arr(w_code, np.uint8)
    lw, uw = _arr(lw, np.float32), _arr(uw, np.float32)
    idx = _arr(flat_idx, np.int64)
    g = _geom(a.shape, w.shape, stride, pad)
    vals = np.empty(idx.shape, dtype=np.float32)
    accs = np.empty(idx.shape, dtype=np.int32)
    _check(_load().dsq_oracle_conv_at(
        _ptr(a, C.c_uint8), la, ua, _ptr(w, C.c_uint8), _ptr(lw, C.c_float),
        _ptr(uw, C.c_float), bits, *g, _ptr(idx, C.c_int64), idx.size,
        _ptr(vals, C.c_float), _ptr(accs, C.c_int32)), "conv_at")
    return vals, accs
