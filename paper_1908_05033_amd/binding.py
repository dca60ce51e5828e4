"""ctypes binding of libdsqconv: the same names as ``include/dsqconv.h``.

Argument marshalling only.  PyTorch supplies device memory (``data_ptr()``)
and the HIP stream handle (``torch.cuda.current_stream().cuda_stream`` is
PyTorch-ROCm's name for the hipStream_t); every step of the path runs in the
library's HIP kernels.  There is no CPU fallback: if the shared library has
not been built, the first call raises.
"""
import ctypes as C
import os
from dataclasses import dataclass

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdsqconv.so")

DSQ_NHWC, DSQ_NCHW = 0, 1
DSQ_OK = 0
DSQ_CONV_MANY_IN_FLIGHT = 0x10
DSQ_CONV_ACT_DENSE3 = 0x20
DSQ_CONV_NEXT_DENSE3 = 0x40
DSQ_CONV_NEXT_SUMS_ZERO = 0x80
DSQ_PACK_CONTAINER, DSQ_PACK_DENSE3 = 0, 1


def DSQ_CONV_KERNEL(k):
    return k & 15

EXPORTS = [
    "dsq_act_packed_bytes", "dsq_act_packed_bytes_ex", "dsq_wgt_packed_bytes", "dsq_wgt_aux_bytes",
    "dsq_quantize_act", "dsq_quantize_act_ex", "dsq_pack_weights", "dsq_pack_weights_for", "dsq_conv2d", "dsq_conv2d_requant", "dsq_conv2d_wq",
    "dsq_soft_quantize_fwd", "dsq_soft_quantize_bwd",
    "dsq_conv2d_plan", "dsq_status_string",
]


class DsqError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("libdsqconv: %s (status %d)" % (message, status))
        self.status = status


class dsq_conv_desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("N", "C_in", "H", "W", "C_out", "R", "S", "stride", "pad", "bits", "flags")]


_lib = None


def load_library():
    """Load libdsqconv.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libdsqconv.so is missing at %s: build it first "
            "(python -c 'import __graft_entry__ as g; g.build()'). "
            "There is no fallback path." % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, sz, i, f = C.c_void_p, C.c_size_t, C.c_int, C.c_float
    lib.dsq_act_packed_bytes.restype = sz
    lib.dsq_act_packed_bytes.argtypes = [i] * 5
    lib.dsq_act_packed_bytes_ex.restype = sz
    lib.dsq_act_packed_bytes_ex.argtypes = [i] * 6
    lib.dsq_quantize_act_ex.restype = i
    lib.dsq_quantize_act_ex.argtypes = [vp, i, i, i, i, i, f, f, i, i, vp, sz, vp, vp]
    lib.dsq_wgt_packed_bytes.restype = sz
    lib.dsq_wgt_packed_bytes.argtypes = [i] * 5
    lib.dsq_wgt_aux_bytes.restype = sz
    lib.dsq_wgt_aux_bytes.argtypes = [i] * 3
    lib.dsq_quantize_act.restype = i
    lib.dsq_quantize_act.argtypes = [vp, i, i, i, i, i, f, f, i, vp, sz, vp, vp]
    lib.dsq_pack_weights.restype = i
    lib.dsq_pack_weights.argtypes = [vp, vp, vp, vp, i, i, i, i, i, vp, sz, vp, sz, vp]
    lib.dsq_pack_weights_for.restype = i
    lib.dsq_pack_weights_for.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, vp, sz, vp, sz, vp]
    lib.dsq_conv2d.restype = i
    lib.dsq_conv2d.argtypes = [C.POINTER(dsq_conv_desc), vp, vp, f, f, vp, vp, vp, i, vp, vp]
    lib.dsq_conv2d_requant.restype = i
    lib.dsq_conv2d_requant.argtypes = [C.POINTER(dsq_conv_desc), vp, vp, f, f, vp, vp, vp, vp, i, f, f, i,
                                       vp, sz, vp, vp]
    lib.dsq_conv2d_wq.restype = i
    lib.dsq_conv2d_wq.argtypes = [C.POINTER(dsq_conv_desc), vp, i, vp, vp, vp, i, vp]
    lib.dsq_soft_quantize_fwd.restype = i
    lib.dsq_soft_quantize_fwd.argtypes = [vp, sz, f, f, f, i, vp, vp]
    lib.dsq_soft_quantize_bwd.restype = i
    lib.dsq_soft_quantize_bwd.argtypes = [vp, vp, sz, f, f, f, i, vp, vp, vp]
    lib.dsq_conv2d_plan.restype = i
    lib.dsq_conv2d_plan.argtypes = [C.POINTER(dsq_conv_desc), i, f, C.c_char_p, sz]
    lib.dsq_status_string.restype = C.c_char_p
    lib.dsq_status_string.argtypes = [i]
    _lib = lib
    return lib


def _check(status):
    if status != DSQ_OK:
        raise DsqError(status, load_library().dsq_status_string(status).decode())


def _dev_ptr(t, dtype=None, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise DsqError(1, "a required tensor is None")
    if isinstance(t, int):          # raw device address
        return t
    if not t.is_cuda:
        raise TypeError("libdsqconv takes device tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, t.dtype))
    if not t.is_contiguous():
        raise TypeError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def dsq_act_packed_bytes(N, H, W, C, bits):
    return int(load_library().dsq_act_packed_bytes(N, H, W, C, bits))


def dsq_act_packed_bytes_ex(N, H, W, C, bits, packing):
    return int(load_library().dsq_act_packed_bytes_ex(N, H, W, C, bits, packing))


def dsq_wgt_packed_bytes(C_out, C_in, R, S, bits):
    return int(load_library().dsq_wgt_packed_bytes(C_out, C_in, R, S, bits))


def dsq_wgt_aux_bytes(C_out, R, S):
    return int(load_library().dsq_wgt_aux_bytes(C_out, R, S))


def dsq_quantize_act(x, layout, N, C, H, W, l, u, bits, codes_packed, pix_code_sum, stream=None):
    _check(load_library().dsq_quantize_act(
        _dev_ptr(x, torch.float32), layout, N, C, H, W, l, u, bits,
        _dev_ptr(codes_packed, torch.uint8), codes_packed.numel() if codes_packed is not None else 0,
        _dev_ptr(pix_code_sum, torch.int32), _stream(stream)))


def dsq_quantize_act_ex(x, layout, N, C, H, W, l, u, bits, packing, codes_packed, pix_code_sum, stream=None):
    _check(load_library().dsq_quantize_act_ex(
        _dev_ptr(x, torch.float32), layout, N, C, H, W, l, u, bits, packing,
        _dev_ptr(codes_packed, torch.uint8), codes_packed.numel() if codes_packed is not None else 0,
        _dev_ptr(pix_code_sum, torch.int32), _stream(stream)))


def dsq_pack_weights(w_oihw, l_w, u_w, codes_oihw, C_out, C_in, R, S, bits, w_packed, w_aux,
                     stream=None):
    _check(load_library().dsq_pack_weights(
        _dev_ptr(w_oihw, torch.float32, True), _dev_ptr(l_w, torch.float32),
        _dev_ptr(u_w, torch.float32), _dev_ptr(codes_oihw, torch.uint8, True),
        C_out, C_in, R, S, bits,
        _dev_ptr(w_packed, torch.uint8), w_packed.numel() if w_packed is not None else 0,
        _dev_ptr(w_aux, torch.uint8), w_aux.numel() if w_aux is not None else 0,
        _stream(stream)))


def dsq_pack_weights_for(w_oihw, l_w, u_w, codes_oihw, C_out, C_in, R, S, bits_w, bits_act, w_packed, w_aux,
                         stream=None):
    _check(load_library().dsq_pack_weights_for(
        _dev_ptr(w_oihw, torch.float32, True), _dev_ptr(l_w, torch.float32),
        _dev_ptr(u_w, torch.float32), _dev_ptr(codes_oihw, torch.uint8, True),
        C_out, C_in, R, S, bits_w, bits_act,
        _dev_ptr(w_packed, torch.uint8), w_packed.numel() if w_packed is not None else 0,
        _dev_ptr(w_aux, torch.uint8), w_aux.numel() if w_aux is not None else 0,
        _stream(stream)))


def dsq_conv2d(desc, act_packed, pix_code_sum, l_a, u_a, w_packed, w_aux, out, out_layout,
               acc_or_none=None, stream=None):
    _check(load_library().dsq_conv2d(
        C.byref(desc) if desc is not None else None,
        _dev_ptr(act_packed, torch.uint8), _dev_ptr(pix_code_sum, torch.int32), l_a, u_a,
        _dev_ptr(w_packed, torch.uint8), _dev_ptr(w_aux, torch.uint8),
        _dev_ptr(out, torch.float32), out_layout,
        _dev_ptr(acc_or_none, torch.int32, True), _stream(stream)))


def dsq_conv2d_requant(desc, act_packed, pix_code_sum, l_a, u_a, w_packed, w_aux, scale, shift, relu,
                       l_next, u_next, bits_next, codes_next, pix_code_sum_next, stream=None):
    _check(load_library().dsq_conv2d_requant(
        C.byref(desc) if desc is not None else None,
        _dev_ptr(act_packed, torch.uint8), _dev_ptr(pix_code_sum, torch.int32), l_a, u_a,
        _dev_ptr(w_packed, torch.uint8), _dev_ptr(w_aux, torch.uint8),
        _dev_ptr(scale, torch.float32, True), _dev_ptr(shift, torch.float32, True), int(bool(relu)),
        l_next, u_next, bits_next,
        _dev_ptr(codes_next, torch.uint8), codes_next.numel() if codes_next is not None else 0,
        _dev_ptr(pix_code_sum_next, torch.int32), _stream(stream)))


def dsq_conv2d_wq(desc, x, x_layout, w_packed, w_aux, out, out_layout, stream=None):
    _check(load_library().dsq_conv2d_wq(
        C.byref(desc) if desc is not None else None, _dev_ptr(x, torch.float32), x_layout,
        _dev_ptr(w_packed, torch.uint8), _dev_ptr(w_aux, torch.uint8), _dev_ptr(out, torch.float32), out_layout,
        _stream(stream)))


def dsq_soft_quantize_fwd(x, l, u, alpha, bits, y, stream=None):
    _check(load_library().dsq_soft_quantize_fwd(_dev_ptr(x, torch.float32), x.numel(), l, u, alpha, bits,
                                                _dev_ptr(y, torch.float32), _stream(stream)))


def dsq_soft_quantize_bwd(x, grad_y, l, u, alpha, bits, grad_x, grad_alpha_l_u, stream=None):
    _check(load_library().dsq_soft_quantize_bwd(
        _dev_ptr(x, torch.float32), _dev_ptr(grad_y, torch.float32), x.numel(), l, u, alpha, bits,
        _dev_ptr(grad_x, torch.float32), _dev_ptr(grad_alpha_l_u, torch.float64), _stream(stream)))


def dsq_conv2d_plan(desc, chained=False, l_a=0.0):
    buf = C.create_string_buffer(512)
    _check(load_library().dsq_conv2d_plan(C.byref(desc), int(bool(chained)), l_a, buf, len(buf)))
    return buf.value.decode()


# ---------------------------------------------------------------------------
# Small conveniences: buffer allocation for one layer (still no arithmetic).
# ---------------------------------------------------------------------------

@dataclass
class LayerBuffers:
    desc: dsq_conv_desc
    act_packed: torch.Tensor
    pix_code_sum: torch.Tensor
    w_packed: torch.Tensor
    w_aux: torch.Tensor
    out: torch.Tensor          # NHWC float32 [N, Ho, Wo, C_out]
    acc: torch.Tensor = None   # NHWC int32, optional


def make_desc(N, C_in, H, W, C_out, R, S, stride, pad, bits, flags=0):
    return dsq_conv_desc(N, C_in, H, W, C_out, R, S, stride, pad, bits, flags)


def alloc_layer(N, C_in, H, W, C_out, R, S, stride, pad, bits, device="cuda", with_acc=False, flags=0):
    """Device buffers for one layer, sized by the library's own size queries."""
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - S) // stride + 1
    u8 = dict(dtype=torch.uint8, device=device)
    return LayerBuffers(
        desc=make_desc(N, C_in, H, W, C_out, R, S, stride, pad, bits, flags),
        act_packed=torch.empty(dsq_act_packed_bytes(N, H, W, C_in, bits), **u8),
        pix_code_sum=torch.empty(N * H * W, dtype=torch.int32, device=device),
        w_packed=torch.empty(dsq_wgt_packed_bytes(C_out, C_in, R, S, bits), **u8),
        w_aux=torch.empty(dsq_wgt_aux_bytes(C_out, R, S), **u8),
        out=torch.empty((N, Ho, Wo, C_out), dtype=torch.float32, device=device),
        acc=torch.empty((N, Ho, Wo, C_out), dtype=torch.int32, device=device) if with_acc else None,
    )
