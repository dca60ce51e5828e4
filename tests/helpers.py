"""Host-side helpers for the GPU parity tests: unpacking of the documented
packed formats with numpy, running one layer through the C ABI, and the
tolerance of the float output."""
import numpy as np
import torch

import oracle
from paper_1908_05033_amd import binding as B


def container(bits):
    return 2 if bits <= 2 else 4


def round_up(x, m):
    return (x + m - 1) // m * m


def unpack_words(words_u32, bits):
    """[..., nwords] uint32 -> [..., nwords * channels_per_word] uint8 codes in
    channel order (format: byte j of a word = c[j] | c[j+4]<<cont | ...)."""
    cont = container(bits)
    cpd = 32 // cont
    mask = (1 << cont) - 1
    w = words_u32.astype(np.uint32)
    out = np.empty(w.shape + (cpd,), dtype=np.uint8)
    for j in range(cpd):
        shift = 8 * (j & 3) + cont * (j >> 2)
        out[..., j] = (w >> np.uint32(shift)) & np.uint32(mask)
    return out.reshape(w.shape[:-1] + (w.shape[-1] * cpd,))


def unpack_act(packed_u8, N, H, W, C, bits):
    """Packed activation bytes -> codes [N, H, W, Cp]."""
    Cp = round_up(C, 64)
    words = packed_u8.view(np.uint32).reshape(N, H, W, Cp * container(bits) // 32)
    return unpack_words(words, bits)


def unpack_act_dense3(packed_u8, N, H, W, C):
    """Dense 3-bit activation bytes -> codes [N, H, W, Cp] (format: 12-byte units of
    32 channels; words 0 / 1 = low two bits of channels 0..15 / 16..31 as in the
    2-bit container format, word 2 bit 8j+g = bit 2 of channel 4g+j)."""
    Cp = round_up(C, 64)
    w = packed_u8.view(np.uint32).reshape(N, H, W, Cp // 32, 3)
    out = np.empty((N, H, W, Cp // 32, 32), dtype=np.uint8)
    for c in range(32):
        low_word = w[..., c // 16]
        k = c % 16
        low = (low_word >> np.uint32(8 * (k & 3) + 2 * (k >> 2))) & np.uint32(3)
        g, j = c // 4, c % 4
        high = (w[..., 2] >> np.uint32(8 * j + g)) & np.uint32(1)
        out[..., c] = (low | (high << np.uint32(2))).astype(np.uint8)
    return out.reshape(N, H, W, Cp)


def pack_act_dense3(codes_nhwc):
    """Codes [N, H, W, Cp] (Cp a multiple of 32, values < 8) -> dense 3-bit bytes, by the
    definition of the format (the inverse of unpack_act_dense3)."""
    N, H, W, Cp = codes_nhwc.shape
    c = codes_nhwc.reshape(N, H, W, Cp // 32, 32).astype(np.uint32)
    w = np.zeros((N, H, W, Cp // 32, 3), dtype=np.uint32)
    for ch in range(32):
        k = ch % 16
        w[..., ch // 16] |= (c[..., ch] & 3) << np.uint32(8 * (k & 3) + 2 * (k >> 2))
        g, j = ch // 4, ch % 4
        w[..., 2] |= ((c[..., ch] >> 2) & 1) << np.uint32(8 * j + g)
    return w.reshape(-1).view(np.uint8)


def unpack_weights(packed_u8, C_out, C_in, R, bits):
    """Packed weight bytes -> codes [Cop, Cp, R, R] (OIHW order, padded)."""
    Cp, Cop = round_up(C_in, 64), round_up(C_out, 256)
    T = R * R
    if bits <= 2:
        # one code per 4-bit field; [ct][cb][tap][lane = 32h + row][word d], word d
        # nibble n = channel 64cb + 32h + 16(d/2) + 4(d%2) + 8(n%2) + n/2
        words = packed_u8.view(np.uint32).reshape(Cop // 32, Cp // 64, T, 2, 32, 4)
        codes = np.empty((Cop // 32, 32, Cp // 64, 64, T), dtype=np.uint8)
        for d in range(4):
            for n in range(8):
                nib = ((words[..., d] >> np.uint32(4 * n)) & np.uint32(15)).astype(np.uint8)   # [ct, cb, tap, h, row]
                for h in range(2):
                    ch = 32 * h + 16 * (d // 2) + 4 * (d % 2) + 8 * (n % 2) + n // 2
                    codes[:, :, :, ch, :] = nib[:, :, :, h, :].transpose(0, 3, 1, 2)
        return codes.reshape(Cop, Cp, R, R)
    wpl = 2
    words = packed_u8.view(np.uint32).reshape(Cop // 32, Cp // 64, T, 64, 2, wpl)
    codes = unpack_words(words, bits)                 # [ct, cb, tap, lane, kh, 16]
    codes = codes.reshape(Cop // 32, Cp // 64, T, 2, 32, 2, 16)   # lane = 32*h + row
    # axes: ct, cb, tap, h, row, kh, k16 -> channel = 64*cb + 32*kh + 16*h + k16
    codes = codes.transpose(0, 4, 1, 5, 3, 6, 2).reshape(Cop, Cp, R, R)
    return codes


def split_aux(aux_u8, C_out, R):
    Cop = round_up(C_out, 256)
    T = R * R
    f = aux_u8.view(np.float32)
    i = aux_u8.view(np.int32)
    return {"delta_w": f[:Cop], "l_w": f[Cop:2 * Cop], "sw_total": i[2 * Cop:3 * Cop],
            "sw_tap": i[3 * Cop:3 * Cop + Cop * T].reshape(Cop, T)}


def run_layer_gpu(layer, inp, x_layout=B.DSQ_NHWC, out_layout=B.DSQ_NHWC, w_codes=None,
                  kernel=0, with_acc=True, many_in_flight=False):
    """quantize + pack + conv through the C ABI.  Returns a dict of host arrays
    (out / acc always as [N, C_out, Ho, Wo])."""
    L = layer
    buf = B.alloc_layer(L.N, L.C_in, L.H, L.W, L.C_out, L.R, L.S, L.stride, L.pad, L.bits,
                        with_acc=with_acc)
    x = inp["x"]
    if x_layout == B.DSQ_NHWC:
        xd = x.permute(0, 2, 3, 1).contiguous().cuda()
    else:
        xd = x.contiguous().cuda()
    B.dsq_quantize_act(xd, x_layout, L.N, L.C_in, L.H, L.W, inp["l_a"], inp["u_a"], L.bits,
                       buf.act_packed, buf.pix_code_sum)
    lw = torch.from_numpy(np.ascontiguousarray(inp["l_w"])).cuda()
    uw = torch.from_numpy(np.ascontiguousarray(inp["u_w"])).cuda()
    wd = inp["w"].contiguous().cuda() if w_codes is None else None
    wc = torch.from_numpy(np.ascontiguousarray(w_codes)).cuda() if w_codes is not None else None
    B.dsq_pack_weights(wd, lw, uw, wc, L.C_out, L.C_in, L.R, L.S, L.bits, buf.w_packed, buf.w_aux)
    if out_layout == B.DSQ_NCHW:
        buf.out = torch.empty((L.N, L.C_out, L.Ho, L.Wo), dtype=torch.float32, device="cuda")
        if with_acc:
            buf.acc = torch.empty((L.N, L.C_out, L.Ho, L.Wo), dtype=torch.int32, device="cuda")
    buf.out.fill_(float("nan"))
    buf.desc.flags = B.DSQ_CONV_KERNEL(kernel) | (B.DSQ_CONV_MANY_IN_FLIGHT if many_in_flight else 0)
    B.dsq_conv2d(buf.desc, buf.act_packed, buf.pix_code_sum, inp["l_a"], inp["u_a"],
                 buf.w_packed, buf.w_aux, buf.out, out_layout, buf.acc)
    torch.cuda.synchronize()
    out = buf.out.cpu().numpy()
    acc = buf.acc.cpu().numpy() if with_acc else None
    if out_layout == B.DSQ_NHWC:
        out = out.transpose(0, 3, 1, 2)
        acc = acc.transpose(0, 3, 1, 2) if with_acc else None
    return {"out": out, "acc": acc,
            "act_packed": buf.act_packed.cpu().numpy(), "pix_sum": buf.pix_code_sum.cpu().numpy(),
            "w_packed": buf.w_packed.cpu().numpy(), "w_aux": buf.w_aux.cpu().numpy(), "buf": buf}


def oracle_layer(layer, inp, w_codes=None):
    """Codes, accumulators and float output of the oracle for the same inputs."""
    L = layer
    a_code = oracle.quantize(inp["x"].numpy(), inp["l_a"], inp["u_a"], L.bits)
    w_code = w_codes if w_codes is not None else \
        oracle.quantize_weights(inp["w"].numpy(), inp["l_w"], inp["u_w"], L.bits)
    return a_code, w_code


def assert_out_close(gpu, ref, delta_a, delta_w, rel=1e-5):
    """|gpu-ref| <= rel*|ref| + rel*Da*Dw[o] per element, and
    max|gpu-ref| <= rel*max|ref| per tensor.  gpu/ref are [N, C_out, Ho, Wo]."""
    g = gpu.astype(np.float64)
    r = ref.astype(np.float64)
    floor = rel * float(delta_a) * np.asarray(delta_w, np.float64).reshape(1, -1, 1, 1)
    err = np.abs(g - r)
    bad = err > rel * np.abs(r) + floor
    assert not bad.any(), "%d elements off, worst %.3e (ref %.3e)" % (
        bad.sum(), err.max(), np.abs(r).max())
    assert err.max() <= rel * np.abs(r).max()


def pack_codes_reference(oc, bits):
    """Codes [P, 64] (uint8 torch tensor) -> the packed bytes the header
    documents: 4-bit containers, byte j of word w = c[8w+j] | c[8w+4+j] << 4;
    2-bit containers, byte j = c[16w+j] | c[16w+4+j] << 2 | c[16w+8+j] << 4 | c[16w+12+j] << 6."""
    P = oc.shape[0]
    if container(bits) == 4:
        g = oc.reshape(P, 8, 2, 4)
        return (g[:, :, 0, :] | (g[:, :, 1, :] << 4)).reshape(P, 32)
    g = oc.reshape(P, 4, 4, 4)
    return (g[:, :, 0, :] | (g[:, :, 1, :] << 2) | (g[:, :, 2, :] << 4) | (g[:, :, 3, :] << 6)).reshape(P, 16)
