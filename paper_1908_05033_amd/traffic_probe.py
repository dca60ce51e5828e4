"""Workload for HBM-traffic counters (run under ``rocprofv3 --pmc FETCH_SIZE``
or ``--pmc WRITE_SIZE``):

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d out -- \\
        python3 -m paper_1908_05033_amd.traffic_probe --cfg 2

It launches (1) a plain device-to-device copy of a known size, which calibrates
the counter (bytes the counter reports per byte really moved), and (2) the
quantize and convolution kernels of one layer of a config (with --chained also
dsq_conv2d_requant), each over several distinct buffer sets so that the
last-level cache cannot serve them.
"""
import argparse

import torch

from . import binding as B
from . import inputs

COPY_BYTES = 256 * 1024 * 1024


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cfg", type=int, default=2)
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--bits", type=int, default=None)
    ap.add_argument("--sets", type=int, default=0, help="buffer sets (0 = enough to exceed 600 MB, at most 48)")
    ap.add_argument("--many-in-flight", action="store_true", help="pass DSQ_CONV_MANY_IN_FLIGHT")
    ap.add_argument("--chained", action="store_true", help="also launch dsq_conv2d_requant (same layer, codes out)")
    a = ap.parse_args()
    flags = B.DSQ_CONV_MANY_IN_FLIGHT if a.many_in_flight else 0
    L = inputs.config_layers(a.cfg, a.bits)[a.layer]
    per_set = (L.N * L.H * L.W * L.C_in * 4 + L.N * L.Ho * L.Wo * L.C_out * 4 +
               B.dsq_act_packed_bytes(L.N, L.H, L.W, L.C_in, L.bits) + L.N * L.H * L.W * 4)
    a.sets = a.sets or int(min(48, max(2, -(-600e6 // per_set))))
    dev = "cuda"
    gen = torch.Generator(device=dev).manual_seed(inputs.BASE_SEED)

    src = torch.empty(COPY_BYTES // 4, dtype=torch.float32, device=dev).normal_(generator=gen)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)            # calibration: reads and writes COPY_BYTES
    torch.cuda.synchronize()

    w = torch.randn((L.C_out, L.C_in, L.R, L.S), device=dev, generator=gen) * 0.05
    uw = w.reshape(L.C_out, -1).abs().amax(dim=1).contiguous()
    lw = (-uw).contiguous()
    bufs = []
    for _ in range(a.sets):
        b = B.alloc_layer(L.N, L.C_in, L.H, L.W, L.C_out, L.R, L.S, L.stride, L.pad, L.bits, flags=flags)
        b.x = torch.randn((L.N, L.H, L.W, L.C_in), device=dev, generator=gen).abs_()
        bufs.append(b)
    wp, aux = bufs[0].w_packed, bufs[0].w_aux
    B.dsq_pack_weights(w, lw, uw, None, L.C_out, L.C_in, L.R, L.S, L.bits, wp, aux)
    torch.cuda.synchronize()
    for b in bufs:
        B.dsq_quantize_act(b.x, B.DSQ_NHWC, L.N, L.C_in, L.H, L.W, 0.0, 2.5, L.bits,
                           b.act_packed, b.pix_code_sum)
    torch.cuda.synchronize()
    for b in bufs:
        B.dsq_conv2d(b.desc, b.act_packed, b.pix_code_sum, 0.0, 2.5, wp, aux, b.out, B.DSQ_NHWC, None)
    torch.cuda.synchronize()
    if a.chained:
        scale = torch.rand(L.C_out, device=dev, generator=gen) + 0.5
        shift = torch.randn(L.C_out, device=dev, generator=gen) * 0.1
        nxt = [(torch.empty(B.dsq_act_packed_bytes(L.N, L.Ho, L.Wo, L.C_out, L.bits), dtype=torch.uint8, device=dev),
                torch.empty(L.N * L.Ho * L.Wo, dtype=torch.int32, device=dev)) for _ in bufs]
        for b, (codes, pix) in zip(bufs, nxt):
            B.dsq_conv2d_requant(b.desc, b.act_packed, b.pix_code_sum, 0.0, 2.5, wp, aux, scale, shift, True, 0.0, 1.0,
                                 L.bits, codes, pix)
        torch.cuda.synchronize()
    print("copy_bytes", COPY_BYTES, "layer", L.name, "sets", a.sets)


if __name__ == "__main__":
    main()
