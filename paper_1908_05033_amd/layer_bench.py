"""Per-layer timing of dsq_quantize_act and dsq_conv2d on one GPU.

    python -m paper_1908_05033_amd.layer_bench --cfg 3 [--bits 4] [--kernel 0] [--chained]
    python -m paper_1908_05033_amd.layer_bench --fc [--kernel 2]      (fully connected layers)

For every layer of a config (shapes from :mod:`paper_1908_05033_amd.inputs`)
it prints one JSON line: kernel time, effective int-TOPS (2*MACs/s, padding taps
included), fraction of the matrix peak of the instruction the layer runs on
(int8: 5000 TOP/s; 2-bit layers use the FP4 form: 10100), algorithmic bytes (packed codes in,
packed weights, pixel sums, fp32 out) and the GB/s they amount to.  Inputs are
random tensors drawn on the GPU (timing does not depend on the values); launches
are captured in a hipGraph that rotates over enough buffer sets to exceed the
256 MB last-level cache, and timed with events on the launch stream.

With --chained it also times dsq_conv2d_requant (the layer's output written as
the next layer's packed codes) and, for comparison, the two calls it replaces:
dsq_conv2d to fp32 followed by dsq_quantize_act of that tensor.
"""
import argparse
import json

import torch

from . import binding as B
from . import inputs

INT8_PEAK_TOPS = 5000.0      # dense int8 matrix peak (3- and 4-bit layers)
FP4_PEAK_TOPS = 10100.0      # dense FP4 matrix peak (2-bit layers run on the FP4 instruction)
HBM_PEAK_GBS = 8000.0


def _time_graph(fn, bufs, stream, reps):
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        for b in bufs:
            fn(b)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        g.replay()
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(reps):
            g.replay()
        e1.record(stream)
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / (reps * len(bufs))


def bench_layer(L, kernel=0, min_bytes=600e6, max_sets=16, reps=5, chained=False):
    dev = "cuda"
    gen = torch.Generator(device=dev).manual_seed(inputs.BASE_SEED)
    in_bytes = L.N * L.H * L.W * L.C_in * 4
    out_bytes = L.N * L.Ho * L.Wo * L.C_out * 4
    code_bytes = B.dsq_act_packed_bytes(L.N, L.H, L.W, L.C_in, L.bits)
    pix_bytes = L.N * L.H * L.W * 4
    w_bytes = B.dsq_wgt_packed_bytes(L.C_out, L.C_in, L.R, L.S, L.bits)
    per_set = in_bytes + out_bytes + code_bytes + pix_bytes
    sets = int(min(max_sets, max(2, -(-min_bytes // per_set))))

    w = torch.randn((L.C_out, L.C_in, L.R, L.S), device=dev, generator=gen) * 0.05
    uw = w.reshape(L.C_out, -1).abs().amax(dim=1).contiguous()
    lw = (-uw).contiguous()
    bufs = []
    for _ in range(sets):
        b = B.alloc_layer(L.N, L.C_in, L.H, L.W, L.C_out, L.R, L.S, L.stride, L.pad, L.bits)
        b.x = torch.randn((L.N, L.H, L.W, L.C_in), device=dev, generator=gen).abs_()
        bufs.append(b)
    wp, aux = bufs[0].w_packed, bufs[0].w_aux
    B.dsq_pack_weights(w, lw, uw, None, L.C_out, L.C_in, L.R, L.S, L.bits, wp, aux)
    l_a, u_a = 0.0, 2.5

    def quant(b):
        B.dsq_quantize_act(b.x, B.DSQ_NHWC, L.N, L.C_in, L.H, L.W, l_a, u_a, L.bits,
                           b.act_packed, b.pix_code_sum)

    def conv(b):
        B.dsq_conv2d(b.desc, b.act_packed, b.pix_code_sum, l_a, u_a, wp, aux, b.out, B.DSQ_NHWC, None)

    if chained:
        scale = torch.rand(L.C_out, device=dev, generator=gen) + 0.5
        shift = torch.randn(L.C_out, device=dev, generator=gen) * 0.1
        l_n, u_n = 0.0, 1.0
        next_bytes = B.dsq_act_packed_bytes(L.N, L.Ho, L.Wo, L.C_out, L.bits)
        for b in bufs:
            b.codes_next = torch.empty(next_bytes, dtype=torch.uint8, device=dev)
            b.pix_next = torch.empty(L.N * L.Ho * L.Wo, dtype=torch.int32, device=dev)

    def conv_chained(b):
        B.dsq_conv2d_requant(b.desc, b.act_packed, b.pix_code_sum, l_a, u_a, wp, aux, scale, shift, True,
                             l_n, u_n, L.bits, b.codes_next, b.pix_next)

    def quant_next(b):      # what the chained call saves: quantizing the fp32 output for the next layer
        B.dsq_quantize_act(b.out, B.DSQ_NHWC, L.N, L.C_out, L.Ho, L.Wo, l_n, u_n, L.bits,
                           b.codes_next, b.pix_next)

    prev = B.dsq_set_conv_kernel(kernel)
    try:
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            for b in bufs:
                quant(b)
                conv(b)
                if chained:
                    conv_chained(b)
            torch.cuda.synchronize()
        tq = _time_graph(quant, bufs, stream, reps)
        tc = _time_graph(conv, bufs, stream, reps)
        if chained:
            tcc = _time_graph(conv_chained, bufs, stream, reps)
            tqn = _time_graph(quant_next, bufs, stream, reps)
    finally:
        B.dsq_set_conv_kernel(prev)
    # algorithmic conv bytes: packed weights are counted at the packed code width
    cont = 2 if L.bits <= 2 else 4
    w_alg = L.C_out * L.C_in * L.R * L.S * cont // 8
    conv_bytes = code_bytes + pix_bytes + w_alg + out_bytes
    quant_bytes = in_bytes + code_bytes + pix_bytes
    tops = 2.0 * L.macs / tc / 1e12
    extra = {}
    if chained:
        ch_bytes = code_bytes + pix_bytes + w_alg + next_bytes + L.N * L.Ho * L.Wo * 4
        extra = {
            "chained_us": round(tcc * 1e6, 2), "chained_TOPS": round(2.0 * L.macs / tcc / 1e12, 1),
            "chained_alg_MB": round(ch_bytes / 1e6, 2), "chained_GBps": round(ch_bytes / tcc / 1e9, 1),
            "unchained_us": round((tc + tqn) * 1e6, 2), "quant_next_us": round(tqn * 1e6, 2),
            "chained_speedup": round((tc + tqn) / tcc, 2),
        }
    return {**extra, **{
        "layer": L.name, "bits": L.bits, "count": L.count,
        "gemm_MxNxK": [L.N * L.Ho * L.Wo, L.C_out, L.C_in * L.R * L.S],
        "conv_us": round(tc * 1e6, 2), "conv_TOPS": round(tops, 1),
        "conv_frac_int8_peak": round(tops / INT8_PEAK_TOPS, 4),
        "matrix_peak_TOPS": FP4_PEAK_TOPS if L.bits <= 2 else INT8_PEAK_TOPS,
        "conv_frac_matrix_peak": round(tops / (FP4_PEAK_TOPS if L.bits <= 2 else INT8_PEAK_TOPS), 4),
        "conv_alg_MB": round(conv_bytes / 1e6, 2), "conv_GBps": round(conv_bytes / tc / 1e9, 1),
        "conv_frac_hbm_peak": round(conv_bytes / tc / 1e9 / HBM_PEAK_GBS, 4),
        "quant_us": round(tq * 1e6, 2), "quant_GBps": round(quant_bytes / tq / 1e9, 1),
        "quant_frac_hbm_peak": round(quant_bytes / tq / 1e9 / HBM_PEAK_GBS, 4),
        "buffer_sets": sets, "w_buffer_bytes": w_bytes,
    }}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cfg", type=int, default=None)
    ap.add_argument("--fc", action="store_true",
                    help="fully connected layers (1x1 layers on 1x1 images) instead of a benchmark config")
    ap.add_argument("--bits", type=int, default=None)
    ap.add_argument("--kernel", type=int, default=0)
    ap.add_argument("--layer", type=int, default=None)
    ap.add_argument("--chained", action="store_true")
    ap.add_argument("--policy", type=int, default=0,
                    help="dsq_set_conv_policy value (0 = shortest single call: kernels are timed one at a time here)")
    a = ap.parse_args()
    B.dsq_set_conv_policy(a.policy)
    if a.fc:
        layers = [inputs.ConvLayer("fc.%d-%d@batch%d" % (ci, co, n), n, ci, 1, 1, co, 1, 1, 1, 0, b)
                  for n, ci, co, b in ((64, 4096, 4096, 4), (64, 4096, 4096, 2), (256, 4096, 4096, 4),
                                       (64, 25088, 4096, 4), (64, 4096, 1000, 4), (1024, 4096, 4096, 4))]
    else:
        if a.cfg is None:
            ap.error("--cfg or --fc")
        layers = inputs.config_layers(a.cfg, a.bits)
    if a.layer is not None:
        layers = [layers[a.layer]]
    tot_t, tot_macs = 0.0, 0
    for L in layers:
        r = bench_layer(L, kernel=a.kernel, chained=a.chained)
        print(json.dumps(r), flush=True)
        tot_t += (r["conv_us"] + r["quant_us"]) * 1e-6 * L.count
        tot_macs += L.macs * L.count
    print(json.dumps({"config": "fc" if a.fc else a.cfg, "layers": sum(L.count for L in layers),
                      "total_GMAC": round(tot_macs / 1e9, 2),
                      "quant_plus_conv_ms": round(tot_t * 1e3, 3),
                      "TOPS_over_quant_plus_conv": round(2 * tot_macs / tot_t / 1e12, 1)}))


if __name__ == "__main__":
    main()
