"""Per-layer timing of dsq_quantize_act, dsq_conv2d and dsq_conv2d_requant on one GPU.

    python -m paper_1908_05033_amd.layer_bench --cfg 3 [--bits 4] [--kernel 0] [--chained]
    python -m paper_1908_05033_amd.layer_bench --fc [--kernel 2]      (fully connected layers)

For every layer of a config (shapes from :mod:`paper_1908_05033_amd.inputs`)
it prints one JSON line: kernel time, effective int-TOPS (2*MACs/s, padding taps
included), fraction of the matrix peak of the instruction the layer runs on
(int8: 5000 TOP/s; 1- and 2-bit layers use the FP4 form: 10100), algorithmic
bytes (packed codes in, packed weights, pixel sums, fp32 out) and the GB/s they
amount to.  Inputs are random tensors of the config's distribution drawn on the
GPU (timing does not depend on the values).  Each call is timed twice:

  cold   launches captured in a hipGraph that rotates over as many buffer sets
         as it takes to exceed 600 MB, so that the 256 MB last-level cache
         cannot serve them (what a layer inside a large network sees);
  warm   a graph of as many launches over two buffer sets only, whose tensors
         stay in the last-level cache when they fit (what a small layer
         called in a tight loop sees).

Both are timed with events on the launch stream.  With --chained it also times
dsq_conv2d_requant (the layer's output written as the next layer's packed
codes) and, for comparison, the two calls it replaces: dsq_conv2d to fp32
followed by dsq_quantize_act of that tensor.
"""
import argparse
import json
import math

import torch

from . import binding as B
from . import inputs

INT8_PEAK_TOPS = 5000.0      # dense int8 matrix peak (3- and 4-bit layers)
FP4_PEAK_TOPS = 10100.0      # dense FP4 matrix peak (1- and 2-bit layers run on the FP4 instruction)
HBM_PEAK_GBS = 8000.0
RIDGE_INT8 = INT8_PEAK_TOPS * 1e12 / (HBM_PEAK_GBS * 1e9)     # ops per byte where the two bounds meet
MAX_SETS = 1024              # most buffer sets (graph nodes) of one measurement

# clip bound of |N(0,1)| activations at the percentile the config's recipe names
HALF_NORMAL_Q = {99.9: 3.2905, 99.5: 2.8070}


def matrix_peak_tops(bits):
    return FP4_PEAK_TOPS if bits <= 2 else INT8_PEAK_TOPS


def time_graph(fns, stream, reps, warm_reps=1):
    """Average seconds per call of the calls ``fns`` (closures without
    arguments), captured once as a hipGraph and replayed ``reps`` times
    between two events on the launch stream."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        for fn in fns:
            fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        for _ in range(warm_reps):
            g.replay()
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(reps):
            g.replay()
        e1.record(stream)
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / (reps * len(fns))


class LayerState:
    """Device buffers and call closures of one layer over ``sets`` buffer sets.
    Weights are packed once (model-load time)."""

    def __init__(self, L, sets, flags=0, chained=False, u_a=2.5, gen=None, bits_next=None, dense3=False):
        dev = "cuda"
        self.L = L
        self.dense3 = dense3          # 3-bit layers: dense 3-bit codes in (and out of the chained call)
        self.packing = B.DSQ_PACK_DENSE3 if dense3 else B.DSQ_PACK_CONTAINER
        if dense3:
            flags |= B.DSQ_CONV_ACT_DENSE3
        gen = gen or torch.Generator(device=dev).manual_seed(inputs.BASE_SEED)
        self.in_bytes = L.N * L.H * L.W * L.C_in * 4
        self.out_bytes = L.N * L.Ho * L.Wo * L.C_out * 4
        self.code_bytes = B.dsq_act_packed_bytes_ex(L.N, L.H, L.W, L.C_in, L.bits, self.packing)
        self.pix_bytes = L.N * L.H * L.W * 4
        self.w_bytes = B.dsq_wgt_packed_bytes(L.C_out, L.C_in, L.R, L.S, L.bits)
        w = torch.randn((L.C_out, L.C_in, L.R, L.S), device=dev, generator=gen) * math.sqrt(2.0 / (L.C_in * L.R * L.S))
        wf = w.reshape(L.C_out, -1)
        self.w, self.lw, self.uw = w, wf.amin(dim=1).contiguous(), wf.amax(dim=1).contiguous()
        self.bufs = []
        for _ in range(sets):
            b = B.alloc_layer(L.N, L.C_in, L.H, L.W, L.C_out, L.R, L.S, L.stride, L.pad, L.bits, flags=flags)
            b.x = torch.randn((L.N, L.H, L.W, L.C_in), device=dev, generator=gen).abs_()
            if dense3:
                b.act_packed = torch.empty(self.code_bytes, dtype=torch.uint8, device=dev)
            # (the chained call's descriptor: the same, plus the format of the codes it writes)
            b.desc_chained = B.make_desc(L.N, L.C_in, L.H, L.W, L.C_out, L.R, L.S, L.stride, L.pad, L.bits,
                                         flags | (B.DSQ_CONV_NEXT_DENSE3 if dense3 else 0))
            # (and for a caller that clears the next layer's pixel sums itself)
            b.desc_chained_z = B.make_desc(L.N, L.C_in, L.H, L.W, L.C_out, L.R, L.S, L.stride, L.pad, L.bits,
                                           flags | B.DSQ_CONV_NEXT_SUMS_ZERO | (B.DSQ_CONV_NEXT_DENSE3 if dense3 else 0))
            self.bufs.append(b)
        self.wp, self.aux = self.bufs[0].w_packed, self.bufs[0].w_aux
        self.l_a, self.u_a = 0.0, float(u_a)
        self.pack()
        self.chained = chained
        if chained:
            self.bits_next = bits_next or L.bits
            self.scale = torch.rand(L.C_out, device=dev, generator=gen) + 0.5
            self.shift = torch.randn(L.C_out, device=dev, generator=gen) * 0.1
            self.l_n, self.u_n = 0.0, 1.0
            self.next_bytes = B.dsq_act_packed_bytes_ex(L.N, L.Ho, L.Wo, L.C_out, self.bits_next, self.packing)
            for b in self.bufs:
                b.codes_next = torch.empty(self.next_bytes, dtype=torch.uint8, device=dev)
                b.pix_next = torch.empty(L.N * L.Ho * L.Wo, dtype=torch.int32, device=dev)

    @staticmethod
    def bytes_per_set(L):
        return (L.N * L.H * L.W * L.C_in * 4 + L.N * L.Ho * L.Wo * L.C_out * 4 +
                B.dsq_act_packed_bytes(L.N, L.H, L.W, L.C_in, L.bits) + L.N * L.H * L.W * 4)

    def pack(self):
        L = self.L
        B.dsq_pack_weights(self.w, self.lw, self.uw, None, L.C_out, L.C_in, L.R, L.S, L.bits, self.wp, self.aux)

    def quant(self, b):
        L = self.L
        B.dsq_quantize_act_ex(b.x, B.DSQ_NHWC, L.N, L.C_in, L.H, L.W, self.l_a, self.u_a, L.bits, self.packing,
                              b.act_packed, b.pix_code_sum)

    def conv(self, b):
        B.dsq_conv2d(b.desc, b.act_packed, b.pix_code_sum, self.l_a, self.u_a, self.wp, self.aux, b.out,
                     B.DSQ_NHWC, None)

    def conv_chained(self, b):
        B.dsq_conv2d_requant(b.desc_chained, b.act_packed, b.pix_code_sum, self.l_a, self.u_a, self.wp, self.aux,
                             self.scale, self.shift, True, self.l_n, self.u_n, self.bits_next,
                             b.codes_next, b.pix_next)

    def conv_chained_zeroed(self, b, pix_next):
        """The chained call into pixel sums the caller has cleared (DSQ_CONV_NEXT_SUMS_ZERO)."""
        B.dsq_conv2d_requant(b.desc_chained_z, b.act_packed, b.pix_code_sum, self.l_a, self.u_a, self.wp, self.aux,
                             self.scale, self.shift, True, self.l_n, self.u_n, self.bits_next,
                             b.codes_next, pix_next)

    def quant_next(self, b):
        """What the chained call saves: quantizing the fp32 output for the next layer."""
        L = self.L
        B.dsq_quantize_act_ex(b.out, B.DSQ_NHWC, L.N, L.C_out, L.Ho, L.Wo, self.l_n, self.u_n, self.bits_next,
                              self.packing, b.codes_next, b.pix_next)

    def calls(self, method, bufs=None):
        return [(lambda b=b: method(b)) for b in (bufs if bufs is not None else self.bufs)]

    # algorithmic bytes per call (packed weights counted at the packed code width)
    def conv_alg_bytes(self):
        L = self.L
        cont = 2 if L.bits <= 2 else 4
        return self.code_bytes + self.pix_bytes + L.C_out * L.C_in * L.R * L.S * cont // 8 + self.out_bytes

    def chained_alg_bytes(self):
        L = self.L
        cont = 2 if L.bits <= 2 else 4
        return (self.code_bytes + self.pix_bytes + L.C_out * L.C_in * L.R * L.S * cont // 8 +
                self.next_bytes + L.N * L.Ho * L.Wo * 4)

    def quant_alg_bytes(self):
        return self.in_bytes + self.code_bytes + self.pix_bytes


def cold_sets(L, min_bytes=600e6):
    return int(min(MAX_SETS, max(2, -(-min_bytes // LayerState.bytes_per_set(L)))))


def bench_layer(L, kernel=0, many_in_flight=False, min_bytes=600e6, reps=5, chained=False, u_a=2.5, dense3=False):
    sets = cold_sets(L, min_bytes)
    flags = B.DSQ_CONV_KERNEL(kernel) | (B.DSQ_CONV_MANY_IN_FLIGHT if many_in_flight else 0)
    st = LayerState(L, sets, flags=flags, chained=chained, u_a=u_a, dense3=dense3)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for b in st.bufs:
            st.quant(b)
            st.conv(b)
            if chained:
                st.conv_chained(b)
        torch.cuda.synchronize()
    # warm: two buffer sets, repeated inside the graph so that a replay holds at least as
    # many launches as a cold one (the cost of starting a graph is spread the same way)
    warm = st.bufs[:2] * max(16, sets // 2)
    warm_reps = reps
    tq = time_graph(st.calls(st.quant), stream, reps)
    tc = time_graph(st.calls(st.conv), stream, reps)
    tq_warm = time_graph(st.calls(st.quant, warm), stream, warm_reps)
    tc_warm = time_graph(st.calls(st.conv, warm), stream, warm_reps)
    conv_bytes, quant_bytes = st.conv_alg_bytes(), st.quant_alg_bytes()
    tops = 2.0 * L.macs / tc / 1e12
    peak = matrix_peak_tops(L.bits)
    extra = {}
    if chained:
        tcc = time_graph(st.calls(st.conv_chained), stream, reps)
        tqn = time_graph(st.calls(st.quant_next), stream, reps)
        tcc_warm = time_graph(st.calls(st.conv_chained, warm), stream, warm_reps)
        ch_bytes = st.chained_alg_bytes()
        extra = {
            "chained_us": round(tcc * 1e6, 2), "chained_warm_us": round(tcc_warm * 1e6, 2),
            "chained_TOPS": round(2.0 * L.macs / tcc / 1e12, 1),
            "chained_alg_MB": round(ch_bytes / 1e6, 2), "chained_GBps": round(ch_bytes / tcc / 1e9, 1),
            "unchained_us": round((tc + tqn) * 1e6, 2), "quant_next_us": round(tqn * 1e6, 2),
            "chained_speedup": round((tc + tqn) / tcc, 2), "chained_vs_plain_conv": round(tc / tcc, 2),
        }
    return {**extra, **{
        "layer": L.name, "bits": L.bits, "count": L.count, "codes": "dense 3-bit" if dense3 else "containers",
        "gemm_MxNxK": [L.N * L.Ho * L.Wo, L.C_out, L.C_in * L.R * L.S],
        "conv_us": round(tc * 1e6, 2), "conv_warm_us": round(tc_warm * 1e6, 2), "conv_TOPS": round(tops, 1),
        "conv_frac_int8_peak": round(tops / INT8_PEAK_TOPS, 4),
        "matrix_peak_TOPS": peak,
        "conv_frac_matrix_peak": round(tops / peak, 4),
        "conv_alg_MB": round(conv_bytes / 1e6, 2), "conv_GBps": round(conv_bytes / tc / 1e9, 1),
        "conv_frac_hbm_peak": round(conv_bytes / tc / 1e9 / HBM_PEAK_GBS, 4),
        "quant_us": round(tq * 1e6, 2), "quant_warm_us": round(tq_warm * 1e6, 2),
        "quant_GBps": round(quant_bytes / tq / 1e9, 1),
        "quant_frac_hbm_peak": round(quant_bytes / tq / 1e9 / HBM_PEAK_GBS, 4),
        "buffer_sets": sets, "cold_working_set_MB": round(sets * LayerState.bytes_per_set(L) / 1e6, 1),
        "w_buffer_bytes": st.w_bytes,
    }}


FP32_MATRIX_PEAK_TFLOPS = 157.3


def bench_weight_only(L, bits_w=1, reps=3):
    """dsq_conv2d_wq (b-bit weights, binary32 activations) on one layer shape: cold timing."""
    dev = "cuda"
    gen = torch.Generator(device=dev).manual_seed(inputs.BASE_SEED)
    per_set = L.N * L.H * L.W * L.C_in * 4 + L.N * L.Ho * L.Wo * L.C_out * 4
    sets = int(min(MAX_SETS, max(2, -(-600e6 // per_set))))
    w = torch.randn((L.C_out, L.C_in, L.R, L.S), device=dev, generator=gen) * math.sqrt(2.0 / (L.C_in * L.R * L.S))
    wf = w.reshape(L.C_out, -1)
    lw, uw = wf.amin(dim=1).contiguous(), wf.amax(dim=1).contiguous()
    wp = torch.empty(B.dsq_wgt_packed_bytes(L.C_out, L.C_in, L.R, L.S, 4), dtype=torch.uint8, device=dev)
    aux = torch.empty(B.dsq_wgt_aux_bytes(L.C_out, L.R, L.S), dtype=torch.uint8, device=dev)
    B.dsq_pack_weights_for(w, lw, uw, None, L.C_out, L.C_in, L.R, L.S, bits_w, 4, wp, aux)
    d = B.make_desc(L.N, L.C_in, L.H, L.W, L.C_out, L.R, L.S, L.stride, L.pad, bits_w)
    xs = [torch.randn((L.N, L.H, L.W, L.C_in), device=dev, generator=gen) for _ in range(sets)]
    outs = [torch.empty((L.N, L.Ho, L.Wo, L.C_out), device=dev) for _ in range(sets)]
    stream = torch.cuda.Stream()
    calls = [(lambda x=x, o=o: B.dsq_conv2d_wq(d, x, B.DSQ_NHWC, wp, aux, o, B.DSQ_NHWC)) for x, o in zip(xs, outs)]
    with torch.cuda.stream(stream):
        for fn in calls:
            fn()
        torch.cuda.synchronize()
    t = time_graph(calls, stream, reps)
    tf = 2.0 * L.macs / t / 1e12
    return {"layer": L.name, "weight_bits": bits_w, "activations": "binary32", "conv_us": round(t * 1e6, 2),
            "TFLOPs": round(tf, 1), "frac_fp32_matrix_peak": round(tf / FP32_MATRIX_PEAK_TFLOPS, 4),
            "GBps": round(per_set / t / 1e9, 1), "buffer_sets": sets}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cfg", type=int, default=None)
    ap.add_argument("--fc", action="store_true",
                    help="fully connected layers (1x1 layers on 1x1 images) instead of a benchmark config")
    ap.add_argument("--bits", type=int, default=None)
    ap.add_argument("--kernel", type=int, default=0)
    ap.add_argument("--layer", type=int, default=None)
    ap.add_argument("--chained", action="store_true")
    ap.add_argument("--dense3", action="store_true",
                    help="3-bit layers (--bits 3): dense 3-bit activation codes instead of 4-bit containers")
    ap.add_argument("--weight-only", type=int, default=0, metavar="BITS",
                    help="time dsq_conv2d_wq (BITS-bit weights, binary32 activations) on the config's shapes instead")
    ap.add_argument("--many-in-flight", action="store_true",
                    help="pass DSQ_CONV_MANY_IN_FLIGHT (the default optimises a single call; kernels are "
                         "timed one at a time here)")
    a = ap.parse_args()
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
    if a.weight_only:
        for L in layers:
            print(json.dumps(bench_weight_only(L, a.weight_only)), flush=True)
        return
    tot_t, tot_macs = 0.0, 0
    for L in layers:
        try:
            r = bench_layer(L, kernel=a.kernel, many_in_flight=a.many_in_flight, chained=a.chained, dense3=a.dense3)
        except B.DsqError as e:
            if e.status != 5 or a.kernel < 2:
                raise
            # a forced tile that does not take this layer (or has no chained variant for it)
            try:
                r = bench_layer(L, kernel=a.kernel, many_in_flight=a.many_in_flight, chained=False, dense3=a.dense3)
            except B.DsqError:
                print(json.dumps({"layer_skipped": L.name, "reason": "kernel %d does not take it" % a.kernel}), flush=True)
                continue
        print(json.dumps(r), flush=True)
        tot_t += (r["conv_us"] + r["quant_us"]) * 1e-6 * L.count
        tot_macs += L.macs * L.count
    print(json.dumps({"config": "fc" if a.fc else a.cfg, "layers": sum(L.count for L in layers),
                      "total_GMAC": round(tot_macs / 1e9, 2),
                      "quant_plus_conv_ms": round(tot_t * 1e3, 3),
                      "TOPS_over_quant_plus_conv": round(2 * tot_macs / tot_t / 1e12, 1)}))


if __name__ == "__main__":
    main()
