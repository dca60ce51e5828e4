#!/usr/bin/env python3
"""Benchmark of the b-bit quantized convolution hot path on one MI355X.

A step is one pass of the per-batch hot path over one batch of synthetic
input: dsq_quantize_act (fp32 activations -> packed codes + pixel sums)
followed by dsq_conv2d (integer implicit GEMM + dequantizing epilogue -> fp32).
dsq_pack_weights runs once per layer when a model is loaded; it is timed
separately and is not part of the step.  The workload is the 3x3, 256->256,
14x14, batch-32, 4-bit layer (the ResNet stage-3 shape).  Inputs live in HBM
before the timed region; the steps rotate over enough buffer sets that the
working set exceeds twice the 256 MB last-level cache (their number is chosen so
that whole passes over them make exactly --steps steps).  By default the steps are dealt
to four chains (four batches in flight, each running its own quantize -> conv
in order), one hipGraph and one stream per chain, which is how a server with
several requests in flight drives the library; --serial runs them strictly one
after the other and is reported too.

Prints ONE JSON line:  value = effective int-TOPS = 2*MACs*steps / time.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0     # MI355X dense int8 matrix peak
HBM_PEAK_GBS = 8000.0

# HBM bytes per dsq_conv2d launch on this workload from two rocprofv3 --pmc runs
# (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, factors from a 256 MiB copy kernel;
# profiles/traffic_cfg2.md).  Algorithmic bytes are 7.55 MB.
MEASURED_CONV_TRAFFIC_BYTES = {2: 9954687}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=2, help="benchmark config (1 or 2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--serial", action="store_true", help="no overlap between steps of different batches")
    ap.add_argument("--sets", type=int, default=0, help="buffer sets to rotate over (0 = auto)")
    ap.add_argument("--streams", type=int, default=4,
                    help="run the steps as this many independent serial chains, one stream each "
                         "(0 = the two-stream pipeline: quantize of batch i+1 beside conv of batch i)")
    ap.add_argument("--latency-policy", action="store_true",
                    help="keep the library's default kernel choice (shortest single call) although several "
                         "steps are in flight; the default here is dsq_set_conv_policy(1)")
    ap.add_argument("--one-graph", action="store_true",
                    help="the chains as branches of a single graph instead of one graph per chain")
    return ap.parse_args()


def choose_sets(per_set, args):
    """Number of buffer sets: the working set must exceed twice the 256 MB
    last-level cache, a pass over the sets must deal every chain the same number
    of steps, and whole passes should make up exactly --steps (and --warmup)
    steps; the smallest such count is taken.  If none fits, the smallest count
    of the right size is used and the step counts are rounded up to whole passes
    (the JSON line reports what was run).  At most 256 sets."""
    chains = 1 if args.serial else (args.streams if args.streams > 0 else 2)
    lo = max(2, -(-520000000 // per_set))
    lo = -(-lo // chains) * chains
    cap = 256                     # (a tiny layer would need thousands of sets: the largest count that fits)
    if lo > cap:
        lo = cap - cap % chains
        cands = range(lo, 0, -chains)
    else:
        cands = range(lo, min(4 * lo, cap) + 1, chains)
    for ok in (lambda n: args.steps % n == 0 and args.warmup % n == 0, lambda n: args.steps % n == 0):
        fit = [n for n in cands if ok(n)]
        if fit:
            return fit[0]
    return lo


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path shards over the batch "
              "with no exchange step); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1908_05033_amd import binding as B
    from paper_1908_05033_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.load_library()
    # several batches in flight: tell the library (it then spreads a layer differently);
    # every figure of this run, the kernel durations included, is taken under the same policy
    many_in_flight = not args.serial and not args.latency_policy
    B.dsq_set_conv_policy(1 if many_in_flight else 0)

    layer, inp = inputs.make_config_layer(args.config)
    L = layer
    macs = L.macs

    # ---- buffers: one weight set, `sets` activation/output sets ------------
    in_bytes = L.N * L.C_in * L.H * L.W * 4
    out_bytes = L.N * L.Ho * L.Wo * L.C_out * 4
    code_bytes = B.dsq_act_packed_bytes(L.N, L.H, L.W, L.C_in, L.bits)
    per_set = in_bytes + out_bytes + code_bytes + L.N * L.H * L.W * 4
    sets = min(args.sets or choose_sets(per_set, args), 256)   # (same cap as in choose_sets)

    x_nhwc = inp["x"].permute(0, 2, 3, 1).contiguous()
    bufs = []
    for s in range(sets):
        b = B.alloc_layer(L.N, L.C_in, L.H, L.W, L.C_out, L.R, L.S, L.stride, L.pad, L.bits)
        b.x = x_nhwc.cuda() if s == 0 else bufs[0].x.clone()
        bufs.append(b)
    w = inp["w"].contiguous().cuda()
    lw = torch.from_numpy(inp["l_w"]).cuda()
    uw = torch.from_numpy(inp["u_w"]).cuda()
    w_packed, w_aux = bufs[0].w_packed, bufs[0].w_aux
    l_a, u_a = inp["l_a"], inp["u_a"]

    stream = torch.cuda.Stream()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def pack():
        B.dsq_pack_weights(w, lw, uw, None, L.C_out, L.C_in, L.R, L.S, L.bits, w_packed, w_aux)

    def quant(b):
        B.dsq_quantize_act(b.x, B.DSQ_NHWC, L.N, L.C_in, L.H, L.W, l_a, u_a, L.bits,
                           b.act_packed, b.pix_code_sum)

    def conv(b):
        B.dsq_conv2d(b.desc, b.act_packed, b.pix_code_sum, l_a, u_a, w_packed, w_aux, b.out,
                     B.DSQ_NHWC, None)

    def capture(fn):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for b in bufs:
                fn(b)
        return g

    side = torch.cuda.Stream()

    def capture_pipelined():
        """All steps of one pass over the buffer sets, software-pipelined over two
        streams the way a serving loop double-buffers batches: the activations of
        batch i+1 are quantized (side stream) while batch i is convolved (launch
        stream).  Every step still runs quantize then conv on its own batch; only
        steps of different batches overlap."""
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            ready = []
            side.wait_stream(stream)
            with torch.cuda.stream(side):
                quant(bufs[0])
                e = torch.cuda.Event()
                e.record(side)
                ready.append(e)
            for i, b in enumerate(bufs):
                if i + 1 < len(bufs):
                    with torch.cuda.stream(side):
                        quant(bufs[i + 1])
                        e = torch.cuda.Event()
                        e.record(side)
                        ready.append(e)
                stream.wait_event(ready[i])
                conv(b)
            stream.wait_stream(side)
        return g

    def capture_chains(n_chains):
        """The steps dealt round-robin to n_chains streams; each stream runs its
        steps (quantize then conv of one batch) strictly in order, the streams run
        side by side, the way a server keeps several requests in flight."""
        chains = [torch.cuda.Stream() for _ in range(n_chains)]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for c, st in enumerate(chains):
                st.wait_stream(stream)
                with torch.cuda.stream(st):
                    for b in bufs[c::n_chains]:
                        quant(b)
                        conv(b)
            for st in chains:
                stream.wait_stream(st)
        return g

    def capture_chain_graphs(n_chains):
        """One graph per chain: the steps dealt round-robin to n_chains chains, each
        captured as a strictly serial graph of its own."""
        graphs = []
        for c in range(n_chains):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for b in bufs[c::n_chains]:
                    quant(b)
                    conv(b)
            graphs.append(g)
        return graphs

    def timed_chain_replays(graphs, streams, n):
        """n replays of every chain graph, chain c on streams[c], between two events
        on the launch stream (which the chain streams wait for and are joined to)."""
        torch.cuda.synchronize()
        ev0.record(stream)
        for st in streams:
            st.wait_event(ev0)
        for _ in range(n):
            for g, st in zip(graphs, streams):
                with torch.cuda.stream(st):
                    g.replay()
        for st in streams:
            stream.wait_stream(st)
        ev1.record(stream)
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) * 1e-3

    def pick_streams(graphs, n_chains):
        """HIP multiplexes its streams onto a few hardware queues; chains whose
        streams share a queue run one after the other.  Which streams share one is
        not visible from here, so a short calibration run tries windows of
        consecutive streams from a small pool and keeps the fastest."""
        pool = [torch.cuda.Stream() for _ in range(n_chains + 6)]
        best, best_t = None, None
        for o in range(len(pool) - n_chains + 1):
            cand = pool[o:o + n_chains]
            timed_chain_replays(graphs, cand, 1)
            t = min(timed_chain_replays(graphs, cand, 2) for _ in range(2))
            if best_t is None or t < best_t:
                best, best_t = cand, t
        return best

    def timed_replays(g, n):
        """n replays of a graph between two events on the launch stream."""
        with torch.cuda.stream(stream):
            torch.cuda.synchronize()
            ev0.record(stream)
            for _ in range(n):
                g.replay()
            ev1.record(stream)
            torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) * 1e-3

    with torch.cuda.stream(stream):
        pack()
        for b in bufs:
            quant(b)
            conv(b)
        torch.cuda.synchronize()
        # weight packing, timed on its own (model-load time, not part of a step)
        ev0.record(stream)
        for _ in range(10):
            pack()
        ev1.record(stream)
        torch.cuda.synchronize()
        pack_ms = ev0.elapsed_time(ev1) / 10

    def step(b):
        quant(b)
        conv(b)

    g_step, g_quant, g_conv = capture(step), capture(quant), capture(conv)
    chain_graphs = chain_streams = None
    if args.serial:
        g_pipe = g_step
    elif args.streams > 0 and not args.one_graph:
        g_pipe = None
        chain_graphs = capture_chain_graphs(args.streams)
        chain_streams = pick_streams(chain_graphs, args.streams)
    elif args.streams > 0:
        g_pipe = capture_chains(args.streams)
    else:
        g_pipe = capture_pipelined()

    def timed_pass(n):
        if chain_graphs is not None:
            return timed_chain_replays(chain_graphs, chain_streams, n)
        return timed_replays(g_pipe, n)

    # ---- the timed region: exactly `steps` steps ---------------------------
    n_warm = max(1, -(-args.warmup // sets))
    n_rep = max(1, -(-args.steps // sets))
    steps = n_rep * sets
    warmup = n_warm * sets
    timed_pass(n_warm)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    gpu_s = timed_pass(n_rep)
    wall_s = time.perf_counter() - t0
    step_s = max(gpu_s, 0.0) / steps
    value = 2.0 * macs / step_s / 1e12
    # the same steps strictly one after the other on one stream
    timed_replays(g_step, n_warm)
    serial_step_s = timed_replays(g_step, n_rep) / steps

    # ---- per-kernel average launch durations, same stream, HIP events ------
    timed_replays(g_conv, n_warm)
    conv_s = timed_replays(g_conv, n_rep) / steps
    timed_replays(g_quant, n_warm)
    quant_s = timed_replays(g_quant, n_rep) / steps

    # the same kernel call under the other policy, for the record
    B.dsq_set_conv_policy(0 if many_in_flight else 1)
    g_conv_other = capture(conv)
    B.dsq_set_conv_policy(1 if many_in_flight else 0)
    timed_replays(g_conv_other, n_warm)
    conv_other_s = timed_replays(g_conv_other, n_rep) / steps

    conv_tops = 2.0 * macs / conv_s / 1e12
    quant_bytes = in_bytes + code_bytes + L.N * L.H * L.W * 4
    result = {
        "metric": "effective int-TOPS of b-bit conv2d (2*MACs/s), 1 GPU",
        "value": round(value, 3),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(step_s * 1e3, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u%d codes, int8 MFMA, int32 accumulate, f64 epilogue -> f32" % L.bits,
        "data": "synthetic",
        "config": {
            "workload": "config %d: %dx%d conv stride %d pad %d, N=%d, C_in=%d, C_out=%d, %dx%d, %d-bit "
                        "acts and weights" % (args.config, L.R, L.S, L.stride, L.pad, L.N, L.C_in, L.C_out,
                                              L.H, L.W, L.bits),
            "step": "dsq_quantize_act + dsq_conv2d (weights packed once, outside the step)",
            "gemm_MxNxK": [L.N * L.Ho * L.Wo, L.C_out, L.C_in * L.R * L.S],
            "macs_per_step": macs,
            "buffer_sets": sets,
            "kernel_policy": "dsq_set_conv_policy(1): several calls in flight" if many_in_flight else
                             "dsq_set_conv_policy(0): shortest single call",
            "launch": ("%d steps per pass, %d passes; " % (sets, n_rep)) +
                      ("one hipGraph, steps strictly serial on one stream" if args.serial else
                       "%d hipGraphs, each a serial chain of every %dth step, replayed side by side on %d streams "
                       "(picked from a pool of %d by a calibration run: streams that share a hardware queue "
                       "would serialise)" % (args.streams, args.streams, args.streams, args.streams + 6)
                       if chain_graphs is not None else
                       "one hipGraph with %d independent chains of serial steps as branches" % args.streams
                       if args.streams > 0 else
                       "one hipGraph, quantize of batch i+1 overlaps conv of batch i (two streams)"),
        },
        "kernels": {
            "serial_step_us": round(serial_step_s * 1e6, 3),
            "dsq_conv2d_us": round(conv_s * 1e6, 3),
            "dsq_conv2d_TOPS": round(conv_tops, 2),
            "dsq_conv2d_us_under_policy_%d" % (0 if many_in_flight else 1): round(conv_other_s * 1e6, 3),
            "dsq_quantize_act_us": round(quant_s * 1e6, 3),
            "dsq_quantize_act_GBps": round(quant_bytes / quant_s / 1e9, 1),
            "dsq_pack_weights_us_not_in_step": round(pack_ms * 1e3, 2),
            "host_wall_s_timed_region": round(wall_s, 4),
        },
        "roofline": {
            "kernel": "dsq_conv2d",
            "bound": "mfma",
            "achieved": round(conv_tops, 2),
            "peak": INT8_MFMA_PEAK_TOPS,
            "unit": "TOP/s",
            "frac": round(conv_tops / INT8_MFMA_PEAK_TOPS, 4),
            "traffic": MEASURED_CONV_TRAFFIC_BYTES.get(args.config),
            "algorithmic_ops_per_launch": 2 * macs,
        },
    }

    if not args.no_cpu_baseline:
        import oracle
        xs = inp["x"].numpy()
        ws = inp["w"].numpy()
        w_code = oracle.quantize_weights(ws, inp["l_w"], inp["u_w"], L.bits)   # once per layer, like the GPU
        t0 = time.perf_counter()
        passes = 0
        while passes < 64 and (passes == 0 or time.perf_counter() - t0 < 6.0):
            a_code = oracle.quantize(xs, l_a, u_a, L.bits)
            oracle.conv_real(a_code, l_a, u_a, w_code, inp["l_w"], inp["u_w"], L.bits, L.stride, L.pad)
            passes += 1
        cpu_s = (time.perf_counter() - t0) / passes
        result["cpu_baseline"] = {
            "value": round(2.0 * macs / cpu_s / 1e12, 6),
            "unit": "TOPS",
            "cores": oracle.threads(),
            "kind": "oracle",
            "sample": "%d passes over one full batch of the same workload (quantize + direct conv on "
                      "dequantized doubles), %.3f s per pass, %.1f s in all" % (passes, cpu_s, cpu_s * passes),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
