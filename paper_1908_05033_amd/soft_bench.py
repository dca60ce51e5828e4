"""Timing of the training-mode DSQ kernels on one GPU.

    python -m paper_1908_05033_amd.soft_bench

For activation-sized tensors of the benchmark configs it prints one JSON line
per size: time of dsq_soft_quantize_fwd (8 B per element: fp32 in, fp32 out)
and dsq_soft_quantize_bwd (12 B per element: x and the upstream gradient in,
dL/dx out; the fill kernel of the three sums included), the GB/s those bytes
amount to and the fraction of the 8 TB/s HBM peak.  Launches are captured in a
hipGraph that rotates over enough buffer sets to exceed the 256 MB last-level
cache.
"""
import json

import torch

from . import binding as B

HBM_PEAK_GBS = 8000.0
SIZES = [("cfg2 activation 32x256x14x14", 32 * 256 * 14 * 14),
         ("ResNet-18 stage-1 activation 64x64x56x56", 64 * 64 * 56 * 56),
         ("VGG-16 first quantized activation 32x64x224x224", 32 * 64 * 224 * 224)]


def _time(fn, sets, stream, reps):
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        for s in sets:
            fn(s)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        g.replay()
        torch.cuda.synchronize()
        e0.record(stream)
        for _ in range(reps):
            g.replay()
        e1.record(stream)
        torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / (reps * len(sets))


def main():
    l, u, alpha, bits = 0.0, 2.5, 0.2, 4
    stream = torch.cuda.Stream()
    for name, n in SIZES:
        n_sets = int(min(16, max(2, -(-600e6 // (16 * n)))))
        sets = []
        for _ in range(n_sets):
            x = torch.randn(n, device="cuda").abs_() * 1.2
            sets.append((x, torch.randn(n, device="cuda"), torch.empty(n, device="cuda"), torch.empty(n, device="cuda"),
                         torch.empty(4, dtype=torch.float64, device="cuda")))
        fwd = lambda s: B.dsq_soft_quantize_fwd(s[0], l, u, alpha, bits, s[2])
        bwd = lambda s: B.dsq_soft_quantize_bwd(s[0], s[1], l, u, alpha, bits, s[3], s[4])
        with torch.cuda.stream(stream):
            fwd(sets[0]); bwd(sets[0])
            torch.cuda.synchronize()
        tf = _time(fwd, sets, stream, 5)
        tb = _time(bwd, sets, stream, 5)
        print(json.dumps({
            "tensor": name, "elements": n, "buffer_sets": n_sets,
            "fwd_us": round(tf * 1e6, 2), "fwd_GBps": round(8 * n / tf / 1e9, 1),
            "fwd_frac_hbm_peak": round(8 * n / tf / 1e9 / HBM_PEAK_GBS, 4),
            "bwd_us": round(tb * 1e6, 2), "bwd_GBps": round(12 * n / tb / 1e9, 1),
            "bwd_frac_hbm_peak": round(12 * n / tb / 1e9 / HBM_PEAK_GBS, 4)}), flush=True)
        del sets


if __name__ == "__main__":
    main()
