"""The library's calls inside a captured HIP graph: every replay must give the
eager result.  (The calls that clear a buffer do it with a fill kernel, not a
memset node, precisely so that they can be captured.)"""
import numpy as np
import pytest
import torch

from paper_1908_05033_amd import binding as B
from paper_1908_05033_amd import inputs

pytestmark = pytest.mark.gpu


def test_replays_match_eager_results():
    layer, inp = inputs.make_config_layer(1)
    L = layer
    buf = B.alloc_layer(L.N, L.C_in, L.H, L.W, L.C_out, L.R, L.S, L.stride, L.pad, L.bits)
    x = inp["x"].permute(0, 2, 3, 1).contiguous().cuda()
    B.dsq_pack_weights(inp["w"].contiguous().cuda(), torch.from_numpy(inp["l_w"]).cuda(),
                       torch.from_numpy(inp["u_w"]).cuda(), None, L.C_out, L.C_in, L.R, L.S, L.bits,
                       buf.w_packed, buf.w_aux)
    codes_next = torch.empty(B.dsq_act_packed_bytes(L.N, L.Ho, L.Wo, L.C_out, 4), dtype=torch.uint8, device="cuda")
    pix_next = torch.empty(L.N * L.Ho * L.Wo, dtype=torch.int32, device="cuda")
    gx = torch.empty_like(x)
    sums = torch.empty(4, dtype=torch.float64, device="cuda")
    gy = torch.randn(x.shape, generator=torch.Generator().manual_seed(3)).cuda()

    def step():
        B.dsq_quantize_act(x, B.DSQ_NHWC, L.N, L.C_in, L.H, L.W, inp["l_a"], inp["u_a"], L.bits,
                           buf.act_packed, buf.pix_code_sum)
        B.dsq_conv2d(buf.desc, buf.act_packed, buf.pix_code_sum, inp["l_a"], inp["u_a"], buf.w_packed, buf.w_aux,
                     buf.out, B.DSQ_NHWC, None)
        B.dsq_conv2d_requant(buf.desc, buf.act_packed, buf.pix_code_sum, inp["l_a"], inp["u_a"], buf.w_packed,
                             buf.w_aux, None, None, True, 0.0, 1.5, 4, codes_next, pix_next)
        B.dsq_soft_quantize_bwd(x, gy, inp["l_a"], inp["u_a"], 0.2, L.bits, gx, sums)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (buf.act_packed, buf.pix_code_sum, buf.out, codes_next, pix_next, gx, sums)]

    def scramble():
        for t in (buf.act_packed, buf.pix_code_sum, codes_next, pix_next):
            t.fill_(77)
        for t in (buf.out, gx, sums):
            t.fill_(float("nan"))

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()
        want = snapshot()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            step()
        for _ in range(3):
            scramble()                       # eager work between the replays
            torch.cuda.synchronize()
            g.replay()
            got = snapshot()
            for a, b in zip(got[:-1], want[:-1]):
                assert torch.equal(a, b)
            # binary64 atomics: the order of the partial sums may differ between runs
            assert np.allclose(got[-1][:3].cpu().numpy(), want[-1][:3].cpu().numpy(), rtol=1e-12, atol=0)


@pytest.mark.parametrize("caller_clears", [False, True])
def test_chained_call_on_a_wide_layer_replays(caller_clears):
    """A layer wider than a workgroup's tile: the chained call adds to the next layer's
    pixel sums with atomics after clearing them with its own fill kernel, or after the
    caller's fill (DSQ_CONV_NEXT_SUMS_ZERO); both forms must replay to the eager result."""
    layer, inp = inputs.small_random_case(31, 2, 256, 6, 6, 256, 3, 1, 1, 4, l_a=0.0, u_a=2.1)
    L = layer
    buf = B.alloc_layer(L.N, L.C_in, L.H, L.W, L.C_out, L.R, L.S, L.stride, L.pad, L.bits,
                        flags=B.DSQ_CONV_NEXT_SUMS_ZERO if caller_clears else 0)
    x = inp["x"].permute(0, 2, 3, 1).contiguous().cuda()
    B.dsq_pack_weights(inp["w"].contiguous().cuda(), torch.from_numpy(np.ascontiguousarray(inp["l_w"])).cuda(),
                       torch.from_numpy(np.ascontiguousarray(inp["u_w"])).cuda(), None, L.C_out, L.C_in, L.R, L.S,
                       L.bits, buf.w_packed, buf.w_aux)
    scale, shift = inputs.affine_params(31, L.C_out)
    sc, sh = torch.from_numpy(scale).cuda(), torch.from_numpy(shift).cuda()
    codes_next = torch.empty(B.dsq_act_packed_bytes(L.N, L.Ho, L.Wo, L.C_out, 4), dtype=torch.uint8, device="cuda")
    pix_next = torch.empty(L.N * L.Ho * L.Wo, dtype=torch.int32, device="cuda")

    def step():
        B.dsq_quantize_act(x, B.DSQ_NHWC, L.N, L.C_in, L.H, L.W, inp["l_a"], inp["u_a"], L.bits,
                           buf.act_packed, buf.pix_code_sum)
        if caller_clears:
            pix_next.zero_()
        B.dsq_conv2d_requant(buf.desc, buf.act_packed, buf.pix_code_sum, inp["l_a"], inp["u_a"], buf.w_packed,
                             buf.w_aux, sc, sh, True, 0.0, 2.0, 4, codes_next, pix_next)

    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()
        torch.cuda.synchronize()
        want = [codes_next.clone(), pix_next.clone()]
        assert int(want[1].sum()) > 0
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            step()
        for _ in range(3):
            codes_next.fill_(77)
            pix_next.fill_(12345)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(codes_next, want[0]) and torch.equal(pix_next, want[1])
