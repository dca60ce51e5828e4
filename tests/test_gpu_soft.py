"""GPU parity of the training-mode DSQ kernels (dsq_soft_quantize_fwd / _bwd)
against the float64 oracle.

Tolerances: the kernels evaluate ~15 binary32 operations per element on
constants rounded from binary64, so an element may be off by a few units of
6e-8 relative to the magnitudes involved: values are compared to 2e-6 of
max(|l|, |u|, u - l), derivatives to 1e-5 of their largest magnitude, and the
three sums (accumulated in binary64) to 1e-5 of the sum of the absolute values
of their terms."""
import numpy as np
import pytest
import torch

from oracle import dsq_soft as S
from paper_1908_05033_amd import binding as B
from paper_1908_05033_amd import inputs

pytestmark = pytest.mark.gpu

CASES = [  # l, u, alpha, bits
    (-1.0, 2.0, 0.2, 2),
    (0.0, 3.0, 0.05, 4),
    (-0.7, 0.9, 0.45, 3),
    (0.0, 6.0, 0.2, 4),
    (0.0, 0.01, 0.2, 4),          # k capped at 1000
    (-0.004, 0.004, 0.3, 2),      # capped, symmetric (a weight tensor)
]
SIZES = [1, 3, 4, 1023, 4096 + 1, (1 << 20) + 3]


def run_fwd(x, l, u, alpha, bits):
    xd = x.cuda()
    y = torch.full_like(xd, float("nan"))
    B.dsq_soft_quantize_fwd(xd, l, u, alpha, bits, y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def run_bwd(x, g, l, u, alpha, bits):
    xd, gd = x.cuda(), g.cuda()
    gx = torch.full_like(xd, float("nan"))
    sums = torch.full((4,), 7.0, dtype=torch.float64, device="cuda")     # stale contents must be overwritten
    B.dsq_soft_quantize_bwd(xd, gd, l, u, alpha, bits, gx, sums)
    torch.cuda.synchronize()
    return gx.cpu().numpy(), sums.cpu().numpy()[:3]


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("l,u,alpha,bits", CASES)
def test_forward(l, u, alpha, bits, n):
    x, _ = inputs.soft_quant_case(n % 97, n, l, u)
    ref = S.forward(x.numpy().astype(np.float64), np.float32(l), np.float32(u), np.float32(alpha), bits)
    got = run_fwd(x, l, u, alpha, bits)
    scale = max(abs(l), abs(u), u - l)
    assert np.abs(got - ref).max() <= 2e-6 * scale


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("l,u,alpha,bits", CASES)
def test_backward(l, u, alpha, bits, n):
    x, g = inputs.soft_quant_case(n % 89, n, l, u)
    xs, gs = x.numpy().astype(np.float64), g.numpy().astype(np.float64)
    lf, uf, af = np.float32(l), np.float32(u), np.float32(alpha)
    dx, da, dl, du = S.partials(xs, lf, uf, af, bits)
    got_gx, got_sums = run_bwd(x, g, l, u, alpha, bits)
    assert np.abs(got_gx - gs * dx).max() <= 1e-5 * max(1.0, np.abs(dx).max()) * np.abs(gs).max()
    for got, d in zip(got_sums, (da, dl, du)):
        terms = gs * d
        assert abs(got - terms.sum()) <= 1e-5 * np.abs(terms).sum() + 1e-12


def test_largest_tensor():
    """n = 2^31 - 1 elements (the limit, and an odd count): forward values and the
    elementwise gradient at the head, the tail and a million places in between,
    and the three gradient sums over all elements.  The tensor repeats one seeded
    block of 4 194 301 elements (an odd length, so that the repeats fall differently
    into the kernel's vectors and workgroups each time); the sums the oracle gives
    for the block and for the ragged last repeat then add up to the expected sums
    of the whole tensor, which an element dropped or counted twice anywhere in the
    2^31 would change."""
    l, u, alpha, bits = -1.0, 2.0, 0.2, 4
    n = (1 << 31) - 1
    P = 4194301
    g = torch.Generator(device="cuda").manual_seed(inputs.BASE_SEED + 91)
    xb = torch.empty((P,), dtype=torch.float32, device="cuda").normal_(0.5, 1.2, generator=g)
    gb = torch.empty((P,), dtype=torch.float32, device="cuda").normal_(0.0, 1.0, generator=g)
    x = torch.empty((n,), dtype=torch.float32, device="cuda")
    gy = torch.empty((n,), dtype=torch.float32, device="cuda")
    for s in range(0, n, P):
        m = min(P, n - s)
        x[s:s + m] = xb[:m]
        gy[s:s + m] = gb[:m]
    y = torch.empty_like(x)
    B.dsq_soft_quantize_fwd(x, l, u, alpha, bits, y)
    gx = torch.empty_like(x)
    sums = torch.zeros((4,), dtype=torch.float64, device="cuda")
    B.dsq_soft_quantize_bwd(x, gy, l, u, alpha, bits, gx, sums)
    torch.cuda.synchronize()
    rs = np.random.RandomState(3)
    sample = np.unique(np.concatenate([np.arange(4096), np.arange(n - 4096, n), rs.randint(0, n, 1 << 20)]))
    idx = torch.from_numpy(sample).cuda()
    xs = x[idx].cpu().numpy().astype(np.float64)
    gs = gy[idx].cpu().numpy().astype(np.float64)
    lf, uf, af = np.float32(l), np.float32(u), np.float32(alpha)
    ref = S.forward(xs, lf, uf, af, bits)
    assert np.abs(y[idx].cpu().numpy() - ref).max() <= 2e-6 * max(abs(l), abs(u), u - l)
    dx, da, dl, du = S.partials(xs, lf, uf, af, bits)
    assert np.abs(gx[idx].cpu().numpy() - gs * dx).max() <= 1e-5 * max(1.0, np.abs(dx).max()) * np.abs(gs).max()
    # the three sums over all 2^31 - 1 elements: whole repeats of the block plus the ragged last one
    q, r = divmod(n, P)
    xbh, gbh = xb.cpu().numpy().astype(np.float64), gb.cpu().numpy().astype(np.float64)
    _, da, dl, du = S.partials(xbh, lf, uf, af, bits)
    got_sums = sums.cpu().numpy()[:3]
    for got, d in zip(got_sums, (da, dl, du)):
        terms = gbh * d
        want = q * terms.sum() + terms[:r].sum()
        assert abs(got - want) <= 1e-5 * (q * np.abs(terms).sum() + np.abs(terms[:r]).sum())
    with pytest.raises(B.DsqError) as e:                      # one element more is refused
        B._check(B.load_library().dsq_soft_quantize_fwd(x.data_ptr(), n + 1, l, u, alpha, bits, y.data_ptr(), None))
    assert e.value.status == 4


def test_special_values():
    l, u, alpha, bits = -1.0, 2.0, 0.2, 3
    d = (u - l) / 7
    x = torch.tensor([l, u, l - 1e-3, u + 1e-3, l + d, l + 0.5 * d, l + 3 * d, -1e30, 1e30, float("inf"),
                      -float("inf")], dtype=torch.float32)
    ref = S.forward(x.numpy().astype(np.float64), np.float32(l), np.float32(u), np.float32(alpha), bits)
    got = run_fwd(x, l, u, alpha, bits)
    assert np.abs(got - ref).max() <= 4e-6
    nan = run_fwd(torch.tensor([float("nan")] * 4), l, u, alpha, bits)
    assert np.isnan(nan).all()
    gx, sums = run_bwd(x, torch.ones_like(x), l, u, alpha, bits)
    dx, da, dl, du = S.partials(x.numpy().astype(np.float64), np.float32(l), np.float32(u), np.float32(alpha), bits)
    assert np.abs(gx - dx).max() <= 1e-5 * max(1.0, np.abs(dx).max())
    assert abs(sums[1] - dl.sum()) <= 1e-5 * np.abs(dl).sum() and abs(sums[2] - du.sum()) <= 1e-5 * np.abs(du).sum()


def test_argument_errors():
    x = torch.zeros(16, device="cuda")
    y = torch.zeros(16, device="cuda")
    sums = torch.zeros(4, dtype=torch.float64, device="cuda")
    for args, status in (((x, 0.0, 1.0, 0.5, 4, y), 3), ((x, 0.0, 1.0, 0.0, 4, y), 3), ((x, 1.0, 1.0, 0.2, 4, y), 3),
                         ((x, 0.0, 1.0, 0.2, 5, y), 2), ((x, 0.0, 1.0, 0.2, 4, None), 1)):
        with pytest.raises(B.DsqError) as e:
            B.dsq_soft_quantize_fwd(*args)
        assert e.value.status == status
    with pytest.raises(B.DsqError) as e:
        B.dsq_soft_quantize_bwd(x, y, 0.0, 1.0, 0.2, 4, y, None)
    assert e.value.status == 1
    with pytest.raises(B.DsqError) as e:
        B.dsq_soft_quantize_bwd(x, y, 0.0, 1.0, 0.7, 4, y, sums)
    assert e.value.status == 3
