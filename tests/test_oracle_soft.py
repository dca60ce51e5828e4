"""Pins of the training-mode oracle (oracle/dsq_soft.py): the properties the
paper states for the DSQ function, its limits, automatic differentiation of an
independently written expression, finite differences, and two invariances."""
import numpy as np
import pytest
import torch

import oracle
from oracle import dsq_soft as S

CASES = [  # l, u, alpha, bits
    (-1.0, 2.0, 0.2, 2),
    (0.0, 3.0, 0.05, 4),
    (-0.7, 0.9, 0.45, 3),
    (0.0, 1.0, 0.2, 1),           # one interval: the binary special case (Sec. 3.2, Fig. 2b)
    (0.0, 0.01, 0.2, 4),          # Delta so small that k = log(2/alpha-1)/Delta would exceed 1000
]


def grid(l, u, bits):
    L = (1 << bits) - 1
    d = (u - l) / L
    return d, L


@pytest.mark.parametrize("l,u,alpha,bits", CASES)
def test_properties_stated_in_the_paper(l, u, alpha, bits):
    d, L = grid(l, u, bits)
    delta, k, s, capped = S.shape_parameters(l, u, alpha, bits)
    assert capped == (np.log(2 / alpha - 1) / d > 1000) and k <= 1000
    # Sec. 3.3: alpha = 1 - tanh(0.5 k Delta) = 1 - 1/s (while k is not capped)
    if not capped:
        assert abs((1 - np.tanh(0.5 * k * delta)) - alpha) < 1e-12 and abs(s - 1 / (1 - alpha)) < 1e-12
    # Sec. 3.2: s makes phi reach -1 / +1 at the ends of every interval, so Q_S passes
    # through the grid points l + i*Delta and is continuous there; Q_S(m_i) = m_i
    eps = 1e-9 * d
    for i in range(L):
        lo, hi, mid = l + i * d, l + (i + 1) * d, l + (i + 0.5) * d
        y = S.forward(np.array([lo + eps, hi - eps, mid]), l, u, alpha, bits)
        assert abs(y[0] - lo) < 1e-6 * d and abs(y[1] - hi) < 1e-6 * d and abs(y[2] - mid) < 1e-12
    # the outer cases
    assert np.abs(S.forward(np.array([l - 1.0, u + 1.0, l, u]), l, u, alpha, bits) - [l, u, l, u]).max() < 1e-12
    # monotone, and within half an interval of x inside the range
    x = np.linspace(l - 0.1, u + 0.1, 20001)
    y = S.forward(x, l, u, alpha, bits)
    assert np.all(np.diff(y) >= -1e-12)
    inside = (x >= l) & (x <= u)
    assert np.abs(y - x)[inside].max() <= 0.5 * d + 1e-9


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_sign_of_phi_and_small_alpha_give_the_hard_quantizer(bits):
    """Sec. 3.2: phi followed by sgn is the uniform quantizer; as alpha -> 0 the
    soft curve itself approaches it.  The hard quantizer is the deployment
    oracle's binary32 recipe (pinned separately)."""
    l, u = -0.5, 1.75
    d, L = grid(l, u, bits)
    rng = np.random.default_rng(bits)
    x = rng.uniform(l - 0.2, u + 0.2, 5000).astype(np.float32).astype(np.float64)
    frac = ((x - l) / d) % 1.0
    x = x[np.abs(frac - 0.5) > 0.02]                     # away from the midpoints
    hard = oracle.dequantize(oracle.quantize(x.astype(np.float32), l, u, bits), l, u, bits)
    delta, k, s, _ = S.shape_parameters(l, u, 0.2, bits)
    i = S.interval_index(x, l, u, bits)
    phi = s * np.tanh(k * (x - (l + (i + 0.5) * d)))
    via_sign = l + d * (i + (np.where(phi >= 0, 1.0, -1.0) + 1) / 2)
    via_sign = np.where(x < l, l, np.where(x > u, u, via_sign))
    assert np.abs(via_sign - hard).max() < 1e-6
    # (the approach is only logarithmic in alpha: compare away from the midpoints)
    far = np.abs((((x - l) / d) % 1.0) - 0.5) > 0.3
    soft = S.forward(x[far], l, u, 1e-12, bits)
    assert np.abs(soft - hard[far]).max() < 1e-6 * d


def torch_forward(x, l, u, alpha, bits):
    """The same function typed again with torch ops, for automatic differentiation."""
    L = float((1 << bits) - 1)
    delta = (u - l) / L
    k = torch.clamp(torch.log(2.0 / alpha - 1.0) / delta, max=1000.0)
    s = 1.0 / torch.tanh(0.5 * k * delta)
    i = torch.clamp(torch.floor((x - l) / delta), 0, L - 1).detach()
    m = l + (i + 0.5) * delta
    y = l + delta * (i + 0.5 * (s * torch.tanh(k * (x - m)) + 1.0))
    return torch.where(x < l, l + 0 * x, torch.where(x > u, u + 0 * x, y))


@pytest.mark.parametrize("l,u,alpha,bits", CASES)
def test_partials_against_autograd_and_finite_differences(l, u, alpha, bits):
    d, L = grid(l, u, bits)
    rng = np.random.default_rng(7)
    x = rng.uniform(l - 0.3 * (u - l), u + 0.3 * (u - l), 400)
    frac = ((x - l) / d) % 1.0
    x = x[(frac > 0.02) & (frac < 0.98)]
    dx, da, dl, du = S.partials(x, l, u, alpha, bits)
    assert np.allclose(S.forward(x, l, u, alpha, bits),
                       torch_forward(torch.tensor(x), torch.tensor(l, dtype=torch.float64),
                                     torch.tensor(u, dtype=torch.float64),
                                     torch.tensor(alpha, dtype=torch.float64), bits).numpy(), rtol=0, atol=1e-12)
    # automatic differentiation, one element at a time for the three parameters
    xt = torch.tensor(x, requires_grad=True)
    lt, ut, at = (torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in (l, u, alpha))
    y = torch_forward(xt, lt, ut, at, bits)
    (gx,) = torch.autograd.grad(y.sum(), xt, retain_graph=True)
    scale = max(1.0, np.abs(dx).max())
    assert np.abs(gx.numpy() - dx).max() < 1e-9 * scale
    for j in range(0, len(x), 7):
        ga, gl, gu = torch.autograd.grad(y[j], (at, lt, ut), retain_graph=True)
        for got, want in ((da[j], ga), (dl[j], gl), (du[j], gu)):
            assert abs(got - float(want)) < 1e-8 * max(1.0, abs(float(want)))
    # central differences in float64
    h = 1e-6 * (u - l)
    fd = lambda f: (f(+1) - f(-1))
    fdx = fd(lambda sgn: S.forward(x + sgn * h, l, u, alpha, bits)) / (2 * h)
    fdl = fd(lambda sgn: S.forward(x, l + sgn * h, u, alpha, bits)) / (2 * h)
    fdu = fd(lambda sgn: S.forward(x, l, u + sgn * h, alpha, bits)) / (2 * h)
    ha = 1e-5 * alpha
    fda = fd(lambda sgn: S.forward(x, l, u, alpha + sgn * ha, bits)) / (2 * ha)
    for got, want in ((dx, fdx), (da, fda), (dl, fdl), (du, fdu)):
        assert np.abs(got - want).max() < 2e-5 * max(1.0, np.abs(want).max())


@pytest.mark.parametrize("l,u,alpha,bits", CASES)
def test_invariances_and_outer_cases(l, u, alpha, bits):
    """Shifting x, l, u together shifts Q_S by the same amount, and scaling them
    scales it: dy/dx + dy/dl + dy/du = 1 and x*dy/dx + l*dy/dl + u*dy/du = y.
    Outside the range only the clipped bound receives gradient (Sec. 3.4)."""
    rng = np.random.default_rng(3)
    x = rng.uniform(l - 0.3 * (u - l), u + 0.3 * (u - l), 3000)
    dx, da, dl, du = S.partials(x, l, u, alpha, bits)
    y = S.forward(x, l, u, alpha, bits)
    assert np.abs(dx + dl + du - 1).max() < 1e-9
    if not S.shape_parameters(l, u, alpha, bits)[3]:      # a capped k is an absolute constant: no scaling law
        assert np.abs(x * dx + l * dl + u * du - y).max() < 1e-9 * max(1.0, abs(l), abs(u))
    lo, hi = x < l, x > u
    assert lo.any() and hi.any()
    assert not dx[lo | hi].any() and not da[lo | hi].any()
    assert np.all(dl[lo] == 1) and np.all(du[lo] == 0) and np.all(dl[hi] == 0) and np.all(du[hi] == 1)
    # continuously differentiable across interval ends (Sec. 3.2)
    d, L = grid(l, u, bits)
    for i in range(1, L):
        b = l + i * d
        left, right = S.partials(np.array([b - 1e-9 * d, b + 1e-9 * d]), l, u, alpha, bits)[0]
        assert abs(left - right) < 1e-5 * max(1.0, abs(left))


def test_backward_sums():
    rng = np.random.default_rng(5)
    x = rng.normal(0.5, 1.0, 1000)
    g = rng.normal(0, 1, 1000)
    gx, ga, gl, gu = S.backward(x, g, -1.0, 2.0, 0.2, 3)
    dx, da, dl, du = S.partials(x, -1.0, 2.0, 0.2, 3)
    assert np.array_equal(gx, g * dx)
    assert abs(ga - np.dot(g, da)) < 1e-9 and abs(gl - np.dot(g, dl)) < 1e-9 and abs(gu - np.dot(g, du)) < 1e-9
