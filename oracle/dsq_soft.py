"""TEST INFRASTRUCTURE ONLY -- plain float64 statement of the training-mode
DSQ function and its partial derivatives.

Differentiable soft quantization (paper Sec. 3.2): inside interval P_i the
asymptotic function phi(x) = s*tanh(k*(x - m_i)) with m_i = l + (i+0.5)*Delta
replaces the step of the uniform quantizer, and
    Q_S(x) = l                              x < l
             u                              x > u
             l + Delta*(i + (phi(x)+1)/2)   x in P_i
Sec. 3.3 ties the shape to the characteristic variable alpha:
    k = log(2/alpha - 1)/Delta,  s = 1/(1 - alpha) = 1/tanh(0.5*k*Delta).
Sec. 4.3 limits alpha to (0, 0.5) and k to at most 1000; when that cap is
active s is taken from its definition 1/tanh(0.5*k*Delta) so that neighbouring
intervals still join (phi = +-1 at the interval ends).

The derivatives with respect to x, alpha, l and u (Sec. 3.3 / 3.4, Algorithm 1
back-propagation) are written out from the chain rule with the interval index
held fixed, as the paper does (q = i + (phi+1)/2).  numpy, float64, no
blocking; nothing in the product path may import this module.
"""
import numpy as np

K_MAX = 1000.0


def shape_parameters(l, u, alpha, bits):
    """Delta, k, s and whether the cap on k is active."""
    levels = float((1 << bits) - 1)
    delta = (float(u) - float(l)) / levels
    k = np.log(2.0 / alpha - 1.0) / delta
    capped = k > K_MAX
    if capped:
        k = K_MAX
        s = 1.0 / np.tanh(0.5 * k * delta)
    else:
        s = 1.0 / (1.0 - alpha)
    return delta, k, s, capped


def interval_index(x, l, u, bits):
    """i with x in P_i = [l + i*Delta, l + (i+1)*Delta), the last one closed at u."""
    levels = (1 << bits) - 1
    delta = (float(u) - float(l)) / levels
    i = np.floor((x - l) / delta)
    return np.clip(i, 0, levels - 1)


def forward(x, l, u, alpha, bits):
    """Q_S(x), float64, same shape as x."""
    x = np.asarray(x, dtype=np.float64)
    delta, k, s, _ = shape_parameters(l, u, alpha, bits)
    i = interval_index(x, l, u, bits)
    m = l + (i + 0.5) * delta
    phi = s * np.tanh(k * (x - m))
    y = l + delta * (i + 0.5 * (phi + 1.0))
    return np.where(x < l, float(l), np.where(x > u, float(u), y))


def partials(x, l, u, alpha, bits):
    """(dy/dx, dy/dalpha, dy/dl, dy/du), each float64 with the shape of x."""
    x = np.asarray(x, dtype=np.float64)
    # (infinite inputs produce invalid intermediates in the branch that the final
    # selection discards)
    with np.errstate(invalid="ignore", over="ignore"):
        return _partials(x, l, u, alpha, bits)


def _partials(x, l, u, alpha, bits):
    levels = float((1 << bits) - 1)
    delta, k, s, capped = shape_parameters(l, u, alpha, bits)
    i = interval_index(x, l, u, bits)
    m = l + (i + 0.5) * delta
    t = np.tanh(k * (x - m))
    sech2 = 1.0 - t * t
    phi = s * t
    q = i + 0.5 * (phi + 1.0)

    # how k, s and m_i move with alpha, l, u (Delta_l = -1/levels, Delta_u = +1/levels)
    if capped:
        k_a = k_l = k_u = 0.0
        T = np.tanh(0.5 * k * delta)
        s_a = 0.0
        s_l = (1.0 - T * T) * k / (2.0 * levels * T * T)
        s_u = -s_l
    else:
        c = np.log(2.0 / alpha - 1.0)
        k_a = -2.0 / (alpha * (2.0 - alpha)) / delta
        k_l = c / (levels * delta * delta)
        k_u = -k_l
        s_a = 1.0 / ((1.0 - alpha) ** 2)
        s_l = s_u = 0.0
    m_l = 1.0 - (i + 0.5) / levels
    m_u = (i + 0.5) / levels

    phi_a = s_a * t + s * sech2 * (k_a * (x - m))
    phi_l = s_l * t + s * sech2 * (k_l * (x - m) - k * m_l)
    phi_u = s_u * t + s * sech2 * (k_u * (x - m) - k * m_u)

    dx = 0.5 * delta * s * sech2 * k
    da = 0.5 * delta * phi_a
    dl = 1.0 - q / levels + 0.5 * delta * phi_l
    du = q / levels + 0.5 * delta * phi_u

    below, above = x < l, x > u
    zero = np.zeros_like(x)
    dx = np.where(below | above, zero, dx)
    da = np.where(below | above, zero, da)
    dl = np.where(below, 1.0, np.where(above, 0.0, dl))
    du = np.where(below, 0.0, np.where(above, 1.0, du))
    return dx, da, dl, du


def backward(x, grad_y, l, u, alpha, bits):
    """Back-propagation of Algorithm 1 for one tensor: grad_x (float64 array) and
    the three sums (dL/dalpha, dL/dl, dL/du)."""
    g = np.asarray(grad_y, dtype=np.float64)
    dx, da, dl, du = partials(x, l, u, alpha, bits)
    return g * dx, float((g * da).sum()), float((g * dl).sum()), float((g * du).sum())
