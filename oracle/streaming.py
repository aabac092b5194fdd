"""Scalar, one-logit-at-a-time fp64 renditions of the paper's streaming
algorithms, for tiny inputs only (pure Python loops).

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE: it exists to pin
``flce_oracle`` (the two-stage definition) against the streaming formulation
the paper claims is equivalent to it, independently of any GPU code.

  * ``alg1_forward``   - Alg. 1: running maximum m, accumulator a relative to
                         it, and the target logit, per position; loss summed
                         and divided by the number of positions.
  * ``alg2_backward``  - Alg. 2: logits recomputed, p = exp(z - m) / a,
                         g = Gamma * (p - [v == y]), rank-one updates of the
                         row of dH and of the row of dW.
  * ``alg3_forward_partial`` / ``alg4_scale`` - Alg. 3 and 4: unscaled
                         gradients produced next to the loss, then multiplied
                         by the scalar upstream gradient.
  * ``merge_windows``  - the epilogue Section 3.2.1 asks for when the
                         vocabulary loop is cut into windows; the paper does
                         not print it, the log-sum-exp merge is the reading
                         taken.

Targets are 0-based here (the paper's are 1-based).  Every position counts,
exactly as in the paper: the ignore mask is not part of these algorithms.
"""
from __future__ import annotations

import math

import numpy as np


def _dot(h, w):
    s = 0.0
    for k in range(len(h)):
        s += float(h[k]) * float(w[k])
    return s


def stream_row(h, W, target, v_begin=0, v_end=None):
    """Inner vocabulary loop of Alg. 1 over [v_begin, v_end): returns
    (m, a, z_target, found)."""
    v_end = len(W) if v_end is None else v_end
    m, a, zt, found = -math.inf, 0.0, 0.0, False
    for v in range(v_begin, v_end):
        z = _dot(h, W[v])
        if z > m:
            a = a * math.exp(m - z) + 1.0
            m = z
        else:
            a = a + math.exp(z - m)
        if v == target:
            zt, found = z, True
    return m, a, zt, found


def alg1_forward(H, W, y, as_printed=False):
    """Alg. 1.  Returns (loss, m[N], a[N]).

    ``as_printed`` evaluates the last two steps literally, s = exp(m) * a and
    L -= log(exp(z_t) / s); the default uses the algebraically equal
    m + log(a) - z_t, which cannot overflow.
    """
    N = len(H)
    L = 0.0
    ms, As = np.empty(N), np.empty(N)
    for i in range(N):
        m, a, zt, _ = stream_row(H[i], W, int(y[i]))
        if as_printed:
            s = math.exp(m) * a
            L -= math.log(math.exp(zt) / s)
        else:
            L += m + math.log(a) - zt
        ms[i], As[i] = m, a
    return L / N, ms, As


def alg2_backward(H, W, y, m, a, Gamma):
    """Alg. 2.  ``Gamma`` is a scalar or one value per position."""
    N, d = np.shape(H)
    V = len(W)
    Gam = np.broadcast_to(np.asarray(Gamma, dtype=np.float64), (N,))
    dH = np.zeros((N, d))
    dW = np.zeros((V, d))
    for i in range(N):
        for v in range(V):
            z = _dot(H[i], W[v])
            p = math.exp(z - m[i]) / a[i]
            g = Gam[i] * (p - (1.0 if v == int(y[i]) else 0.0))
            for k in range(d):
                dH[i, k] += g * float(W[v][k])
                dW[v, k] += g * float(H[i][k])
    return dH, dW


def alg3_forward_partial(H, W, y):
    """Alg. 3: loss plus gradients not yet scaled by the upstream gradient."""
    loss, m, a = alg1_forward(H, W, y)
    dHp, dWp = alg2_backward(H, W, y, m, a, 1.0)
    return loss, dHp, dWp, m, a


def alg4_scale(dHp, dWp, Gamma):
    """Alg. 4, scalar branch."""
    return Gamma * dHp, Gamma * dWp


def merge_windows(parts):
    """Combine per-window (m, a, z_target, found) tuples of one row, in window
    order, into (lse, z_target).  A window that saw no logit carries
    (m, a) = (-inf, 0) and is the identity of the merge."""
    M = -math.inf
    for m, a, _, _ in parts:
        if a > 0.0 and m > M:
            M = m
    A, zt = 0.0, 0.0
    for m, a, z, found in parts:
        if a > 0.0:
            A += a * math.exp(m - M)
        if found:
            zt = z
    return M + math.log(A), zt
