"""The streaming formulation of the loss in fp64, for tiny inputs only (Python
loops over vocabulary entries).

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE: it exists to pin
``flce_oracle`` (the two-stage definition) against the streaming formulation
the paper claims is equivalent to it, independently of any GPU code.

The paper's forward (Alg. 1) never holds a row of logits: it carries, per
position, a pair (m, a) with the meaning

    m = max of the logits seen so far,   a = sum over them of exp(z - m),

so that m + log(a) is the log-sum-exp of what has been seen.  Everything here
is written from that meaning.  Two such summaries of disjoint sets of logits
combine into the summary of their union,

    M = max(m1, m2),   A = a1 * exp(m1 - M) + a2 * exp(m2 - M),

with (-inf, 0) (nothing seen) as the neutral element.  One more logit is the
summary (z, 1) combined in; the windows of Section 3.2.1 are summaries of
parts of the vocabulary combined in order, which is the reading taken for the
merging step the paper asks for but does not print.  The backward (Alg. 2)
turns each logit, recomputed, into a probability with the pair it kept,
p = exp(z - m) / a, and accumulates Gamma * (p - [v == y]) times the other
factor into the two gradients; Alg. 3 is that sweep with Gamma left out,
Alg. 4 the multiplication by Gamma afterwards.

Targets are 0-based here (the paper's are 1-based).  Every position counts,
exactly as in the paper: the ignore mask is not part of these algorithms.
"""
from __future__ import annotations

import math

import numpy as np

NOTHING = (-math.inf, 0.0)        # summary of no logits at all


def combine(s1, s2):
    """Summary (m, a) of the union of two disjoint sets of logits."""
    (m1, a1), (m2, a2) = s1, s2
    if a1 == 0.0:
        return (m2, a2)
    if a2 == 0.0:
        return (m1, a1)
    M = max(m1, m2)
    return (M, a1 * math.exp(m1 - M) + a2 * math.exp(m2 - M))


def logit(h, w):
    """One entry of Eq. 1: the inner product of a hidden state and a vocabulary row."""
    return math.fsum(float(a) * float(b) for a, b in zip(h, w))


def stream_row(h, W, target, v_begin=0, v_end=None):
    """One position's pass over the vocabulary entries [v_begin, v_end), one logit at a time:
    returns (m, a, z_target, found), found = the target lies in the range."""
    v_end = len(W) if v_end is None else v_end
    state, zt, found = NOTHING, 0.0, False
    for v in range(v_begin, v_end):
        z = logit(h, W[v])
        state = combine(state, (z, 1.0))
        if v == target:
            zt, found = z, True
    return state[0], state[1], zt, found


def closing_steps_as_printed(m, a, zt):
    """The last steps of Alg. 1 exactly as the paper prints them: the denominator s = exp(m) * a, then
    -log(exp(z_t) / s).  Overflows once |m| or |z_t| passes about 709; equal to m + log(a) - z_t below that."""
    s = math.exp(m) * a
    return -math.log(math.exp(zt) / s)


def alg1_forward(H, W, y, as_printed=False):
    """Alg. 1.  Returns (loss, m[N], a[N]): the mean over all positions of log-sum-exp minus target logit, and
    the pair each position ends with."""
    N = len(H)
    rows = [stream_row(H[i], W, int(y[i])) for i in range(N)]
    if as_printed:
        per_row = [closing_steps_as_printed(m, a, zt) for m, a, zt, _ in rows]
    else:
        per_row = [m + math.log(a) - zt for m, a, zt, _ in rows]
    return math.fsum(per_row) / N, np.array([r[0] for r in rows]), np.array([r[1] for r in rows])


def alg2_backward(H, W, y, m, a, Gamma):
    """Alg. 2 with the pairs (m, a) the forward kept.  ``Gamma`` is a scalar or one value per position."""
    H, W = np.asarray(H, dtype=np.float64), np.asarray(W, dtype=np.float64)
    N, V = len(H), len(W)
    Gam = np.broadcast_to(np.asarray(Gamma, dtype=np.float64), (N,))
    dH, dW = np.zeros_like(H), np.zeros_like(W)
    for i in range(N):
        for v in range(V):
            p = math.exp(logit(H[i], W[v]) - m[i]) / a[i]
            g = Gam[i] * (p - (v == int(y[i])))
            dH[i] += g * W[v]
            dW[v] += g * H[i]
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
    """Per-window (m, a, z_target, found) tuples of one row, combined in window order: (lse, z_target)."""
    state, zt = NOTHING, 0.0
    for m, a, z, found in parts:
        state = combine(state, (m, a))
        if found:
            zt = z
    return state[0] + math.log(state[1]), zt
