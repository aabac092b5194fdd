"""CPU fp64 oracle for the fused projection + cross-entropy path.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke
check and the benchmark's ``cpu_baseline`` leg may import it.  It shares no
code with the HIP path and never calls it.

What it computes is the plain two-stage pipeline the paper says its fused
method is exactly equivalent to (Section 3.1 and the equivalence claim at the
end of Section 3.2's first paragraph; "exact gradients" in Appendix A.1):

    Z      = H . W^T                                        (Eq. 1)
    lse_i  = log sum_v exp(Z_iv)                            (denominator of Eq. 2)
    loss_i = lse_i - Z_{i, y_i}                             (Eq. 2 / Eq. 3, one row)
    loss   = sum_i loss_i / n_valid   (mean)   or   sum_i loss_i   (sum)
    G_iv   = Gamma * (exp(Z_iv - lse_i) - [v == y_i])       (Appendix A.1, dL/dz)
    dH     = G . W                                          (Eq. 4)
    dW     = G^T . H                                        (Eq. 5)

with Gamma = grad_loss / n_valid for the mean and grad_loss for the sum (the
"upstream gradient" input of Alg. 2).  The logits ARE materialised here, on
purpose.  All arithmetic is IEEE fp64; numpy's matmul is the only library
primitive used as a step.

Readings taken where the paper is silent:
  * targets are 0-based, in [0, V) (the paper writes {1..V});
  * rows whose target equals ``ignore_index`` contribute loss 0, a zero row of
    G, and are left out of the mean's denominator;
  * a non-ignored target outside [0, V) is an input error: the row is treated
    as ignored and ``out_of_range`` is reported;
  * n_valid == 0 gives loss 0 and zero gradients;
  * the denominator is evaluated as max + log(sum exp(z - max)) rather than
    exp(m) * a, which overflows as printed (Alg. 1's last two steps).

Rows are processed in blocks only to bound the size of the materialised Z;
each row's result is independent of the blocking, dW is the sum of the
per-block G^T . H products.

Every public function here is pinned by tests/test_oracle_pins.py (closed
forms, invariants, finite differences, an independent scalar transcription of
Alg. 1/2, and the fp64 log-softmax/NLL of two numerical libraries; the
label-smoothed per-row variant also by a library's own label-smoothed loss).
"""
from __future__ import annotations

import numpy as np

MEAN = "mean"
SUM = "sum"


def _f64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def classify_targets(y, V, ignore_index):
    """Integer facts about the targets: which rows count, how many, any bad id.

    Returns (valid[N] bool, n_valid int, out_of_range bool).  The ignore test
    comes first, so ``ignore_index`` may be any int64, inside [0, V) included.
    """
    y = np.asarray(y, dtype=np.int64)
    not_ignored = y != np.int64(ignore_index)
    in_range = (y >= 0) & (y < V)
    valid = not_ignored & in_range
    out_of_range = bool(np.any(not_ignored & ~in_range))
    return valid, int(valid.sum()), out_of_range


def gamma(n_valid, reduction, grad_loss=1.0):
    """Scalar upstream gradient of every counted row (Alg. 2's Gamma)."""
    if reduction == MEAN:
        return 0.0 if n_valid == 0 else float(grad_loss) / float(n_valid)
    if reduction == SUM:
        return float(grad_loss)
    raise ValueError("reduction must be 'mean' or 'sum'")


def row_stats(H_rows, W, y_rows, valid_rows):
    """lse, target logit and per-row loss of the given rows (Eq. 1, Eq. 2).

    ``valid_rows`` marks rows that count; others get zt = 0 and loss 0 but
    still get their lse.
    """
    H_rows, W = _f64(H_rows), _f64(W)
    Z = H_rows @ W.T                                   # Eq. 1, materialised
    mx = Z.max(axis=1)
    lse = mx + np.log(np.exp(Z - mx[:, None]).sum(axis=1))
    zt = np.zeros(len(H_rows))
    idx = np.nonzero(valid_rows)[0]
    zt[idx] = Z[idx, np.asarray(y_rows, dtype=np.int64)[idx]]
    loss_rows = np.where(valid_rows, lse - zt, 0.0)
    return lse, zt, loss_rows


def forward(H, W, y, ignore_index=-100, reduction=MEAN, block_rows=1024):
    """Two-stage loss.  Returns a dict: loss, lse[N], loss_rows[N], n_valid,
    valid[N], out_of_range."""
    H, W = _f64(H), _f64(W)
    N, V = H.shape[0], W.shape[0]
    y = np.asarray(y, dtype=np.int64)
    valid, n_valid, oor = classify_targets(y, V, ignore_index)
    lse = np.empty(N)
    loss_rows = np.empty(N)
    for r0 in range(0, N, block_rows):
        r1 = min(N, r0 + block_rows)
        lse[r0:r1], _, loss_rows[r0:r1] = row_stats(H[r0:r1], W, y[r0:r1], valid[r0:r1])
    total = float(loss_rows.sum())
    if reduction == MEAN:
        loss = 0.0 if n_valid == 0 else total / n_valid
    elif reduction == SUM:
        loss = total
    else:
        raise ValueError("reduction must be 'mean' or 'sum'")
    return dict(loss=loss, lse=lse, loss_rows=loss_rows, n_valid=n_valid,
                valid=valid, out_of_range=oor)


def grad_logits(H_rows, W, y_rows, valid_rows, gam):
    """G for the given rows: Gamma * (softmax(Z) - onehot), zero on rows that
    do not count (Appendix A.1; Alg. 2's p_v and g_v)."""
    H_rows, W = _f64(H_rows), _f64(W)
    Z = H_rows @ W.T
    mx = Z.max(axis=1, keepdims=True)
    E = np.exp(Z - mx)
    P = E / E.sum(axis=1, keepdims=True)
    idx = np.nonzero(valid_rows)[0]
    P[idx, np.asarray(y_rows, dtype=np.int64)[idx]] -= 1.0
    P[~np.asarray(valid_rows, dtype=bool)] = 0.0
    return gam * P


def backward(H, W, y, ignore_index=-100, reduction=MEAN, grad_loss=1.0, block_rows=1024):
    """Analytic gradients.  Returns a dict: dH[N,d], dW[V,d], gamma, n_valid."""
    H, W = _f64(H), _f64(W)
    N, V = H.shape[0], W.shape[0]
    y = np.asarray(y, dtype=np.int64)
    valid, n_valid, _ = classify_targets(y, V, ignore_index)
    gam = gamma(n_valid, reduction, grad_loss)
    dH = np.zeros_like(H)
    dW = np.zeros_like(W)
    for r0 in range(0, N, block_rows):
        r1 = min(N, r0 + block_rows)
        G = grad_logits(H[r0:r1], W, y[r0:r1], valid[r0:r1], gam)
        dH[r0:r1] = G @ W                              # Eq. 4
        dW += G.T @ H[r0:r1]                           # Eq. 5
    return dict(dH=dH, dW=dW, gamma=gam, n_valid=n_valid)


# ---------------------------------------------------------------------------
# Per-position upstream gradients and label smoothing.
#
# Alg. 2 takes an upstream gradient Gamma that may differ per position (the
# non-scalar branch of Alg. 4 says the same); with one loss value per row
# ("no reduction") that is the natural interface.  Label smoothing is the loss
# variant the Discussion names.  The paper gives no formula for it; the reading
# taken is the usual one: the target distribution of a counted row is
#     q_v = (1 - eps) [v == y_i] + eps / V,
#     loss_i = - sum_v q_v log softmax(Z_i)_v
#            = (1 - eps) (lse_i - Z_{i,y_i}) + eps (lse_i - mean_v Z_iv),
#     dloss_i / dZ_iv = softmax(Z_i)_v - q_v,
# which is Eq. 2 and Appendix A.1 for eps = 0.
# ---------------------------------------------------------------------------

def forward_per_row(H, W, y, ignore_index=-100, label_smoothing=0.0, block_rows=1024):
    """One loss value per row (0 for rows that do not count) and every row's
    lse.  Returns a dict: loss_rows[N], lse[N], valid[N], n_valid, out_of_range."""
    H, W = _f64(H), _f64(W)
    N, V = H.shape[0], W.shape[0]
    eps = float(label_smoothing)
    y = np.asarray(y, dtype=np.int64)
    valid, n_valid, oor = classify_targets(y, V, ignore_index)
    lse = np.empty(N)
    loss_rows = np.zeros(N)
    for r0 in range(0, N, block_rows):
        r1 = min(N, r0 + block_rows)
        Z = H[r0:r1] @ W.T
        mx = Z.max(axis=1)
        lse[r0:r1] = mx + np.log(np.exp(Z - mx[:, None]).sum(axis=1))
        logp = Z - lse[r0:r1, None]                    # log softmax, materialised
        idx = np.nonzero(valid[r0:r1])[0]
        nll = -logp[idx, y[r0:r1][idx]]
        uniform = -logp[idx].mean(axis=1)
        loss_rows[r0 + idx] = (1.0 - eps) * nll + eps * uniform
    return dict(loss_rows=loss_rows, lse=lse, valid=valid, n_valid=n_valid, out_of_range=oor)


def backward_per_row(H, W, y, grad_rows, ignore_index=-100, label_smoothing=0.0, block_rows=1024):
    """Gradients of sum_i grad_rows[i] * loss_i: G_iv = grad_rows[i] * (softmax(Z_i)_v - q_v) on
    counted rows, 0 elsewhere; dH = G . W (Eq. 4), dW = G^T . H (Eq. 5)."""
    H, W = _f64(H), _f64(W)
    N, V = H.shape[0], W.shape[0]
    eps = float(label_smoothing)
    y = np.asarray(y, dtype=np.int64)
    gr = _f64(grad_rows)
    valid, n_valid, _ = classify_targets(y, V, ignore_index)
    dH = np.zeros_like(H)
    dW = np.zeros_like(W)
    for r0 in range(0, N, block_rows):
        r1 = min(N, r0 + block_rows)
        Z = H[r0:r1] @ W.T
        mx = Z.max(axis=1, keepdims=True)
        E = np.exp(Z - mx)
        G = E / E.sum(axis=1, keepdims=True)
        G -= eps / V
        idx = np.nonzero(valid[r0:r1])[0]
        G[idx, y[r0:r1][idx]] -= 1.0 - eps
        G[~valid[r0:r1]] = 0.0
        G *= gr[r0:r1, None]
        dH[r0:r1] = G @ W
        dW += G.T @ H[r0:r1]
    return dict(dH=dH, dW=dW, n_valid=n_valid)


# ---------------------------------------------------------------------------
# Row- and vocabulary-sampled entry points, for shapes where the full pipeline
# (3*N*d*V fp64 multiply-adds) does not finish in seconds.  Each returns exactly
# what the full functions above would return at the sampled positions.
# ---------------------------------------------------------------------------

def forward_rows(H_rows, W, y_rows, ignore_index=-100):
    """lse, zt, loss_rows for a subset of rows (rows are independent in Eq. 2)."""
    V = np.asarray(W).shape[0]
    valid, _, _ = classify_targets(y_rows, V, ignore_index)
    return row_stats(H_rows, W, y_rows, valid)


def dH_rows(H_rows, W, y_rows, gam, ignore_index=-100):
    """Rows of dH for a subset of rows (Eq. 4 touches only row i of H)."""
    V = np.asarray(W).shape[0]
    valid, _, _ = classify_targets(y_rows, V, ignore_index)
    return grad_logits(H_rows, W, y_rows, valid, gam) @ _f64(W)


def dW_rows(H, W_rows, vocab_ids, y, lse, gam, ignore_index=-100, V=None, block_rows=4096):
    """Rows ``vocab_ids`` of dW (Eq. 5), given every row's lse from this
    oracle's own forward.  ``W_rows`` = W[vocab_ids]; V is the full vocabulary
    size (needed only to classify the targets)."""
    H, W_rows = _f64(H), _f64(W_rows)
    vocab_ids = np.asarray(vocab_ids, dtype=np.int64)
    y = np.asarray(y, dtype=np.int64)
    lse = _f64(lse)
    V = int(V if V is not None else vocab_ids.max() + 1)
    valid, _, _ = classify_targets(y, V, ignore_index)
    out = np.zeros_like(W_rows)
    for r0 in range(0, H.shape[0], block_rows):
        r1 = min(H.shape[0], r0 + block_rows)
        Zs = H[r0:r1] @ W_rows.T
        G = np.exp(Zs - lse[r0:r1, None])
        G -= (y[r0:r1, None] == vocab_ids[None, :])
        G[~valid[r0:r1]] = 0.0
        out += (gam * G).T @ H[r0:r1]
    return out
