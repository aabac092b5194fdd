"""torch.autograd front end of libflce: hidden states and vocabulary weights in, loss out, gradients through
``backward()``.  Plumbing only: every step of the computation runs inside the library's kernels; torch holds the
tensors, names the stream and chains the autograd graph.

    loss = linear_cross_entropy(H, W, targets)                       # mean over counted rows
    rows = linear_cross_entropy(H, W, targets, reduction="none")     # one loss per row
    loss.backward()                                                   # H.grad, W.grad

H is [..., d] (leading dimensions are flattened to N rows), W is [V, d], both bf16 or both fp32, contiguous, on the
same GPU; targets are int64 with the leading shape of H.  The N x V logits are never formed.
"""
from __future__ import annotations

import torch

from . import binding as B

_DT = {torch.bfloat16: B.FLCE_DTYPE_BF16, torch.float32: B.FLCE_DTYPE_F32}
_RED = {"mean": B.FLCE_REDUCE_MEAN, "sum": B.FLCE_REDUCE_SUM}


def _check(rc):
    if rc != B.FLCE_OK:
        raise RuntimeError(f"libflce: {B.flce_status_string(rc)}")


def _prepare(H, W, targets):
    if H.dtype not in _DT or W.dtype != H.dtype:
        raise TypeError("H and W must both be bfloat16 or both float32")
    if not (H.is_cuda and W.is_cuda and targets.is_cuda):
        raise ValueError("libflce works on GPU tensors only")
    H2 = H.reshape(-1, H.shape[-1]).contiguous()
    W2 = W.contiguous()
    y = targets.reshape(-1).to(torch.int64).contiguous()
    if y.numel() != H2.shape[0] or W2.shape[1] != H2.shape[1]:
        raise ValueError("shapes: H [..., d], W [V, d], targets [...]")
    return H2, W2, y


def _workspace(N, d, V, dt, backward, device):
    nb = B.flce_workspace_bytes(N, d, V, dt, backward)
    if nb == 0:
        raise ValueError("unsupported shape (d must be a multiple of 8)")
    return torch.empty(nb, dtype=torch.uint8, device=device), nb


class _ScalarLoss(torch.autograd.Function):
    """Alg. 1 forward, Alg. 2 backward; mean or sum over the counted rows."""

    @staticmethod
    def forward(ctx, H, W, targets, ignore_index, reduction):
        H2, W2, y = _prepare(H, W, targets)
        N, d = H2.shape
        V = W2.shape[0]
        dt = _DT[H2.dtype]
        st = torch.cuda.current_stream(H2.device)
        loss = torch.empty(1, dtype=torch.float32, device=H2.device)
        lse = torch.empty(N, dtype=torch.float32, device=H2.device)
        ws, nb = _workspace(N, d, V, dt, 0, H2.device)
        _check(B.flce_forward(H2, W2, y, N, d, V, ignore_index, _RED[reduction], dt, loss, lse, ws, nb, st))
        ctx.save_for_backward(H2, W2, y, lse)
        ctx.meta = (H.shape, ignore_index, reduction)
        return loss[0]

    @staticmethod
    def backward(ctx, grad_out):
        H2, W2, y, lse = ctx.saved_tensors
        shape, ignore_index, reduction = ctx.meta
        N, d = H2.shape
        V = W2.shape[0]
        dt = _DT[H2.dtype]
        st = torch.cuda.current_stream(H2.device)
        dH = torch.empty_like(H2)
        dW = torch.empty_like(W2)
        ws, nb = _workspace(N, d, V, dt, 1, H2.device)
        # the library takes the upstream gradient as a host scalar: reading it waits for the stream
        g = float(grad_out)
        _check(B.flce_backward(H2, W2, y, lse, N, d, V, ignore_index, _RED[reduction], dt, g, dH, dW, ws, nb, st))
        return dH.reshape(shape), dW, None, None, None


class _RowLosses(torch.autograd.Function):
    """One loss per row (optionally label-smoothed); the backward takes one upstream gradient per row."""

    @staticmethod
    def forward(ctx, H, W, targets, ignore_index, label_smoothing):
        H2, W2, y = _prepare(H, W, targets)
        N, d = H2.shape
        V = W2.shape[0]
        dt = _DT[H2.dtype]
        st = torch.cuda.current_stream(H2.device)
        rows = torch.empty(N, dtype=torch.float32, device=H2.device)
        lse = torch.empty(N, dtype=torch.float32, device=H2.device)
        ws, nb = _workspace(N, d, V, dt, 0, H2.device)
        _check(B.flce_forward_rows(H2, W2, y, N, d, V, ignore_index, label_smoothing, dt, rows, lse, ws, nb, st))
        ctx.save_for_backward(H2, W2, y, lse)
        ctx.meta = (H.shape, ignore_index, label_smoothing)
        return rows.reshape(targets.shape)

    @staticmethod
    def backward(ctx, grad_rows):
        H2, W2, y, lse = ctx.saved_tensors
        shape, ignore_index, label_smoothing = ctx.meta
        N, d = H2.shape
        V = W2.shape[0]
        dt = _DT[H2.dtype]
        st = torch.cuda.current_stream(H2.device)
        dH = torch.empty_like(H2)
        dW = torch.empty_like(W2)
        gr = grad_rows.reshape(-1).to(torch.float32).contiguous()
        ws, nb = _workspace(N, d, V, dt, 1, H2.device)
        _check(B.flce_backward_rows(H2, W2, y, lse, gr, N, d, V, ignore_index, label_smoothing, dt, dH, dW, ws, nb,
                                    st))
        return dH.reshape(shape), dW, None, None, None


def linear_cross_entropy(H, W, targets, ignore_index=-100, reduction="mean", label_smoothing=0.0):
    """Cross-entropy of softmax(H . W^T) against `targets` without the logits tensor.

    reduction: "mean" (over rows whose target is not `ignore_index`), "sum" or "none".  Label smoothing comes
    with one loss per row only (reduction="none", the library's per-row call): reduce the rows with torch as
    needed, autograd hands the per-row upstream gradients back to the library.
    """
    if reduction not in ("mean", "sum", "none"):
        raise ValueError("reduction must be 'mean', 'sum' or 'none'")
    if reduction != "none":
        if label_smoothing != 0.0:
            raise ValueError("label smoothing is available with reduction='none' only")
        return _ScalarLoss.apply(H, W, targets, int(ignore_index), reduction)
    return _RowLosses.apply(H, W, targets, int(ignore_index), float(label_smoothing))
