"""Device-side plumbing around the C-ABI calls: PyTorch is used only to hold
device memory and name a stream.  Every step of the path runs inside libflce.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B

_DT = {"bf16": B.FLCE_DTYPE_BF16, "f32": B.FLCE_DTYPE_F32}
_RED = {"mean": B.FLCE_REDUCE_MEAN, "sum": B.FLCE_REDUCE_SUM}


def to_device(a, device):
    """numpy array (fp32, or uint16 bf16 bit patterns, or int64) -> device tensor, bit for bit."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(a).to(device)


def to_host_f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


class Session:
    """Holds the device buffers of one problem and calls the library on them."""

    def __init__(self, N, d, V, dtype, reduction, ignore_index, H, W, y, device="cuda:0", grad_loss=1.0):
        self.N, self.d, self.V = int(N), int(d), int(V)
        self.dt, self.red = _DT[dtype], _RED[reduction]
        self.ignore_index, self.grad_loss = int(ignore_index), float(grad_loss)
        self.device = torch.device(device)
        self.H = H if torch.is_tensor(H) else to_device(H, self.device)
        self.W = W if torch.is_tensor(W) else to_device(W, self.device)
        self.y = y if torch.is_tensor(y) else to_device(np.asarray(y, dtype=np.int64), self.device)
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        self.loss = torch.empty(1, dtype=torch.float32, device=self.device)
        self.lse = torch.empty(self.N, dtype=torch.float32, device=self.device)
        self.dH = torch.empty(self.N, self.d, dtype=tdt, device=self.device)
        self.dW = torch.empty(self.V, self.d, dtype=tdt, device=self.device)
        self.fwd_bytes = B.flce_workspace_bytes(self.N, self.d, self.V, self.dt, 0)
        self.bwd_bytes = B.flce_workspace_bytes(self.N, self.d, self.V, self.dt, 1)
        if self.fwd_bytes == 0 or self.bwd_bytes == 0:
            raise ValueError("unsupported shape")
        # one buffer serves both calls (torch allocations are 512-byte aligned)
        self.ws = torch.empty(max(self.fwd_bytes, self.bwd_bytes), dtype=torch.uint8, device=self.device)

    def stream(self):
        return torch.cuda.current_stream(self.device)

    def forward(self):
        return B.flce_forward(self.H, self.W, self.y, self.N, self.d, self.V, self.ignore_index, self.red, self.dt,
                              self.loss, self.lse, self.ws, self.fwd_bytes, self.stream())

    def backward(self):
        return B.flce_backward(self.H, self.W, self.y, self.lse, self.N, self.d, self.V, self.ignore_index, self.red,
                               self.dt, self.grad_loss, self.dH, self.dW, self.ws, self.bwd_bytes, self.stream())

    def forward_with_grads(self):
        """Alg. 3: loss, lse and the unscaled gradients (left in dH, dW)."""
        return B.flce_forward_with_grads(self.H, self.W, self.y, self.N, self.d, self.V, self.ignore_index, self.red,
                                         self.dt, self.loss, self.lse, self.dH, self.dW, self.ws, self.ws.numel(),
                                         self.stream())

    def scale(self):
        """Alg. 4: dH, dW scaled in place by the upstream gradient."""
        return B.flce_scale(self.dH, self.dW, self.N, self.d, self.V, self.red, self.dt, self.grad_loss, self.ws,
                            self.dH, self.dW, self.stream())

    def forward_rows(self, loss_rows, label_smoothing=0.0):
        """One loss per row into `loss_rows` (device, N floats)."""
        return B.flce_forward_rows(self.H, self.W, self.y, self.N, self.d, self.V, self.ignore_index, label_smoothing,
                                   self.dt, loss_rows, self.lse, self.ws, self.fwd_bytes, self.stream())

    def backward_rows(self, grad_rows, label_smoothing=0.0):
        """Gradients of sum_i grad_rows[i] * loss_i (grad_rows: device, N floats)."""
        return B.flce_backward_rows(self.H, self.W, self.y, self.lse, grad_rows, self.N, self.d, self.V,
                                    self.ignore_index, label_smoothing, self.dt, self.dH, self.dW, self.ws,
                                    self.bwd_bytes, self.stream())

    def device_status(self):
        return B.flce_last_device_status(self.ws, self.stream())

    def tensor_bytes(self):
        """Bytes of every buffer the path touches (inputs, outputs, workspace)."""
        ts = (self.H, self.W, self.y, self.loss, self.lse, self.dH, self.dW, self.ws)
        return sum(t.numel() * t.element_size() for t in ts)


def session_for(wl, x, device="cuda:0", grad_loss=1.0):
    return Session(wl.N, wl.d, wl.V, wl.dtype, wl.reduction, wl.ignore_index, x["H"], x["W"], x["y"], device,
                   grad_loss)


def run_workload(wl, x, device="cuda:0", grad_loss=1.0):
    """Forward + backward once; results as host arrays (fp64 images of what the device wrote)."""
    s = session_for(wl, x, device, grad_loss)
    st_f = s.forward()
    st_dev_f, n_valid = s.device_status()
    loss = float(s.loss.item())
    lse = to_host_f64(s.lse)
    st_b = s.backward()
    st_dev_b, n_valid_b = s.device_status()
    status = next((c for c in (st_f, st_b, st_dev_f, st_dev_b) if c != B.FLCE_OK), B.FLCE_OK)
    return dict(status=status, loss=loss, lse=lse, n_valid=n_valid, n_valid_bwd=n_valid_b,
                dH=to_host_f64(s.dH), dW=to_host_f64(s.dW), session=s)
