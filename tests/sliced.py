"""Test helper: one problem through the vocabulary-sliced calls, every slice on this one GPU in turn.  The sum of
the slices' partial dH (what a tensor-parallel group would get from its all-reduce) is formed here, on the host,
in fp64: it is the test's stand-in for the exchange, not a step of the library."""
import numpy as np
import torch

from paper_2511_17599_amd import binding as B
from paper_2511_17599_amd.runner import _DT, _RED, to_device, to_host_f64


def run_sliced(wl, x, cuts, device="cuda:0", grad_loss=1.0):
    """The same problem through the vocabulary-sliced calls: slice k is rows [cuts[k], cuts[k+1]) of W.  Every
    slice runs on this one GPU, one after the other; the partial dH are summed on the host in fp64 (the sum a
    tensor-parallel group would get from its all-reduce).  Returns host arrays like run_workload, plus the
    per-slice (m, a, z_target)."""
    dev = torch.device(device)
    dt, red = _DT[wl.dtype], _RED[wl.reduction]
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    H, W = to_device(x["H"], dev), to_device(x["W"], dev)
    y = to_device(np.asarray(x["y"], dtype=np.int64), dev)
    N, d, V = wl.N, wl.d, wl.V
    P = len(cuts) - 1
    parts = torch.empty(3, P, N, dtype=torch.float32, device=dev)
    st = torch.cuda.current_stream(dev)
    for k in range(P):
        v0, v1 = cuts[k], cuts[k + 1]
        nb = B.flce_workspace_bytes(N, d, v1 - v0, dt, 0)
        ws = torch.empty(nb, dtype=torch.uint8, device=dev)
        rc = B.flce_forward_partial(H, W[v0:v1], y, N, d, v1 - v0, v0, V, wl.ignore_index, dt, parts[0, k],
                                    parts[1, k], parts[2, k], ws, nb, st)
        assert rc == B.FLCE_OK, B.flce_status_string(rc)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    lse = torch.empty(N, dtype=torch.float32, device=dev)
    nb = B.flce_merge_workspace_bytes(N)
    wsm = torch.empty(nb, dtype=torch.uint8, device=dev)
    rc = B.flce_merge_partials(parts[0], parts[1], parts[2], P, y, N, V, wl.ignore_index, red, loss, lse, wsm, nb, st)
    assert rc == B.FLCE_OK, B.flce_status_string(rc)
    status, n_valid = B.flce_last_device_status(wsm, st)
    dH = np.zeros((N, d))
    dW = torch.empty(V, d, dtype=tdt, device=dev)
    dHk = torch.empty(N, d, dtype=tdt, device=dev)
    dH_bits_of_dead_rows = []
    for k in range(P):
        v0, v1 = cuts[k], cuts[k + 1]
        nb = B.flce_workspace_bytes(N, d, v1 - v0, dt, 1)
        ws = torch.empty(nb, dtype=torch.uint8, device=dev)
        rc = B.flce_backward_partial(H, W[v0:v1], y, lse, N, d, v1 - v0, v0, V, wl.ignore_index, red, dt, grad_loss,
                                     dHk, dW[v0:v1], ws, nb, st)
        assert rc == B.FLCE_OK, B.flce_status_string(rc)
        stb, nvb = B.flce_last_device_status(ws, st)
        assert nvb == n_valid and stb == status
        dH += to_host_f64(dHk)
        dH_bits_of_dead_rows.append(dHk.view(torch.int16 if wl.dtype == "bf16" else torch.int32).cpu().numpy().copy())
    return dict(status=status, loss=float(loss.item()), lse=to_host_f64(lse), n_valid=n_valid, dH=dH,
                dW=to_host_f64(dW), parts=parts.cpu().numpy().astype(np.float64), dH_bits=dH_bits_of_dead_rows)
