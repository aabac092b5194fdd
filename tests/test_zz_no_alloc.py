"""flce_forward_static (the forward whose scratch is a device array inside the library, for callers that cannot
allocate) against flce_forward on the same inputs, through the C ABI: two calls in a row on one GPU, the second on
a smaller problem of another type, so that whatever the first call left in the shared array is stale for it."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2511_17599_amd import binding as B             # noqa: E402
from paper_2511_17599_amd import inputs as I              # noqa: E402
from paper_2511_17599_amd.runner import session_for, to_host_f64   # noqa: E402


@pytest.fixture(autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def both_forwards(wl, x):
    print(f"[case] static-scratch forward {wl.name} N={wl.N} d={wl.d} V={wl.V} {wl.dtype} seed={wl.seed}", flush=True)
    s = session_for(wl, x)
    assert s.forward() == B.FLCE_OK
    st_ref, nv_ref = s.device_status()
    loss_ref, lse_ref = float(s.loss.item()), to_host_f64(s.lse)
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device=s.device)
    lse = torch.full((wl.N,), float("nan"), dtype=torch.float32, device=s.device)
    status = torch.full((1,), -1, dtype=torch.int32, device=s.device)
    n_valid = torch.full((1,), -1, dtype=torch.int64, device=s.device)
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    rc = B.flce_forward_static(s.H, s.W, s.y, wl.N, wl.d, wl.V, wl.ignore_index, s.red, s.dt, loss, lse, status,
                               n_valid, s.stream())
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert rc == B.FLCE_OK, B.flce_status_string(rc)
    assert free_after == free_before                       # the call took no device memory
    # integer facts: exact
    assert int(status.item()) == st_ref and int(n_valid.item()) == nv_ref
    tol = 1e-5 if wl.dtype == "f32" else 2e-3
    lse_tol = 2e-6 if wl.dtype == "f32" else 2e-3
    got_lse = to_host_f64(lse)
    assert np.all(np.isfinite(got_lse))
    assert abs(float(loss.item()) - loss_ref) <= tol * max(abs(loss_ref), 1e-30), (float(loss.item()), loss_ref)
    assert np.abs(got_lse - lse_ref).max() <= lse_tol * np.abs(lse_ref).max()
    print(f"       loss {float(loss.item()):.7g} vs {loss_ref:.7g}; max |lse diff| {np.abs(got_lse - lse_ref).max():.2e}; "
          f"n_valid {int(n_valid.item())}", flush=True)


def test_static_scratch_forward_matches_the_workspace_forward_twice_in_a_row():
    big = I.Workload("static_big", 1500, 256, 5000, "bf16", "zipf", zipf_s=1.1, ignore_frac=0.1, seed=401)
    xb = I.make_inputs(big)
    xb["y"][7] = 6000                                        # a counted target outside the vocabulary: flagged
    both_forwards(big, xb)
    small = I.Workload("static_small", 300, 72, 700, "f32", "uniform", ignore_frac=0.2, reduction="sum", seed=402)
    both_forwards(small, I.make_inputs(small))
    tiny = I.Workload("static_tiny", 3, 64, 5, "bf16", "uniform", seed=403)
    both_forwards(tiny, I.make_inputs(tiny))


def test_static_scratch_forward_rejects_what_does_not_fit():
    p = 4096  # fake aligned device addresses: the size check comes before any launch
    # 12 bytes x 4 windows x 400 000 rows alone exceed the 16 MiB array
    rc = B.flce_forward_static(p, p, p, 400000, 4096, 128256, -100, B.FLCE_REDUCE_MEAN, B.FLCE_DTYPE_BF16, p, p)
    assert rc == B.FLCE_ERR_WORKSPACE
    assert B.flce_forward_static(None, p, p, 256, 64, 512, -100, B.FLCE_REDUCE_MEAN, B.FLCE_DTYPE_BF16, p, p) == \
        B.FLCE_ERR_BAD_ARG
    assert B.flce_forward_static(p, p, p, 256, 60, 512, -100, B.FLCE_REDUCE_MEAN, B.FLCE_DTYPE_BF16, p, p) == \
        B.FLCE_ERR_BAD_SHAPE
