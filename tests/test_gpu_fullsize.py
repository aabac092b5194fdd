"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.

The full fp64 pipeline costs 3*N*d*V multiply-adds (1.3e13 for the Llama-3-8B shape), so
the oracle is evaluated on sampled outputs it can compute one by one:
  * a seeded sample of rows: lse_i, the per-row loss and the dH row, exactly;
  * the scalar loss through sum_i (lse_i - z_{i,y_i}) with the oracle's own z_{i,y_i} for
    every row (N*d multiply-adds) and the oracle's lse on the sampled rows;
and dW through properties that hold at any size: its column sums vanish (every row of G
sums to zero) up to the rounding of its entries and <dH, H> = <dW, W> (both equal sum_iv G_iv Z_iv).  Where affordable
(all but the long-sequence shape) the oracle's lse of EVERY row is computed too, which gives exact dW rows
for a sample of vocabulary ids (hot, cold, tile-edge, last).
"""
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import flce_oracle as O                       # noqa: E402
from paper_2511_17599_amd import binding as B             # noqa: E402
from paper_2511_17599_amd import inputs as I              # noqa: E402
from paper_2511_17599_amd.runner import session_for, to_host_f64   # noqa: E402


@pytest.fixture(autouse=True)
def _need_gpu(monkeypatch):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    for k in ("FLCE_WINDOWS", "FLCE_VC_TILES", "FLCE_NC_TILES", "FLCE_GENERIC", "FLCE_SPLITK_DH", "FLCE_SPLITK_DW"):
        monkeypatch.delenv(k, raising=False)
    yield


def sample_rows(wl, y, k, seed):
    r = np.random.default_rng(seed)
    rows = set(r.choice(wl.N, size=k, replace=False).tolist())
    rows |= {0, wl.N - 1, 255, 256}
    ign = np.nonzero(y == wl.ignore_index)[0]
    rows |= set(ign[:4].tolist())
    return np.array(sorted(rows), dtype=np.int64)


def run_fullsize(name, n_rows, full_lse):
    wl = I.WORKLOADS[name] if isinstance(name, str) else name
    print(f"[case] full size {wl.name} N={wl.N} d={wl.d} V={wl.V} seed={wl.seed}", flush=True)
    t0 = time.time()
    x = I.make_inputs(wl)
    s = session_for(wl, x)
    assert s.forward() == B.FLCE_OK
    st, n_valid = s.device_status()
    assert st == B.FLCE_OK
    assert s.backward() == B.FLCE_OK
    st, n_valid_b = s.device_status()
    assert st == B.FLCE_OK
    print(f"       gpu done after {time.time() - t0:.1f} s", flush=True)

    y = x["y"]
    valid, nv, oor = O.classify_targets(y, wl.V, wl.ignore_index)
    assert n_valid == nv == n_valid_b and not oor                       # integer facts: exact
    gam = O.gamma(nv, wl.reduction, 1.0)
    Wd = I.to_f64(x["W"])
    rows = sample_rows(wl, y, n_rows, wl.seed)
    Hs = I.to_f64(x["H"][rows])
    lse_o, zt_o, loss_rows_o = O.forward_rows(Hs, Wd, y[rows], wl.ignore_index)
    lse_g = to_host_f64(s.lse)
    assert np.abs(lse_g[rows] - lse_o).max() <= 2e-3 * np.abs(lse_o).max()
    print(f"       sampled lse max abs err {np.abs(lse_g[rows] - lse_o).max():.2e}", flush=True)
    # dH rows of the sample
    dH_o = O.dH_rows(Hs, Wd, y[rows], gam, wl.ignore_index)
    dH_g = s.dH[torch.from_numpy(rows).to(s.dH.device)].float().cpu().numpy().astype(np.float64)
    scale = np.abs(dH_o).max()
    assert np.abs(dH_g - dH_o).max() <= 2e-2 * scale
    dead = ~valid[rows]
    raw = s.dH.view(torch.int16)[torch.from_numpy(rows[dead]).to(s.dH.device)].cpu().numpy()
    assert not raw.any()                                                # ignored rows: exactly +0
    # scalar loss: oracle target logits for every row, oracle lse where sampled, GPU lse elsewhere
    zt_all = np.zeros(wl.N)
    idx = np.nonzero(valid)[0]
    for b0 in range(0, len(idx), 8192):
        ii = idx[b0:b0 + 8192]
        zt_all[ii] = np.einsum("ij,ij->i", I.to_f64(x["H"][ii]), Wd[y[ii]])
    lse_mix = lse_g.copy()
    lse_mix[rows] = lse_o
    total = float(np.where(valid, lse_mix - zt_all, 0.0).sum())
    want = total / nv if wl.reduction == "mean" else total
    got = float(s.loss.item())
    assert abs(got - want) <= 2e-3 * abs(want), (got, want)
    print(f"       loss {got:.6f} vs {want:.6f} (mixed-lse check), n_valid {nv}", flush=True)

    # dW properties at full size (fp32 accumulation on the device, no big host copies)
    dW = s.dW.float()
    colsum = dW.sum(dim=0, dtype=torch.float64).abs()
    mx = dW.abs().max().item()
    # A column of dW sums to zero in exact arithmetic.  Every stored entry was rounded to bf16 to nearest, an error
    # of at most ulp/2, so |column sum| <= sum ulp/2 (the rounding of G adds a few per cent: 0.55 instead of 0.5).
    # The errors are not independent (a target row holds -H_ic plus a small term that the rounding absorbs whole,
    # and these small terms share the sign of sum_i H_ic), so no square-root law is claimed.
    _, e = torch.frexp(dW)                                   # |x| = m * 2^e, m in [0.5, 1): ulp = 2^(e - 8)
    ulp = torch.where(dW != 0, torch.ldexp(torch.ones_like(dW), e - 8), torch.zeros_like(dW))
    col = (colsum / (0.55 * ulp.sum(dim=0, dtype=torch.float64)).clamp_min(1e-300)).max().item()
    del ulp, e
    assert col <= 1.0, (col, mx)
    lhs = (s.dH.float() * s.H.float()).sum(dtype=torch.float64).item()
    rhs = (dW * s.W.float()).sum(dtype=torch.float64).item()
    assert abs(lhs - rhs) <= 2e-2 * max(abs(lhs), abs(rhs)), (lhs, rhs)
    print(f"       dW column sums: largest is {col:.3f} of its rounding bound (max |dW| {mx:.3e}); <dH,H> {lhs:.6e} <dW,W> {rhs:.6e}", flush=True)
    del dW

    if full_lse:
        t1 = time.time()
        f = O.forward(I.to_f64(x["H"]), Wd, y, wl.ignore_index, wl.reduction, block_rows=512)
        print(f"       oracle lse of all rows: {time.time() - t1:.1f} s", flush=True)
        assert abs(got - f["loss"]) <= 2e-3 * abs(f["loss"])
        assert np.abs(lse_g - f["lse"]).max() <= 2e-3 * np.abs(f["lse"]).max()
        hot = np.bincount(y[valid], minlength=wl.V).argsort()[::-1][:4]
        ids = np.unique(np.concatenate([hot, [0, 255, 256, wl.V - 257, wl.V - 256, wl.V - 1],
                                        np.random.default_rng(5).integers(0, wl.V, 6)]))
        dW_o = O.dW_rows(I.to_f64(x["H"]), Wd[ids], ids, y, f["lse"], gam, wl.ignore_index, V=wl.V)
        dW_g = s.dW[torch.from_numpy(ids).to(s.dW.device)].float().cpu().numpy().astype(np.float64)
        err = np.abs(dW_g - dW_o).max() / np.abs(dW_o).max()
        print(f"       sampled dW rows err {err:.2e}", flush=True)
        assert err <= 2e-2


def test_llama3_8b_full_size():
    run_fullsize("llama3_8b", 48, full_lse=True)


def test_large_vocab_full_size():
    run_fullsize("large_vocab", 24, full_lse=True)


def test_long_seq_full_size():
    run_fullsize("long_seq", 24, full_lse=False)


def test_hidden_states_beyond_2_31_elements():
    """N * d above 2^31: every offset into H, dH and the compacted copy needs 64 bits (2344 row blocks)."""
    wl = I.Workload("big_rows", 600000, 4096, 600, "bf16", "uniform", ignore_frac=0.01, seed=2101)
    run_fullsize(wl, 24, full_lse=True)


def test_weights_beyond_2_31_elements():
    """V * d above 2^31: every offset into W and dW needs 64 bits (2344 vocabulary tiles, 19 chunks)."""
    wl = I.Workload("big_vocab", 600, 4096, 600000, "bf16", "zipf", zipf_s=1.05, ignore_frac=0.01, seed=2102)
    run_fullsize(wl, 24, full_lse=True)
