"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle on
the same seeded inputs, element by element.

Tolerances (fixed by the benchmark definition): loss 1e-5 relative (fp32) / 2e-3
(bf16); dH and dW max|x - ref| / max|ref| <= 1e-4 (fp32) / 2e-2 (bf16); n_valid, the
ignore mask (rows of dH that are exactly +0) and target indexing bit-exact.
"""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import flce_oracle as O                       # noqa: E402
from paper_2511_17599_amd import binding as B             # noqa: E402
from paper_2511_17599_amd import inputs as I              # noqa: E402
from paper_2511_17599_amd.runner import run_workload      # noqa: E402
from conftest import set_plan                              # noqa: E402

TOL = {"f32": dict(loss=1e-5, grad=1e-4, lse=2e-6), "bf16": dict(loss=2e-3, grad=2e-2, lse=2e-3)}


@pytest.fixture(autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def nerr(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))


def check_against_oracle(wl, x, grad_loss=1.0, expect_status=B.FLCE_OK):
    print(f"[case] {wl.name} N={wl.N} d={wl.d} V={wl.V} {wl.dtype} {wl.reduction} seed={wl.seed}", flush=True)
    got = run_workload(wl, x, grad_loss=grad_loss)
    Hd, Wd = I.to_f64(x["H"]), I.to_f64(x["W"])
    f = O.forward(Hd, Wd, x["y"], wl.ignore_index, wl.reduction)
    b = O.backward(Hd, Wd, x["y"], wl.ignore_index, wl.reduction, grad_loss)
    tol = TOL[wl.dtype]
    assert got["status"] == expect_status
    assert got["n_valid"] == f["n_valid"] == got["n_valid_bwd"]
    assert np.all(np.isfinite(got["lse"]))
    lse_err = np.abs(got["lse"] - f["lse"]).max() / np.abs(f["lse"]).max()
    assert lse_err <= tol["lse"], lse_err
    assert abs(got["loss"] - f["loss"]) <= tol["loss"] * max(abs(f["loss"]), 1e-30), (got["loss"], f["loss"])
    # rows that do not count: dH exactly +0, bit for bit
    dead = ~f["valid"]
    s = got["session"]
    if dead.any():
        raw = s.dH.view(torch.int16 if wl.dtype == "bf16" else torch.int32).cpu().numpy()
        assert not raw[dead].any()
    if f["n_valid"] > 0:
        eH, eW = nerr(got["dH"], b["dH"]), nerr(got["dW"], b["dW"])
        print(f"       loss {got['loss']:.7g} vs {f['loss']:.7g}  lse_err {lse_err:.2e}  dH {eH:.2e}  dW {eW:.2e}",
              flush=True)
        assert eH <= tol["grad"], eH
        assert eW <= tol["grad"], eW
    else:
        assert not got["dH"].any() and not got["dW"].any() and got["loss"] == 0.0
    return got, f, b


def custom(name, N, d, V, dtype, seed, targets="uniform", ignore_frac=0.0, reduction="mean", w_std=0.02, zipf_s=1.1):
    return I.Workload(name, N, d, V, dtype, targets, zipf_s=zipf_s, ignore_frac=ignore_frac, reduction=reduction,
                      seed=seed, w_std=w_std)


def test_tiny_f32_workload():
    wl = I.WORKLOADS["tiny_f32"]
    check_against_oracle(wl, I.make_inputs(wl))


@pytest.mark.parametrize("wl", [
    custom("bf16_ragged", 600, 200, 1000, "bf16", 11, ignore_frac=0.1),
    custom("f32_ragged", 300, 72, 777, "f32", 12, ignore_frac=0.2, reduction="sum"),
    custom("bf16_one_tile", 256, 64, 256, "bf16", 13),
    custom("bf16_small_everything", 5, 8, 3, "bf16", 14),
    custom("f32_single_row", 1, 8, 1, "f32", 15),
    custom("bf16_zipf_sum", 1030, 256, 2049, "bf16", 16, targets="zipf", reduction="sum"),
    # the tuned bf16 loop (d a multiple of 32) at degenerate extents
    custom("bf16_tuned_one_row_one_word", 1, 32, 1, "bf16", 17),
    custom("bf16_tuned_few_rows", 3, 64, 300, "bf16", 18),
    custom("bf16_tuned_two_words", 300, 64, 2, "bf16", 19, ignore_frac=0.3),
    custom("bf16_tuned_257", 257, 32, 257, "bf16", 20, ignore_frac=0.5),
], ids=lambda w: w.name)
def test_ragged_and_small_shapes(wl):
    check_against_oracle(wl, I.make_inputs(wl), grad_loss=1.0 if wl.reduction == "mean" else -0.75)


@pytest.mark.parametrize("dtype,generic", [("bf16", 0), ("bf16", 1), ("f32", 0)])
@pytest.mark.parametrize("windows,vc,nc", [(1, 1, 1), (3, 2, 1), (5, 1, 2), (64, 3, 3)])
def test_chunk_and_window_splits(monkeypatch, dtype, generic, windows, vc, nc):
    """Forces several vocabulary windows in the forward and several vocabulary / token chunks in
    the backward on a small problem, so the merge and the fixed-order accumulation are exercised;
    for bf16 once with the tuned main loop (operands read in place) and once with the generic one
    (transposed copies)."""
    set_plan(monkeypatch, FLCE_WINDOWS=windows, FLCE_VC_TILES=vc, FLCE_NC_TILES=nc, FLCE_GENERIC=generic)
    wl = custom(f"split_{dtype}_{generic}_{windows}_{vc}_{nc}", 700, 160, 1500, dtype, 21, ignore_frac=0.05)
    check_against_oracle(wl, I.make_inputs(wl))


@pytest.mark.parametrize("dtype,generic", [("bf16", 0), ("bf16", 1), ("f32", 0)])
@pytest.mark.parametrize("sdh,sdw,vc,nc", [(3, 2, 128, 32), (2, 3, 4, 2), (5, 1, 2, 1)])
def test_split_k_contractions(monkeypatch, dtype, generic, sdh, sdw, vc, nc):
    """K of the dH / dW contractions cut into slices whose fp32 tiles are summed in slice order, with and
    without chunk accumulation on top."""
    set_plan(monkeypatch, FLCE_SPLITK_DH=sdh, FLCE_SPLITK_DW=sdw, FLCE_VC_TILES=vc, FLCE_NC_TILES=nc,
             FLCE_GENERIC=generic)
    wl = custom(f"splitk_{dtype}_{generic}_{sdh}_{sdw}_{vc}_{nc}", 1100, 288, 1800, dtype, 22, ignore_frac=0.08)
    check_against_oracle(wl, I.make_inputs(wl))


@pytest.mark.parametrize("name,N,d,V,ignore_frac", [
    # dW: 90 x 3 = 270 output tiles = one round of 256 workgroups + 5 output-row tiles (15 tiles) cut into 2 K slices
    ("tail_dW", 1024, 768, 23040, 0.1),
    # dH: 20 x 14 = 280 output tiles = one round + 2 row tiles (28 tiles) cut into 4 K slices; with a twentieth of
    # the rows ignored the compacted rows end inside the tail
    ("tail_dH", 5120, 3584, 2048, 0.05),
    # the same with so many rows ignored that the tail launch has no rows left at all
    ("tail_dH_empty", 5120, 3584, 2048, 0.15),
])
def test_k_split_tail_of_a_contraction_launch(name, N, d, V, ignore_frac):
    """Launches of a little more than one round of workgroups: the output-row tiles beyond the whole rounds go
    out as a second launch with K cut into slices (default plan; the plan line says which tails it has)."""
    plan = B.flce_plan_describe(N, d, V, B.FLCE_DTYPE_BF16)
    print(plan, flush=True)
    assert ("tail_dW=5x2" in plan) if name == "tail_dW" else ("tail_dH=2x4" in plan)
    wl = custom(name, N, d, V, "bf16", 25, ignore_frac=ignore_frac)
    check_against_oracle(wl, I.make_inputs(wl))


@pytest.mark.parametrize("d", [32, 96, 416])
def test_tuned_loop_short_and_odd_k(d):
    """K extents of 1, 3 and 13 stages of the tuned bf16 loop (prologue / drain paths), hidden size not a
    multiple of the 256-wide output tile."""
    wl = custom(f"bf16_k{d}", 515, d, 1027, "bf16", 23, ignore_frac=0.07)
    check_against_oracle(wl, I.make_inputs(wl))


def test_generic_loop_matches_tuned_loop_closely(monkeypatch):
    wl = custom("both_loops", 520, 256, 2100, "bf16", 24, ignore_frac=0.1)
    x = I.make_inputs(wl)
    a = run_workload(wl, x)
    set_plan(monkeypatch, FLCE_GENERIC=1)
    b = run_workload(wl, x)
    assert abs(a["loss"] - b["loss"]) <= 1e-6 * abs(a["loss"])
    assert nerr(a["dH"], b["dH"]) < 1e-2 and nerr(a["dW"], b["dW"]) < 1e-2


@pytest.mark.parametrize("dtype,w_std", [("bf16", 1.0), ("f32", 0.5)])
def test_peaked_softmax_large_logits(dtype, w_std):
    """Logits with a standard deviation of tens: exercises the max shift of the online softmax."""
    wl = custom(f"peaked_{dtype}", 512, 1024, 3000, dtype, 31, ignore_frac=0.03, w_std=w_std)
    check_against_oracle(wl, I.make_inputs(wl))


def test_target_positions_and_mask_are_exact():
    """Targets on tile edges, first / last id, a hot id, and ignored rows in between."""
    V, N, d = 777, 520, 64
    wl = custom("edges", N, d, V, "f32", 41)
    x = I.make_inputs(wl)
    y = np.full(N, 3, dtype=np.int64)                       # hot id
    special = [0, 255, 256, 511, 512, 767, 768, 776, 1, 254, 257]
    y[:len(special)] = special
    y[100:140] = wl.ignore_index
    y[255:258] = [776, wl.ignore_index, 0]                  # across a row-tile edge
    x["y"] = y
    got, f, b = check_against_oracle(wl, x)
    # W = 0 makes G exactly Gamma * (1/V - onehot): the -Gamma term must sit on row y_i of dW
    x0 = dict(x, W=np.zeros_like(x["W"]))
    got0, f0, b0 = check_against_oracle(custom("edges_w0", N, d, V, "f32", 41), x0)
    np.testing.assert_allclose(got0["lse"], np.log(V), rtol=1e-6)
    assert not got0["dH"].any()


def test_all_rows_ignored():
    wl = custom("all_ignored", 300, 64, 500, "bf16", 51)
    x = I.make_inputs(wl)
    x["y"][:] = wl.ignore_index
    for red in ("mean", "sum"):
        w2 = custom("all_ignored_" + red, 300, 64, 500, "bf16", 51, reduction=red)
        got, f, _ = check_against_oracle(w2, x)
        assert got["loss"] == 0.0 and got["n_valid"] == 0


def test_ignore_index_inside_vocabulary():
    wl = I.Workload("ignore_in_range", 400, 64, 300, "f32", "uniform", seed=52, ignore_index=7)
    x = I.make_inputs(wl)
    x["y"][::5] = 7
    check_against_oracle(wl, x)


def test_out_of_range_target_is_flagged_and_dropped():
    wl = custom("oor", 300, 64, 500, "f32", 53)
    x = I.make_inputs(wl)
    x["y"][17] = 500
    x["y"][290] = -5
    got, f, _ = check_against_oracle(wl, x, expect_status=B.FLCE_ERR_TARGET_RANGE)
    assert f["out_of_range"] and got["n_valid"] == 298


@pytest.mark.parametrize("env", [
    {},
    # several vocabulary and token chunks (fp32 running sums read and written back between launches) and K slices
    # summed by the second kernel: the places where an order that depended on scheduling would show
    {"FLCE_VC_TILES": "2", "FLCE_NC_TILES": "2", "FLCE_SPLITK_DH": "3", "FLCE_SPLITK_DW": "2", "FLCE_WINDOWS": "5"},
    {"FLCE_VC_TILES": "3", "FLCE_NC_TILES": "1", "FLCE_SPLITK_DH": "2", "FLCE_SPLITK_DW": "1", "FLCE_GENERIC": "1"},
    # a dW launch with a K-split tail (90 x 3 output tiles)
    {"shape": (1024, 768, 23040)},
], ids=["default_plan", "chunks_and_k_slices", "generic_loop_chunks", "k_split_tail"])
def test_results_are_bit_identical_between_runs(monkeypatch, env):
    env = dict(env)
    N, d, V = env.pop("shape", (1024, 256, 5000))
    set_plan(monkeypatch, **env)
    wl = custom("determinism", N, d, V, "bf16", 61, targets="zipf", ignore_frac=0.05)
    x = I.make_inputs(wl)
    a = run_workload(wl, x)
    b = run_workload(wl, x)
    c = run_workload(wl, x)
    for k in ("lse", "dH", "dW"):
        assert np.array_equal(a[k], b[k]) and np.array_equal(a[k], c[k]), k
    assert a["loss"] == b["loss"] == c["loss"]


def test_gpt2_small_workload():
    wl = I.WORKLOADS["gpt2_small"]
    check_against_oracle(wl, I.make_inputs(wl))


def test_largest_staging_tile():
    """128 x 128 tiles of G in one launch (2 GiB in bf16): the contraction that walks G over memory
    rows uses buffer offsets beyond 2^31 (they are unsigned 32-bit)."""
    wl = custom("g_2gib", 32768, 64, 32750, "bf16", 71, ignore_frac=0.001)     # > 32704 counted rows x 65664 bytes
    check_against_oracle(wl, I.make_inputs(wl))


@pytest.mark.parametrize("dtype,reduction,grad_loss", [("bf16", "mean", 1.0), ("bf16", "sum", -0.5), ("f32", "mean", 3.0)])
def test_partial_gradients_then_scaling(dtype, reduction, grad_loss):
    """Alg. 3 (loss + gradients without the upstream gradient) and Alg. 4 (scaling) through their own
    entry points, against the two-stage oracle: the partial gradients are the gradients of the summed
    loss, the scaled ones those of the requested reduction."""
    wl = custom(f"alg3_{dtype}_{reduction}", 700, 160, 1500, dtype, 81, ignore_frac=0.1, reduction=reduction)
    x = I.make_inputs(wl)
    print(f"[case] {wl.name} partial gradients + scaling", flush=True)
    from paper_2511_17599_amd.runner import session_for, to_host_f64
    s = session_for(wl, x, grad_loss=grad_loss)
    assert s.forward_with_grads() == B.FLCE_OK
    st, nv = s.device_status()
    Hd, Wd = I.to_f64(x["H"]), I.to_f64(x["W"])
    f = O.forward(Hd, Wd, x["y"], wl.ignore_index, wl.reduction)
    part = O.backward(Hd, Wd, x["y"], wl.ignore_index, "sum", 1.0)
    full = O.backward(Hd, Wd, x["y"], wl.ignore_index, wl.reduction, grad_loss)
    tol = TOL[dtype]
    assert st == B.FLCE_OK and nv == f["n_valid"]
    assert abs(float(s.loss.item()) - f["loss"]) <= tol["loss"] * abs(f["loss"])
    assert np.abs(to_host_f64(s.lse) - f["lse"]).max() <= tol["lse"] * np.abs(f["lse"]).max()
    assert nerr(to_host_f64(s.dH), part["dH"]) <= tol["grad"]
    assert nerr(to_host_f64(s.dW), part["dW"]) <= tol["grad"]
    assert s.scale() == B.FLCE_OK
    assert nerr(to_host_f64(s.dH), full["dH"]) <= tol["grad"]
    assert nerr(to_host_f64(s.dW), full["dW"]) <= tol["grad"]
    raw = s.dH.view(torch.int16 if dtype == "bf16" else torch.int32).cpu().numpy()
    assert not raw[~f["valid"]].any()                      # rows that do not count stay exactly +0


def test_partial_gradients_against_streaming_algorithms():
    """A case small enough for the per-row, per-vocabulary-entry loops of Alg. 3 and Alg. 4 as stated."""
    from oracle import streaming as S
    from paper_2511_17599_amd.runner import session_for, to_host_f64
    wl = custom("alg3_stream", 7, 8, 37, "f32", 82)
    x = I.make_inputs(wl)
    s = session_for(wl, x, grad_loss=2.5)
    assert s.forward_with_grads() == B.FLCE_OK
    Hd, Wd = I.to_f64(x["H"]), I.to_f64(x["W"])
    loss, dHp, dWp, m, a = S.alg3_forward_partial(Hd, Wd, x["y"])
    assert abs(float(s.loss.item()) - loss) <= 1e-5 * abs(loss)           # Alg. 1 ends with the division by B*T
    assert nerr(to_host_f64(s.dH), dHp) <= 1e-4 and nerr(to_host_f64(s.dW), dWp) <= 1e-4
    assert s.scale() == B.FLCE_OK
    dH, dW = S.alg4_scale(dHp, dWp, 2.5 / wl.N)
    assert nerr(to_host_f64(s.dH), dH) <= 1e-4 and nerr(to_host_f64(s.dW), dW) <= 1e-4


@pytest.mark.parametrize("dtype,reduction", [("bf16", "mean"), ("f32", "sum")])
def test_vocabulary_slices_merge_to_the_whole(dtype, reduction):
    """The vocabulary cut into uneven slices (one exactly a tile, one a single row, ragged ends), each run through
    the partial calls and merged: per slice (m, a, z_target) against their definitions, the merged loss / lse and
    the assembled dW / summed dH against the two-stage oracle on the whole vocabulary."""
    from sliced import run_sliced
    wl = custom(f"slices_{dtype}", 700, 160, 1500, dtype, 91, ignore_frac=0.1, reduction=reduction)
    x = I.make_inputs(wl)
    x["y"][5] = 1700                                         # one target outside the whole vocabulary
    cuts = [0, 256, 257, 700, 1333, 1500]
    print(f"[case] {wl.name} cuts {cuts}", flush=True)
    got = run_sliced(wl, x, cuts, grad_loss=0.5)
    Hd, Wd = I.to_f64(x["H"]), I.to_f64(x["W"])
    f = O.forward(Hd, Wd, x["y"], wl.ignore_index, wl.reduction)
    b = O.backward(Hd, Wd, x["y"], wl.ignore_index, wl.reduction, 0.5)
    tol = TOL[dtype]
    assert f["out_of_range"] and got["status"] == B.FLCE_ERR_TARGET_RANGE and got["n_valid"] == f["n_valid"]
    Z = Hd @ Wd.T
    for k in range(len(cuts) - 1):
        v0, v1 = cuts[k], cuts[k + 1]
        m, a, zt = got["parts"][:, k]
        # (m, a) is one of many equal representations of the slice's log-sum-exp; m itself is its largest logit
        lse_k = np.log(np.exp(Z[:, v0:v1] - Z[:, v0:v1].max(axis=1, keepdims=True)).sum(axis=1)) + Z[:, v0:v1].max(axis=1)
        assert np.abs(m - Z[:, v0:v1].max(axis=1)).max() <= 1e-5 * np.abs(Z).max()
        assert np.abs(m + np.log(a) - lse_k).max() <= tol["lse"] * np.abs(lse_k).max()
        inside = f["valid"] & (x["y"] >= v0) & (x["y"] < v1)
        want = np.where(inside, Z[np.arange(wl.N), np.clip(x["y"], 0, wl.V - 1)], 0.0)
        assert np.abs(zt - want).max() <= 1e-5 * np.abs(Z).max()
        assert not zt[~inside].any()                        # exactly 0 where the target is elsewhere
    assert abs(got["loss"] - f["loss"]) <= tol["loss"] * abs(f["loss"])
    assert np.abs(got["lse"] - f["lse"]).max() <= tol["lse"] * np.abs(f["lse"]).max()
    assert nerr(got["dW"], b["dW"]) <= tol["grad"]
    assert nerr(got["dH"], b["dH"]) <= tol["grad"]
    for bits in got["dH_bits"]:
        assert not bits[~f["valid"]].any()
    # and against the unsliced call on the same device
    whole = run_workload(wl, x, grad_loss=0.5)
    assert np.abs(whole["lse"] - got["lse"]).max() <= 4e-6 * np.abs(f["lse"]).max()
    assert nerr(whole["dW"], got["dW"]) <= (1e-2 if dtype == "bf16" else 1e-5)


@pytest.mark.parametrize("dtype,eps,generic", [("bf16", 0.0, 0), ("bf16", 0.1, 0), ("bf16", 0.1, 1), ("f32", 0.2, 0)])
def test_per_row_losses_and_gradients(monkeypatch, dtype, eps, generic):
    """No reduction: one loss per row out, one upstream gradient per row in, with and without label smoothing,
    against the oracle's per-row functions (several chunks in the backward)."""
    from paper_2511_17599_amd.runner import session_for, to_host_f64, to_device
    set_plan(monkeypatch, FLCE_GENERIC=generic, FLCE_VC_TILES=3, FLCE_NC_TILES=2)
    wl = custom(f"rows_{dtype}_{eps}_{generic}", 900, 160, 1700, dtype, 95, ignore_frac=0.1)
    x = I.make_inputs(wl)
    x["y"][11] = 5000                                        # outside the vocabulary: dropped and flagged
    print(f"[case] {wl.name} per-row, label smoothing {eps}", flush=True)
    gr = (np.random.default_rng(9).standard_normal(wl.N) * 0.5 + 1.0).astype(np.float32)
    s = session_for(wl, x)
    loss_rows = torch.empty(wl.N, dtype=torch.float32, device=s.device)
    assert s.forward_rows(loss_rows, eps) == B.FLCE_OK
    st, nv = s.device_status()
    assert s.backward_rows(to_device(gr, s.device), eps) == B.FLCE_OK
    stb, nvb = s.device_status()
    Hd, Wd = I.to_f64(x["H"]), I.to_f64(x["W"])
    f = O.forward_per_row(Hd, Wd, x["y"], wl.ignore_index, eps)
    b = O.backward_per_row(Hd, Wd, x["y"], gr.astype(np.float64), wl.ignore_index, eps)
    tol = TOL[dtype]
    assert st == stb == B.FLCE_ERR_TARGET_RANGE and nv == nvb == f["n_valid"]
    lr = to_host_f64(loss_rows)
    assert not lr[~f["valid"]].any()                         # rows that do not count: exactly 0
    assert np.abs(lr - f["loss_rows"]).max() <= tol["loss"] * np.abs(f["loss_rows"]).max()
    assert np.abs(to_host_f64(s.lse) - f["lse"]).max() <= tol["lse"] * np.abs(f["lse"]).max()
    eH, eW = nerr(to_host_f64(s.dH), b["dH"]), nerr(to_host_f64(s.dW), b["dW"])
    print(f"       dH {eH:.2e}  dW {eW:.2e}", flush=True)
    assert eH <= tol["grad"] and eW <= tol["grad"]
    raw = s.dH.view(torch.int16 if dtype == "bf16" else torch.int32).cpu().numpy()
    assert not raw[~f["valid"]].any()


def _random_cases(n, seed):
    r = np.random.default_rng(seed)
    cases = []
    for k in range(n):
        dtype = "bf16" if r.random() < 0.75 else "f32"
        d = int(r.choice([8, 24, 32, 64, 96, 160, 256, 320, 512]))
        N = int(r.integers(1, 1400))
        V = int(r.integers(1, 3000))
        cases.append(dict(
            wl=custom(f"rand{k}", N, d, V, dtype, 500 + k, targets="zipf" if r.random() < 0.4 else "uniform",
                      ignore_frac=float(r.choice([0.0, 0.05, 0.5, 0.95])), reduction="sum" if r.random() < 0.4 else "mean",
                      w_std=float(r.choice([0.02, 0.3]))),
            env=dict(FLCE_WINDOWS=str(int(r.choice([0, 1, 2, 7]))), FLCE_VC_TILES=str(int(r.choice([1, 2, 3, 128]))),
                     FLCE_NC_TILES=str(int(r.choice([1, 2, 128]))), FLCE_SPLITK_DH=str(int(r.choice([0, 0, 2, 3]))),
                     FLCE_SPLITK_DW=str(int(r.choice([0, 0, 2])))),
            grad_loss=float(r.choice([1.0, -0.5, 3.0]))))
    return cases


@pytest.mark.parametrize("case", _random_cases(24, 2024), ids=lambda c: c["wl"].name)
def test_seeded_random_shapes_and_plans(monkeypatch, case):
    """A fixed, seeded set of arbitrary shapes (ragged everywhere, d with and without the tuned loop), target
    mixes and launch plans (windows, chunk sizes, K splits)."""
    set_plan(monkeypatch, **case["env"])
    wl = case["wl"]
    print(f"[plan] {case['env']}", flush=True)
    check_against_oracle(wl, I.make_inputs(wl), grad_loss=case["grad_loss"])
