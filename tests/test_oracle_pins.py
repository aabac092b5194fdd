"""Pins for the CPU oracle: what the paper and the mathematics fix.

None of these compares the oracle with itself through the same formula: each
uses a closed form, an invariant, finite differences of the loss, an
independent scalar rendition of the paper's streaming algorithms, or the
fp64 log-softmax / NLL of a numerical library.
"""
import math

import numpy as np
import pytest

from oracle import flce_oracle as O
from oracle import streaming as S

IGN = -100


def rand_case(seed, N, d, V, n_ignored=0, w_std=0.5):
    r = np.random.default_rng(seed)
    H = r.standard_normal((N, d))
    W = w_std * r.standard_normal((V, d))
    y = r.integers(0, V, size=N).astype(np.int64)
    if n_ignored:
        y[r.permutation(N)[:n_ignored]] = IGN
    return H, W, y


# ---- P1: W = 0  =>  uniform softmax --------------------------------------
@pytest.mark.parametrize("reduction", ["mean", "sum"])
def test_zero_weights_closed_form(reduction):
    N, d, V = 13, 5, 11
    H, _, y = rand_case(1, N, d, V, n_ignored=3)
    W = np.zeros((V, d))
    f = O.forward(H, W, y, IGN, reduction)
    nv = 10
    assert f["n_valid"] == nv
    np.testing.assert_allclose(f["lse"], math.log(V), rtol=0, atol=1e-15)
    expect = math.log(V) if reduction == "mean" else nv * math.log(V)
    assert abs(f["loss"] - expect) < 1e-13
    b = O.backward(H, W, y, IGN, reduction, grad_loss=1.0)
    gam = 1.0 / nv if reduction == "mean" else 1.0
    assert np.all(b["dH"] == 0.0)
    valid = y != IGN
    dW = np.zeros((V, d))
    for v in range(V):
        dW[v] = gam * (H[valid].sum(0) / V - H[valid & (y == v)].sum(0))
    np.testing.assert_allclose(b["dW"], dW, rtol=0, atol=1e-14)


# ---- P2: H = 0 ------------------------------------------------------------
def test_zero_hidden_closed_form():
    N, d, V = 7, 4, 9
    _, W, y = rand_case(2, N, d, V, n_ignored=2)
    H = np.zeros((N, d))
    f = O.forward(H, W, y, IGN, "mean")
    assert abs(f["loss"] - math.log(V)) < 1e-14
    b = O.backward(H, W, y, IGN, "mean")
    assert np.all(b["dW"] == 0.0)
    gam = 1.0 / 5
    for i in range(N):
        want = gam * (W.mean(0) - W[y[i]]) if y[i] != IGN else np.zeros(d)
        np.testing.assert_allclose(b["dH"][i], want, rtol=0, atol=1e-15)


# ---- P3: one-hot dominance, exercises the exponent range ------------------
@pytest.mark.parametrize("c", [0.0, 1.0, 30.0, 100.0, 800.0])
def test_scaled_identity_closed_form(c):
    V = d = 16
    W = c * np.eye(V)
    y = np.arange(V, dtype=np.int64)[::-1].copy()
    H = np.eye(V)[y]
    f = O.forward(H, W, y, IGN, "sum")
    # ln(e^c + V - 1) - c, written so it stays finite for large c
    per_row = math.log1p((V - 1) * math.exp(-c))
    # lse - z_t cancels at size c: fp64 leaves an absolute error of a few ulp(c)
    np.testing.assert_allclose(f["loss_rows"], per_row, rtol=1e-12, atol=4e-16 * (1.0 + c))
    np.testing.assert_allclose(f["lse"], c + per_row, rtol=1e-14)
    G = O.grad_logits(H, W, y, np.ones(V, bool), 1.0)
    p_t = 1.0 / (1.0 + (V - 1) * math.exp(-c))
    np.testing.assert_allclose(G[np.arange(V), y], p_t - 1.0, rtol=1e-10, atol=1e-16)


# ---- P4 / P5: invariants --------------------------------------------------
def test_gradient_invariants():
    H, W, y = rand_case(3, 40, 12, 50, n_ignored=6)
    valid, nv, _ = O.classify_targets(y, 50, IGN)
    G = O.grad_logits(H, W, y, valid, 1.0 / nv)
    np.testing.assert_allclose(G.sum(1), 0.0, atol=1e-16)
    b = O.backward(H, W, y, IGN, "mean")
    np.testing.assert_allclose(b["dW"].sum(0), 0.0, atol=1e-15)
    lhs, rhs = (b["dH"] * H).sum(), (b["dW"] * W).sum()
    assert abs(lhs - rhs) < 1e-13
    assert abs(lhs - (G * (H @ W.T)).sum()) < 1e-13


# ---- P7: central finite differences of the loss ---------------------------
@pytest.mark.parametrize("reduction,grad_loss", [("mean", 1.0), ("sum", 1.0), ("mean", -2.5)])
def test_finite_differences(reduction, grad_loss):
    N, d, V = 6, 5, 9
    H, W, y = rand_case(4, N, d, V, n_ignored=2, w_std=1.0)
    b = O.backward(H, W, y, IGN, reduction, grad_loss)
    eps = 1e-6

    def L(Hx, Wx):
        return grad_loss * O.forward(Hx, Wx, y, IGN, reduction)["loss"]

    fdH = np.zeros_like(H)
    for i in range(N):
        for k in range(d):
            Hp, Hm = H.copy(), H.copy()
            Hp[i, k] += eps
            Hm[i, k] -= eps
            fdH[i, k] = (L(Hp, W) - L(Hm, W)) / (2 * eps)
    fdW = np.zeros_like(W)
    for v in range(V):
        for k in range(d):
            Wp, Wm = W.copy(), W.copy()
            Wp[v, k] += eps
            Wm[v, k] -= eps
            fdW[v, k] = (L(H, Wp) - L(H, Wm)) / (2 * eps)
    np.testing.assert_allclose(b["dH"], fdH, rtol=0, atol=2e-8)
    np.testing.assert_allclose(b["dW"], fdW, rtol=0, atol=2e-8)
    assert np.all(b["dH"][y == IGN] == 0.0)


# ---- P8: the paper's streaming algorithms reach the two-stage result ------
def test_streaming_algorithms_match_two_stage():
    N, d, V = 5, 4, 13
    H, W, y = rand_case(5, N, d, V, w_std=1.5)
    f = O.forward(H, W, y, IGN, "mean")
    loss, m, a = S.alg1_forward(H, W, y)
    assert abs(loss - f["loss"]) < 1e-13
    np.testing.assert_allclose(m + np.log(a), f["lse"], rtol=1e-14)
    np.testing.assert_allclose(m, (H @ W.T).max(1), rtol=1e-15)
    loss_p, _, _ = S.alg1_forward(H, W, y, as_printed=True)
    assert abs(loss_p - loss) < 1e-12
    b = O.backward(H, W, y, IGN, "mean", grad_loss=1.0)
    dH, dW = S.alg2_backward(H, W, y, m, a, 1.0 / N)
    np.testing.assert_allclose(dH, b["dH"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(dW, b["dW"], rtol=0, atol=1e-15)
    # Alg. 3 + Alg. 4 equal Alg. 2 for a scalar upstream gradient
    _, dHp, dWp, _, _ = S.alg3_forward_partial(H, W, y)
    dH4, dW4 = S.alg4_scale(dHp, dWp, 0.37 / N)
    b37 = O.backward(H, W, y, IGN, "mean", grad_loss=0.37)
    np.testing.assert_allclose(dH4, b37["dH"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(dW4, b37["dW"], rtol=0, atol=1e-15)


def test_streaming_per_position_gamma_matches_row_scaling():
    N, d, V = 4, 3, 7
    H, W, y = rand_case(6, N, d, V)
    _, m, a = S.alg1_forward(H, W, y)
    gam = np.array([0.5, -1.0, 0.0, 2.0])
    dH, dW = S.alg2_backward(H, W, y, m, a, gam)
    G = gam[:, None] * O.grad_logits(H, W, y, np.ones(N, bool), 1.0)
    np.testing.assert_allclose(dH, G @ W, atol=1e-15)
    np.testing.assert_allclose(dW, G.T @ H, atol=1e-15)


def test_streaming_pair_means_max_and_shifted_sum_on_every_prefix_and_split():
    """The pair (m, a) the streaming forward carries IS (max, sum exp(z - max)) of what it has seen: after every
    prefix of the vocabulary, for any cut of a range in two, in either order of combination, and with empty
    parts; large logits (|z| ~ 300) so that a missing max shift would overflow."""
    r = np.random.default_rng(77)
    d, V = 5, 23
    h = r.standard_normal(d) * 40.0
    W = r.standard_normal((V, d)) * 3.0
    z = W @ h
    assert np.abs(z).max() > 200
    for end in range(1, V + 1):
        m, a, _, _ = S.stream_row(h, W, -1, 0, end)
        assert m == z[:end].max()
        assert abs(a - np.exp(z[:end] - z[:end].max()).sum()) <= 1e-12 * a
    for lo, cut, hi in [(0, 7, 23), (3, 3, 19), (0, 22, 23), (5, 23, 23), (0, 0, 23)]:
        left = S.stream_row(h, W, -1, lo, cut)[:2]
        right = S.stream_row(h, W, -1, cut, hi)[:2]
        whole = S.stream_row(h, W, -1, lo, hi)[:2]
        for got in (S.combine(left, right), S.combine(right, left)):
            assert got[0] == whole[0] and abs(got[1] - whole[1]) <= 1e-12 * whole[1]
    assert S.combine(S.NOTHING, S.NOTHING) == S.NOTHING
    # associativity on summaries of three ranges
    a1, a2, a3 = (S.stream_row(h, W, -1, lo, hi)[:2] for lo, hi in ((0, 4), (4, 15), (15, 23)))
    x, y_ = S.combine(S.combine(a1, a2), a3), S.combine(a1, S.combine(a2, a3))
    assert x[0] == y_[0] and abs(x[1] - y_[1]) <= 1e-12 * x[1]
    # the printed closing steps agree with m + log a - z_t where they are finite, and overflow where they are not
    assert abs(S.closing_steps_as_printed(2.5, 3.0, 1.25) - (2.5 + np.log(3.0) - 1.25)) < 1e-14
    with pytest.raises(OverflowError):
        S.closing_steps_as_printed(800.0, 2.0, 1.0)


@pytest.mark.parametrize("cuts", [[0, 13], [0, 4, 13], [0, 1, 2, 12, 13], [0, 0, 5, 5, 13]])
def test_window_merge_equals_single_pass(cuts):
    N, d, V = 4, 6, 13
    H, W, y = rand_case(7, N, d, V, w_std=3.0)
    f = O.forward(H, W, y, IGN, "sum")
    for i in range(N):
        parts = [S.stream_row(H[i], W, int(y[i]), cuts[k], cuts[k + 1]) for k in range(len(cuts) - 1)]
        assert sum(p[3] for p in parts) == 1          # exactly one window owns the target
        lse, zt = S.merge_windows(parts)
        assert abs(lse - f["lse"][i]) < 1e-13
        assert abs((lse - zt) - f["loss_rows"][i]) < 1e-13


# ---- P9: adding one vector to every vocabulary row changes nothing --------
def test_shift_invariance():
    H, W, y = rand_case(8, 20, 8, 30, n_ignored=3)
    u = 40.0 * np.random.default_rng(9).standard_normal(8)
    f0, f1 = O.forward(H, W, y, IGN, "mean"), O.forward(H, W + u, y, IGN, "mean")
    assert abs(f0["loss"] - f1["loss"]) < 1e-11
    np.testing.assert_allclose(f1["lse"] - f0["lse"], H @ u, atol=1e-11)
    b0, b1 = O.backward(H, W, y, IGN, "mean"), O.backward(H, W + u, y, IGN, "mean")
    np.testing.assert_allclose(b0["dW"], b1["dW"], atol=1e-12)
    np.testing.assert_allclose(b0["dH"], b1["dH"], atol=1e-12)


# ---- P10: the definition is log_softmax + nll_loss of a numerical library -
@pytest.mark.parametrize("reduction", ["mean", "sum"])
def test_against_torch_fp64_autograd(reduction):
    torch = pytest.importorskip("torch")
    H, W, y = rand_case(10, 33, 16, 70, n_ignored=5, w_std=1.0)
    Ht = torch.tensor(H, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    loss = torch.nn.functional.cross_entropy(Ht @ Wt.T, torch.tensor(y), ignore_index=IGN, reduction=reduction)
    (1.7 * loss).backward()
    f = O.forward(H, W, y, IGN, reduction)
    b = O.backward(H, W, y, IGN, reduction, grad_loss=1.7)
    assert abs(f["loss"] - loss.item()) < 1e-12 * max(1.0, abs(loss.item()))
    np.testing.assert_allclose(b["dH"], Ht.grad.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(b["dW"], Wt.grad.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(f["lse"], torch.logsumexp(Ht @ Wt.T, 1).detach().numpy(), rtol=1e-14)


def test_against_scipy_logsumexp_softmax():
    sp = pytest.importorskip("scipy.special")
    H, W, y = rand_case(11, 9, 7, 21, w_std=4.0)
    Z = H @ W.T
    f = O.forward(H, W, y, IGN, "sum")
    np.testing.assert_allclose(f["lse"], sp.logsumexp(Z, axis=1), rtol=1e-14)
    G = O.grad_logits(H, W, y, np.ones(9, bool), 1.0)
    P = sp.softmax(Z, axis=1)
    P[np.arange(9), y] -= 1
    np.testing.assert_allclose(G, P, atol=1e-15)


# ---- P11: integer facts ---------------------------------------------------
def test_mask_and_index_facts():
    V = 8
    y = np.array([0, V - 1, IGN, 3, IGN, 3], dtype=np.int64)
    valid, nv, oor = O.classify_targets(y, V, IGN)
    assert valid.tolist() == [True, True, False, True, False, True] and nv == 4 and not oor
    # ignore_index inside the vocabulary range is still ignored
    valid, nv, oor = O.classify_targets(y, V, 3)
    assert valid.tolist() == [True, True, False, False, False, False] and nv == 2 and oor
    # a counted target outside [0, V) is flagged and dropped
    valid, nv, oor = O.classify_targets(np.array([V, -1, 2]), V, IGN)
    assert valid.tolist() == [False, False, True] and nv == 1 and oor
    # the -Gamma term lands on column y_i and nowhere else (W = 0 makes G exact)
    H = np.ones((6, 2))
    G = O.grad_logits(H, np.zeros((V, 2)), y, y != IGN, 1.0)
    for i, t in enumerate(y):
        want = np.full(V, 1.0 / V) if t != IGN else np.zeros(V)
        if t != IGN:
            want[t] -= 1.0
        assert np.array_equal(G[i], want)


def test_all_ignored_gives_zero():
    H, W, _ = rand_case(12, 5, 3, 6)
    y = np.full(5, IGN, dtype=np.int64)
    for red in ("mean", "sum"):
        f = O.forward(H, W, y, IGN, red)
        b = O.backward(H, W, y, IGN, red)
        assert f["loss"] == 0.0 and f["n_valid"] == 0
        assert np.all(b["dH"] == 0) and np.all(b["dW"] == 0)
        assert np.all(np.isfinite(f["lse"]))


# ---- sampled entry points return what the full functions return -----------
def test_sampled_entry_points_match_full():
    H, W, y = rand_case(13, 50, 10, 40, n_ignored=7)
    f = O.forward(H, W, y, IGN, "mean", block_rows=16)
    b = O.backward(H, W, y, IGN, "mean", grad_loss=0.9, block_rows=16)
    f1 = O.forward(H, W, y, IGN, "mean", block_rows=1000)
    assert np.array_equal(f["lse"], f1["lse"])
    rows = np.array([0, 3, 17, 49])
    lse, zt, lr = O.forward_rows(H[rows], W, y[rows], IGN)
    np.testing.assert_allclose(lse, f["lse"][rows], rtol=1e-15)
    np.testing.assert_allclose(lr, f["loss_rows"][rows], rtol=1e-15, atol=1e-15)
    np.testing.assert_allclose(O.dH_rows(H[rows], W, y[rows], b["gamma"], IGN), b["dH"][rows], atol=1e-16)
    ids = np.array([0, 5, 39, int(y[y != IGN][0])])
    got = O.dW_rows(H, W[ids], ids, y, f["lse"], b["gamma"], IGN, V=40, block_rows=13)
    np.testing.assert_allclose(got, b["dW"][ids], atol=1e-15)


# ---- P13: per-row upstream gradients and label smoothing ------------------
def test_per_row_variant_reduces_to_the_scalar_one():
    """eps = 0 and a constant upstream gradient are the mean / sum pipeline."""
    H, W, y = rand_case(21, 19, 7, 23, n_ignored=4, w_std=1.0)
    f = O.forward(H, W, y, IGN, "sum")
    pr = O.forward_per_row(H, W, y, IGN, 0.0)
    np.testing.assert_allclose(pr["loss_rows"], f["loss_rows"], rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(pr["lse"], f["lse"], rtol=1e-15)
    assert np.all(pr["loss_rows"][y == IGN] == 0.0)
    b = O.backward(H, W, y, IGN, "mean", 0.7)
    br = O.backward_per_row(H, W, y, np.full(len(y), 0.7 / f["n_valid"]), IGN, 0.0)
    np.testing.assert_allclose(br["dH"], b["dH"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(br["dW"], b["dW"], rtol=0, atol=1e-15)


@pytest.mark.parametrize("eps", [0.0, 0.1, 0.35])
def test_label_smoothing_closed_forms_and_invariants(eps):
    N, d, V = 9, 6, 11
    H, W, y = rand_case(22, N, d, V, n_ignored=2, w_std=1.0)
    # W = 0: every log-probability is -ln V, so the loss is ln V whatever eps; G = 1/V - q
    z = O.forward_per_row(H, np.zeros_like(W), y, IGN, eps)
    np.testing.assert_allclose(z["loss_rows"][y != IGN], math.log(V), rtol=1e-15)
    gr = np.linspace(0.5, 1.5, N)
    b0 = O.backward_per_row(H, np.zeros_like(W), y, gr, IGN, eps)
    assert np.abs(b0["dH"]).max() == 0.0
    want = np.zeros((V, d))
    for i in range(N):
        if y[i] == IGN:
            continue
        q = np.full(V, eps / V)
        q[y[i]] += 1.0 - eps
        want += np.outer(gr[i] * (1.0 / V - q), H[i])
    np.testing.assert_allclose(b0["dW"], want, rtol=0, atol=1e-15)
    # rows of G sum to zero (p and q both sum to one): dW's column sums vanish, <dH,H> = <dW,W>
    b = O.backward_per_row(H, W, y, gr, IGN, eps)
    assert np.abs(b["dW"].sum(axis=0)).max() < 1e-14
    assert abs((b["dH"] * H).sum() - (b["dW"] * W).sum()) < 1e-13
    # the smoothed loss is the plain loss mixed with the cross-entropy against the uniform distribution
    p0 = O.forward_per_row(H, W, y, IGN, 0.0)
    Z = H @ W.T
    unif = p0["lse"] - Z.mean(axis=1)
    pe = O.forward_per_row(H, W, y, IGN, eps)
    ok = y != IGN
    np.testing.assert_allclose(pe["loss_rows"][ok], ((1 - eps) * p0["loss_rows"] + eps * unif)[ok], rtol=1e-13)


@pytest.mark.parametrize("eps", [0.0, 0.2])
def test_per_row_finite_differences(eps):
    N, d, V = 5, 4, 7
    H, W, y = rand_case(23, N, d, V, n_ignored=1, w_std=1.0)
    gr = np.array([0.3, -1.2, 2.0, 0.9, 1.1])
    b = O.backward_per_row(H, W, y, gr, IGN, eps)
    h = 1e-6

    def L(Hx, Wx):
        return float(gr @ O.forward_per_row(Hx, Wx, y, IGN, eps)["loss_rows"])

    for A, dA, which in ((H, b["dH"], 0), (W, b["dW"], 1)):
        fd = np.zeros_like(A)
        for idx in np.ndindex(*A.shape):
            Ap, Am = A.copy(), A.copy()
            Ap[idx] += h
            Am[idx] -= h
            fd[idx] = ((L(Ap, W) - L(Am, W)) if which == 0 else (L(H, Ap) - L(H, Am))) / (2 * h)
        np.testing.assert_allclose(dA, fd, rtol=0, atol=5e-8)


@pytest.mark.parametrize("eps", [0.0, 0.1])
def test_per_row_against_torch_label_smoothing(eps):
    torch = pytest.importorskip("torch")
    H, W, y = rand_case(24, 29, 12, 41, n_ignored=4, w_std=1.0)
    gr = np.random.default_rng(3).standard_normal(len(y))
    Ht = torch.tensor(H, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    rows = torch.nn.functional.cross_entropy(Ht @ Wt.T, torch.tensor(y), ignore_index=IGN, reduction="none",
                                             label_smoothing=eps)
    (rows * torch.tensor(gr)).sum().backward()
    f = O.forward_per_row(H, W, y, IGN, eps)
    b = O.backward_per_row(H, W, y, gr, IGN, eps)
    np.testing.assert_allclose(f["loss_rows"], rows.detach().numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(b["dH"], Ht.grad.numpy(), rtol=0, atol=1e-13)
    np.testing.assert_allclose(b["dW"], Wt.grad.numpy(), rtol=0, atol=1e-13)
