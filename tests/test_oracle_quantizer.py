"""Pins for oracle/quantizer.py (CPU only): what the paper and the mathematics fix."""
import itertools

import numpy as np

from oracle import fuse, quantizer as Q


def _layer(M, N, T, seed):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((M, N)) * 0.05
    A = rng.standard_normal((N, N)) * 0.3 + np.eye(N)          # correlated input channels
    X = A @ rng.standard_normal((N, T))
    return W, X


def test_scale_grid_stays_inside_the_interval_of_eq7():
    g = Q.scale_grid(-1.0, 2.0, 5, 7)
    lo, hi = 3.0 / 63, 3.0 / 15
    assert len(g) == 7 and np.all(g > lo) and np.all(g < hi) and np.all(np.diff(g) > 0)
    assert np.isclose(g[3], (lo + hi) / 2)                      # odd grid: the middle point is the midpoint


def test_quant_row_reproduces_the_papers_example():
    """Eq. 6: W_int = [0,2,3,1,1,6,5], BCchoice = [0,1,6,7] -> [0,1,1,1,1,6,6]; with S = 1, qbias = 0 the
    linear step is the identity on these integers."""
    w = np.array([0, 2, 3, 1, 1, 6, 5], dtype=np.float64)
    assert Q.quant_row(w, 1.0, 0.0, [0, 1, 6, 7], 3).tolist() == [0, 1, 1, 1, 1, 6, 6]


def test_search_is_the_brute_force_argmin():
    """Tiny layer: every (scale, tied-plane set) pair enumerated independently with explicit
    matrix products on X (not on H)."""
    W, X = _layer(5, 12, 40, 1)
    n, q, grid = 3, 2, 5
    S, b, pi, err = Q.search(W, Q.hessian(X), n, q, grid)
    parts = fuse.all_partitions(n, q)
    for m in range(W.shape[0]):
        w = W[m]
        best = None
        for s, (k, p) in itertools.product(Q.scale_grid(w.min(), w.max(), n, grid), enumerate(parts)):
            w_int = np.clip(np.rint((w - w.min()) / s), 0, 2 ** n - 1)
            choice = np.array(fuse.bcchoice(p, n))
            w_q = choice[np.abs(w_int[:, None] - choice[None, :]).argmin(axis=1)]
            e = float(np.sum(((s * w_q + w.min() - w) @ X) ** 2))
            if best is None or e < best[0] - 1e-12 * abs(best[0]):
                best = (e, s, k)
        assert np.isclose(err[m], best[0], rtol=1e-9)
        assert np.isclose(S[m], best[1]) and pi[m] == best[2] and b[m] == w.min()


def test_gptq_with_uncorrelated_inputs_is_round_to_nearest():
    """Diagonal H: the inverse Hessian has no off-diagonal terms, so Eq. 2 changes no other
    weight and every weight is simply quantised in place."""
    W, _ = _layer(4, 10, 8, 2)
    H = np.diag(np.linspace(1.0, 3.0, 10))
    n, q = 4, 3
    part = fuse.all_partitions(n, q)[2]
    choice = fuse.bcchoice(part, n)
    S = (W.max(1) - W.min(1)) / (2 ** n - 1)
    b = W.min(1)
    for f in (Q.gptq_definition, Q.gptq):
        Wq = f(W, H, S, b, [choice] * 4, n)
        for m in range(4):
            assert np.array_equal(Wq[m], Q.quant_row(W[m], S[m], b[m], choice, n))


def test_eq2_is_the_least_squares_compensation():
    """One step of Eq. 2 on one row: fixing w_0 to its quantised value and moving the others by
    delta_F must minimise the output change ||(w' - w) X||^2 over all w' with w'_0 fixed --
    compared with numpy's least-squares solution of that constrained problem."""
    rng = np.random.default_rng(3)
    N, T = 6, 30
    X = rng.standard_normal((N, T))
    w = rng.standard_normal(N)
    target0 = w[0] + 0.37                                       # "quant(w_0)"
    H = Q.hessian(X)
    Hinv = np.linalg.inv(H)
    delta = Q.eq2_delta(w[0] - target0, Hinv)                   # the oracle's Eq. 2
    assert np.isclose(w[0] + delta[0], target0)
    # minimise ||d X||^2 with d_0 = target0 - w_0: d_rest = argmin || d_0 X_0 + d_rest X_rest ||
    d0 = target0 - w[0]
    d_rest = np.linalg.lstsq(X[1:].T, -d0 * X[0], rcond=None)[0]
    assert np.allclose(delta[1:], d_rest, rtol=1e-9, atol=1e-12)


def test_cholesky_form_equals_the_definition():
    """Recomputing the remaining inverse Hessian at every column (Eq. 1-2 as printed) and the
    single Cholesky factorisation give the same integers."""
    W, X = _layer(6, 16, 64, 4)
    n, q = 4, 3
    H = Q.hessian(X)
    parts = fuse.all_partitions(n, q)
    choices = [fuse.bcchoice(parts[m % len(parts)], n) for m in range(6)]
    S = (W.max(1) - W.min(1)) / (2 ** n - 1)
    b = W.min(1)
    A = Q.gptq_definition(W, H, S, b, choices, n)
    B = Q.gptq(W, H, S, b, choices, n)
    assert np.array_equal(A, B)
    for m in range(6):
        assert set(A[m]).issubset(set(choices[m]))


def test_compensation_lowers_the_output_error():
    """The point of Eq. 2: on correlated inputs GPTQ's output error is below round-to-nearest's
    (a property of the method, on average over rows)."""
    W, X = _layer(24, 48, 256, 5)
    n, q = 4, 3
    H = Q.hessian(X)
    part = fuse.all_partitions(n, q)[0]
    choice = fuse.bcchoice(part, n)
    S = (W.max(1) - W.min(1)) / (2 ** n - 1)
    b = W.min(1)
    Wq = Q.gptq(W, H, S, b, [choice] * 24, n)
    rtn = np.stack([Q.quant_row(W[m], S[m], b[m], choice, n) for m in range(24)])
    e_gptq = Q.output_error(W, Wq, S, b, H)
    e_rtn = Q.output_error(W, rtn, S, b, H)
    assert e_gptq.sum() < 0.8 * e_rtn.sum()
    assert np.mean(e_gptq < e_rtn) > 0.7


def test_output_error_is_the_squared_error_of_the_layer_outputs():
    """Eq. 5's criterion, read as the row's output error: output_error (evaluated through H = 2 X X^T) equals
    || w_hat X - w X ||^2 computed on the calibration inputs themselves, row by row."""
    W, X = _layer(7, 24, 96, 11)
    rng = np.random.default_rng(12)
    n = 3
    S = rng.uniform(0.01, 0.05, size=7)
    b = rng.uniform(-0.2, 0.0, size=7)
    Wq = rng.integers(0, 2 ** n, size=W.shape).astype(np.float64)
    e = Q.output_error(W, Wq, S, b, Q.hessian(X))
    for m in range(7):
        w_hat = S[m] * Wq[m] + b[m]
        direct = sum((w_hat @ X[:, t] - W[m] @ X[:, t]) ** 2 for t in range(X.shape[1]))
        assert np.isclose(e[m], direct, rtol=1e-10, atol=0.0)
    assert np.all(Q.output_error(W, (W - b[:, None]) / S[:, None], S, b, Q.hessian(X)) < 1e-20)  # w_hat = w: no error


def test_cholesky_factor_is_the_upper_factor_of_the_dampened_inverse():
    """U of the GPTQ pass: upper triangular with positive diagonal, U^T U (H + damp mean(diag H) I) = I;
    damp = 0 on a diagonal H gives diag(1 / sqrt(h))."""
    _, X = _layer(1, 20, 64, 13)
    H = Q.hessian(X)
    for damp in (0.01, 0.25):
        U = Q.cholesky_factor(H, damp)
        assert np.allclose(U, np.triu(U)) and np.all(np.diag(U) > 0)
        Hd = H + damp * np.mean(np.diag(H)) * np.eye(20)
        assert np.allclose(U.T @ U @ Hd, np.eye(20), atol=1e-9)
    h = np.array([4.0, 0.25, 9.0])
    assert np.allclose(Q.cholesky_factor(np.diag(h), 0.0), np.diag(1.0 / np.sqrt(h)))


def test_search_then_fuse_round_trip():
    """The searched parameters feed oracle.fuse unchanged: dequantising the fused planes gives
    S W_q + qbias for every row's own tied-plane set."""
    W, X = _layer(3, 64, 96, 6)
    n, q = 5, 3
    H = Q.hessian(X)
    S, b, pi, _ = Q.search(W, H, n, q, 4)
    parts = fuse.all_partitions(n, q)
    for m in range(3):
        choice = fuse.bcchoice(parts[pi[m]], n)
        Wq = Q.quant_row(W[m], S[m], b[m], choice, n)[None, :]
        planes, alpha, z = fuse.fuse(Wq, S[m:m + 1, None], b[m:m + 1, None], parts[pi[m]], n, 64)
        signs = np.stack([2.0 * ((planes[i, 0, :, None] >> np.arange(32)) & 1).reshape(-1) - 1 for i in range(q)])
        w_hat = (alpha[0, 0][:, None] * signs).sum(0) + z[0, 0]
        assert np.allclose(w_hat, S[m] * Wq[0] + b[m], rtol=1e-12, atol=1e-15)


def test_constant_row_is_reproduced():
    """Degenerate case: W_max = W_min leaves Eq. 7's interval empty; the row is then reproduced exactly
    (scale 1, integers 0, qbias = the constant)."""
    rng = np.random.default_rng(3)
    W = rng.standard_normal((3, 32)) * 0.02
    W[1] = 0.0173
    H = Q.hessian(rng.standard_normal((32, 64)))
    S, b, p, e = Q.search(W, H, 3, 2, 4)
    assert S[1] == 1.0 and b[1] == 0.0173 and e[1] == 0.0 and p[1] == 0
    parts = fuse.all_partitions(3, 2)
    choices = [fuse.bcchoice(parts[i], 3) for i in p]
    Wq = Q.gptq(W, H, S, b, choices, 3)
    assert (Wq[1] == 0).all()


def test_gptq_follow_replays_gptq_and_reports_forced_columns():
    """gptq_follow with gptq()'s own integers reports nothing; with one integer replaced it reports
    exactly that column (with the working weight gptq() had there), and the later columns of that
    row, re-derived by gptq() from the changed history, are reproduced by following them."""
    W, X = _layer(6, 24, 60, 7)
    H = Q.hessian(X)
    n, q = 3, 2
    part = fuse.all_partitions(n, q)[1]
    choice = fuse.bcchoice(part, n)
    S = (W.max(1) - W.min(1)) / (2 ** n - 1)
    b = W.min(1)
    choices = [choice] * W.shape[0]
    Wq = Q.gptq(W, H, S, b, choices, n)
    U = Q.cholesky_factor(H)
    assert Q.gptq_follow(W, U, S, b, choices, n, Wq) == []
    # force another member of the set at (2, 5); rebuild the rest of the row as the definition would
    forced = Wq.copy()
    other = [c for c in choice if c != Wq[2, 5]][0]
    forced[2, 5] = other
    w = W[2].astype(np.float64).copy()
    for j in range(W.shape[1]):
        wq = forced[2, j] if j <= 5 else Q.quant_row(w[j:j + 1], S[2], b[2], choice, n)[0]
        forced[2, j] = wq
        w[j:] -= (w[j] - (S[2] * wq + b[2])) / U[j, j] * U[j, j:]
    ev = Q.gptq_follow(W, U, S, b, choices, n, forced)
    assert len(ev) == 1 and ev[0][:2] == (2, 5) and ev[0][3] == Wq[2, 5] and ev[0][4] == other
