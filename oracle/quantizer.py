"""Oracle for the GPTQT quantiser itself (paper Sec. II-A Eq. 1-2, Sec. II-B Eq. 5-6, Sec. II-C
Eq. 7 and the algorithm that closes Sec. II-D).  TEST INFRASTRUCTURE; numpy, fp64, written for
clarity: loops over rows, columns and candidates exactly as the paper states them.

Notation follows the paper: W [M][N] full-precision weights, X [N][T] calibration inputs,
H = 2 X X^T (Sec. II-A), n = bits of the intermediate linear quantisation, q = number of
binary-coding planes, S / qbias the linear scale and bias of a row (GPTQ fixes them row-wise).

Readings where the paper is silent (also listed in the design notes):
  * quantisation parameters are per row (Sec. II-A: "row-wisely"); the grid search of Eq. 7 and
    the choice of the tied-plane set are done per row, keeping the row's best pair;
  * qbias = W_min of the row; the first-step scale is (W_max - W_min) / (2^n - 1); Eq. 7's open
    interval is searched on `grid` equidistant interior points, ascending; for a constant row
    (W_max = W_min, Eq. 7's interval is empty) the scale is 1 and every integer is 0;
  * the search criterion of Eq. 5 ("argmin (W_q X)") is the output error of the row,
    ||(w_hat - w) X||^2 = (w_hat - w) (X X^T) (w_hat - w)^T, with w_hat = S' W_q + qbias and
    W_q = nearest-BCchoice(linear-quant(w)) -- no error compensation inside the search;
  * candidates are visited scale-major, tied-plane sets in the order of oracle.fuse.all_partitions;
    the first candidate with the smallest error wins;
  * the final pass is GPTQ (Eq. 1-2) with quant() = that row's S', qbias and BCchoice;
    dampening lambda = damp * mean(diag H) is added to H before inversion (standard for GPTQ;
    the paper does not give a value).
"""
import numpy as np

from oracle import fuse


def hessian(X):
    """H_F for the full set: 2 X X^T (Sec. II-A)."""
    X = np.asarray(X, dtype=np.float64)
    return 2.0 * X @ X.T


def scale_grid(w_min, w_max, n, grid):
    """Eq. 7: `grid` equidistant points strictly inside ((Wmax-Wmin)/(2^(n+1)-1), (Wmax-Wmin)/(2^(n-1)-1))."""
    if w_max == w_min:                                  # a constant row: every scale reproduces it (W_int = 0)
        return np.ones(grid)
    lo = (w_max - w_min) / (2 ** (n + 1) - 1)
    hi = (w_max - w_min) / (2 ** (n - 1) - 1)
    return lo + (hi - lo) * (np.arange(1, grid + 1) / (grid + 1.0))


def quant_row(w, S, qbias, choice, n):
    """Both steps of Eq. 5 for one row: linear quantisation, then nearest BCchoice (Eq. 6).
    Returns the integers W_q (members of `choice`)."""
    return fuse.nearest_bcchoice(fuse.linear_quantize(w, S, qbias, n), choice)


def search(W, H, n, q, grid):
    """Per row: the pair (S', tied-plane set) of smallest output error (Eq. 5, Eq. 7).
    Returns S [M], qbias [M], index into fuse.all_partitions(n, q) [M], error [M]."""
    W = np.asarray(W, dtype=np.float64)
    G = np.asarray(H, dtype=np.float64) / 2.0          # X X^T
    parts = fuse.all_partitions(n, q)
    choices = [fuse.bcchoice(p, n) for p in parts]
    M = W.shape[0]
    S_out, b_out = np.empty(M), np.empty(M)
    p_out, e_out = np.empty(M, dtype=np.int64), np.empty(M)
    for m in range(M):
        w = W[m]
        qbias = w.min()
        best = (np.inf, None, None)
        for S in scale_grid(w.min(), w.max(), n, grid):
            for pi, choice in enumerate(choices):
                d = S * quant_row(w, S, qbias, choice, n) + qbias - w
                err = float(d @ G @ d)
                if err < best[0]:
                    best = (err, S, pi)
        e_out[m], S_out[m], p_out[m] = best
        b_out[m] = qbias
    return S_out, b_out, p_out, e_out


def eq2_delta(err, Hinv):
    """Eq. 2: the change of the remaining weights F (first entry: the weight being quantised, which so
    lands on its quantised value) that compensates quantising it with error err = w_q - quant(w_q);
    Hinv = H_F^-1."""
    return -err / Hinv[0, 0] * Hinv[:, 0]


def gptq_definition(W, H, S, qbias, choices, n, damp=0.01):
    """GPTQ as Eq. 1-2 state it, with the inverse Hessian of the REMAINING weights recomputed
    from scratch at every column (slow; the definition).  choices[m] = BCchoice of row m.
    Returns W_q ints [M][N]."""
    W = np.array(W, dtype=np.float64)
    H = np.array(H, dtype=np.float64)
    M, N = W.shape
    H = H + damp * np.mean(np.diag(H)) * np.eye(N)
    Wq = np.empty((M, N), dtype=np.int64)
    for j in range(N):
        Hinv = np.linalg.inv(H[j:, j:])                # H_F^-1, F = columns j .. N-1
        for m in range(M):
            wq = quant_row(W[m, j:j + 1], S[m], qbias[m], choices[m], n)[0]
            Wq[m, j] = wq
            err = W[m, j] - (S[m] * wq + qbias[m])     # w_q - quant(w_q)
            W[m, j:] += eq2_delta(err, Hinv)           # Eq. 2 (its own component becomes quant(w_q))
    return Wq


def gptq(W, H, S, qbias, choices, n, damp=0.01):
    """The same pass through one Cholesky factorisation of H^-1 (the usual arrangement: with
    H^-1 = U^T U, U upper triangular, row j of U scaled by 1/U[j,j] is the column of the remaining
    inverse Hessian that Eq. 2 needs).  Returns W_q ints [M][N]."""
    W = np.array(W, dtype=np.float64)
    H = np.array(H, dtype=np.float64)
    M, N = W.shape
    H = H + damp * np.mean(np.diag(H)) * np.eye(N)
    U = np.linalg.cholesky(np.linalg.inv(H)).T         # upper, H^-1 = U^T U
    Wq = np.empty((M, N), dtype=np.int64)
    for j in range(N):
        for m in range(M):
            wq = quant_row(W[m, j:j + 1], S[m], qbias[m], choices[m], n)[0]
            Wq[m, j] = wq
            err = (W[m, j] - (S[m] * wq + qbias[m])) / U[j, j]
            W[m, j:] -= err * U[j, j:]
    return Wq


def gptq_follow(W, U, S, qbias, choices, n, follow):
    """The pass of gptq() with a given factor U (upper triangular, H^-1 = U^T U), replayed against the
    integers `follow` [M][N] of a second implementation: at every column the oracle takes its own
    decision (Eq. 5 step 1, Eq. 6) from its own binary64 working weight; where `follow` differs, the
    event is recorded and `follow`'s integer is taken instead, so that the compensation of Eq. 2 for the
    later columns follows the implementation under test.  Returns the list of such events as
    (m, j, t, own, taken) with t = (w - qbias) / S, the working weight in quantisation steps at that
    moment.  A parity test then shows that every event is a near-tie of the rounding of t (and that
    `taken` is what the other side of the tie gives); with an empty list `follow` equals gptq()'s result."""
    W = np.array(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    M, N = W.shape
    events = []
    for j in range(N):
        for m in range(M):
            own = int(quant_row(W[m, j:j + 1], S[m], qbias[m], choices[m], n)[0])
            wq = int(follow[m, j])
            if wq != own:
                events.append((m, j, float((W[m, j] - qbias[m]) / S[m]), own, wq))
            err = (W[m, j] - (S[m] * wq + qbias[m])) / U[j, j]
            W[m, j:] -= err * U[j, j:]
    return events


def cholesky_factor(H, damp=0.01):
    """U of gptq(): upper Cholesky factor of (H + damp * mean(diag H) I)^-1."""
    H = np.array(H, dtype=np.float64)
    H = H + damp * np.mean(np.diag(H)) * np.eye(H.shape[0])
    return np.linalg.cholesky(np.linalg.inv(H)).T


def output_error(W, Wq, S, qbias, H):
    """Per row (w_hat - w) (X X^T) (w_hat - w)^T with w_hat = S W_q + qbias."""
    D = S[:, None] * Wq + qbias[:, None] - np.asarray(W, dtype=np.float64)
    G = np.asarray(H, dtype=np.float64) / 2.0
    return np.einsum("mk,kl,ml->m", D, G, D)
