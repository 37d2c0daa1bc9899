"""Plain fp64 CPU oracle for the computation GuidedQuant adds to layer-wise PTQ.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
what the HIP path must compute.  It shares no code with the HIP path and is
never imported by the product package; only tests, the smoke check and the
benchmark's cpu_baseline leg call it.

Every function is the definition from the paper written out in numpy float64
(a matmul is used as a library step where the definition is a matrix product;
there is no blocking, fusion or reordering beyond what the definition states).

Notation (paper, Section 3 "GuidedQuant", Algorithm 1):
    X   [n, d_in]    input feature map of one linear layer, rows = tokens
    dZ  [n, d_out]   gradient of the end loss w.r.t. the layer output Z = X W
    g   (here G)     number of groups of output channels
    J_k              k-th group: d_out/G consecutive output channels
    s_k [n]          mean over j in J_k of dZ[:, j]**2
    Hbar_k           X^T Diag(s_k) X                       [d_in, d_in]
    W, What          weights before/after quantization; HERE stored
                     [d_out, d_in] (row j = output channel j), i.e. the
                     transpose of the paper's [d_in, d_out] layout.

The assignment step that consumes Hbar_k (Section 4.2, Algorithm 2 lines 6-12 with
the closed form of Eq. "cd_closed") is `cd_assign`; being an iterative heuristic it
follows the algorithm's steps in the paper's order: cycles, then coordinates in
increasing order, one closed-form minimisation each.

`damped_cholesky`, `gptq_assign` and `ldlq_assign` cover the sequential-rounding quantizers the
paper feeds its Hessians to (GPTQ in SpinQuant, LDLQ in QTIP): published algorithms, restated.

Pins (tests/test_oracle_pins.py) check every function against closed forms,
a hand-worked example, an independent BLAS routine (dsyrk), and brute-force
evaluation of the paper's *un-averaged* definitions (per-channel Hessians,
the Frobenius form of the objective) on tiny inputs.  No function here is
"parity unpinned".
"""
from __future__ import annotations

import numpy as np

_F64 = np.float64


def group_partition(d_out: int, G: int):
    """Algorithm 1, line 1: contiguous groups J_k of d_out/G channels.

    Returns a list of (start, stop) half-open, 0-based channel ranges.
    The paper assumes G divides d_out; anything else is an error.
    """
    if G <= 0 or d_out <= 0 or d_out % G != 0:
        raise ValueError("G must be positive and divide d_out")
    m = d_out // G
    return [(k * m, (k + 1) * m) for k in range(G)]


def group_weights(dZ, G: int, grad_scale: float = 1.0) -> np.ndarray:
    """Algorithm 1, line 2: s[i, k] = (1/|J_k|) * sum_{j in J_k} (c * dZ[i, j])**2.

    `grad_scale` (c) is the constant the paper multiplies the gradients by while
    computing the averaged Hessians (Section 3.2, last paragraph before
    Algorithm 1; 1e3 in its experiments).  It is applied to dZ before squaring
    and is not undone.
    """
    dZ = np.asarray(dZ, dtype=_F64)
    n, d_out = dZ.shape
    s = np.empty((n, G), dtype=_F64)
    for k, (j0, j1) in enumerate(group_partition(d_out, G)):
        g = grad_scale * dZ[:, j0:j1]
        s[:, k] = np.sum(g * g, axis=1) / (j1 - j0)
    return s


def fisher_gram(X, s, H=None) -> np.ndarray:
    """Algorithm 1, line 4: Hbar_k = X^T Diag(s_k) X for every group k.

    X [n, d_in], s [n, G] -> H [G, d_in, d_in] (full squares).  If `H` is given
    the result is added to it (accumulation over token chunks: the sum over
    tokens in the definition splits over disjoint chunks).
    """
    X = np.asarray(X, dtype=_F64)
    s = np.asarray(s, dtype=_F64)
    n, d_in = X.shape
    G = s.shape[1]
    assert s.shape[0] == n
    if H is None:
        H = np.zeros((G, d_in, d_in), dtype=_F64)
    for k in range(G):
        H[k] += X.T @ (s[:, k][:, None] * X)
    return H


def fisher_gram_block(X, s_k, rows, cols) -> np.ndarray:
    """Entries Hbar_k[rows, cols] of Algorithm 1, line 4, for one group.

    s_k is the length-n weight vector of that group; rows/cols are slices or
    index arrays into the d_in axis.  Same definition as `fisher_gram`,
    restricted to a block of entries so that large shapes can be sampled.
    """
    X = np.asarray(X)
    s_k = np.asarray(s_k, dtype=_F64)
    A = np.asarray(X[:, rows], dtype=_F64)
    B = np.asarray(X[:, cols], dtype=_F64)
    return A.T @ (s_k[:, None] * B)


def objective(W, What, H, G: int | None = None):
    """Eq. (ours2): sum_k sum_{j in J_k} (w_j - what_j)^T Hbar_k (w_j - what_j).

    W, What [d_out, d_in] (row j = channel j), H [G, d_in, d_in].
    Returns (obj[G], obj_row[d_out]); obj[k] is the inner sum over J_k and
    obj_row[j] the single quadratic form of channel j.  The layer objective of
    the paper is obj.sum().
    """
    W = np.asarray(W, dtype=_F64)
    What = np.asarray(What, dtype=_F64)
    H = np.asarray(H, dtype=_F64)
    if G is None:
        G = H.shape[0]
    d_out, d_in = W.shape
    assert H.shape == (G, d_in, d_in)
    delta = W - What
    obj = np.zeros(G, dtype=_F64)
    obj_row = np.zeros(d_out, dtype=_F64)
    for k, (j0, j1) in enumerate(group_partition(d_out, G)):
        Dk = delta[j0:j1]
        obj_row[j0:j1] = np.sum((Dk @ H[k]) * Dk, axis=1)
        obj[k] = obj_row[j0:j1].sum()
    return obj, obj_row


# ----------------------------------------------------------------------------
# Definitional variants: the paper's un-averaged quantities.  They never go
# through s or Hbar and are used by the tests to pin the functions above.
# ----------------------------------------------------------------------------

def per_channel_hessian(X, dZ, j: int, grad_scale: float = 1.0) -> np.ndarray:
    """H_j = X^T Diag(dZ[:, j])^2 X (Section 3.2, the chain-rule identity for
    H_j = n F_j), built as an explicit sum of outer products over tokens."""
    X = np.asarray(X, dtype=_F64)
    dZ = np.asarray(dZ, dtype=_F64)
    n, d_in = X.shape
    Hj = np.zeros((d_in, d_in), dtype=_F64)
    for i in range(n):
        g = grad_scale * dZ[i, j]
        Hj += (g * g) * np.outer(X[i], X[i])
    return Hj


def unaveraged_objective(X, dZ, W, What, grad_scale: float = 1.0) -> float:
    """Eq. (ours): || dZ (.) (X W - X What) ||_F^2, with W stored [d_out, d_in]
    so that Z = X W^T in this layout.  Written as the double sum over tokens
    and channels of the right-hand side of that equation."""
    X = np.asarray(X, dtype=_F64)
    dZ = np.asarray(dZ, dtype=_F64)
    W = np.asarray(W, dtype=_F64)
    What = np.asarray(What, dtype=_F64)
    n, d_out = dZ.shape
    total = 0.0
    for i in range(n):
        for j in range(d_out):
            z = float(np.dot(X[i], W[j]))
            zhat = float(np.dot(X[i], What[j]))
            total += (grad_scale * dZ[i, j] * (z - zhat)) ** 2
    return total


def objective_from_tokens(X, s_k, delta_j) -> float:
    """sum_i s_k[i] * (x_i . delta_j)^2: the quadratic form delta^T Hbar_k delta
    evaluated from X without ever forming Hbar_k (same step as in the proof of
    Remark 3.1, applied to the averaged weights)."""
    X = np.asarray(X, dtype=_F64)
    s_k = np.asarray(s_k, dtype=_F64)
    delta_j = np.asarray(delta_j, dtype=_F64)
    total = 0.0
    for i in range(X.shape[0]):
        t = float(np.dot(X[i], delta_j))
        total += s_k[i] * t * t
    return total


def objective_rows_from_tokens(X, s_k, delta_rows) -> np.ndarray:
    """sum_i s_k[i] * (x_i . delta_j)^2 for several channels j at once (rows of
    `delta_rows`), i.e. `objective_from_tokens` with the token loop written as
    one matrix product.  Used to sample the objective at sizes where Hbar_k is
    too large to form on the host."""
    X = np.asarray(X, dtype=_F64)
    s_k = np.asarray(s_k, dtype=_F64)
    D = np.asarray(delta_rows, dtype=_F64)
    T = X @ D.T                      # [n, rows]: x_i . delta_j
    return (s_k[:, None] * T * T).sum(axis=0)



def cd_coordinate_target(w_j, what_j, H_k, i: int) -> float:
    """Eq. "cd_closed" (Section 4.2): the unconstrained minimiser of
    (what - w)^T H (what - w) over coordinate i alone, all others fixed:
        t = w[i] - sum_{i' != i} H[i, i'] / H[i, i] * (what[i'] - w[i']).
    """
    w_j = np.asarray(w_j, dtype=_F64)
    delta = np.asarray(what_j, dtype=_F64) - w_j
    H_k = np.asarray(H_k, dtype=_F64)
    off = H_k[i] @ delta - H_k[i, i] * delta[i]
    return float(w_j[i] - off / H_k[i, i])


def cd_assign(W, What, codebook, H, G: int | None = None, n_cycles: int = 1):
    """Cyclic coordinate descent on the assignments (Algorithm 2, lines 6-12, with the
    closed-form coordinate update of Eq. "cd_closed_par"), every output channel of
    group k against that group's Hbar_k.

    W, What   [d_out, d_in]  original weights and the current feasible quantized weights
    codebook  [d_out, m]     the grid {c_1..c_m} of every output channel
    H         [G, d_in, d_in] full symmetric matrices with positive diagonals

    For cycle = 1..n_cycles, for i = 0..d_in-1 (in this order): every channel j replaces
    What[j, i] by the point of its grid nearest to the coordinate target t of Eq.
    "cd_closed", computed from the current What (coordinates < i already updated in
    this cycle).  Among equally near grid points the one with the lowest index wins.
    Returns (Q [d_out, d_in] int64 grid indices, What_new [d_out, d_in] float64); a
    coordinate's index is that of its last update.
    """
    W = np.asarray(W, dtype=_F64)
    What = np.array(What, dtype=_F64, copy=True)
    C = np.asarray(codebook, dtype=_F64)
    H = np.asarray(H, dtype=_F64)
    if H.ndim == 2:
        H = H[None]
    G = H.shape[0] if G is None else G
    d_out, d_in = W.shape
    Q = np.zeros((d_out, d_in), dtype=np.int64)
    for k, (j0, j1) in enumerate(group_partition(d_out, G)):
        Hk = H[k]
        diag = np.diag(Hk)
        if np.any(diag <= 0):
            raise ValueError("H must have a positive diagonal")
        Wk, Ck = W[j0:j1], C[j0:j1]
        delta = What[j0:j1] - Wk                       # [rows, d_in]
        rows = np.arange(j1 - j0)
        for _ in range(n_cycles):
            for i in range(d_in):
                off = delta @ Hk[i] - Hk[i, i] * delta[:, i]     # sum over i' != i
                t = Wk[:, i] - off / Hk[i, i]
                q = np.argmin(np.abs(Ck - t[:, None]), axis=1)   # first minimum = lowest index
                Q[j0:j1, i] = q
                What[j0:j1, i] = Ck[rows, q]               # the grid value itself, not w + (c - w)
                delta[:, i] = What[j0:j1, i] - Wk[:, i]
    return Q, What


def lnq_codebook(W, Q, H, n_levels: int, G: int | None = None, lam: float = 1e-7):
    """Closed-form codebook update of LNQ for fixed assignments (Section 4.2, Eq. "conti-sol",
    Algorithm 2 lines 4 and 14), every output channel j of group k against that group's Hbar_k:

        c^(j) = (P^T H P + lam I)^-1 P^T H w_j,     P[i, q] = 1 if Q[j, i] == q else 0,

    with the small constant lam (1e-7 in the paper) on the diagonal, which also settles grid
    points that no coordinate is assigned to (their value becomes 0).
    W [d_out, d_in], Q [d_out, d_in] integer grid indices in [0, n_levels), H [G, d_in, d_in].
    Returns (codebook [d_out, n_levels] float64, What [d_out, d_in] = P c).
    """
    W = np.asarray(W, dtype=_F64)
    Q = np.asarray(Q)
    H = np.asarray(H, dtype=_F64)
    if H.ndim == 2:
        H = H[None]
    G = H.shape[0] if G is None else G
    d_out, d_in = W.shape
    if Q.shape != W.shape or Q.min() < 0 or Q.max() >= n_levels:
        raise ValueError("Q must hold grid indices in [0, n_levels) for every weight")
    C = np.zeros((d_out, n_levels), dtype=_F64)
    What = np.empty_like(W)
    for k, (j0, j1) in enumerate(group_partition(d_out, G)):
        Hk = H[k]
        for j in range(j0, j1):
            P = np.zeros((d_in, n_levels), dtype=_F64)
            P[np.arange(d_in), Q[j]] = 1.0
            A = P.T @ Hk @ P + lam * np.eye(n_levels)
            b = P.T @ (Hk @ W[j])
            C[j] = np.linalg.solve(A, b)
            What[j] = P @ C[j]
    return C, What


def lnq(W, Q, H, n_levels: int, G: int | None = None, n_iters: int = 2, n_cycles: int = 4, lam: float = 1e-7):
    """Algorithm 2 (LNQ) against the group Hessians: starting from the assignments Q, n_iters (T) times
    {closed-form grids for the current assignments (line 4), What = P c (line 5), n_cycles (K) cycles of
    coordinate descent on the assignments (lines 6-12)}, then the grids once more (line 14).
    Returns (Q, What, codebook, trace) with trace the layer objective summed over the groups after every
    codebook step and every batch of CD cycles, in order."""
    W = np.asarray(W, dtype=_F64)
    H = np.asarray(H, dtype=_F64)
    if H.ndim == 2:
        H = H[None]
    G = H.shape[0] if G is None else G
    Q = np.array(Q, dtype=np.int64, copy=True)
    trace = []
    for _ in range(n_iters):
        C, What = lnq_codebook(W, Q, H, n_levels, G, lam)
        trace.append(float(objective(W, What, H, G)[0].sum()))
        if n_cycles > 0:
            Q, What = cd_assign(W, What, C, H, G, n_cycles)
            trace.append(float(objective(W, What, H, G)[0].sum()))
    C, What = lnq_codebook(W, Q, H, n_levels, G, lam)
    trace.append(float(objective(W, What, H, G)[0].sum()))
    return Q, What, C, trace


def damped_cholesky(H, damp_rel: float = 0.01, damp_abs: float = 0.0, reverse: bool = False) -> np.ndarray:
    """The triangular factor of the damped group Hessians (Algorithm 2, line 1; Section 4.2:
    a small constant is added to the diagonal so that the matrix is positive definite).

        eps_k = damp_abs + damp_rel * mean_i H[k][i, i]
        reverse=False:  H[k] + eps_k I = L L^T,  L lower triangular, positive diagonal
        reverse=True:   H[k] + eps_k I = R R^T,  R UPPER triangular, positive diagonal
                        (the factorization taken from the last coordinate backwards; it is the one
                        whose columns give the feedback of sequential rounding in the order
                        0, 1, ..., d_in-1, see `ldlq_assign`)

    The paper leaves the constant open; the relative form is the convention of the GPTQ line of
    work it cites (a fraction of the mean diagonal).  H [G, d, d] (or [d, d]) full symmetric.
    numpy's Cholesky routine is the library step; the reverse form is the same routine applied to
    the matrix with rows and columns in reverse order.
    """
    H = np.asarray(H, dtype=_F64)
    squeeze = H.ndim == 2
    if squeeze:
        H = H[None]
    out = np.empty_like(H)
    d = H.shape[1]
    for k in range(H.shape[0]):
        A = H[k] + (damp_abs + damp_rel * np.mean(np.diag(H[k]))) * np.eye(d)
        if reverse:
            out[k] = np.linalg.cholesky(A[::-1, ::-1])[::-1, ::-1]
        else:
            out[k] = np.linalg.cholesky(A)
    return out[0] if squeeze else out


def _nearest(grid_rows, t):
    """Index of the grid point nearest to t, per row; the lowest index among equals."""
    return np.argmin(np.abs(grid_rows - t[:, None]), axis=1)


def gptq_assign(W, codebook, H, G: int | None = None, damp_rel: float = 0.01, damp_abs: float = 0.0):
    """Sequential rounding with error feedback as published by Frantar et al. (GPTQ, the weight
    quantizer the paper plugs its Hessians into for SpinQuant, Appendix "Implementation Details
    for Different Quantization Types", and the alternative assignment step of its LNQ ablation),
    without the lazy batching, which does not change the result: with A = H[k] + eps_k I
    (eps_k as in `damped_cholesky`), A^-1 = T^T T, T upper triangular, for i = 0..d_in-1:

        q_i = nearest grid point of the current w_i;  e = (w_i - q_i) / T[i, i];
        w_{i'} -= e * T[i, i']   for i' > i.

    W [d_out, d_in], codebook [d_out, m] (the grid of every channel; a uniform grid is a special
    case), H [G, d_in, d_in].  Returns (Q int64 indices, What float64 grid values).
    """
    W = np.asarray(W, dtype=_F64)
    C = np.asarray(codebook, dtype=_F64)
    H = np.asarray(H, dtype=_F64)
    if H.ndim == 2:
        H = H[None]
    G = H.shape[0] if G is None else G
    d_out, d_in = W.shape
    Q = np.zeros((d_out, d_in), dtype=np.int64)
    What = np.empty_like(W)
    for k, (j0, j1) in enumerate(group_partition(d_out, G)):
        A = H[k] + (damp_abs + damp_rel * np.mean(np.diag(H[k]))) * np.eye(d_in)
        T = np.linalg.cholesky(np.linalg.inv(A)).T          # A^-1 = T^T T, T upper
        Wk = W[j0:j1].copy()
        Ck = C[j0:j1]
        rows = np.arange(j1 - j0)
        for i in range(d_in):
            q = _nearest(Ck, Wk[:, i])
            Q[j0:j1, i] = q
            What[j0:j1, i] = Ck[rows, q]
            e = (Wk[:, i] - What[j0:j1, i]) / T[i, i]
            Wk[:, i + 1:] -= e[:, None] * T[i, i + 1:][None, :]
    return Q, What


def ldlq_assign(W, codebook, R, G: int | None = None):
    """The same rounding written with the factor of the matrix itself instead of its inverse
    (the LDLQ form of Chee et al., which the QTIP quantizer the paper also builds on uses
    block-wise): with A = R R^T, R upper triangular (`damped_cholesky(..., reverse=True)`),
    for i = 0..d_in-1

        What[j, i] = nearest grid point of  W[j, i] - sum_{i' < i} (What[j, i'] - W[j, i']) * R[i', i] / R[i, i].

    R [G, d_in, d_in].  Returns (Q, What, Tgt) with Tgt the targets that were rounded.
    """
    W = np.asarray(W, dtype=_F64)
    C = np.asarray(codebook, dtype=_F64)
    R = np.asarray(R, dtype=_F64)
    if R.ndim == 2:
        R = R[None]
    G = R.shape[0] if G is None else G
    d_out, d_in = W.shape
    Q = np.zeros((d_out, d_in), dtype=np.int64)
    What = np.empty_like(W)
    Tgt = np.empty_like(W)
    for k, (j0, j1) in enumerate(group_partition(d_out, G)):
        Rk = R[k]
        Wk, Ck = W[j0:j1], C[j0:j1]
        rows = np.arange(j1 - j0)
        delta = np.zeros_like(Wk)
        for i in range(d_in):
            t = Wk[:, i] - delta[:, :i] @ (Rk[:i, i] / Rk[i, i])
            q = _nearest(Ck, t)
            Q[j0:j1, i] = q
            What[j0:j1, i] = Ck[rows, q]
            Tgt[j0:j1, i] = t
            delta[:, i] = What[j0:j1, i] - Wk[:, i]
    return Q, What, Tgt
