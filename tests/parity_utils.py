"""Helpers shared by the GPU parity tests (comparison metrics, host copies)."""
import numpy as np
import torch

TOL_F32 = 1e-5     # relative Frobenius error, fp32 path
TOL_BF16 = 3e-3    # relative Frobenius error, bf16 matrix-core path
TOL_S = 2e-6       # relative, per element of s


def to_np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_fro(a: np.ndarray, ref: np.ndarray) -> float:
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(a - ref) / den) if den > 0 else float(np.linalg.norm(a))


def upper(a: np.ndarray) -> np.ndarray:
    """Entries on or above the diagonal of the last two axes (others zeroed)."""
    return np.triu(a)


def say(msg: str) -> None:
    print(msg, flush=True)


# ------------------------------------------------------------------ sampled oracle for full-size shapes
def _host_cols(X: torch.Tensor, idx) -> np.ndarray:
    """Columns idx of a (GPU) matrix as fp64 on the host (exact for bf16/fp32 values)."""
    return X[:, torch.as_tensor(idx, device=X.device)].to(torch.float64).cpu().numpy()


def sampled_gram_check(oracle, X, s, H, tol, n_random=24, block=128, n_probe=4, seed=0, what=""):
    """Compare a (mirrored, full-square) GPU result H[G,d,d] with the fp64 oracle on
    (i) blocks of `block` x `block` entries: random ones, a run along the diagonal, the last
    block row/column and the blocks holding the largest-norm (outlier) columns, and
    (ii) probe vectors: H[k] v against X^T (s_k * (X v)), evaluated chunk-wise in fp64 on the host.
    Returns (rel-Frobenius over the sampled entries, max probe rel error, entries compared)."""
    rng = np.random.default_rng(seed)
    n, d = X.shape
    G = s.shape[1]
    nb = (d + block - 1) // block
    s64 = s.to(torch.float64).cpu().numpy()
    col_norm = X.to(torch.float32).pow(2).sum(0)
    hot = int(torch.argmax(col_norm).item()) // block
    pairs = {(nb - 1, nb - 1), (0, nb - 1), (0, 0), (hot, hot), (min(hot, nb - 1), nb - 1), (0, hot)}
    for t in range(min(3, nb)):
        b = int(rng.integers(0, nb))
        pairs.add((b, b))
        if b + 1 < nb:
            pairs.add((b, b + 1))
    while len(pairs) < n_random + 8 and len(pairs) < nb * (nb + 1) // 2:
        a, b = sorted(int(v) for v in rng.integers(0, nb, size=2))
        pairs.add((a, b))
    worst, entries = 0.0, 0
    num, den = np.zeros(G), np.zeros(G)
    for (bi, bj) in sorted(pairs):
        rows = np.arange(bi * block, min(d, (bi + 1) * block))
        cols = np.arange(bj * block, min(d, (bj + 1) * block))
        Xs = np.concatenate([_host_cols(X, rows), _host_cols(X, cols)], axis=1)
        for k in range(G):
            ref = oracle.fisher_gram_block(Xs, s64[:, k], slice(0, len(rows)), slice(len(rows), len(rows) + len(cols)))
            got = H[k][bi * block:bi * block + len(rows), bj * block:bj * block + len(cols)].to(torch.float64).cpu().numpy()
            err = rel_fro(got, ref)
            worst = max(worst, err)
            num[k] += float(np.sum((got - ref) ** 2))
            den[k] += float(np.sum(ref ** 2))
            entries += ref.size
            # the mirrored entry must be the same number
            if bi != bj:
                low = H[k][bj * block:bj * block + len(cols), bi * block:bi * block + len(rows)].to(torch.float64).cpu().numpy()
                assert np.array_equal(low, got.T)
    # probe vectors
    V = rng.standard_normal((d, n_probe))
    V[hot * block:min(d, (hot + 1) * block), 0] += 1.0
    Y = np.zeros((G, d, n_probe))
    chunk = 4096
    for r0 in range(0, n, chunk):
        Xc = X[r0:r0 + chunk].to(torch.float64).cpu().numpy()
        T = Xc @ V
        for k in range(G):
            Y[k] += Xc.T @ (s64[r0:r0 + chunk, k][:, None] * T)
    Vg = torch.as_tensor(V, device=H.device)
    worst_probe = 0.0
    for k in range(G):
        got = (H[k].to(torch.float64) @ Vg).cpu().numpy()
        worst_probe = max(worst_probe, rel_fro(got, Y[k]))
    pooled = float(np.max(np.sqrt(num / den)))     # rel-Frobenius over all sampled entries of a group (max over groups)
    say(f"{what}: sampled H check: {len(pairs)} blocks x {G} groups ({entries} entries): rel-Frobenius over the "
        f"sampled entries {pooled:.2e} (worst single block {worst:.2e}); {n_probe} probe vectors worst "
        f"{worst_probe:.2e} (tol {tol:g})")
    # the verdict is the relative Frobenius error over what was sampled (per group) and the
    # whole-matrix probes; a single small-norm off-diagonal block may sit a little above it,
    # but a localized indexing mistake would put it near 1
    assert pooled <= tol and worst_probe <= tol and worst <= 5 * tol
    return pooled, worst_probe, entries


def sampled_objective_check(oracle, X, s, W, What, obj, obj_row, G, tol, rows_per_group=32, seed=0, what=""):
    """obj_row[j] for sampled channels against sum_i s_k[i] (x_i . delta_j)^2 computed from X in
    fp64 on the host, and obj[k] against the fp64 sum of the GPU's own obj_row."""
    rng = np.random.default_rng(seed)
    n, d = X.shape
    d_out = W.shape[0]
    m = d_out // G
    s64 = s.to(torch.float64).cpu().numpy()
    rows = np.concatenate([k * m + np.sort(rng.choice(m, size=min(rows_per_group, m), replace=False)) for k in range(G)])
    D = (W[torch.as_tensor(rows, device=W.device)].to(torch.float64) - What[torch.as_tensor(rows, device=W.device)].to(torch.float64)).cpu().numpy()
    ref = np.zeros(len(rows))
    chunk = 4096
    for r0 in range(0, n, chunk):
        Xc = X[r0:r0 + chunk].to(torch.float64).cpu().numpy()
        for k in range(G):
            sel = (rows // m) == k
            ref[sel] += oracle.objective_rows_from_tokens(Xc, s64[r0:r0 + chunk, k], D[sel])
    got = obj_row.to(torch.float64).cpu().numpy()
    e_rows = rel_fro(got[rows], ref)
    sums = got.reshape(G, m).sum(1)
    e_sum = float(np.max(np.abs(obj.cpu().numpy() - sums) / sums))
    say(f"{what}: objective on {len(rows)} sampled channels rel-Frobenius {e_rows:.2e}; obj vs sum of rows {e_sum:.2e} (tol {tol:g})")
    assert e_rows <= tol and e_sum <= 1e-6
    return e_rows


# ------------------------------------------------------------------ sequential rounding decisions
def check_rounding_decisions(T, S, Cn, Qg, new, what):
    """The GPU rounded, for every (channel, coordinate), a target to a grid point.  T holds the exact
    (fp64) targets for the state the GPU was in, S the sum of the absolute values of the terms of each
    target's sum.  The GPU forms every product of the sum from two-term bf16 splits of both factors and
    drops the lo*lo product, a relative error below 2^-15 per term in the worst case, and adds the terms
    in fp32; so its target is within 2^-14 * S + 2^-20 * |t| of the exact one, and the grid point it picks
    can be farther from the exact target than the nearest one by at most twice that."""
    dist = np.abs(Cn[:, None, :] - T[:, :, None])                     # [d_out, d_in, m]
    chosen = np.take_along_axis(dist, Qg[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    best = dist.min(axis=2)
    slack = 2.0 ** -14 * S + 2.0 ** -20 * np.abs(T)
    excess = chosen - best
    bad = excess > 2 * slack
    spacing = np.median(np.diff(np.sort(Cn, axis=1), axis=1))
    say(f"{what}: decisions off the nearest grid point by more than the slack: {int(bad.sum())} of {bad.size}; "
        f"max excess {float(excess.max()):.2e}, largest slack {float(2 * slack.max()):.2e}, median grid spacing {spacing:.2e}")
    assert not bad.any()
    assert 2 * slack.max() <= 0.1 * spacing                            # the bound is small against the grid itself,
    assert np.mean(excess > 0) <= 2e-3                                 # and almost every decision IS the exact nearest point
    assert np.array_equal(new, np.take_along_axis(Cn, Qg.astype(np.int64), axis=1))   # What is the grid value of its code, exactly


def cd_targets_along(Wn, old, new, Hn, G):
    """t[j, i] of Eq. (cd_closed) for the state in which coordinate i was updated during one cycle
    that turned `old` into `new` (coordinates < i new, coordinates > i old), and the sum of the
    absolute values of the terms of its sum, S[j, i] = sum_i' |Ht[i, i']| |delta[j, i']|."""
    d_out, d_in = Wn.shape
    m = d_out // G
    T, S = np.empty_like(Wn), np.empty_like(Wn)
    for k in range(G):
        r = slice(k * m, (k + 1) * m)
        Ht = Hn[k] / np.diag(Hn[k])[:, None]
        lower, upper = np.tril(Ht, -1), np.triu(Ht, 1)
        dn, do = new[r] - Wn[r], old[r] - Wn[r]
        T[r] = Wn[r] - dn @ lower.T - do @ upper.T
        S[r] = np.abs(dn) @ np.abs(lower).T + np.abs(do) @ np.abs(upper).T
    return T, S


def ldlq_targets(Wn, new, Rn, G):
    """t[j, i] = w[j, i] - sum_{i' < i} (new[j, i'] - w[j, i']) R[i', i] / R[i, i] and the sum of the
    absolute values of the terms, for the rounded weights `new` the GPU produced."""
    d_out, d_in = Wn.shape
    m = d_out // G
    T, S = np.empty_like(Wn), np.empty_like(Wn)
    for k in range(G):
        r = slice(k * m, (k + 1) * m)
        U = np.triu(Rn[k], 1) / np.diag(Rn[k])[None, :]                # U[i', i] = R[i', i] / R[i, i], i' < i
        dn = new[r] - Wn[r]
        T[r] = Wn[r] - dn @ U
        S[r] = np.abs(dn) @ np.abs(U)
    return T, S


# ------------------------------------------------------------------ codebook step
def check_codebook_channels(oracle, Wn, Qn, Hk, Cg, m, lam, what):
    """Wn, Qn, Cg: the rows of some channels of ONE group; Hk that group's Hessian (fp64)."""
    d_in = Wn.shape[1]
    Habs = np.abs(Hk)
    worst_back, worst_obj, worst_fwd = 0.0, 0.0, 0.0
    Co, _ = oracle.lnq_codebook(Wn, Qn, Hk[None], m, 1, lam)
    for j in range(Wn.shape[0]):
        P = np.zeros((d_in, m))
        P[np.arange(d_in), Qn[j]] = 1.0
        A = P.T @ Hk @ P + lam * np.eye(m)
        b = P.T @ (Hk @ Wn[j])
        c = Cg[j]
        scale = (P.T @ Habs @ P) @ np.abs(c) + P.T @ (Habs @ np.abs(Wn[j]))
        used = P.sum(axis=0) > 0
        resid = np.abs(A @ c - b)
        back = float(np.max(resid[used] / scale[used]))
        worst_back = max(worst_back, back)
        assert np.all(c[~used] == 0.0), f"{what}: channel {j}: an unused grid point is not 0"
        e_g, e_o = Wn[j] - P @ c, Wn[j] - P @ Co[j]
        o_g, o_o = e_g @ Hk @ e_g, e_o @ Hk @ e_o
        worst_obj = max(worst_obj, float((o_g - o_o) / o_o))
        cond = np.linalg.cond(A[np.ix_(used, used)])
        fwd = float(np.max(np.abs(c - Co[j])) / max(np.max(np.abs(Co[j])), np.max(np.abs(Wn[j]))))   # on the scale of the weights
        worst_fwd = max(worst_fwd, fwd / cond)
    say(f"{what}: backward error {worst_back:.2e} (bound 9.5e-07), objective above the minimum by {worst_obj:.2e} (rel), "
        f"grid error / condition number {worst_fwd:.2e}")
    assert worst_back <= 2.0 ** -20
    assert worst_obj <= 1e-6
    assert worst_fwd <= 1e-5
