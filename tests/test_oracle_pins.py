"""Pins for the CPU oracle: closed forms, a hand-worked example, an independent
BLAS routine, and brute force through the paper's *un-averaged* definitions.
None of these tests touches the HIP path."""
import json
import os

import numpy as np
import pytest
import scipy.linalg.blas as blas

import oracle


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- worked example
# Worked by hand from Algorithm 1 (lines 1, 2, 4) and Eq. (ours2); n=3, d_in=2,
# d_out=4, G=2 so J_0={0,1}, J_1={2,3}.  The numbers live in tests/golden/.
def _golden(name):
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)) as f:
        return json.load(f)


_EX = _golden("alg1_worked_example.json")
X_EX, DZ_EX, S_EX, H_EX = (np.array(_EX[k]) for k in ("X", "dZ", "s", "H"))
DELTA_EX, OBJ_ROW_EX, OBJ_EX = (np.array(_EX[k]) for k in ("delta", "obj_row", "obj"))


def test_worked_example_group_weights():
    np.testing.assert_allclose(oracle.group_weights(DZ_EX, 2), S_EX, rtol=0, atol=1e-15)


def test_worked_example_gram():
    np.testing.assert_allclose(oracle.fisher_gram(X_EX, S_EX), H_EX, rtol=0, atol=1e-13)


def test_worked_example_objective():
    What = np.zeros((4, 2))
    obj, obj_row = oracle.objective(DELTA_EX, What, H_EX, 2)
    np.testing.assert_allclose(obj_row, OBJ_ROW_EX, rtol=0, atol=1e-13)
    np.testing.assert_allclose(obj, OBJ_EX, rtol=0, atol=1e-13)
    # sign convention: only the difference W - What matters
    obj2, _ = oracle.objective(What, DELTA_EX, H_EX, 2)
    np.testing.assert_allclose(obj2, OBJ_EX, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- group partition / s
def test_partition_is_contiguous_and_rejects_nondivisible():
    assert oracle.group_partition(8, 4) == [(0, 2), (2, 4), (4, 6), (6, 8)]
    with pytest.raises(ValueError):
        oracle.group_partition(10, 4)
    with pytest.raises(ValueError):
        oracle.group_weights(np.ones((3, 10)), 4)


def test_s_constant_gradient_closed_form():
    s = oracle.group_weights(np.full((7, 12), -0.5), 3, grad_scale=4.0)
    np.testing.assert_allclose(s, np.full((7, 3), 16.0 * 0.25), rtol=1e-15)


def test_s_one_hot_column_lands_in_its_group_only():
    n, d_out, G = 5, 12, 3
    v = np.arange(1.0, n + 1)
    for j in range(d_out):
        dZ = np.zeros((n, d_out))
        dZ[:, j] = v
        s = oracle.group_weights(dZ, G)
        expect = np.zeros((n, G))
        expect[:, j // 4] = v * v / 4.0
        np.testing.assert_allclose(s, expect, rtol=1e-15)


def test_s_g_equals_dout_is_elementwise_square_and_g1_is_row_mean():
    dZ = _rng(0).standard_normal((9, 6))
    np.testing.assert_allclose(oracle.group_weights(dZ, 6), dZ ** 2, rtol=1e-15)
    np.testing.assert_allclose(oracle.group_weights(dZ, 1)[:, 0], np.mean(dZ ** 2, axis=1), rtol=1e-14)


def test_scale_law_s_h_obj():
    r = _rng(1)
    X, dZ = r.standard_normal((20, 5)), r.standard_normal((20, 8))
    W, What = r.standard_normal((8, 5)), r.standard_normal((8, 5))
    c = 1e3
    s1, sc = oracle.group_weights(dZ, 2), oracle.group_weights(dZ, 2, grad_scale=c)
    np.testing.assert_allclose(sc, c * c * s1, rtol=1e-13)
    H1, Hc = oracle.fisher_gram(X, s1), oracle.fisher_gram(X, sc)
    np.testing.assert_allclose(Hc, c * c * H1, rtol=1e-12)
    np.testing.assert_allclose(oracle.objective(W, What, Hc)[0], c * c * oracle.objective(W, What, H1)[0], rtol=1e-12)


# ---------------------------------------------------------------- Gram
def test_gram_g1_unit_gradient_is_plain_xtx_dsyrk():
    X = _rng(2).standard_normal((37, 11))
    H = oracle.fisher_gram(X, oracle.group_weights(np.ones((37, 4)), 1))[0]
    C = blas.dsyrk(1.0, X, trans=1, lower=0)           # upper triangle of X^T X
    iu = np.triu_indices(11)
    np.testing.assert_allclose(H[iu], C[iu], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(H, H.T, rtol=1e-14, atol=1e-14)


@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_gram_is_group_mean_of_per_channel_hessians(G):
    r = _rng(3 + G)
    n, d_in, d_out = 64, 16, 8
    X, dZ = r.standard_normal((n, d_in)), r.standard_normal((n, d_out)) * np.exp(r.standard_normal((n, 1)))
    H = oracle.fisher_gram(X, oracle.group_weights(dZ, G))
    m = d_out // G
    for k in range(G):
        Hbar = sum(oracle.per_channel_hessian(X, dZ, j) for j in range(k * m, (k + 1) * m)) / m
        np.testing.assert_allclose(H[k], Hbar, rtol=1e-12, atol=1e-12 * np.abs(Hbar).max())


def test_gram_entrywise_brute_force_nonsquare_and_block():
    r = _rng(9)
    n, d_in, G = 13, 7, 3
    X, s = r.standard_normal((n, d_in)), r.random((n, G))
    H = oracle.fisher_gram(X, s)
    assert H.shape == (G, d_in, d_in)
    for k in range(G):
        for a in range(d_in):
            for b in range(d_in):
                ref = sum(s[i, k] * X[i, a] * X[i, b] for i in range(n))
                assert abs(H[k, a, b] - ref) <= 1e-12 * (1 + abs(ref))
    blk = oracle.fisher_gram_block(X, s[:, 1], slice(1, 4), np.array([6, 0, 2]))
    np.testing.assert_allclose(blk, H[1][1:4][:, [6, 0, 2]], rtol=1e-13, atol=1e-13)


def test_gram_symmetric_psd_rank_and_single_token():
    r = _rng(10)
    n, d_in, G = 6, 10, 2
    X, s = r.standard_normal((n, d_in)), r.random((n, G))
    H = oracle.fisher_gram(X, s)
    for k in range(G):
        np.testing.assert_allclose(H[k], H[k].T, rtol=1e-13, atol=1e-13)
        ev = np.linalg.eigvalsh(0.5 * (H[k] + H[k].T))
        assert ev.min() >= -1e-12 * ev.max()
        assert np.linalg.matrix_rank(H[k]) <= n
    H1 = oracle.fisher_gram(X[:1], s[:1])
    for k in range(G):
        np.testing.assert_allclose(H1[k], s[0, k] * np.outer(X[0], X[0]), rtol=1e-14)


def test_gram_chunk_additivity():
    r = _rng(11)
    X, s = r.standard_normal((50, 6)), r.random((50, 2))
    H = oracle.fisher_gram(X[:20], s[:20])
    H = oracle.fisher_gram(X[20:], s[20:], H=H)
    np.testing.assert_allclose(H, oracle.fisher_gram(X, s), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- objective
def test_objective_equals_sum_over_tokens_form():
    r = _rng(12)
    n, d_in, d_out, G = 40, 6, 8, 4
    X, dZ = r.standard_normal((n, d_in)), r.standard_normal((n, d_out))
    W, What = r.standard_normal((d_out, d_in)), r.standard_normal((d_out, d_in))
    s = oracle.group_weights(dZ, G)
    obj, obj_row = oracle.objective(W, What, oracle.fisher_gram(X, s), G)
    m = d_out // G
    for j in range(d_out):
        ref = oracle.objective_from_tokens(X, s[:, j // m], W[j] - What[j])
        assert abs(obj_row[j] - ref) <= 1e-11 * ref
    np.testing.assert_allclose(obj, obj_row.reshape(G, m).sum(1), rtol=1e-13)


def test_objective_with_one_group_per_channel_is_the_unaveraged_frobenius_form():
    # Remark 3.1 / Eq. (ours): with |J_k| = 1 nothing is averaged away.
    r = _rng(13)
    n, d_in, d_out = 30, 5, 6
    X, dZ = r.standard_normal((n, d_in)), r.standard_normal((n, d_out))
    W, What = r.standard_normal((d_out, d_in)), r.standard_normal((d_out, d_in))
    H = oracle.fisher_gram(X, oracle.group_weights(dZ, d_out, grad_scale=3.0))
    obj, _ = oracle.objective(W, What, H, d_out)
    ref = oracle.unaveraged_objective(X, dZ, W, What, grad_scale=3.0)
    assert abs(obj.sum() - ref) <= 1e-11 * ref


def test_objective_zero_nonneg_single_perturbation_and_group_routing():
    r = _rng(14)
    n, d_in, d_out, G = 25, 7, 6, 3
    X, s = r.standard_normal((n, d_in)), r.random((n, G))
    H = oracle.fisher_gram(X, s)
    W = r.standard_normal((d_out, d_in))
    obj0, row0 = oracle.objective(W, W.copy(), H, G)
    assert np.all(obj0 == 0) and np.all(row0 == 0)
    eps, a, j = 0.25, 4, 3                              # row 3 lives in group 1
    What = W.copy()
    What[j, a] += eps
    obj, row = oracle.objective(W, What, H, G)
    assert abs(obj[1] - eps * eps * H[1, a, a]) <= 1e-13 * obj[1]
    assert obj[0] == 0 and obj[2] == 0 and row[j] == obj[1]
    objr, _ = oracle.objective(W, r.standard_normal((d_out, d_in)), H, G)
    assert np.all(objr > 0)


def test_objective_rows_from_tokens_matches_the_token_loop_and_the_hessian_form():
    r = _rng(15)
    n, d_in = 33, 5
    X, s_k = r.standard_normal((n, d_in)), r.random(n)
    D = r.standard_normal((4, d_in))
    got = oracle.objective_rows_from_tokens(X, s_k, D)
    H = oracle.fisher_gram(X, s_k[:, None])[0]
    for j in range(4):
        assert abs(got[j] - oracle.objective_from_tokens(X, s_k, D[j])) <= 1e-12 * got[j]
        assert abs(got[j] - D[j] @ H @ D[j]) <= 1e-11 * got[j]


# ---------------------------------------------------------------- cyclic CD assignment step
def _cd_case(seed, d_out=6, d_in=7, G=2, m=4, n=40):
    r = _rng(seed)
    X = r.standard_normal((n, d_in))
    s = r.random((n, G)) + 0.1
    H = oracle.fisher_gram(X, s)
    W = r.standard_normal((d_out, d_in))
    C = np.sort(r.standard_normal((d_out, m)), axis=1)
    q0 = r.integers(0, m, size=(d_out, d_in))
    What0 = C[np.arange(d_out)[:, None], q0]
    return W, What0, C, H


def test_cd_worked_example():
    ex = _golden("cd_worked_example.json")          # worked by hand from Eq. (cd_closed)
    H, W, C, start = (np.array(ex[k]) for k in ("H", "W", "grid", "start"))
    assert abs(oracle.cd_coordinate_target(W[0], start[0], H[0], 0) - ex["targets"][0]) < 1e-15
    assert abs(oracle.cd_coordinate_target(W[0], [1.0, 0.0], H[0], 1) - ex["targets"][1]) < 1e-15
    Q, What = oracle.cd_assign(W, start, C, H)
    assert Q.tolist() == ex["codes"] and What.tolist() == ex["What"]
    assert abs(oracle.objective(W, start, H)[0][0] - ex["objective_before"]) < 1e-14
    assert abs(oracle.objective(W, What, H)[0][0] - ex["objective_after"]) < 1e-14


def test_cd_each_update_is_the_exhaustive_argmin_of_the_objective():
    # Algorithm 2, line 8 defines the update as the grid point that minimises the layer objective;
    # replay the cycle with that definition evaluated exhaustively and compare the assignments.
    W, What0, C, H = _cd_case(20)
    d_out, d_in = W.shape
    G = H.shape[0]
    Q, What = oracle.cd_assign(W, What0, C, H, G, n_cycles=2)
    cur = What0.copy()
    for _ in range(2):
        for i in range(d_in):
            for j in range(d_out):
                best, best_q = None, None
                for q in range(C.shape[1]):
                    trial = cur.copy()
                    trial[j, i] = C[j, q]
                    val = oracle.objective(W, trial, H, G)[1][j]
                    if best is None or val < best - 1e-12 * abs(best):
                        best, best_q = val, q
                cur[j, i] = C[j, best_q]
                last = best_q
                if _ == 1:
                    assert Q[j, i] == last
    np.testing.assert_array_equal(What, cur)


def test_cd_is_a_descent_method_and_reaches_a_fixed_point():
    W, What0, C, H = _cd_case(21, d_out=8, d_in=12, G=2, m=8)
    prev = oracle.objective(W, What0, H, 2)[1]
    cur = What0
    for cycle in range(30):
        Q, nxt = oracle.cd_assign(W, cur, C, H, 2, n_cycles=1)
        val = oracle.objective(W, nxt, H, 2)[1]
        assert np.all(val <= prev * (1 + 1e-12))          # Prop. 4.1: feasible start => monotone descent, per channel
        if np.array_equal(nxt, cur):
            break
        prev, cur = val, nxt
    else:
        raise AssertionError("no fixed point within 30 cycles")
    # several cycles in one call are the same as the calls chained
    Qk, Wk = oracle.cd_assign(W, What0, C, H, 2, n_cycles=cycle + 1)
    np.testing.assert_array_equal(Wk, cur)
    assert np.all(C[np.arange(8)[:, None], Qk] == Wk)


def test_cd_with_diagonal_hessian_is_round_to_nearest_and_groups_use_their_own_matrix():
    W, What0, C, H = _cd_case(22, d_out=6, d_in=9, G=2, m=4)
    H = H.copy()
    H[1] = np.diag(np.diag(H[1]))                                  # group 1: no coupling between coordinates
    Q, What = oracle.cd_assign(W, What0, C, H, 2)
    rtn = np.argmin(np.abs(C[3:, None, :] - W[3:, :, None]), axis=2)
    np.testing.assert_array_equal(Q[3:], rtn)
    assert not np.array_equal(Q[:3], np.argmin(np.abs(C[:3, None, :] - W[:3, :, None]), axis=2))   # group 0 is coupled


def test_cd_tie_goes_to_the_lower_index_and_rejects_nonpositive_diagonal():
    H = np.array([[[1.0, 0.0], [0.0, 1.0]]])
    W = np.array([[0.5, 0.25]])
    C = np.array([[0.0, 1.0, 0.5]])                                # 0.25 is equally far from 0 (index 0) and 0.5 (index 2)
    Q, What = oracle.cd_assign(W, np.zeros((1, 2)), C, H)
    assert Q.tolist() == [[2, 0]] and What.tolist() == [[0.5, 0.0]]
    with pytest.raises(ValueError):
        oracle.cd_assign(W, np.zeros((1, 2)), C, np.zeros((1, 2, 2)))


def test_gram_of_stacked_layer_weights_is_the_layers_grams_one_after_the_other():
    # layers that read the same X: Algorithm 1, line 4 is linear in s column by column
    r = _rng(40)
    X = r.standard_normal((30, 6))
    dZa, dZb = r.standard_normal((30, 8)), r.standard_normal((30, 12))
    sa, sb = oracle.group_weights(dZa, 2), oracle.group_weights(dZb, 3)
    H = oracle.fisher_gram(X, np.concatenate([sa, sb], axis=1))
    np.testing.assert_array_equal(H[:2], oracle.fisher_gram(X, sa))
    np.testing.assert_array_equal(H[2:], oracle.fisher_gram(X, sb))


# ---------------------------------------------------------------- LNQ codebook step
def test_lnq_codebook_worked_example():
    ex = _golden("lnq_codebook_worked_example.json")      # worked by hand from Eq. (conti-sol)
    C, What = oracle.lnq_codebook(np.array(ex["W"]), np.array(ex["Q"]), np.array(ex["H"]), 2, lam=0.0)
    np.testing.assert_allclose(C, ex["codebook"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(What, ex["What"], rtol=0, atol=1e-14)


def test_lnq_codebook_with_identity_hessian_is_the_cluster_mean_and_empty_clusters_get_zero():
    # H = I: the problem is 1-D k-means' centroid step (textbook): c_q = mean of the weights assigned to q
    r = _rng(50)
    d_out, d_in, m = 5, 40, 4
    W = r.standard_normal((d_out, d_in))
    Q = r.integers(0, 3, size=(d_out, d_in))                 # grid point 3 is never used
    C, What = oracle.lnq_codebook(W, Q, np.eye(d_in)[None], m, lam=1e-12)
    for j in range(d_out):
        for q in range(3):
            np.testing.assert_allclose(C[j, q], W[j, Q[j] == q].mean(), rtol=1e-9)
        assert C[j, 3] == 0.0
    np.testing.assert_array_equal(What, np.take_along_axis(C, Q, axis=1))


def test_lnq_codebook_is_the_minimiser_of_the_layer_objective_over_the_grid_values():
    W, What0, C0, H = _cd_case(51, d_out=6, d_in=14, G=2, m=4)
    Q = np.argmin(np.abs(C0[:, None, :] - What0[:, :, None]), axis=2)
    lam = 1e-9
    C, What = oracle.lnq_codebook(W, Q, H, 4, 2, lam=lam)
    base = oracle.objective(W, What, H, 2)[1]
    # Prop. 4.1, first inequality: the update cannot increase any channel's objective
    assert np.all(base <= oracle.objective(W, What0, H, 2)[1] * (1 + 1e-12))
    # stationarity (normal equations of Eq. (conti-sol)): P^T H (w - P c) = lam c
    for j in range(6):
        P = np.eye(4)[Q[j]]
        g = P.T @ H[j // 3] @ (W[j] - What[j])
        np.testing.assert_allclose(g, lam * C[j], atol=1e-9 * np.abs(H).max())
    # and brute force: moving any grid value of any channel either way does not help
    r = _rng(52)
    for _ in range(200):
        j, q = r.integers(0, 6), r.integers(0, 4)
        C2 = C.copy()
        C2[j, q] += r.choice([-1, 1]) * 10.0 ** r.uniform(-4, -1)
        trial = np.take_along_axis(C2, Q, axis=1)
        assert oracle.objective(W, trial, H, 2)[1][j] >= base[j] * (1 - 1e-9)


def test_lnq_codebook_recovers_an_exactly_representable_weight_and_is_relabeling_invariant():
    r = _rng(53)
    d_in, m = 20, 4
    H = oracle.fisher_gram(r.standard_normal((50, d_in)), r.random((50, 1)) + 0.1)
    c_true = np.array([[-1.5, -0.25, 0.5, 2.0]])
    Q = r.integers(0, m, size=(1, d_in))
    W = np.take_along_axis(c_true, Q, axis=1)
    C, What = oracle.lnq_codebook(W, Q, H, m, lam=0.0)
    np.testing.assert_allclose(C, c_true, rtol=1e-9)
    perm = np.array([2, 0, 3, 1])
    C2, What2 = oracle.lnq_codebook(W, perm[Q], H, m, lam=0.0)
    np.testing.assert_allclose(C2[0, perm], C[0], rtol=1e-9)
    np.testing.assert_allclose(What2, What, rtol=1e-9)
    with pytest.raises(ValueError):
        oracle.lnq_codebook(W, Q + 1, H, m)


def test_lnq_alternation_descends_and_reduces_to_its_parts():
    # Prop. 4.1: neither step can increase the objective; with no iterations the alternation is the codebook
    # step alone; one iteration is codebook step -> CD cycles -> codebook step, composed by hand here
    r = _rng(55)
    d_out, d_in, G, m = 6, 24, 2, 4
    X = r.normal(size=(80, d_in))
    H = np.stack([X.T @ (r.uniform(0.5, 2.0, 80)[:, None] * X) for _ in range(G)]) + 0.01 * np.eye(d_in)
    W = r.normal(size=(d_out, d_in))
    Q0 = r.integers(0, m, size=(d_out, d_in))
    Q, What, C, trace = oracle.lnq(W, Q0, H, m, G, n_iters=3, n_cycles=2)
    assert len(trace) == 7 and all(b <= a * (1 + 1e-12) for a, b in zip(trace[:-1], trace[1:]))
    assert trace[-1] < 0.7 * trace[0]
    np.testing.assert_array_equal(What, np.take_along_axis(C, Q, axis=1))
    Qz, Wz, Cz, tz = oracle.lnq(W, Q0, H, m, G, n_iters=0)
    C0, W0 = oracle.lnq_codebook(W, Q0, H, m, G)
    np.testing.assert_array_equal(Qz, Q0)
    np.testing.assert_array_equal(Wz, W0)
    np.testing.assert_array_equal(Cz, C0)
    Q1, W1 = oracle.cd_assign(W, W0, C0, H, G, n_cycles=2)
    C1, W1b = oracle.lnq_codebook(W, Q1, H, m, G)
    Qo, Wo, Co, _ = oracle.lnq(W, Q0, H, m, G, n_iters=1, n_cycles=2)
    np.testing.assert_array_equal(Qo, Q1)
    np.testing.assert_array_equal(Wo, W1b)
    np.testing.assert_array_equal(Co, C1)


# ---------------------------------------------------------------- damped Cholesky, sequential rounding (GPTQ / LDLQ)
def _spd(r, G, d, cond=50.0):
    out = []
    for _ in range(G):
        B = r.normal(size=(3 * d, d)) * np.linspace(1.0, np.sqrt(cond), d)[None, :]
        out.append(B.T @ B / (3 * d))
    return np.stack(out)


def test_sequential_rounding_worked_example():
    ex = _golden("sequential_rounding_worked_example.json")
    np.testing.assert_allclose(oracle.damped_cholesky(np.array(ex["chol_A"]), 0.0, 0.0), ex["chol_L"], rtol=0, atol=1e-13)
    A, W, C = np.array(ex["A"]), np.array(ex["W"]), np.array(ex["codebook"])
    Q, What = oracle.gptq_assign(W, C, A, damp_rel=0.0)
    assert Q.tolist() == ex["Q"] and What.tolist() == ex["What"]
    Q2, What2, Tgt = oracle.ldlq_assign(W, C, oracle.damped_cholesky(A, 0.0, 0.0, reverse=True))
    assert Q2.tolist() == ex["Q"] and What2.tolist() == ex["What"]
    np.testing.assert_allclose(Tgt, ex["targets"], rtol=0, atol=1e-14)


def test_damped_cholesky_is_the_unique_triangular_factor_of_the_damped_matrix():
    # a positive definite matrix has exactly one lower (upper) triangular factor with positive diagonal:
    # shape, sign and the product pin the result without reference to how it was computed
    r = _rng(60)
    H = _spd(r, 3, 9)
    for rel, ab in ((0.0, 0.0), (0.01, 0.0), (0.05, 0.3)):
        L = oracle.damped_cholesky(H, rel, ab)
        R = oracle.damped_cholesky(H, rel, ab, reverse=True)
        for k in range(3):
            eps = ab + rel * np.trace(H[k]) / 9
            A = H[k] + eps * np.eye(9)
            assert np.all(np.triu(L[k], 1) == 0) and np.all(np.diag(L[k]) > 0)
            assert np.all(np.tril(R[k], -1) == 0) and np.all(np.diag(R[k]) > 0)
            np.testing.assert_allclose(L[k] @ L[k].T, A, rtol=1e-13, atol=1e-13)
            np.testing.assert_allclose(R[k] @ R[k].T, A, rtol=1e-13, atol=1e-13)
    # the two factors differ (they are not transposes of each other) unless the matrix is diagonal
    assert np.abs(oracle.damped_cholesky(H[0], 0, 0, reverse=True) - oracle.damped_cholesky(H[0], 0, 0).T).max() > 1e-3
    D = np.diag([4.0, 9.0, 16.0])
    np.testing.assert_allclose(oracle.damped_cholesky(D, 0.0, 0.0, reverse=True), np.diag([2.0, 3.0, 4.0]), atol=1e-15)
    with pytest.raises(np.linalg.LinAlgError):
        oracle.damped_cholesky(np.array([[1.0, 2.0], [2.0, 1.0]]), 0.0, 0.0)       # indefinite without damping


def test_each_rounding_target_is_the_conditional_minimiser_given_the_coordinates_already_rounded():
    # the defining property (optimal-brain-surgeon update, textbook constrained least squares): before
    # coordinate i is rounded, the free coordinates i.. sit at the minimiser of (w' - w)^T A (w' - w)
    # subject to the coordinates < i being fixed at their rounded values:
    #   w'_R = w_R - A_RR^-1 A_RF (what_F - w_F),   R = {i, ..., d-1}, F = {0, ..., i-1}
    r = _rng(61)
    d_out, d_in, G, m = 4, 7, 2, 4
    H = _spd(r, G, d_in)
    W = r.normal(size=(d_out, d_in))
    C = np.sort(r.normal(size=(d_out, m)), axis=1)
    rel = 0.02
    Q, What = oracle.gptq_assign(W, C, H, G, damp_rel=rel)
    Rf = oracle.damped_cholesky(H, rel, 0.0, reverse=True)
    Q2, What2, Tgt = oracle.ldlq_assign(W, C, Rf, G)
    np.testing.assert_array_equal(Q, Q2)                                   # inverse-factor form == factor form
    np.testing.assert_array_equal(What, What2)
    for j in range(d_out):
        k = j // (d_out // G)
        A = H[k] + rel * np.trace(H[k]) / d_in * np.eye(d_in)
        for i in range(d_in):
            Rset, F = np.arange(i, d_in), np.arange(0, i)
            free = W[j, Rset] - np.linalg.solve(A[np.ix_(Rset, Rset)], A[np.ix_(Rset, F)] @ (What[j, F] - W[j, F]))
            assert abs(free[0] - Tgt[j, i]) < 1e-11
            assert Q[j, i] == int(np.argmin(np.abs(C[j] - free[0])))
            assert What[j, i] == C[j, Q[j, i]]
        # and the error decomposes over the coordinates: (what - w)^T A (what - w) = sum_i R[i,i]^2 (what_i - t_i)^2
        e = What[j] - W[j]
        assert abs(e @ A @ e - np.sum(np.diag(Rf[k]) ** 2 * (What[j] - Tgt[j]) ** 2)) < 1e-10


def test_sequential_rounding_special_cases():
    r = _rng(62)
    d_out, d_in, m = 6, 11, 8
    W = r.normal(size=(d_out, d_in))
    C = r.normal(size=(d_out, m))                                          # grids in any order
    Hd = np.stack([np.diag(r.uniform(0.5, 2.0, d_in)) for _ in range(2)])
    rtn = np.argmin(np.abs(C[:, None, :] - W[:, :, None]), axis=2)
    Q, What = oracle.gptq_assign(W, C, Hd, 2)                              # diagonal matrix: no feedback, plain rounding
    np.testing.assert_array_equal(Q, rtn)
    np.testing.assert_array_equal(What, np.take_along_axis(C, rtn, axis=1))
    # a weight already on its grid everywhere is left alone, whatever the matrix
    H = _spd(r, 2, d_in)
    Won = np.take_along_axis(C, r.integers(0, m, size=(d_out, d_in)), axis=1)
    _, What = oracle.gptq_assign(Won, C, H, 2)
    np.testing.assert_array_equal(What, Won)
    # ties go to the lower index: w exactly between two grid points
    Qt, _ = oracle.gptq_assign(np.array([[0.5]]), np.array([[1.0, 0.0]]), np.array([[[1.0]]]), 1, damp_rel=0.0)
    assert Qt[0, 0] == 0
    # every group uses its own matrix: swapping the matrices changes the result of a coupled problem
    Wb = r.normal(size=(4, d_in))
    Cb = np.tile(np.array([[-1.0, 0.0, 1.0]]), (4, 1))
    Qa, _ = oracle.gptq_assign(Wb, Cb, H, 2)
    Qb, _ = oracle.gptq_assign(Wb, Cb, H[::-1], 2)
    assert np.any(Qa != Qb)
    # feedback does better than plain rounding on the objective it is built for, on average
    obj_seq = oracle.objective(Wb, oracle.gptq_assign(Wb, Cb, H, 2, damp_rel=0.0)[1], H, 2)[0].sum()
    obj_rtn = oracle.objective(Wb, np.take_along_axis(Cb, np.argmin(np.abs(Cb[:, None, :] - Wb[:, :, None]), axis=2), axis=1), H, 2)[0].sum()
    assert obj_seq < obj_rtn
