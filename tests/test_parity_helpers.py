"""The fp64 replay helpers of the GPU parity tests (tests/parity_utils.py) restate Eq. "cd_closed"
and the sequential-rounding recursion in matrix form.  These CPU tests tie them to the pinned
oracle: along the oracle's own trajectory the helpers must reproduce, coordinate by coordinate,
the targets the oracle rounded -- and a transposed or mis-signed helper must not."""
import numpy as np

import oracle
from parity_utils import cd_targets_along, ldlq_targets


def _problem(seed, d_out=12, d_in=9, G=3, m=4, n=40):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, d_in)) * (1.0 + 3.0 * (rng.random(d_in) < 0.2))
    s = rng.random((n, G)) + 0.05
    H = oracle.fisher_gram(X, s)
    H = H + 0.01 * np.mean(np.diagonal(H, axis1=1, axis2=2), axis=1)[:, None, None] * np.eye(d_in)
    W = rng.standard_normal((d_out, d_in)) * 0.5
    C = np.sort(rng.standard_normal((d_out, m)), axis=1)
    What = np.take_along_axis(C, np.argmin(np.abs(C[:, None, :] - W[:, :, None]), axis=2), axis=1)
    return W, What, C, H, G


def _oracle_cd_targets(W, old, C, H, G):
    """Targets along the oracle's own cycle: coordinate i sees coordinates < i as the oracle left them."""
    _, new = oracle.cd_assign(W, old, C, H, G, n_cycles=1)
    d_out, d_in = W.shape
    m = d_out // G
    T = np.empty_like(W)
    for j in range(d_out):
        for i in range(d_in):
            state = np.concatenate([new[j, :i], old[j, i:]])
            T[j, i] = oracle.cd_coordinate_target(W[j], state, H[j // m], i)
    return new, T


def test_cd_targets_along_equals_the_oracle_coordinate_by_coordinate():
    for seed in (1, 2, 3):
        W, old, C, H, G = _problem(seed)
        new, T_ref = _oracle_cd_targets(W, old, C, H, G)
        T, S = cd_targets_along(W, old, new, H, G)
        assert np.allclose(T, T_ref, rtol=1e-12, atol=1e-12)
        # the rounded value of every target is what the oracle chose
        q = np.argmin(np.abs(C[:, None, :] - T[:, :, None]), axis=2)
        assert np.array_equal(np.take_along_axis(C, q, axis=1), new)
        # S bounds the size of the sum's terms: |t - w| <= S
        assert np.all(np.abs(T - W) <= S * (1 + 1e-12) + 1e-15)


def test_cd_targets_along_detects_a_transposed_or_mis_signed_restatement():
    W, old, C, H, G = _problem(5)
    new, T_ref = _oracle_cd_targets(W, old, C, H, G)
    # the same formula with the roles of the updated and the not-yet-updated coordinates swapped
    T_swapped, _ = cd_targets_along(W, new, old, H, G)
    assert not np.allclose(T_swapped, T_ref, rtol=1e-6, atol=1e-9)
    # ... and with an unsymmetric H (normalised by the wrong diagonal entry) the helper must differ too:
    Hbad = H * np.linspace(1.0, 2.0, H.shape[1])[None, None, :]
    T_bad, _ = cd_targets_along(W, old, new, Hbad, G)
    assert not np.allclose(T_bad, T_ref, rtol=1e-6, atol=1e-9)


def test_ldlq_targets_equals_the_targets_the_oracle_rounded():
    for seed in (7, 8):
        W, _, C, H, G = _problem(seed)
        R = oracle.damped_cholesky(H, 0.0, 0.0, reverse=True)
        _, new, Tgt = oracle.ldlq_assign(W, C, R, G)
        T, S = ldlq_targets(W, new, R, G)
        assert np.allclose(T, Tgt, rtol=1e-12, atol=1e-12)
        assert np.all(np.abs(T - W) <= S * (1 + 1e-12) + 1e-15)
        # a transposed factor gives other targets
        T_t, _ = ldlq_targets(W, new, np.transpose(R, (0, 2, 1)), G)
        assert not np.allclose(T_t, Tgt, rtol=1e-6, atol=1e-9)
