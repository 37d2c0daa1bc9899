"""Damped Cholesky and sequential rounding with error feedback (GPTQ / LDLQ) on the GPU, through
the C ABI, against the fp64 oracle.

Rounding: as for the coordinate-descent step, every decision depends on all earlier ones and the
GPU evaluates the sums in fp32-grade arithmetic, so every decision is re-derived in fp64 from the
GPU's own trajectory and from the factor the GPU was given (exactly representable: fp32 values),
and must be the nearest grid point up to the slack of that arithmetic; codes and objective are then
compared with the oracle's own pass.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_07004_amd import binding as gq
from paper_2505_07004_amd import workloads as wl
from parity_utils import check_rounding_decisions, ldlq_targets, say, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _hessian(n, d_in, d_out, G, seed):
    X = wl.make_x_outlier(n, d_in, max(1, d_in // 64), 20.0, seed, DEV, torch.float32)
    dZ = wl.make_dz(n, d_out, 1.0, 1.5, seed + 1, DEV)
    s = gq.gq_group_weights(dZ, G)
    if d_in % 4:                        # rows of X not 16-byte aligned: an input for the factorization all the same
        return torch.einsum("ia,ik,ib->kab", X, s, X).contiguous()
    return gq.gq_fisher_gram(X, s, mirror=True)


@pytest.mark.parametrize("n,d_in,d_out,G,bits,ld", [
    (512, 256, 128, 2, 3, None),        # two blocks
    (400, 200, 96, 4, 2, 208),          # ragged last block, padded pitch
    (600, 384, 192, 1, 4, None),        # 16 grid points, three blocks
    (300, 132, 40, 2, 3, 136),          # last block of 4 coordinates
    (256, 96, 64, 2, 3, None),          # a single, ragged block
])
def test_sequential_rounding_decisions_are_valid_and_match_the_oracle(n, d_in, d_out, G, bits, ld):
    say(f"ldlq n={n} d_in={d_in} d_out={d_out} G={G} bits={bits} ld={ld}")
    H = _hessian(n, d_in, d_out, G, 41 + d_in)
    Rn = oracle.damped_cholesky(to_np64(H), 0.01, 0.0, reverse=True).astype(np.float32)   # what the GPU is given
    R = torch.from_numpy(Rn).to(DEV)
    W = wl.make_w(d_out, d_in, 43 + d_in, DEV)
    _, C = wl.quantize_codebook_per_row(W, bits, return_codebook=True)
    C = C.contiguous()
    if ld:
        buf = torch.full((d_out, ld), float("nan"), device=DEV)
        buf[:, :d_in] = W
        W = buf[:, :d_in]
    What, Q = gq.gq_ldlq_assign(W, C, R)
    torch.cuda.synchronize()
    Wn, Cn, new, Qg = to_np64(W), to_np64(C), to_np64(What), Q.cpu().numpy()
    R64 = Rn.astype(np.float64)
    T, S = ldlq_targets(Wn, new, R64, G)
    check_rounding_decisions(T, S, Cn, Qg, new, "sequential rounding")
    Qo, ref, _ = oracle.ldlq_assign(Wn, Cn, R64, G)
    differ = float(np.mean(Qo != Qg))
    A = R64 @ np.transpose(R64, (0, 2, 1))
    og, oo = oracle.objective(Wn, new, A, G)[0], oracle.objective(Wn, ref, A, G)[0]
    rtn = np.take_along_axis(Cn, np.argmin(np.abs(Cn[:, None, :] - Wn[:, :, None]), axis=2), axis=1)
    o_rtn = oracle.objective(Wn, rtn, A, G)[0]
    say(f"  codes that differ from the oracle's: {100 * differ:.3f} %; objective gpu {og}, oracle {oo}, plain rounding {o_rtn}")
    assert differ <= 5e-3
    assert np.all(np.abs(og - oo) <= 1e-3 * oo) and np.all(og < o_rtn)


def test_sequential_rounding_with_a_diagonal_factor_is_plain_rounding():
    d_out, d_in = 64, 160
    W = wl.make_w(d_out, d_in, 5, DEV)
    _, C = wl.quantize_codebook_per_row(W, 3, return_codebook=True)
    C = C.contiguous()
    R = torch.diag_embed(torch.rand(2, d_in, device=DEV) + 0.5)
    What, Q = gq.gq_ldlq_assign(W, C, R)
    torch.cuda.synchronize()
    rtn = torch.argmin((C[:, None, :] - W[:, :, None]).abs(), dim=2)
    assert torch.equal(Q.long(), rtn)
    assert torch.equal(What, torch.gather(C, 1, rtn))


# ------------------------------------------------------------------ damped Cholesky
def _check_factor(Hn, Fg, rel, ab, reverse, what):
    """A positive definite matrix has ONE triangular factor with positive diagonal, so shape, sign and
    the product pin the result.  Backward: ||F F^T - A||_F / ||A||_F (fp32 arithmetic, blocks of 128:
    a few 2^-24 times a slowly growing function of d; bar 1e-5, the fp32 bar of this build).  Forward:
    against the oracle's fp64 factor, relative to the condition number of A."""
    G, d, _ = Hn.shape
    Fo = oracle.damped_cholesky(Hn, rel, ab, reverse=reverse)
    worst_b = worst_f = 0.0
    for k in range(G):
        A = Hn[k] + (ab + rel * np.trace(Hn[k]) / d) * np.eye(d)
        F = Fg[k]
        if reverse:
            assert np.all(np.tril(F, -1) == 0.0)
        else:
            assert np.all(np.triu(F, 1) == 0.0)
        assert np.all(np.diag(F) > 0)
        back = np.linalg.norm(F @ F.T - A) / np.linalg.norm(A)
        fwd = np.linalg.norm(F - Fo[k]) / np.linalg.norm(Fo[k])
        cond = np.linalg.cond(A)
        worst_b, worst_f = max(worst_b, back), max(worst_f, fwd / cond)
        say(f"  {what} group {k}: backward {back:.2e}, forward {fwd:.2e} at condition number {cond:.1e}")
    assert worst_b <= 1e-5
    assert worst_f <= 1e-6


@pytest.mark.parametrize("n,d_in,G,reverse", [
    (512, 256, 2, False),       # two blocks
    (512, 256, 2, True),
    (400, 200, 3, True),        # ragged last block of 72
    (300, 132, 1, False),       # last block of 4
    (300, 100, 2, True),        # a single, ragged block
    (700, 450, 1, True),        # four blocks, d % 4 != 0: the scalar loads of the trailing update
])
def test_damped_cholesky_is_the_factor_of_the_damped_matrix(n, d_in, G, reverse):
    say(f"cholesky n={n} d_in={d_in} G={G} reverse={reverse}")
    H = _hessian(n, d_in, 4 * G, G, 51 + d_in)
    F, info = gq.gq_damped_cholesky(H, 0.01, 0.0, reverse=reverse)
    torch.cuda.synchronize()
    assert info.tolist() == [0] * G
    _check_factor(to_np64(H), to_np64(F), 0.01, 0.0, reverse, "damp 1 %")
    F2, info2 = gq.gq_damped_cholesky(H, 0.0, 0.37, reverse=reverse)      # an absolute constant instead
    torch.cuda.synchronize()
    assert info2.tolist() == [0] * G
    _check_factor(to_np64(H), to_np64(F2), 0.0, 0.37, reverse, "damp 0.37 abs")
    F3, _ = gq.gq_damped_cholesky(H, 0.01, 0.0, reverse=reverse)
    assert torch.equal(F, F3)                                              # deterministic


def test_damped_cholesky_reports_the_first_non_positive_pivot():
    d = 200
    g = torch.Generator().manual_seed(3)
    B = torch.randn(d, d, generator=g, dtype=torch.float64)
    A = (B @ B.T / d + torch.eye(d, dtype=torch.float64))
    bad = A.clone()
    bad[150, 150] = -1.0                                                   # the leading 150 x 150 block stays positive definite
    H = torch.stack([A, bad]).to(torch.float32).to(DEV).contiguous()
    F, info = gq.gq_damped_cholesky(H, 0.0, 0.0)
    torch.cuda.synchronize()
    assert info.tolist() == [0, 151]
    assert torch.isfinite(F).all()
    _check_factor(to_np64(H[:1]), to_np64(F[:1]), 0.0, 0.0, False, "the good group")
    F, info = gq.gq_damped_cholesky(H, 0.0, 0.0, reverse=True)             # from the end: coordinate 150 is the 50th eliminated
    torch.cuda.synchronize()
    assert info.tolist() == [0, 50]


def test_cholesky_then_sequential_rounding_at_the_llama2_7b_shape():
    """Config 2 shape (d_in = d_out = 4096, G = 4): factor on the GPU, check it against the damped matrix
    in fp64, round with it, replay the decisions of sampled channels from the GPU's own factor, and compare
    the objective with the oracle's GPTQ pass (from the inverse, in fp64) on a few channels."""
    spec = wl.CONFIGS["llama2_7b_attn"]
    X = wl.make_x(spec, DEV)
    s = gq.gq_group_weights(wl.make_dz_for(spec, DEV), spec.G)
    H = gq.gq_fisher_gram(X, s, mirror=True)
    del X, s
    R, info = gq.gq_damped_cholesky(H, 0.01, 0.0, reverse=True)
    torch.cuda.synchronize()
    assert info.tolist() == [0] * spec.G
    Hn = to_np64(H[:1])
    _check_factor(Hn, to_np64(R[:1]), 0.01, 0.0, True, "config 2 shape")
    W = wl.make_w(spec.d_out, spec.d_in, 7, DEV)
    _, C = wl.quantize_codebook_per_row(W, 3, return_codebook=True)
    C = C.contiguous()
    What, Q = gq.gq_ldlq_assign(W, C, R)
    rtn = torch.gather(C, 1, torch.argmin((C[:, None, :] - W[:, :, None]).abs(), dim=2))
    Hd = gq.gq_damp_diagonal(H.clone(), 0.01, 0.0)
    o_seq, o_rtn = gq.gq_objective(W, What, Hd), gq.gq_objective(W, rtn, Hd)
    torch.cuda.synchronize()
    say(f"  objective: plain rounding {o_rtn.tolist()}, sequential rounding {o_seq.tolist()}")
    assert torch.all(o_seq < 0.8 * o_rtn)
    assert torch.equal(What, torch.gather(C, 1, Q.long()))
    rows = torch.arange(0, 48, device=DEV) * 7                             # 48 channels of group 0
    R64 = to_np64(R[:1])
    Wn, new = to_np64(W[rows]), to_np64(What[rows])
    T, S = ldlq_targets(Wn, new, R64, 1)
    check_rounding_decisions(T, S, to_np64(C[rows]), Q[rows].cpu().numpy(), new, "config 2 shape, 48 sampled channels")
    r4 = rows[:4]
    _, ref = oracle.gptq_assign(to_np64(W[r4]), to_np64(C[r4]), Hn, 1, damp_rel=0.01)
    A = to_np64(Hd[:1])
    o_g = oracle.objective(to_np64(W[r4]), to_np64(What[r4]), A, 1)[1]
    o_o = oracle.objective(to_np64(W[r4]), ref, A, 1)[1]
    say(f"  4 channels: objective gpu {o_g.sum():.5f}, oracle GPTQ {o_o.sum():.5f}")
    assert abs(o_g.sum() - o_o.sum()) <= 1e-2 * o_o.sum()


def test_damp_diagonal_adds_the_same_constant_the_cholesky_uses():
    H = _hessian(300, 200, 8, 2, 9)
    Hn = to_np64(H)
    F0, _ = gq.gq_damped_cholesky(H, 0.02, 0.1)
    Hd = gq.gq_damp_diagonal(H.clone(), 0.02, 0.1)
    F1, _ = gq.gq_damped_cholesky(Hd, 0.0, 0.0)
    torch.cuda.synchronize()
    for k in range(2):
        want = Hn[k] + (0.1 + 0.02 * np.trace(Hn[k]) / 200) * np.eye(200)
        np.testing.assert_allclose(to_np64(Hd[k]), want, rtol=2e-7, atol=0)
    assert torch.equal(F0, F1)
