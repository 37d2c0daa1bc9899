"""The four consumers of H (coordinate-descent step, codebook step, Cholesky, sequential rounding) at the
shape of workload configuration 3, the Llama-2-7B down projection: d_in = 11008 (86 blocks of 128, not a
power of two), d_out = 4096, G = 4.  H comes from 16384 of the configuration's tokens (the consumers do not
care how many tokens went into it) with the scaled operand carried as two bf16 terms for the heaviest
tokens (GQ_HEAVY_TWO_TERMS): the one-term path rounds one operand of every product, which at this shape
(largest eigenvalue 1700 times the mean diagonal, a few tokens carrying most of the weight) leaves H
indefinite by more than the 1 % damping used here, and a factorization needs an H that is positive
definite.  The fp64 checks run on sampled channels of the first and the last group.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_07004_amd import binding as gq
from paper_2505_07004_amd import workloads as wl
from parity_utils import (cd_targets_along, check_codebook_channels, check_rounding_decisions, ldlq_targets, say,
                          to_np64)

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_consumers_of_h_at_the_llama2_7b_down_shape():
    spec = wl.CONFIGS["llama2_7b_down"]
    n, d_in, d_out, G = 16384, spec.d_in, spec.d_out, spec.G
    say(f"consumers at {spec.name}: W[{d_out},{d_in}] G={G}, H from {n} tokens")
    X = wl.make_x(spec, DEV, n=n)
    s = gq.gq_group_weights(wl.make_dz_for(spec, DEV, n=n), G)
    H1 = gq.gq_fisher_gram(X, s, mirror=True)
    _, info1 = gq.gq_damped_cholesky(H1, 0.01, 0.0, reverse=True)
    H = gq.gq_fisher_gram(X, s, mirror=True, heavy_two_terms=True)
    torch.cuda.synchronize()
    say(f"  first non-positive pivot with the one-term H: {info1.tolist()}")
    assert all(v > 0 for v in info1.tolist())                 # the reason for the second term
    del X, s, H1
    W = wl.make_w(d_out, d_in, 7, DEV)
    What0, C = wl.quantize_codebook_per_row(W, 3, return_codebook=True)
    C = C.contiguous()
    per = d_out // G
    groups = (0, G - 1)
    rows = {k: (k * per + torch.arange(0, 12, device=DEV) * 11) for k in groups}     # 12 channels of each

    # --- Cholesky (reverse factor): structure, and F F^T v against (H + eps I) v in fp64 for probe vectors
    R, info = gq.gq_damped_cholesky(H, 0.01, 0.0, reverse=True)
    torch.cuda.synchronize()
    assert info.tolist() == [0] * G
    rng = np.random.default_rng(0)
    for k in groups:
        Rk, Hk = to_np64(R[k]), to_np64(H[k])
        assert np.all(np.tril(Rk, -1) == 0.0) and np.all(np.diag(Rk) > 0)
        eps = 0.01 * np.trace(Hk) / d_in
        worst = 0.0
        for _ in range(4):
            v = rng.normal(size=d_in)
            ref = Hk @ v + eps * v
            worst = max(worst, float(np.linalg.norm(Rk @ (Rk.T @ v) - ref) / np.linalg.norm(ref)))
        unit = np.zeros(d_in)
        unit[d_in - 1] = 1.0                                                           # and one column exactly
        col = Rk @ (Rk.T @ unit)
        ref = Hk[:, d_in - 1] + eps * unit
        worst = max(worst, float(np.linalg.norm(col - ref) / np.linalg.norm(ref)))
        say(f"  cholesky group {k}: ||R R^T v - A v|| / ||A v|| <= {worst:.2e}")
        assert worst <= 1e-5

        # --- sequential rounding with this factor: replay the decisions of the sampled channels
        if k == groups[0]:
            Wq, Q = gq.gq_ldlq_assign(W, C, R)
            torch.cuda.synchronize()
            assert torch.equal(Wq, torch.gather(C, 1, Q.long()))
        r = rows[k]
        Wn, new = to_np64(W[r]), to_np64(Wq[r])
        T, S = ldlq_targets(Wn, new, Rk[None], 1)
        check_rounding_decisions(T, S, to_np64(C[r]), Q[r].cpu().numpy(), new, f"  sequential rounding, group {k}")
        del Rk, T, S

        # --- one coordinate-descent cycle from plain rounding, against the damped H
        if k == groups[0]:
            Hdg = gq.gq_damp_diagonal(H.clone(), 0.01, 0.0)
            Wc = What0.clone()
            before = gq.gq_objective(W, Wc, Hdg)
            Qc = gq.gq_cd_assign(W, Wc, C, Hdg, n_cycles=1)
            after = gq.gq_objective(W, Wc, Hdg)
            seq = gq.gq_objective(W, Wq, Hdg)
            torch.cuda.synchronize()
            say(f"  objective: plain rounding {before.tolist()}, one CD cycle {after.tolist()}, sequential rounding {seq.tolist()}")
            assert torch.all(after < before) and torch.all(seq < before)
            # --- the codebook step for the assignments of that cycle
            Wl = torch.empty_like(W)
            Cl = gq.gq_lnq_codebook(W, Qc, Hdg, 8, 1e-7, What=Wl)
            grid = gq.gq_objective(W, Wl, Hdg)
            torch.cuda.synchronize()
            say(f"  objective after the codebook step {grid.tolist()}")
            assert torch.all(grid <= after)
        Hdn = to_np64(Hdg[k])
        T, S = cd_targets_along(Wn, to_np64(What0[r]), to_np64(Wc[r]), Hdn[None], 1)
        check_rounding_decisions(T, S, to_np64(C[r]), Qc[r].cpu().numpy(), to_np64(Wc[r]), f"  CD cycle, group {k}")
        check_codebook_channels(oracle, Wn[:6], Qc[r[:6]].cpu().numpy().astype(np.int64), Hdn, to_np64(Cl[r[:6]]), 8, 1e-7,
                                f"  codebook step, group {k}, 6 channels")
        del Hk, Hdn, T, S
