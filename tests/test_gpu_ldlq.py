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
from parity_utils import check_rounding_decisions, say, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _hessian(n, d_in, d_out, G, seed):
    X = wl.make_x_outlier(n, d_in, max(1, d_in // 64), 20.0, seed, DEV, torch.float32)
    dZ = wl.make_dz(n, d_out, 1.0, 1.5, seed + 1, DEV)
    return gq.gq_fisher_gram(X, gq.gq_group_weights(dZ, G), mirror=True)


def _targets_from_factor(Wn, new, Rn, G):
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


@pytest.mark.parametrize("n,d_in,d_out,G,bits,ld", [
    (512, 256, 128, 2, 3, None),        # two blocks
    (400, 200, 96, 4, 2, 208),          # ragged last block, padded pitch
    (600, 384, 192, 1, 4, None),        # 16 grid points, three blocks
    (300, 132, 40, 2, 3, 136),          # last block of 4 coordinates
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
        buf = torch.zeros((d_out, ld), device=DEV)
        buf[:, :d_in] = W
        W = buf[:, :d_in]
    What, Q = gq.gq_ldlq_assign(W, C, R)
    torch.cuda.synchronize()
    Wn, Cn, new, Qg = to_np64(W), to_np64(C), to_np64(What), Q.cpu().numpy()
    R64 = Rn.astype(np.float64)
    T, S = _targets_from_factor(Wn, new, R64, G)
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
