"""The closed-form codebook step on the GPU (through the C ABI) against the fp64 oracle.

The solution of a linear system is as accurate as the system is well conditioned, and the
conditioning of P^T H P is a property of the data, not of the kernel.  So the first check is a
backward one, independent of conditioning: with the oracle's fp64 A = P^T H P and b = P^T H w, the
GPU's grid c must satisfy |(A + lam I) c - b| <= 2^-20 (|P|^T |H| |P| |c| + |P|^T |H| |w|) entry by
entry (the GPU adds exact products in fp32, a relative error of a few 2^-24 of the sum of the
absolute values of the terms; measured: 3e-8).  The second check is the
one the method cares about: the channel's objective at the GPU's grid exceeds the minimum (the
oracle's) by a relative 1e-6 at most.  The third compares the grids directly, the difference
divided by the condition number of the system (a looser, normwise bound: 1e-5)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_07004_amd import binding as gq
from paper_2505_07004_amd import workloads as wl
from parity_utils import check_codebook_channels, say, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda"
LAM = 1e-7


def _case(n, d_in, d_out, G, bits, seed, ld=None):
    X = wl.make_x_outlier(n, d_in, max(1, d_in // 64), 20.0, seed, DEV, torch.float32)
    dZ = wl.make_dz(n, d_out, 1.0, 1.5, seed + 1, DEV)
    s = gq.gq_group_weights(dZ, G)
    H = gq.gq_fisher_gram(X, s, mirror=True)
    gq.gq_damp_diagonal(H, 0.01, 0.0)
    W = wl.make_w(d_out, d_in, seed + 2, DEV)
    What, C = wl.quantize_codebook_per_row(W, bits, return_codebook=True)
    Q = torch.argmin((C[:, None, :] - What[:, :, None]).abs(), dim=2).to(torch.uint8).contiguous()
    if ld:
        buf = torch.full((d_out, ld), float("nan"), device=DEV)
        buf[:, :d_in] = W
        W = buf[:, :d_in]
    return W, Q, H


@pytest.mark.parametrize("n,d_in,d_out,G,bits,ld", [
    (512, 256, 128, 2, 3, None),        # two column tiles, 64 channels x 8 grid points = 4 row tiles per group
    (400, 200, 96, 4, 2, 208),          # ragged contraction and columns, 24 x 4 = 96 rows per group (ragged row tile), padded pitch
    (600, 384, 48, 1, 4, None),         # 16 grid points
    (300, 132, 40, 2, 3, 136),          # 4 coordinates in the last tile, 160 rows per group
])
def test_codebook_step_solves_the_oracles_system(n, d_in, d_out, G, bits, ld):
    say(f"lnq codebook n={n} d_in={d_in} d_out={d_out} G={G} bits={bits} ld={ld}")
    W, Q, H = _case(n, d_in, d_out, G, bits, 131 + d_in, ld)
    m = 1 << bits
    What = torch.zeros_like(W) if ld is None else torch.full((d_out, ld), float("nan"), device=DEV)[:, :d_in]
    C = gq.gq_lnq_codebook(W, Q, H, m, LAM, What=What)
    torch.cuda.synchronize()
    assert torch.equal(What, torch.gather(C, 1, Q.long()))              # What is the grid value of its code, exactly
    Wn, Qn, Hn, Cg = to_np64(W), Q.cpu().numpy().astype(np.int64), to_np64(H), to_np64(C)
    per = d_out // G
    for k in range(G):
        r = slice(k * per, (k + 1) * per)
        check_codebook_channels(oracle, Wn[r], Qn[r], Hn[k], Cg[r], m, LAM, f"group {k}")
    # and without the optional output
    C2 = gq.gq_lnq_codebook(W, Q, H, m, LAM)
    torch.cuda.synchronize()
    assert torch.equal(C, C2)                                           # deterministic


def test_identity_hessian_gives_cluster_means_and_unused_points_are_zero():
    d_out, d_in, m = 64, 200, 8
    W = wl.make_w(d_out, d_in, 3, DEV)
    g = torch.Generator(device="cpu").manual_seed(11)
    Q = torch.randint(0, m - 1, (d_out, d_in), generator=g, dtype=torch.uint8).to(DEV)   # grid point m-1 is never used
    Q[0, :] = 2                                                                            # a channel with a single cluster
    H = torch.eye(d_in, device=DEV).repeat(2, 1, 1).contiguous()
    C = gq.gq_lnq_codebook(W, Q, H, m, LAM)
    torch.cuda.synchronize()
    Wn, Qn, Cg = to_np64(W), Q.cpu().numpy(), to_np64(C)
    for j in range(d_out):
        for q in range(m):
            sel = Qn[j] == q
            want = Wn[j][sel].sum() / (sel.sum() + LAM) if sel.any() else 0.0
            assert abs(Cg[j, q] - want) <= 1e-6 * np.abs(Wn[j]).max(), (j, q, Cg[j, q], want)
    assert np.all(Cg[:, m - 1] == 0.0)


def test_codebook_step_after_a_cd_cycle_does_not_increase_the_objective():
    """Prop. 4.1: each of the two alternating steps of Algorithm 2 can only lower the objective."""
    W, Q0, H = _case(512, 256, 128, 2, 3, 977)
    m = 8
    What = torch.empty_like(W)
    C = gq.gq_lnq_codebook(W, Q0, H, m, LAM, What=What)
    obj = [gq.gq_objective(W, What, H).cpu().numpy()]
    for it in range(3):
        Q = gq.gq_cd_assign(W, What, C, H, n_cycles=1)
        obj.append(gq.gq_objective(W, What, H).cpu().numpy())
        C = gq.gq_lnq_codebook(W, Q, H, m, LAM, What=What)
        obj.append(gq.gq_objective(W, What, H).cpu().numpy())
    torch.cuda.synchronize()
    say("objective along 3 alternations: " + ", ".join(f"{o.sum():.5f}" for o in obj))
    for a, b in zip(obj[:-1], obj[1:]):
        assert np.all(b <= a * (1 + 1e-6))
    assert obj[-1].sum() < 0.9 * obj[0].sum()


def test_codebook_step_at_the_llama2_7b_shape_on_sampled_channels():
    """Full size of workload configuration 2 (d_out = d_in = 4096, G = 4), 3-bit and 4-bit grids;
    the oracle's system is formed for 12 sampled channels of every group."""
    spec = wl.CONFIGS["llama2_7b_attn"]
    X = wl.make_x(spec, DEV)
    s = gq.gq_group_weights(wl.make_dz_for(spec, DEV), spec.G)
    H = gq.gq_fisher_gram(X, s, mirror=True)
    del X, s
    gq.gq_damp_diagonal(H, 0.01, 0.0)
    W = wl.make_w(spec.d_out, spec.d_in, 7, DEV)
    per = spec.d_out // spec.G
    g = torch.Generator().manual_seed(5)
    for bits in (3, 4):
        m = 1 << bits
        say(f"lnq codebook at {spec.name}: W[{spec.d_out},{spec.d_in}] G={spec.G} grid points {m}")
        What0, C0 = wl.quantize_codebook_per_row(W, bits, return_codebook=True)
        Q = torch.argmin((C0[:, None, :] - What0[:, :, None]).abs(), dim=2).to(torch.uint8).contiguous()
        before = gq.gq_objective(W, What0, H)
        What = torch.empty_like(W)
        C = gq.gq_lnq_codebook(W, Q, H, m, LAM, What=What)
        after = gq.gq_objective(W, What, H)
        torch.cuda.synchronize()
        say(f"  objective {before.tolist()} -> {after.tolist()}")
        assert torch.all(after <= before)
        assert torch.equal(What, torch.gather(C, 1, Q.long()))
        for k in range(spec.G):
            rows = (k * per + torch.randperm(per, generator=g)[:12]).to(DEV)
            check_codebook_channels(oracle, to_np64(W[rows]), Q[rows].cpu().numpy().astype(np.int64), to_np64(H[k]), to_np64(C[rows]),
                            m, LAM, f"  group {k}, 12 sampled channels")
        del What, C, What0, C0, Q


@pytest.mark.parametrize("m", [1, 3, 5, 11])
def test_codebook_step_with_a_number_of_grid_points_that_is_not_a_power_of_two(m):
    """Whole channels per workgroup tile: 256 // m of them (at most 64), so tiles end inside a row block."""
    d_out, d_in, G = 140, 200, 2                                         # 70 channels per group: two tiles for m = 5, 11
    X = wl.make_x_outlier(400, d_in, 3, 20.0, 9, DEV, torch.float32)
    H = gq.gq_fisher_gram(X, gq.gq_group_weights(wl.make_dz(400, d_out, 1.0, 1.5, 10, DEV), G), mirror=True)
    gq.gq_damp_diagonal(H, 0.01, 0.0)
    W = wl.make_w(d_out, d_in, 11, DEV)
    g = torch.Generator(device="cpu").manual_seed(12 + m)
    Q = torch.randint(0, m, (d_out, d_in), generator=g, dtype=torch.uint8).to(DEV)
    What = torch.empty_like(W)
    C = gq.gq_lnq_codebook(W, Q, H, m, LAM, What=What)
    torch.cuda.synchronize()
    assert C.shape == (d_out, m) and torch.equal(What, torch.gather(C, 1, Q.long()))
    Wn, Qn, Hn, Cg = to_np64(W), Q.cpu().numpy().astype(np.int64), to_np64(H), to_np64(C)
    per = d_out // G
    for k in range(G):
        r = slice(k * per, (k + 1) * per)
        check_codebook_channels(oracle, Wn[r], Qn[r], Hn[k], Cg[r], m, LAM, f"{m} grid points, group {k}")


def test_lnq_alternation_in_one_call_equals_its_parts_and_reaches_the_oracles_objective():
    """Algorithm 2 with T = 2, K = 2: bit-identical to the same calls made one by one, every step a descent,
    and the final objective within 1e-3 of the fp64 oracle's run from the same start (the two trajectories
    part at rounding-level near-ties, so the assignments themselves are compared only in bulk)."""
    W, Q0, H = _case(512, 256, 128, 2, 3, 555)
    m = 8
    Q = Q0.clone()
    What, C = gq.gq_lnq(W, Q, H, m, n_iters=2, n_cycles=2, lam=LAM)
    torch.cuda.synchronize()
    assert torch.equal(What, torch.gather(C, 1, Q.long()))
    # by hand
    Qh, Wh = Q0.clone(), torch.empty_like(W)
    objs = []
    for _ in range(2):
        Ch = gq.gq_lnq_codebook(W, Qh, H, m, LAM, What=Wh)
        objs.append(gq.gq_objective(W, Wh, H).sum().item())
        Qh = gq.gq_cd_assign(W, Wh, Ch, H, n_cycles=2)
        objs.append(gq.gq_objective(W, Wh, H).sum().item())
    Ch = gq.gq_lnq_codebook(W, Qh, H, m, LAM, What=Wh)
    objs.append(gq.gq_objective(W, Wh, H).sum().item())
    torch.cuda.synchronize()
    assert torch.equal(Qh, Q) and torch.equal(Wh, What) and torch.equal(Ch, C)
    assert all(b <= a * (1 + 1e-6) for a, b in zip(objs[:-1], objs[1:]))
    Qo, Wo, Co, trace = oracle.lnq(to_np64(W), Q0.cpu().numpy(), to_np64(H), m, 2, n_iters=2, n_cycles=2, lam=LAM)
    say("objective gpu " + ", ".join(f"{o:.4f}" for o in objs) + " | oracle " + ", ".join(f"{o:.4f}" for o in trace))
    assert abs(objs[0] - trace[0]) <= 5e-6 * trace[0]                    # the first codebook step: same assignments (gq_objective itself is good to ~2e-6)
    assert abs(objs[-1] - trace[-1]) <= 1e-3 * trace[-1]
    assert float(np.mean(Qo != Q.cpu().numpy())) <= 0.02
    # no iterations: the codebook step alone
    Qz = Q0.clone()
    Wz, Cz = gq.gq_lnq(W, Qz, H, m, n_iters=0, lam=LAM)
    Wc = torch.empty_like(W)
    Cc = gq.gq_lnq_codebook(W, Q0, H, m, LAM, What=Wc)
    torch.cuda.synchronize()
    assert torch.equal(Qz, Q0) and torch.equal(Wz, Wc) and torch.equal(Cz, Cc)
