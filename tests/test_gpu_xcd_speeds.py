"""The schedule tuning of the bf16 Gram kernel: relative XCD speeds decide where the left-over work items
are cut into runs.  Any setting must give the same H within the path's tolerance (only the grouping of the
fp32 sums changes), identical settings identical bits, and the default setting the bits of a process that
never touched it.  The measured speeds come from records every plain call leaves in its workspace."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_07004_amd import binding as gq
from paper_2505_07004_amd import workloads as wl
from parity_utils import TOL_BF16, rel_fro, say, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_xcd_speeds_change_the_cut_of_the_runs_and_nothing_else():
    # 4096 columns, 4 groups: 362 work items on 256 workgroups, one whole round and 106 left-over items
    n, d_in, G = 1024, 4096, 4
    X = wl.make_x_outlier(n, d_in, 40, 20.0, 5, DEV, torch.bfloat16)
    s = gq.gq_group_weights(wl.make_dz(n, 8 * G, 1.0, 1.5, 6, DEV), G)
    ws = torch.empty(gq.gq_fisher_gram_workspace_bytes(X.dtype, n, d_in, G), dtype=torch.uint8, device=DEV)
    iu = torch.triu_indices(d_in, d_in, device=DEV)
    try:
        base = gq.gq_fisher_gram(X, s, workspace=ws)[:, iu[0], iu[1]].clone()
        measured = gq.gq_fisher_gram_measured_xcd_speeds(n, d_in, G, ws)
        say(f"measured XCD speeds: {['%.3f' % v for v in measured]}")
        assert len(measured) == 8 and abs(sum(measured) / 8 - 1.0) < 1e-5 and all(0.5 < v < 2.0 for v in measured)
        skew = [1.08, 0.93, 1.0, 1.04, 0.9, 1.1, 0.97, 1.0]
        gq.gq_fisher_gram_set_xcd_speeds(skew)
        a = gq.gq_fisher_gram(X, s, workspace=ws)[:, iu[0], iu[1]].clone()
        b = gq.gq_fisher_gram(X, s, workspace=ws)[:, iu[0], iu[1]].clone()
        torch.cuda.synchronize()
        assert torch.equal(a, b)                                  # same setting, same bits
        assert not torch.equal(a, base)                           # the cut did move
        ref = oracle.fisher_gram(to_np64(X), to_np64(s))
        H = torch.zeros((G, d_in, d_in), device=DEV)
        H[:, iu[0], iu[1]] = a
        got = to_np64(H)
        errs = [rel_fro(got[k], np.triu(ref[k])) for k in range(G)]
        say(f"skewed speeds: rel-Frobenius per group {['%.2e' % e for e in errs]}")
        assert max(errs) <= TOL_BF16
        assert float((a - base).abs().max() / base.abs().max()) < 1e-5    # only the grouping of fp32 sums differs
        gq.gq_fisher_gram_set_xcd_speeds(None)
        c = gq.gq_fisher_gram(X, s, workspace=ws)[:, iu[0], iu[1]]
        torch.cuda.synchronize()
        assert torch.equal(c, base)                               # back to the default schedule
        with pytest.raises(gq.GQError):
            gq.gq_fisher_gram_set_xcd_speeds([1, 1, 1, 1, 1, 1, 1, 3.0])
        with pytest.raises(gq.GQError):                           # 300 columns: fewer items than workgroups, nothing recorded
            gq.gq_fisher_gram_measured_xcd_speeds(n, 300, G, ws)
    finally:
        gq.gq_fisher_gram_set_xcd_speeds(None)


def test_xcd_speeds_deal_the_whole_rounds_too():
    """With several rounds of work items the speeds also decide how many blocks of whole items each XCD takes
    (which workgroup computes a whole item does not change its bits; the left-over runs move)."""
    n, d_in, G = 512, 5120, 4            # 567 work items on 256 workgroups: two rounds = 16 blocks of 32 items
    X = wl.make_x_outlier(n, d_in, 50, 20.0, 15, DEV, torch.bfloat16)
    s = gq.gq_group_weights(wl.make_dz(n, 8 * G, 1.0, 1.5, 16, DEV), G)
    ws = torch.empty(gq.gq_fisher_gram_workspace_bytes(X.dtype, n, d_in, G), dtype=torch.uint8, device=DEV)
    iu = torch.triu_indices(d_in, d_in, device=DEV)
    try:
        base = gq.gq_fisher_gram(X, s, workspace=ws)[:, iu[0], iu[1]].clone()
        gq.gq_fisher_gram_set_xcd_speeds([1.6, 0.6, 1.0, 1.0, 1.3, 0.7, 1.0, 0.8])      # shares 3.2, 1.2, 2, 2, 2.6, 1.4, 2, 1.6 of 16
        a = gq.gq_fisher_gram(X, s, workspace=ws)[:, iu[0], iu[1]].clone()
        measured = gq.gq_fisher_gram_measured_xcd_speeds(n, d_in, G, ws)
        b = gq.gq_fisher_gram(X, s, workspace=ws)[:, iu[0], iu[1]].clone()
        torch.cuda.synchronize()
        assert len(measured) == 8 and all(0.5 < v < 2.0 for v in measured)
        assert torch.equal(a, b)
        assert float((a - base).abs().max() / base.abs().max()) < 1e-5
        ref = oracle.fisher_gram(to_np64(X), to_np64(s))
        H = torch.zeros((G, d_in, d_in), device=DEV)
        H[:, iu[0], iu[1]] = a
        got = to_np64(H)
        errs = [rel_fro(got[k], np.triu(ref[k])) for k in range(G)]
        say(f"whole rounds dealt by speed: rel-Frobenius per group {['%.2e' % e for e in errs]}")
        assert max(errs) <= TOL_BF16
        gq.gq_fisher_gram_set_xcd_speeds(None)
        c = gq.gq_fisher_gram(X, s, workspace=ws)[:, iu[0], iu[1]]
        torch.cuda.synchronize()
        assert torch.equal(c, base)
    finally:
        gq.gq_fisher_gram_set_xcd_speeds(None)
