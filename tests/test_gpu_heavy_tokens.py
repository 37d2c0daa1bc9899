"""GQ_HEAVY_TWO_TERMS of gq_fisher_gram: the same H (Algorithm 1, line 4), with the scaled operand in two
bf16 terms for the heaviest tokens only.  Checked against the fp64 oracle (the definition is unchanged), and
against the mode's own definition: the call must equal, bit for bit, a one-term call on the weights with the
heavy tokens set to 0 followed by an accumulating two-term call on the heavy tokens' rows, where "heavy" is
decided here on the host straight from the rule in the header."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_07004_amd import binding as gq
from paper_2505_07004_amd import workloads as wl
from parity_utils import TOL_BF16, rel_fro, say, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _capacity(n):
    return 32 * max(1, -(-n // 2048))


def _split_on_host(X, s):
    """The header's rule, spelled out: heavy tokens (first `capacity` of them in token order), the weights with
    those tokens at 0, and their rows and weights padded with zero rows up to the capacity."""
    n, G = s.shape
    thr = (s.double().sum(dim=0) / n).float() * 16.0
    heavy = (s > thr[None, :]).any(dim=1)
    idx = torch.nonzero(heavy).flatten()[: _capacity(n)]
    s_main = s.clone()
    s_main[idx] = 0
    Xh = torch.zeros((_capacity(n), X.shape[1]), dtype=X.dtype, device=X.device)
    sh = torch.zeros((_capacity(n), G), dtype=s.dtype, device=s.device)
    Xh[: idx.numel()] = X[idx]
    sh[: idx.numel()] = s[idx]
    return idx, s_main.contiguous(), Xh, sh, int(heavy.sum())


def _case(n, d_in, G, seed, kind="silu", sigma=1.5):
    X = (wl.make_x_silu(n, d_in, seed, DEV, torch.bfloat16) if kind == "silu"
         else wl.make_x_outlier(n, d_in, max(1, d_in // 64), 20.0, seed, DEV, torch.bfloat16))
    s = gq.gq_group_weights(wl.make_dz(n, 8 * G, 1.0, sigma, seed + 1, DEV), G)
    return X, s


@pytest.mark.parametrize("n,d_in,G,kind", [
    (5000, 520, 4, "silu"),          # wide kernel for the main pass, ragged tokens and columns, capacity 96
    (3000, 264, 3, "outlier"),       # narrow kernel for both passes
    (40, 72, 4, "silu"),             # fewer tokens than the capacity
    (2048, 256, 1, "silu"),
    (2100, 520, 5, "silu"),          # odd group count: the main pass runs as four groups (wide kernel) + one (narrow)
])
def test_heavy_mode_is_its_two_passes_and_matches_the_oracle(n, d_in, G, kind):
    say(f"heavy-token mode n={n} d_in={d_in} G={G} {kind}")
    X, s = _case(n, d_in, G, 900 + n, kind)
    idx, s_main, Xh, sh, n_heavy = _split_on_host(X, s)
    H = gq.gq_fisher_gram(X, s, heavy_two_terms=True)
    ref2 = gq.gq_fisher_gram(X, s_main)
    gq.gq_fisher_gram(Xh, sh, H=ref2, accumulate=True, two_terms=True)
    torch.cuda.synchronize()
    say(f"  {n_heavy} heavy tokens, {idx.numel()} taken (capacity {_capacity(n)})")
    iu = torch.triu_indices(d_in, d_in, device=DEV)
    assert torch.equal(H[:, iu[0], iu[1]], ref2[:, iu[0], iu[1]])
    ref = oracle.fisher_gram(to_np64(X), to_np64(s))
    one = to_np64(gq.gq_fisher_gram(X, s))
    got = to_np64(H)
    e_h = [rel_fro(np.triu(got[k]), np.triu(ref[k])) for k in range(G)]
    e_1 = [rel_fro(np.triu(one[k]), np.triu(ref[k])) for k in range(G)]
    say(f"  rel-Frobenius per group: heavy mode {['%.2e' % e for e in e_h]}, one term {['%.2e' % e for e in e_1]}")
    assert max(e_h) <= TOL_BF16
    if n_heavy:
        assert max(e_h) <= max(e_1)


def test_heavy_mode_without_heavy_tokens_and_with_more_than_the_capacity():
    n, d_in, G = 4096, 264, 4
    X, _ = _case(n, d_in, G, 31)
    # equal weights: nothing is heavy, the call is the plain one
    s = torch.ones((n, G), device=DEV)
    a = gq.gq_fisher_gram(X, s, heavy_two_terms=True)
    b = gq.gq_fisher_gram(X, s)
    torch.cuda.synchronize()
    iu = torch.triu_indices(d_in, d_in, device=DEV)
    assert torch.equal(a[:, iu[0], iu[1]], b[:, iu[0], iu[1]])
    # 150 tokens at 1000 times the weight of the rest: more than the capacity of 64, the first 64 are taken
    s = torch.ones((n, G), device=DEV)
    pos = torch.arange(150, device=DEV) * 27 + 5
    s[pos, 1] = 1000.0
    idx, s_main, Xh, sh, n_heavy = _split_on_host(X, s)
    assert n_heavy == 150 and idx.numel() == 64 and torch.equal(idx, pos[:64])
    H = gq.gq_fisher_gram(X, s, heavy_two_terms=True)
    ref2 = gq.gq_fisher_gram(X, s_main)
    gq.gq_fisher_gram(Xh, sh, H=ref2, accumulate=True, two_terms=True)
    torch.cuda.synchronize()
    assert torch.equal(H[:, iu[0], iu[1]], ref2[:, iu[0], iu[1]])
    ref = oracle.fisher_gram(to_np64(X), to_np64(s))
    got = to_np64(H)
    assert max(rel_fro(np.triu(got[k]), np.triu(ref[k])) for k in range(G)) <= TOL_BF16


def test_heavy_mode_accumulates_over_chunks_mirrors_and_gives_a_factorable_h():
    """Heavy-tailed weights, fewer effective tokens than columns: the one-term H is indefinite beyond the 1 %
    diagonal constant, the heavy-token mode is accepted by the Cholesky factorization."""
    n, d_in, G = 8192, 1024, 4
    X, s = _case(n, d_in, G, 57)
    H = None
    for c0 in range(0, n, 4096):
        H = gq.gq_fisher_gram(X[c0:c0 + 4096], s[c0:c0 + 4096], H=H, accumulate=c0 > 0, heavy_two_terms=True,
                              mirror=c0 > 0)
    H1 = gq.gq_fisher_gram(X, s, mirror=True)
    _, info1 = gq.gq_damped_cholesky(H1, 0.01, 0.0, reverse=True)
    _, info = gq.gq_damped_cholesky(H, 0.01, 0.0, reverse=True)
    torch.cuda.synchronize()
    say(f"first non-positive pivot per group: one term {info1.tolist()}, heavy-token mode {info.tolist()}")
    assert info.tolist() == [0] * G
    got = to_np64(H)
    assert np.array_equal(got, np.transpose(got, (0, 2, 1)))
    ref = oracle.fisher_gram(to_np64(X), to_np64(s))
    assert max(rel_fro(got[k], ref[k]) for k in range(G)) <= TOL_BF16
    a = gq.gq_fisher_gram(X, s, heavy_two_terms=True)
    b = gq.gq_fisher_gram(X, s, heavy_two_terms=True)
    torch.cuda.synchronize()
    assert torch.equal(torch.triu(a), torch.triu(b))              # deterministic


def _deferred(chunks, pool_rows, d_in, G):
    pool = gq.gq_fisher_gram_heavy_pool(d_in, G, pool_rows, DEV)
    H = None
    for i, (Xc, sc) in enumerate(chunks):
        H = gq.gq_fisher_gram_heavy_deferred(Xc, sc, pool, pool_rows, H=H, accumulate=i > 0)
    in_use = int(pool[:4].view(torch.int32).item())
    gq.gq_fisher_gram_heavy_flush(pool, pool_rows, H)
    torch.cuda.synchronize()
    assert int(pool[:4].view(torch.int32).item()) == 0          # the flush leaves the pool empty
    return H, in_use, pool


@pytest.mark.parametrize("sizes,d_in,G,pool_rows", [
    ((3000, 2500, 1777), 520, 4, 256),     # wide main passes; 48 + 64 + 32 rows of capacity fit
    ((2048, 2048, 2048, 2048), 264, 3, 64),   # narrow main passes; the pool fills up: later heavy tokens stay one-term
    ((700,), 136, 1, 32),
])
def test_heavy_rows_gathered_over_chunks_and_flushed_once(sizes, d_in, G, pool_rows):
    """The deferred form: per chunk the same selection as the plain heavy-token call, the rows of all chunks in one
    pool, one two-term pass at the end.  Against the oracle, against the same passes made by hand (selection rule
    retyped on the host; the hand-made second pass sees fewer rows, so fp32 sums may be grouped differently), and
    bit for bit against itself."""
    n = sum(sizes)
    say(f"deferred heavy rows: chunks {sizes} d_in={d_in} G={G} pool of {pool_rows} rows")
    X, s = _case(n, d_in, G, 1300 + n)
    cuts = np.cumsum((0,) + tuple(sizes))
    chunks = [(X[a:b], s[a:b]) for a, b in zip(cuts[:-1], cuts[1:])]
    H, in_use, pool = _deferred(chunks, pool_rows, d_in, G)
    # by hand
    ref2, rows_x, rows_s, room = None, [], [], pool_rows
    for i, (Xc, sc) in enumerate(chunks):
        idx, s_main, _, _, _ = _split_on_host(Xc, sc)
        idx = idx[:room]                                        # what the pool still takes
        s_main = sc.clone()
        s_main[idx] = 0
        room -= idx.numel()
        rows_x.append(Xc[idx])
        rows_s.append(sc[idx])
        ref2 = gq.gq_fisher_gram(Xc, s_main.contiguous(), H=ref2, accumulate=i > 0)
    Xh, sh = torch.cat(rows_x), torch.cat(rows_s)
    assert in_use == Xh.shape[0]
    say(f"  {in_use} rows in the pool before the flush")
    if in_use:
        gq.gq_fisher_gram(Xh.contiguous(), sh.contiguous(), H=ref2, accumulate=True, two_terms=True)
    torch.cuda.synchronize()
    iu = torch.triu_indices(d_in, d_in, device=DEV)
    a, b = H[:, iu[0], iu[1]], ref2[:, iu[0], iu[1]]
    assert float((a - b).abs().max() / b.abs().max()) < 2e-6
    ref = oracle.fisher_gram(to_np64(X), to_np64(s))
    got = to_np64(H)
    errs = [rel_fro(np.triu(got[k]), np.triu(ref[k])) for k in range(G)]
    say(f"  rel-Frobenius per group {['%.2e' % e for e in errs]}")
    assert max(errs) <= TOL_BF16
    again, _, _ = _deferred(chunks, pool_rows, d_in, G)
    assert torch.equal(again[:, iu[0], iu[1]], a)
    # an empty pool adds nothing
    before = H.clone()
    gq.gq_fisher_gram_heavy_flush(pool, pool_rows, H)
    torch.cuda.synchronize()
    assert torch.equal(H[:, iu[0], iu[1]], before[:, iu[0], iu[1]])
