"""The entry point that allocates nothing, gq_fisher_gram_noalloc, against gq_fisher_gram (and the
oracle), through the C ABI: two calls in a row on one GPU, the second with a smaller input, so that the
second call runs over whatever the first left in the library's fixed scratch array."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_07004_amd import binding as gq
from paper_2505_07004_amd import workloads as wl
from parity_utils import TOL_BF16, TOL_F32, rel_fro, say, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _case(n, d_in, G, dtype, seed):
    X = wl.make_x_outlier(n, d_in, max(1, d_in // 64), 20.0, seed, DEV, dtype)
    dZ = wl.make_dz(n, 8 * G, 1.0, 1.5, seed + 1, DEV)
    return X, gq.gq_group_weights(dZ, G)


def _compare(X, s, tol, what, two_terms=False):
    G, d_in = s.shape[1], X.shape[1]
    ref = gq.gq_fisher_gram(X, s, mirror=True, two_terms=two_terms)
    H = torch.full((G, d_in, d_in), float("nan"), device=DEV)
    before = torch.cuda.memory_allocated()
    gq.gq_fisher_gram_noalloc(X, s, H, mirror=True, two_terms=two_terms)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    got, want = to_np64(H), to_np64(ref)
    assert np.all(np.isfinite(got))
    exact = oracle.fisher_gram(to_np64(X), to_np64(s))
    for k in range(G):
        e_ref, e_oracle = rel_fro(got[k], want[k]), rel_fro(got[k], exact[k])
        say(f"{what} group {k}: vs gq_fisher_gram {e_ref:.2e}, vs oracle {e_oracle:.2e}")
        assert np.array_equal(got[k], got[k].T)
        assert e_ref <= 2e-6 and e_oracle <= tol        # same products; only the order of the fp32 additions differs
    return H


def test_two_calls_in_a_row_the_second_smaller():
    X1, s1 = _case(3000, 520, 4, torch.bfloat16, 11)          # wide kernel, ragged token count, several tiles
    _compare(X1, s1, TOL_BF16, "first call (n=3000, d_in=520, G=4)")
    X2, s2 = _case(777, 136, 4, torch.bfloat16, 12)           # smaller in every dimension
    _compare(X2, s2, TOL_BF16, "second call (n=777, d_in=136, G=4)")
    X3, s3 = _case(500, 264, 2, torch.bfloat16, 13)           # the narrow kernel (G not divisible by 4), two terms
    _compare(X3, s3, 2e-5, "third call (n=500, d_in=264, G=2, two terms)", two_terms=True)


def test_accumulation_over_chunks_and_the_fp32_path():
    X, s = _case(2048, 256, 4, torch.bfloat16, 21)
    H = torch.empty((4, 256, 256), device=DEV)
    for i in range(4):
        gq.gq_fisher_gram_noalloc(X[i * 512:(i + 1) * 512], s[i * 512:(i + 1) * 512], H, accumulate=i > 0)
    gq.gq_fisher_mirror(H)
    ref = gq.gq_fisher_gram(X, s, mirror=True)
    torch.cuda.synchronize()
    for k in range(4):
        assert rel_fro(to_np64(H[k]), to_np64(ref[k])) <= 1e-5
    Xf, sf = _case(600, 128, 2, torch.float32, 22)
    _compare(Xf, sf, TOL_F32, "fp32 path")


def test_a_call_beyond_the_fixed_array_is_refused():
    lib = gq.load_library()
    limit = int(lib.gq_fisher_gram_noalloc_max_scratch_bytes())
    assert limit == 4 << 20
    n, G = 65536, 16                                              # 4 * 16 * (65536 + 256) bytes > 4 MiB
    X = torch.zeros((n, 64), dtype=torch.bfloat16, device=DEV)
    s = torch.zeros((n, G), device=DEV)
    H = torch.full((G, 64, 64), 7.0, device=DEV)
    with pytest.raises(gq.GQError) as err:
        gq.gq_fisher_gram_noalloc(X, s, H)
    assert err.value.status == -5                                 # GQ_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((H == 7.0).all())                                 # nothing was enqueued
    gq.gq_fisher_gram_noalloc(X[:, :64], s[:, :15].contiguous(), torch.empty((15, 64, 64), device=DEV))   # G = 15 fits
    torch.cuda.synchronize()
