"""Parity at the full sizes of the five workload configurations, in the launch
configuration bench.py times.  Config 2 is compared with the fp64 oracle element by
element; the larger shapes with the oracle on sampled output blocks, probe vectors and
sampled objective rows (every sampled value is computed exactly in fp64 from X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_07004_amd import binding as gq
from paper_2505_07004_amd import workloads as wl
from parity_utils import (TOL_BF16, TOL_S, rel_fro, sampled_gram_check, sampled_objective_check, say, to_np64)

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _layer(name, G=None):
    spec = wl.CONFIGS[name]
    if G is not None:
        spec = wl.scaled(spec, G=G)
    say(f"{spec.name}: X[{spec.n},{spec.d_in}] dZ[{spec.n},{spec.d_out}] G={spec.G}")
    X = wl.make_x(spec, DEV)
    dZ = wl.make_dz_for(spec, DEV)
    s = gq.gq_group_weights(dZ, spec.G)
    # s against the oracle on sampled tokens (all groups)
    idx = torch.randint(0, spec.n, (512,), device=DEV)
    ref = oracle.group_weights(to_np64(dZ[idx]), spec.G)
    got = to_np64(s[idx])
    assert np.all(np.abs(got - ref) <= TOL_S * np.abs(ref) + 1e-300)
    del dZ
    return spec, X, s


@pytest.mark.parametrize("two_terms,tol_h", [(False, TOL_BF16), (True, 2e-5)])
def test_config2_llama2_7b_attn_full_oracle(two_terms, tol_h):
    spec, X, s = _layer("llama2_7b_attn")
    W, What = wl.make_weights(spec, DEV)
    H = gq.gq_fisher_gram(X, s, mirror=True, two_terms=two_terms)
    obj, rows = gq.gq_objective(W, What, H, want_rows=True)
    torch.cuda.synchronize()
    X64, s64 = to_np64(X), to_np64(s)
    W64, Wh64 = to_np64(W), to_np64(What)
    for k in range(spec.G):
        Hk = oracle.fisher_gram(X64, s64[:, k:k + 1])[0]
        got = to_np64(H[k])
        err = rel_fro(got, Hk)
        o_ref, r_ref = oracle.objective(W64[k * 1024:(k + 1) * 1024], Wh64[k * 1024:(k + 1) * 1024], Hk[None], 1)
        e_obj = abs(float(obj[k]) - o_ref[0]) / o_ref[0]
        e_rows = rel_fro(to_np64(rows[k * 1024:(k + 1) * 1024]), r_ref)
        say(f"config 2 group {k}: H rel-Frobenius {err:.2e}, objective {e_obj:.2e}, per-channel {e_rows:.2e}")
        assert np.array_equal(got, got.T)
        assert err <= tol_h and e_obj <= TOL_BF16 and e_rows <= TOL_BF16
        del Hk, got


def test_config3_llama2_7b_down_eight_chunks():
    spec, X, s = _layer("llama2_7b_down")
    H = None
    c = spec.n // spec.chunks
    for i in range(spec.chunks):
        H = gq.gq_fisher_gram(X[i * c:(i + 1) * c], s[i * c:(i + 1) * c], H=H, accumulate=i > 0)
    gq.gq_fisher_mirror(H)
    sampled_gram_check(oracle, X, s, H, TOL_BF16, seed=3, what="config 3, 8 chunks")
    one = gq.gq_fisher_gram(X, s, mirror=True)
    torch.cuda.synchronize()
    for k in range(spec.G):       # chunked and one-shot differ only by fp32 re-association
        num = torch.linalg.norm((one[k] - H[k]).double())
        assert float(num / torch.linalg.norm(one[k].double())) <= 1e-5
    del one
    W, What = wl.make_weights(spec, DEV)
    obj, rows = gq.gq_objective(W, What, H, want_rows=True)
    sampled_objective_check(oracle, X, s, W, What, obj, rows, spec.G, TOL_BF16, seed=3, what="config 3")


@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_config4_llama2_13b_attn_groups(G):
    spec, X, s = _layer("llama2_13b_attn", G)
    H = gq.gq_fisher_gram(X, s, mirror=True)
    sampled_gram_check(oracle, X, s, H, TOL_BF16, n_random=12, seed=40 + G, what=f"config 4 d_in 5120 G={G}")
    W, What = wl.make_weights(spec, DEV)
    obj, rows = gq.gq_objective(W, What, H, want_rows=True)
    sampled_objective_check(oracle, X, s, W, What, obj, rows, G, TOL_BF16, rows_per_group=16, seed=G, what=f"config 4 G={G}")


@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_config4_llama2_13b_up_wide_gradients(G):
    # gate/up projections: the gradient matrix is 13824 wide, X is the shared attention-side input
    spec, X, s = _layer("llama2_13b_up", G)
    H = gq.gq_fisher_gram(X, s, mirror=True)
    sampled_gram_check(oracle, X, s, H, TOL_BF16, n_random=8, seed=44 + G, what=f"config 4 up_proj G={G}")
    W, What = wl.make_weights(spec, DEV)
    obj, rows = gq.gq_objective(W, What, H, want_rows=True)
    sampled_objective_check(oracle, X, s, W, What, obj, rows, G, TOL_BF16, rows_per_group=16 if G <= 4 else 8, seed=45 + G,
                            what=f"config 4 up_proj G={G}")


@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_config4_llama2_13b_down(G):
    spec, X, s = _layer("llama2_13b_down", G)
    H = gq.gq_fisher_gram(X, s, mirror=True)
    sampled_gram_check(oracle, X, s, H, TOL_BF16, n_random=10, n_probe=2, seed=46 + G, what=f"config 4 down_proj G={G}")
    W, What = wl.make_weights(spec, DEV)
    obj, rows = gq.gq_objective(W, What, H, want_rows=True)
    sampled_objective_check(oracle, X, s, W, What, obj, rows, G, TOL_BF16, rows_per_group=8 if G <= 4 else 4, seed=56 + G,
                            what=f"config 4 down_proj G={G}")


def test_config4_q_k_v_stacked_in_one_gram_call():
    """The three attention projections of the 13B block read the same X: their group weights side by
    side (3 x 4 columns) and ONE Gram call with 12 groups; every layer's four Hessians against the oracle."""
    spec = wl.CONFIGS["llama2_13b_attn"]
    G, layers = spec.G, 3
    say(f"stacked q/k/v: X[{spec.n},{spec.d_in}], {layers} x dZ[{spec.n},{spec.d_out}], G={G} each")
    X = wl.make_x(spec, DEV)
    s_all = torch.empty((spec.n, layers * G), dtype=torch.float32, device=DEV)
    for l in range(layers):
        dZ = wl.make_dz(spec.n, spec.d_out, 1e-4, 1.5, 250507004 + 4000 + 17 * l, DEV)
        gq.gq_group_weights(dZ, G, out=s_all, out_col=l * G)
        one = gq.gq_group_weights(dZ, G)
        assert torch.equal(one, s_all[:, l * G:(l + 1) * G])          # the strided call writes the same numbers
        del dZ, one
    H = gq.gq_fisher_gram(X, s_all, mirror=True)
    assert H.shape == (layers * G, spec.d_in, spec.d_in)
    for l in range(layers):
        sampled_gram_check(oracle, X, s_all[:, l * G:(l + 1) * G].contiguous(), H[l * G:(l + 1) * G], TOL_BF16,
                           n_random=8, n_probe=2, seed=70 + l, what=f"config 4 stacked q/k/v, layer {l}")


@pytest.mark.parametrize("name,G", [("llama2_70b_attn", None), ("llama2_70b_up", None),
                                    ("llama2_70b_attn", 2)])     # 2: the group count of the paper's 70B runs (appendix on hyperparameters)
def test_config5_llama2_70b_8192(name, G):
    spec, X, s = _layer(name, G)
    H = gq.gq_fisher_gram(X, s, mirror=True)
    sampled_gram_check(oracle, X, s, H, TOL_BF16, n_random=12, seed=50, what=f"config 5 {name} G={spec.G}")
    W, What = wl.make_weights(spec, DEV)
    obj, rows = gq.gq_objective(W, What, H, want_rows=True)
    sampled_objective_check(oracle, X, s, W, What, obj, rows, spec.G, TOL_BF16, rows_per_group=8, seed=51, what=f"config 5 {name}")


def test_config5_llama2_70b_down_13gb_hessians():
    spec, X, s = _layer("llama2_70b_down")
    H = gq.gq_fisher_gram(X, s, mirror=True)           # 4 x 28672^2 fp32 = 12.25 GiB, > 2^31 elements
    sampled_gram_check(oracle, X, s, H, TOL_BF16, n_random=10, n_probe=2, seed=52, what="config 5 down_proj")
    W, What = wl.make_weights(spec, DEV)
    obj, rows = gq.gq_objective(W, What, H, want_rows=True)
    sampled_objective_check(oracle, X, s, W, What, obj, rows, spec.G, TOL_BF16, rows_per_group=4, seed=53, what="config 5 down_proj")
