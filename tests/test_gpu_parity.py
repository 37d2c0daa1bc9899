"""Parity of the HIP path (through the C ABI) against the fp64 CPU oracle, element by
element, on seeded inputs small enough for the oracle to finish in seconds."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_07004_amd import binding as gq
from paper_2505_07004_amd import workloads as wl
from parity_utils import TOL_BF16, TOL_F32, TOL_S, rel_fro, say, to_np64

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _pitched(t: torch.Tensor, ld: int) -> torch.Tensor:
    """Same values in a buffer whose row pitch is ld elements; the padding holds NaN (it is not the library's
    to read into a result, nor to write)."""
    buf = torch.full((t.shape[0], ld), float("nan"), dtype=t.dtype, device=t.device)
    buf[:, : t.shape[1]] = t
    return buf[:, : t.shape[1]]


# ------------------------------------------------------------------ group weights
@pytest.mark.parametrize("n,d_out,G,scale,dtype,ld", [
    (2048, 512, 2, 1.0, torch.float32, None),       # config 1
    (333, 4096, 4, 1e3, torch.float32, None),       # Llama width, paper's gradient scale
    (100, 24, 3, 1.0, torch.float32, None),         # m = 8
    (77, 20, 4, 2.0, torch.float32, None),          # m = 5: scalar path
    (50, 12, 12, 1.0, torch.float32, None),         # one channel per group
    (65, 640, 1, 1.0, torch.float32, 648),          # padded pitch
    (129, 1024, 8, 1.0, torch.bfloat16, None),      # bf16 gradients
    (31, 40, 2, 1.0, torch.bfloat16, None),         # bf16, m = 20: scalar path
])
def test_group_weights(n, d_out, G, scale, dtype, ld):
    say(f"group_weights n={n} d_out={d_out} G={G} scale={scale} {dtype} ld={ld}")
    dZ = wl.make_dz(n, d_out, 1.0, 1.0, seed=11 + n, device=DEV).to(dtype)
    if ld:
        dZ = _pitched(dZ, ld)
    s = gq.gq_group_weights(dZ, G, grad_scale=scale)
    torch.cuda.synchronize()
    ref = oracle.group_weights(to_np64(dZ), G, grad_scale=scale)
    got = to_np64(s)
    assert got.shape == ref.shape
    assert np.all(np.abs(got - ref) <= TOL_S * np.abs(ref) + 1e-300)


def test_group_weights_empty():
    s = gq.gq_group_weights(torch.empty((0, 16), device=DEV), 4)
    assert tuple(s.shape) == (0, 4)


# ------------------------------------------------------------------ fisher gram
def _gram_case(n, d_in, G, dtype, seed, ld=None, kind="outlier"):
    if kind == "outlier":
        X = wl.make_x_outlier(n, d_in, max(1, d_in // 64), 20.0, seed, DEV, dtype)
    else:
        X = wl.make_x_silu(n, d_in, seed, DEV, dtype)
    if ld:
        X = _pitched(X, ld)
    dZ = wl.make_dz(n, 8 * G, 1.0, 1.5, seed + 1, DEV)
    s = gq.gq_group_weights(dZ, G)
    return X, s


def _check_gram(H, X, s, tol, what):
    torch.cuda.synchronize()
    ref = oracle.fisher_gram(to_np64(X), to_np64(s))
    got = to_np64(H)
    errs = [rel_fro(np.triu(got[k]), np.triu(ref[k])) for k in range(ref.shape[0])]
    say(f"{what}: rel-Frobenius per group {['%.2e' % e for e in errs]} (tol {tol:g})")
    assert max(errs) <= tol
    return ref


def test_gram_f32_config1_full():
    spec = wl.CONFIGS["tiny_f32"]
    X, dZ = wl.make_x(spec, DEV), wl.make_dz_for(spec, DEV)
    s = gq.gq_group_weights(dZ, spec.G)
    H = gq.gq_fisher_gram(X, s, mirror=True)
    ref = _check_gram(H, X, s, TOL_F32, "config 1 fp32")
    got = to_np64(H)
    assert np.array_equal(got, np.transpose(got, (0, 2, 1)))        # bit-exact symmetry after mirror
    assert max(rel_fro(got[k], ref[k]) for k in range(spec.G)) <= TOL_F32
    for k in range(spec.G):
        ev = np.linalg.eigvalsh(got[k])
        assert ev.min() >= -1e-5 * ev.max()


@pytest.mark.parametrize("n,d_in,G,ld", [
    (1000, 200, 2, None),      # ragged tokens and columns, several tiles
    (1, 128, 1, None),         # single token
    (517, 130, 3, 132),        # padded pitch, odd group count
    (4100, 64, 4, None),       # crosses the accumulator flush boundary
    (40, 7, 2, 8),             # d_in not a multiple of the vector width
])
def test_gram_f32_shapes(n, d_in, G, ld):
    say(f"gram f32 n={n} d_in={d_in} G={G} ld={ld}")
    X, s = _gram_case(n, d_in, G, torch.float32, 100 + n, ld)
    H = gq.gq_fisher_gram(X, s)
    _check_gram(H, X, s, TOL_F32, f"fp32 n={n} d_in={d_in}")


@pytest.mark.parametrize("dtype,tol", [(torch.float32, TOL_F32), (torch.bfloat16, TOL_BF16)])
def test_gram_lower_triangle_untouched_without_mirror_and_zero_tokens(dtype, tol):
    X, s = _gram_case(300, 136, 2, dtype, 7)
    H = torch.full((2, 136, 136), 777.0, device=DEV)
    gq.gq_fisher_gram(X, s, H=H)
    torch.cuda.synchronize()
    got = to_np64(H)
    il = np.tril_indices(136, -1)
    for k in range(2):
        assert np.all(got[k][il] == 777.0)
    # n == 0: overwrite clears the upper triangle, accumulate leaves H alone
    H2 = torch.full((2, 136, 136), 5.0, device=DEV)
    gq.gq_fisher_gram(X[:0], s[:0], H=H2, accumulate=True)
    torch.cuda.synchronize()
    assert bool((H2 == 5.0).all())
    gq.gq_fisher_gram(X[:0], s[:0], H=H2)
    torch.cuda.synchronize()
    g2 = to_np64(H2)
    assert np.all(np.triu(g2[0]) == 0) and np.all(g2[0][il] == 5.0)


@pytest.mark.parametrize("dtype,tol", [(torch.float32, TOL_F32), (torch.bfloat16, TOL_BF16)])
def test_gram_chunk_accumulation(dtype, tol):
    X, s = _gram_case(3000, 264, 4, dtype, 21)
    H = None
    for c0 in range(0, 3000, 1000):
        H = gq.gq_fisher_gram(X[c0:c0 + 1000], s[c0:c0 + 1000], H=H, accumulate=c0 > 0)
    gq.gq_fisher_mirror(H)
    ref = _check_gram(H, X, s, tol, f"3 chunks {dtype}")
    got = to_np64(H)
    assert np.array_equal(got, np.transpose(got, (0, 2, 1)))
    one = to_np64(gq.gq_fisher_gram(X, s, mirror=True))
    assert max(rel_fro(got[k], one[k]) for k in range(4)) <= 1e-5   # only fp32 re-association differs
    assert max(rel_fro(got[k], ref[k]) for k in range(4)) <= tol


def test_gram_bf16_config1_values():
    spec = wl.CONFIGS["tiny_f32"]
    X = wl.make_x(spec, DEV).to(torch.bfloat16)
    s = gq.gq_group_weights(wl.make_dz_for(spec, DEV), spec.G)
    H = gq.gq_fisher_gram(X, s)
    _check_gram(H, X, s, TOL_BF16, "config 1 values, bf16 path")


@pytest.mark.parametrize("n,d_in,G,ld,kind", [
    (4096, 512, 4, None, "outlier"),   # several tiles, group-fused workgroups
    (4096, 512, 1, None, "outlier"),   # one group: 256x256 tiles
    (2048, 768, 2, None, "silu"),      # two groups
    (1500, 520, 8, None, "outlier"),   # two group sets, ragged tokens, ragged column tile
    (1000, 328, 3, None, "silu"),      # odd group count
    (700, 300, 4, 304, "outlier"),     # d_in not a multiple of 8, padded pitch
    (33, 72, 2, None, "outlier"),      # barely more than one token step
    (5, 16, 4, None, "outlier"),       # tiny
    (1999, 1160, 6, 1168, "outlier"),  # even group count, too few items for two row blocks per workgroup
    (3207, 1896, 4, None, "outlier"),  # 97 items on 256 workgroups: three token segments per item, 35 units in runs
    (6001, 1000, 8, 1008, "silu"),     # 56 items: five segments, ragged last token step, 24 units in runs
    (3207, 3584, 1, None, "outlier"),  # one group, 105 items of 256 x 256: three token segments (34, 34, 33 steps)
    (1000, 328, 5, None, "silu"),      # odd group count: four groups on the wide kernel, the fifth on the narrow one
    (2100, 520, 9, 528, "outlier"),    # eight + one, ragged, padded pitch
    (288, 4864, 3, None, "outlier"),   # three groups: two on two row blocks (260 items), the third on the narrow kernel
    (3207, 2304, 2, 2312, "silu"),     # two groups, 99 items of 128 x 256: the same on the other tile shape
    (640, 2304, 2, None, "outlier"),   # the same with more items
])
def test_gram_bf16_shapes(n, d_in, G, ld, kind):
    say(f"gram bf16 n={n} d_in={d_in} G={G} ld={ld} {kind}")
    X, s = _gram_case(n, d_in, G, torch.bfloat16, 300 + n, ld, kind)
    H = gq.gq_fisher_gram(X, s)
    _check_gram(H, X, s, TOL_BF16, f"bf16 n={n} d_in={d_in} G={G}")


def _two_row_block_kernel_ran(X, s, **kw):
    """Runs the Gram call in a workspace of the test's own; the kernel that puts two groups on two row blocks
    per workgroup leaves the timing records that the measured XCD speeds are read from, the others do not."""
    n, d_in = X.shape
    G = int(s.shape[1])
    assert G % 2 == 0 and G % 4 != 0
    ws = torch.empty(gq.gq_fisher_gram_workspace_bytes(X.dtype, n, d_in, G), dtype=torch.uint8, device=DEV)
    H = gq.gq_fisher_gram(X, s, workspace=ws, **kw)
    speeds = gq.gq_fisher_gram_measured_xcd_speeds(n, d_in, G, ws)      # raises if that kernel did not run
    assert len(speeds) == 8
    return H


@pytest.mark.parametrize("n,d_in,G,ld,kind", [
    (1999, 1160, 26, 1168, "outlier"),  # 13 sets of two groups, 286 items: one round and left-over runs; ragged, padded pitch
    (1100, 200, 258, None, "silu"),     # a single tile column, 192 rows do not divide 200; 258 items on 256 workgroups
    (1000, 2304, 10, None, "outlier"),  # 315 items, staircase of the tile columns
    (3207, 3072, 2, None, "outlier"),   # 108 items: three token segments per item make 324 units
])
def test_gram_bf16_two_groups_on_two_row_blocks_shapes(n, d_in, G, ld, kind):
    say(f"gram bf16, two row blocks n={n} d_in={d_in} G={G} ld={ld} {kind}")
    X, s = _gram_case(n, d_in, G, torch.bfloat16, 400 + n, ld, kind)
    H = _two_row_block_kernel_ran(X, s)
    _check_gram(H, X, s, TOL_BF16, f"bf16 n={n} d_in={d_in} G={G}")


def test_gram_bf16_two_groups_accumulate_over_chunks_mirror_and_repeat_bit_for_bit():
    """Even group counts not divisible by four: two groups on two row blocks per workgroup."""
    G = 38                                                                # 15 items per set of two groups: 285 items
    X, s = _gram_case(1300, 1000, G, torch.bfloat16, 91)
    H = None
    for c0 in range(0, 1300, 650):
        H = gq.gq_fisher_gram(X[c0:c0 + 650], s[c0:c0 + 650], H=H, accumulate=c0 > 0, mirror=c0 > 0)
    ref = _check_gram(H, X, s, TOL_BF16, "2 chunks, two groups per workgroup")
    got = to_np64(H)
    assert np.array_equal(got, np.transpose(got, (0, 2, 1)))
    assert max(rel_fro(got[k], ref[k]) for k in range(G)) <= TOL_BF16
    a = _two_row_block_kernel_ran(X, s).clone()
    b = gq.gq_fisher_gram(X, s)
    torch.cuda.synchronize()
    assert torch.equal(torch.triu(a), torch.triu(b))


def test_gram_bf16_token_segments_accumulate_mirror_and_repeat_bit_for_bit():
    """Fewer work items than workgroups: every item is written by the second pass from parked segments and runs;
    accumulating calls add to H there, and the order of the parts is fixed."""
    n, d_in, G = 6414, 1896, 4                        # two chunks of 3207 tokens: 97 items in three segments each
    X, s = _gram_case(n, d_in, G, torch.bfloat16, 93)
    H = None
    for c0 in range(0, n, 3207):
        H = gq.gq_fisher_gram(X[c0:c0 + 3207], s[c0:c0 + 3207], H=H, accumulate=c0 > 0, mirror=c0 > 0)
    ref = _check_gram(H, X, s, TOL_BF16, "2 chunks, token segments")
    got = to_np64(H)
    assert np.array_equal(got, np.transpose(got, (0, 2, 1)))
    assert max(rel_fro(got[k], ref[k]) for k in range(G)) <= TOL_BF16
    a = gq.gq_fisher_gram(X[:3207], s[:3207]).clone()
    b = gq.gq_fisher_gram(X[:3207], s[:3207])
    torch.cuda.synchronize()
    assert torch.equal(torch.triu(a), torch.triu(b))


def test_gram_bf16_one_group_token_segments_accumulate_and_repeat_bit_for_bit():
    n, d_in, G = 6414, 3584, 1                        # two chunks of 3207 tokens: 105 items in three segments each
    X, s = _gram_case(n, d_in, G, torch.bfloat16, 95)
    H = None
    for c0 in range(0, n, 3207):
        H = gq.gq_fisher_gram(X[c0:c0 + 3207], s[c0:c0 + 3207], H=H, accumulate=c0 > 0, mirror=c0 > 0)
    ref = _check_gram(H, X, s, TOL_BF16, "2 chunks, one group, token segments")
    got = to_np64(H)
    assert np.array_equal(got, np.transpose(got, (0, 2, 1)))
    assert rel_fro(got[0], ref[0]) <= TOL_BF16
    a = gq.gq_fisher_gram(X[:3207], s[:3207]).clone()
    b = gq.gq_fisher_gram(X[:3207], s[:3207])
    torch.cuda.synchronize()
    assert torch.equal(torch.triu(a), torch.triu(b))


def _random_gram_shapes(count, seed):
    """Seeded shapes over all the tilings of the bf16 Gram call: group counts 1..12, ragged everything, token counts
    on both sides of what token segments need; sized so that the fp64 oracle stays under a second per shape."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        G = int(rng.choice([1, 1, 2, 2, 3, 4, 4, 6, 8, 10, 12]))
        d_in = int(rng.integers(2, 330)) * 8
        n = int(rng.integers(1, 5200))
        if n * d_in * d_in * G > 3e10:
            continue
        out.append((n, d_in, G, d_in + 8 * int(rng.integers(0, 3)), bool(rng.integers(0, 2)), bool(rng.integers(0, 3) == 0)))
    return out


@pytest.mark.parametrize("n,d_in,G,ld,chunked,heavy", _random_gram_shapes(24, 250507004))
def test_gram_bf16_random_shapes(n, d_in, G, ld, chunked, heavy):
    say(f"gram bf16 random shape n={n} d_in={d_in} G={G} ld={ld} chunked={chunked} heavy={heavy}")
    X, s = _gram_case(n, d_in, G, torch.bfloat16, 7000 + n + d_in, ld if ld != d_in else None, "outlier")
    if chunked and n >= 2:
        cut = n // 2 + 1
        H = gq.gq_fisher_gram(X[:cut], s[:cut], heavy_two_terms=heavy)
        H = gq.gq_fisher_gram(X[cut:], s[cut:], H=H, accumulate=True, heavy_two_terms=heavy)
    else:
        H = gq.gq_fisher_gram(X, s, heavy_two_terms=heavy)
    _check_gram(H, X, s, TOL_BF16, f"random shape n={n} d_in={d_in} G={G}")


def test_gram_bf16_odd_group_count_in_two_parts_accumulates_and_equals_separate_calls():
    """Five groups run as four (wide kernel) + one (narrow kernel): the same bits as those two calls made by hand."""
    n, d_in, G = 1500, 520, 5
    X, s = _gram_case(n, d_in, G, torch.bfloat16, 97)
    H = None
    for c0 in range(0, n, 750):
        H = gq.gq_fisher_gram(X[c0:c0 + 750], s[c0:c0 + 750], H=H, accumulate=c0 > 0, mirror=c0 > 0)
    _check_gram(H, X, s, TOL_BF16, "2 chunks, five groups")
    got = to_np64(H)
    assert np.array_equal(got, np.transpose(got, (0, 2, 1)))
    whole = gq.gq_fisher_gram(X, s)
    four = gq.gq_fisher_gram(X, s[:, :4].contiguous())
    last = gq.gq_fisher_gram(X, s[:, 4:].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(torch.triu(whole[:4]), torch.triu(four)) and torch.equal(torch.triu(whole[4:]), torch.triu(last))


def test_gram_bf16_matches_its_documented_rounding():
    """The bf16 path rounds exactly one operand, bf16_rne(fp32(s)*fp32(x)); with that
    operand reproduced on the host the remaining difference is fp32 accumulation only."""
    n, d_in, G = 2048, 384, 4
    X, s = _gram_case(n, d_in, G, torch.bfloat16, 55)
    H = to_np64(gq.gq_fisher_gram(X, s))
    Xc, sc = X.float().cpu(), s.cpu()
    X64 = Xc.double().numpy()
    for k in range(G):
        A = (sc[:, k:k + 1] * Xc).to(torch.bfloat16).double().numpy()
        ref = A.T @ X64
        err = rel_fro(np.triu(H[k]), np.triu(ref))
        say(f"group {k}: vs rounded-operand model {err:.2e}")
        assert err <= 2e-6


TOL_TWO_TERMS = 2e-5     # two bf16 terms carry s*x to 2^-17 (random sign: ~3e-6 on the sum); fp32 accumulation adds ~1e-5 at most


@pytest.mark.parametrize("n,d_in,G,ld,kind", [
    (4096, 512, 4, None, "outlier"),
    (4096, 512, 1, None, "outlier"),
    (2048, 768, 2, None, "silu"),
    (1500, 520, 8, None, "outlier"),
    (1000, 328, 3, None, "silu"),
    (700, 300, 4, 304, "outlier"),
    (5, 16, 4, None, "outlier"),
    (3207, 3584, 1, None, "outlier"),  # 105 items on 256 workgroups: three token segments per item
])
def test_gram_bf16_two_terms_shapes(n, d_in, G, ld, kind):
    say(f"gram bf16, two terms n={n} d_in={d_in} G={G} ld={ld} {kind}")
    X, s = _gram_case(n, d_in, G, torch.bfloat16, 300 + n, ld, kind)
    H = gq.gq_fisher_gram(X, s, two_terms=True)
    _check_gram(H, X, s, TOL_TWO_TERMS, f"bf16 two terms n={n} d_in={d_in} G={G}")


def test_gram_bf16_two_terms_accumulates_over_chunks_and_is_positive_semidefinite_where_one_term_is_not():
    X, s = _gram_case(3000, 264, 4, torch.bfloat16, 21)
    H = None
    for c0 in range(0, 3000, 1000):
        H = gq.gq_fisher_gram(X[c0:c0 + 1000], s[c0:c0 + 1000], H=H, accumulate=c0 > 0, two_terms=True)
    gq.gq_fisher_mirror(H)
    _check_gram(H, X, s, TOL_TWO_TERMS, "3 chunks, two terms")
    # rank-deficient on purpose (fewer tokens than columns): the exact matrix has 64 zero eigenvalues, and the
    # rounding of the one-term path pushes some of them well below zero
    Xs, ss = X[:200], s[:200]
    H1 = to_np64(gq.gq_fisher_gram(Xs, ss, mirror=True))
    H2 = to_np64(gq.gq_fisher_gram(Xs, ss, mirror=True, two_terms=True))
    for k in range(4):
        e1, e2 = np.linalg.eigvalsh(H1[k]), np.linalg.eigvalsh(H2[k])
        say(f"group {k}: smallest eigenvalue / largest: one term {e1[0] / e1[-1]:.2e}, two terms {e2[0] / e2[-1]:.2e}")
        assert e2[0] >= -2e-6 * e2[-1]
        assert e1[0] < 10 * e2[0] or e1[0] >= -2e-6 * e1[-1]


def test_gram_is_deterministic():
    X, s = _gram_case(2048, 512, 4, torch.bfloat16, 77)
    a = gq.gq_fisher_gram(X, s, mirror=True).clone()
    b = gq.gq_fisher_gram(X, s, mirror=True)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


# ------------------------------------------------------------------ objective
def _check_objective(W, What, H_gpu, H_ref64, G, tol, what):
    obj, rows = gq.gq_objective(W, What, H_gpu, want_rows=True)
    torch.cuda.synchronize()
    ref, ref_rows = oracle.objective(to_np64(W), to_np64(What), H_ref64, G)
    e_obj = np.max(np.abs(to_np64(obj) - ref) / ref)
    e_rows = rel_fro(to_np64(rows), ref_rows)
    say(f"{what}: obj rel err {e_obj:.2e}, per-channel rel-Frobenius {e_rows:.2e} (tol {tol:g})")
    assert e_obj <= tol and e_rows <= tol


def test_objective_config1_isolated_and_end_to_end():
    spec = wl.CONFIGS["tiny_f32"]
    X, dZ = wl.make_x(spec, DEV), wl.make_dz_for(spec, DEV)
    W, What = wl.make_weights(spec, DEV)
    s = gq.gq_group_weights(dZ, spec.G)
    H = gq.gq_fisher_gram(X, s)                       # upper triangle only: lower stays garbage
    H_ref = oracle.fisher_gram(to_np64(X), oracle.group_weights(to_np64(dZ), spec.G))
    # isolation: both sides read the same fp32 H (the oracle sees its symmetric completion)
    Hg = to_np64(H)
    Hsym = np.stack([np.triu(Hg[k]) + np.triu(Hg[k], 1).T for k in range(spec.G)])
    _check_objective(W, What, H, Hsym, spec.G, TOL_F32, "config 1 objective, isolated")
    _check_objective(W, What, H, H_ref, spec.G, TOL_F32, "config 1 objective, end to end fp32")
    Hb = gq.gq_fisher_gram(X.to(torch.bfloat16), s)
    Hb_ref = oracle.fisher_gram(to_np64(X.to(torch.bfloat16)), to_np64(s))
    _check_objective(W, What, Hb, Hb_ref, spec.G, TOL_BF16, "config 1 values, objective on the bf16-path H")


@pytest.mark.parametrize("d_out,d_in,G,ld", [
    (300, 200, 3, None),     # m = 100 < row tile, ragged column tile
    (512, 384, 1, None),     # one group, several row blocks
    (64, 520, 8, 528),       # m = 8, padded pitch
    (12, 6, 2, 8),           # tiny, d_in not a multiple of 4
])
def test_objective_shapes(d_out, d_in, G, ld):
    say(f"objective d_out={d_out} d_in={d_in} G={G} ld={ld}")
    X, s = _gram_case(600, d_in, G, torch.float32, 900 + d_in, ld if d_in % 4 else None)
    H = gq.gq_fisher_gram(X, s, mirror=True)
    W = wl.make_w(d_out, d_in, 5, DEV)
    What = wl.quantize_uniform_per_row(W, 8)
    if ld:
        W, What = _pitched(W, ld), _pitched(What, ld)
    _check_objective(W, What, H, to_np64(H), G, TOL_F32, f"objective {d_out}x{d_in} G={G}")


def test_objective_zero_when_nothing_changed():
    X, s = _gram_case(256, 128, 2, torch.float32, 3)
    H = gq.gq_fisher_gram(X, s)
    W = wl.make_w(64, 128, 9, DEV)
    obj = gq.gq_objective(W, W.clone(), H)
    torch.cuda.synchronize()
    assert bool((obj == 0).all())


# ------------------------------------------------------------------ layers that share X
def test_stacked_group_weights_and_one_gram_call_for_three_layers():
    n, d_in = 700, 320
    X = wl.make_x_outlier(n, d_in, 5, 20.0, 91, DEV, torch.bfloat16)
    layers = [(wl.make_dz(n, 96, 1.0, 1.5, 92, DEV), 4), (wl.make_dz(n, 64, 1.0, 1.5, 93, DEV).to(torch.bfloat16), 2),
              (wl.make_dz(n, 40, 1.0, 1.5, 94, DEV), 1)]
    G_total = sum(G for _, G in layers)
    s_all = torch.full((n, G_total), float("nan"), device=DEV)
    col = 0
    for dZ, G in layers:
        gq.gq_group_weights(dZ, G, out=s_all, out_col=col)
        assert torch.equal(s_all[:, col:col + G], gq.gq_group_weights(dZ, G))      # same kernel, same order: bit-identical
        col += G
    assert not torch.isnan(s_all).any()
    H = gq.gq_fisher_gram(X, s_all, mirror=True)
    torch.cuda.synchronize()
    X64 = to_np64(X)
    col = 0
    for dZ, G in layers:
        ref = oracle.fisher_gram(X64, oracle.group_weights(to_np64(dZ), G))
        for k in range(G):
            err = rel_fro(to_np64(H[col + k]), ref[k])
            say(f"stacked layers: H[{col + k}] rel-Frobenius {err:.2e}")
            assert err <= TOL_BF16
        col += G
