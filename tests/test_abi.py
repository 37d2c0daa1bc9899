"""CPU-side checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments on the host before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2505_07004_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "gq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gq_[a-z_]+)\s*\(", text)))


def test_header_declares_the_expected_calls():
    syms = _declared_symbols()
    for name in ("gq_group_weights", "gq_fisher_gram", "gq_objective", "gq_fisher_mirror",
                 "gq_fisher_gram_workspace_bytes", "gq_objective_workspace_bytes",
                 "gq_cd_assign", "gq_cd_workspace_bytes", "gq_group_weights_strided",
                 "gq_lnq_codebook", "gq_lnq_codebook_workspace_bytes", "gq_ldlq_assign", "gq_damp_diagonal", "gq_lnq", "gq_lnq_workspace_bytes", "gq_damped_cholesky", "gq_cholesky_workspace_bytes", "gq_version", "gq_status_string"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    for name in _declared_symbols():
        assert hasattr(lib, name), name
    assert binding.gq_version() >= 100
    assert binding.status_string(0) == "ok"
    assert "shape" in binding.status_string(-2)


def test_host_side_validation_needs_no_gpu():
    lib = binding.load_library()
    P = ctypes.c_void_p
    a16 = P(0x1000)           # fake, aligned, never dereferenced: every call below must fail before launch
    odd = P(0x1004)
    # group weights
    assert lib.gq_group_weights(a16, 7, 4, 8, 8, 2, 1.0, a16, None) == -3          # dtype
    assert lib.gq_group_weights(a16, 0, 4, 10, 10, 4, 1.0, a16, None) == -2         # G does not divide d_out
    assert lib.gq_group_weights(a16, 0, -1, 8, 8, 2, 1.0, a16, None) == -2
    assert lib.gq_group_weights(a16, 0, 4, 8, 4, 2, 1.0, a16, None) == -2           # ld < width
    assert lib.gq_group_weights(None, 0, 4, 8, 8, 2, 1.0, a16, None) == -1
    assert lib.gq_group_weights(odd, 0, 4, 8, 8, 2, 1.0, a16, None) == -4
    assert lib.gq_group_weights(a16, 0, 4, 6, 6, 2, 1.0, a16, None) == -4           # pitch 24 B
    assert lib.gq_group_weights(None, 0, 0, 8, 8, 2, 1.0, None, None) == 0           # n == 0 is a no-op
    # fisher gram
    assert lib.gq_fisher_gram(a16, 5, 4, 8, 8, a16, 2, a16, 0, None, 0, None) == -3
    assert lib.gq_fisher_gram(a16, 1, 4, 0, 8, a16, 2, a16, 0, None, 0, None) == -2
    assert lib.gq_fisher_gram(a16, 1, 4, 8, 4, a16, 2, a16, 0, None, 0, None) == -2
    assert lib.gq_fisher_gram(a16, 1, 4, 8, 8, a16, 0, a16, 0, None, 0, None) == -2
    assert lib.gq_fisher_gram(a16, 1, 4, 8, 8, a16, 2, None, 0, None, 0, None) == -1
    assert lib.gq_fisher_gram(None, 1, 4, 8, 8, a16, 2, a16, 0, None, 0, None) == -1
    assert lib.gq_fisher_gram(odd, 1, 4, 8, 8, a16, 2, a16, 0, None, 0, None) == -4
    assert lib.gq_fisher_gram(a16, 1, 4, 12, 12, a16, 2, a16, 0, None, 0, None) == -4  # bf16 pitch 24 B
    assert lib.gq_fisher_gram(a16, 1, 4, 8, 8, a16, 2, a16, 64, None, 0, None) == -7   # unknown flag
    assert lib.gq_fisher_gram(a16, 1, 4, 8, 8, a16, 2, a16, 4, None, 0, None) == -5    # two terms: a known flag (no workspace given)
    assert lib.gq_group_weights_strided(a16, 0, 4, 8, 8, 2, 1.0, a16, 1, None) == -2      # output pitch smaller than G
    assert lib.gq_group_weights_strided(a16, 0, 0, 8, 8, 2, 1.0, a16, 6, None) == 0       # no tokens: nothing to do
    # mirror
    assert lib.gq_fisher_mirror(None, 8, 2, None) == -1
    assert lib.gq_fisher_mirror(a16, 0, 2, None) == -2
    # objective
    assert lib.gq_objective(a16, a16, 10, 8, 8, a16, 4, a16, None, a16, 1 << 20, None) == -2
    assert lib.gq_objective(a16, None, 8, 8, 8, a16, 4, a16, None, a16, 1 << 20, None) == -1
    assert lib.gq_objective(a16, a16, 8, 8, 8, a16, 4, a16, None, None, 0, None) == -5
    assert lib.gq_objective(a16, a16, 8, 8, 8, a16, 4, a16, None, P(0x1100), 4, None) == -5
    assert lib.gq_objective(a16, a16, 8, 6, 6, a16, 4, a16, None, P(0x1100), 1 << 20, None) == -4
    assert lib.gq_objective_workspace_bytes(8, 8, 4) > 0
    assert lib.gq_objective_workspace_bytes(10, 8, 4) == 0
    # coordinate-descent assignment step
    big = 1 << 30
    assert lib.gq_cd_assign(a16, a16, a16, 8, 10, 8, 8, a16, 4, 1, None, P(0x1100), big, None) == -2     # G does not divide d_out
    assert lib.gq_cd_assign(a16, a16, a16, 0, 8, 8, 8, a16, 4, 1, None, P(0x1100), big, None) == -2      # no grid points
    assert lib.gq_cd_assign(a16, a16, a16, 8, 8, 8, 8, a16, 4, -1, None, P(0x1100), big, None) == -2     # negative cycles
    assert lib.gq_cd_assign(a16, a16, a16, 17, 8, 8, 8, a16, 4, 1, None, P(0x1100), big, None) == -7     # more than 16 grid points
    assert lib.gq_cd_assign(a16, a16, None, 8, 8, 8, 8, a16, 4, 1, None, P(0x1100), big, None) == -1
    assert lib.gq_cd_assign(a16, a16, a16, 8, 8, 6, 6, a16, 4, 1, None, P(0x1100), big, None) == -4      # pitch not a multiple of 16 bytes
    assert lib.gq_cd_assign(a16, a16, a16, 8, 8, 8, 8, a16, 4, 1, None, P(0x1100), 16, None) == -5
    assert lib.gq_cd_assign(a16, a16, a16, 8, 8, 8, 8, a16, 4, 0, None, P(0x1100), big, None) == 0       # zero cycles: nothing to do
    assert lib.gq_cd_workspace_bytes(8, 8, 4) > 0
    assert lib.gq_cd_workspace_bytes(10, 8, 4) == 0
    # damping
    assert lib.gq_damp_diagonal(None, 8, 2, 0.01, 0.0, None) == -1
    assert lib.gq_damp_diagonal(a16, 0, 2, 0.01, 0.0, None) == -2
    assert lib.gq_damp_diagonal(a16, 8, 2, -0.01, 0.0, None) == -2
    # damped Cholesky
    assert lib.gq_damped_cholesky(a16, 0, 4, 0.01, 0.0, 0, P(0x2000), None, P(0x1100), big, None) == -2       # no coordinates
    assert lib.gq_damped_cholesky(a16, 8, 4, -0.01, 0.0, 0, P(0x2000), None, P(0x1100), big, None) == -2      # negative damping
    assert lib.gq_damped_cholesky(a16, 8, 4, 0.01, float("nan"), 0, P(0x2000), None, P(0x1100), big, None) == -2
    assert lib.gq_damped_cholesky(a16, 8, 4, 0.01, 0.0, 0, a16, None, P(0x1100), big, None) == -2             # in place
    assert lib.gq_damped_cholesky(a16, 8, 4, 0.01, 0.0, 2, P(0x2000), None, P(0x1100), big, None) == -7       # unknown flag
    assert lib.gq_damped_cholesky(a16, 8, 4, 0.01, 0.0, 1, None, None, P(0x1100), big, None) == -1
    assert lib.gq_damped_cholesky(odd, 8, 4, 0.01, 0.0, 1, P(0x2000), None, P(0x1100), big, None) == -4
    assert lib.gq_damped_cholesky(a16, 8, 4, 0.01, 0.0, 1, P(0x2000), None, P(0x1100), 16, None) == -5
    assert lib.gq_cholesky_workspace_bytes(8, 4) >= 4 * 8 * 8 * 4
    assert lib.gq_cholesky_workspace_bytes(0, 4) == 0
    # sequential rounding
    assert lib.gq_ldlq_assign(a16, P(0x2000), a16, 8, 10, 8, 8, a16, 4, None, P(0x1100), big, None) == -2   # G does not divide d_out
    assert lib.gq_ldlq_assign(a16, a16, a16, 8, 8, 8, 8, a16, 4, None, P(0x1100), big, None) == -2          # What == W
    assert lib.gq_ldlq_assign(a16, P(0x2000), a16, 17, 8, 8, 8, a16, 4, None, P(0x1100), big, None) == -7
    assert lib.gq_ldlq_assign(a16, P(0x2000), a16, 8, 8, 8, 8, None, 4, None, P(0x1100), big, None) == -1   # no factor
    assert lib.gq_ldlq_assign(a16, P(0x2004), a16, 8, 8, 8, 8, a16, 4, None, P(0x1100), big, None) == -4
    assert lib.gq_ldlq_assign(a16, P(0x2000), a16, 8, 8, 8, 8, a16, 4, None, P(0x1100), 16, None) == -5
    # the whole alternation
    assert lib.gq_lnq(a16, P(0x2000), a16, a16, 8, 10, 8, 8, a16, 4, 2, 4, 1e-7, P(0x1100), big, None) == -2         # G does not divide d_out
    assert lib.gq_lnq(a16, P(0x2000), a16, a16, 8, 8, 8, 8, a16, 4, -1, 4, 1e-7, P(0x1100), big, None) == -2         # negative iteration count
    assert lib.gq_lnq(a16, a16, a16, a16, 8, 8, 8, 8, a16, 4, 2, 4, 1e-7, P(0x1100), big, None) == -2                # What == W
    assert lib.gq_lnq(a16, P(0x2000), None, a16, 8, 8, 8, 8, a16, 4, 2, 4, 1e-7, P(0x1100), big, None) == -1         # no assignments
    assert lib.gq_lnq(a16, P(0x2000), a16, a16, 17, 8, 8, 8, a16, 4, 2, 4, 1e-7, P(0x1100), big, None) == -7
    assert lib.gq_lnq(a16, P(0x2000), a16, a16, 8, 8, 8, 8, a16, 4, 2, 4, 1e-7, P(0x1100), 16, None) == -5
    assert lib.gq_lnq_workspace_bytes(8, 8, 4, 8) >= lib.gq_cd_workspace_bytes(8, 8, 4)
    # schedule tuning of the Gram kernel: argument checks come before any HIP call
    bad = (ctypes.c_float * 8)(1, 1, 1, 1, 1, 1, 1, 3.0)
    assert lib.gq_fisher_gram_set_xcd_speeds(ctypes.cast(bad, ctypes.c_void_p)) == -2
    assert lib.gq_fisher_gram_measured_xcd_speeds(1024, 4096, 4, None, ctypes.cast(bad, ctypes.c_void_p)) == -1
    assert lib.gq_fisher_gram_measured_xcd_speeds(0, 4096, 4, a16, ctypes.cast(bad, ctypes.c_void_p)) == -2
    # heavy-token rows gathered over chunk calls: the pool and its two calls
    w256 = P(0x1100)
    assert lib.gq_fisher_gram_heavy_pool_bytes(4096, 4, 1024) == 256 + 1024 * 4 * 4 + 1024 * 4096 * 2
    assert lib.gq_fisher_gram_heavy_pool_bytes(4096, 4, 100) == 0                       # not a multiple of 32
    assert lib.gq_fisher_gram_heavy_pool_bytes(4096, 4, 0) == 0
    defer = lambda **kw: lib.gq_fisher_gram_heavy_deferred(
        kw.get("X", a16), kw.get("dt", 1), kw.get("n", 64), 64, kw.get("ld", 64), a16, 4, kw.get("H", a16),
        kw.get("flags", 0), w256, big, kw.get("pool", P(0x2000)), kw.get("rows", 64), None)
    assert defer(rows=48) == -2                                                         # pool_rows not a multiple of 32
    assert defer(dt=0) == -7                                                            # fp32 X: no heavy-token mode
    assert defer(flags=2) == -7                                                         # GQ_MIRROR belongs to the flush
    assert defer(pool=None) == -1
    assert defer(pool=P(0x2010)) == -4                                                  # pool not 256-byte aligned
    assert defer(ld=60) == -2
    assert lib.gq_fisher_gram_heavy_flush(P(0x2000), 64, 64, 4, a16, 1, w256, big, None) == -7    # only GQ_MIRROR
    assert lib.gq_fisher_gram_heavy_flush(P(0x2000), 40, 64, 4, a16, 0, w256, big, None) == -2
    assert lib.gq_fisher_gram_heavy_flush(P(0x2000), 64, 64, 4, None, 0, w256, big, None) == -1
    assert lib.gq_fisher_gram_heavy_flush(P(0x2000), 64, 64, 4, a16, 0, w256, 16, None) == -5     # workspace too small
    # codebook step
    lam = 1e-7
    # no [d_out * m, d_in] intermediate and no full copy of H in three terms: the 70B down projection stays under 1 GiB
    assert 0 < lib.gq_lnq_codebook_workspace_bytes(8192, 28672, 4, 8) < (1 << 30)
    assert 0 < lib.gq_lnq_codebook_workspace_bytes(8192, 28672, 4, 16) < (1 << 30)
    assert lib.gq_lnq_codebook(a16, 10, 8, 8, a16, a16, 4, 4, lam, a16, None, P(0x1100), big, None) == -2   # G does not divide d_out
    assert lib.gq_lnq_codebook(a16, 8, 8, 4, a16, a16, 4, 4, lam, a16, None, P(0x1100), big, None) == -2    # pitch < width
    assert lib.gq_lnq_codebook(a16, 8, 8, 8, a16, a16, 4, 0, lam, a16, None, P(0x1100), big, None) == -2    # no grid points
    assert lib.gq_lnq_codebook(a16, 8, 8, 8, a16, a16, 4, 4, -1.0, a16, None, P(0x1100), big, None) == -2   # negative damping
    assert lib.gq_lnq_codebook(a16, 8, 8, 8, a16, a16, 4, 4, float("nan"), a16, None, P(0x1100), big, None) == -2
    assert lib.gq_lnq_codebook(a16, 8, 8, 8, a16, a16, 4, 17, lam, a16, None, P(0x1100), big, None) == -7   # more than 16 grid points
    assert lib.gq_lnq_codebook(a16, 8, 8, 8, None, a16, 4, 4, lam, a16, None, P(0x1100), big, None) == -1   # no assignments
    assert lib.gq_lnq_codebook(a16, 8, 8, 8, a16, a16, 4, 4, lam, None, None, P(0x1100), big, None) == -1   # no output
    assert lib.gq_lnq_codebook(a16, 8, 8, 8, a16, a16, 4, 4, lam, a16, odd, P(0x1100), big, None) == -4
    assert lib.gq_lnq_codebook(a16, 8, 6, 6, a16, a16, 4, 4, lam, a16, None, P(0x1100), big, None) == -4    # pitch 24 B
    assert lib.gq_lnq_codebook(a16, 8, 8, 8, a16, a16, 4, 4, lam, a16, None, P(0x1100), 16, None) == -5
    assert lib.gq_lnq_codebook_workspace_bytes(8, 8, 4, 4) > 0
    assert lib.gq_lnq_codebook_workspace_bytes(8, 8, 4, 17) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(RuntimeError):
        binding.gq_group_weights(torch.zeros(4, 8), 2)
