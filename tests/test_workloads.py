"""The synthetic input generators: deterministic, right shapes/dtypes, and What lies on
the stated per-row grids."""
import torch

from paper_2505_07004_amd import workloads as wl


def test_configs_cover_the_five_workloads():
    assert {s.cfg for s in wl.CONFIGS.values()} == {1, 2, 3, 4, 5}
    c2 = wl.CONFIGS["llama2_7b_attn"]
    assert (c2.n, c2.d_in, c2.d_out, c2.G, c2.x_dtype) == (65536, 4096, 4096, 4, "bf16")
    c3 = wl.CONFIGS["llama2_7b_down"]
    assert (c3.d_in, c3.chunks) == (11008, 8)


def test_generators_are_seeded_and_shaped():
    spec = wl.scaled(wl.CONFIGS["llama2_7b_attn"], n=256, d_in=512, d_out=128)
    X1, X2 = wl.make_x(spec), wl.make_x(spec)
    assert X1.dtype == torch.bfloat16 and X1.shape == (256, 512) and torch.equal(X1, X2)
    col_rms = X1.float().pow(2).mean(0).sqrt()
    assert int((col_rms > 10).sum()) == 5            # round(1% of 512) outlier columns, x30
    dZ = wl.make_dz_for(spec)
    assert dZ.dtype == torch.float32 and dZ.shape == (256, 128)
    row_rms = dZ.pow(2).mean(1).sqrt()
    assert row_rms.max() / row_rms.min() > 50        # heavy per-token spread
    Xs = wl.make_x(wl.scaled(wl.CONFIGS["llama2_7b_down"], n=128, d_in=64))
    assert Xs.shape == (128, 64) and Xs.float().abs().max() > 1.5


def test_what_lies_on_the_per_row_grids():
    spec = wl.CONFIGS["tiny_f32"]
    W, What = wl.make_weights(spec)
    assert W.shape == (512, 256) and abs(float(W.std()) - 0.02) < 2e-3
    for j in (0, 17, 511):
        assert What[j].unique().numel() <= 16
    assert (W - What).abs().max() <= (W.max(1).values - W.min(1).values).max() / 30 + 1e-7
    spec2 = wl.scaled(wl.CONFIGS["llama2_7b_attn"], d_in=256, d_out=64)
    W2, What2 = wl.make_weights(spec2)
    for j in (0, 63):
        assert What2[j].unique().numel() <= 8
    assert 0 < float((W2 - What2).pow(2).mean()) < float(W2.pow(2).mean()) * 0.1
