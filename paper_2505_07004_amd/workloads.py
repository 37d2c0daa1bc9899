"""Seeded synthetic inputs with the shapes and value structure of the paper's
workloads (Llama-2 linear layers on calibration tokens).

This module only draws random tensors and builds test weights; it contains none
of the method's arithmetic (no squared-gradient averaging, no Gram, no
objective).  Both the HIP path and the CPU checker are fed from here, so that
they always read identical bits.

Conventions: the second parameter of N(., .) and LogNormal(., .) is a standard
deviation; LogNormal(mu, sigma) = exp(mu + sigma * z) multiplies rows of dZ.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import torch

BASE_SEED = 250507004


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, seed, device, chunk_rows: int = 8192) -> torch.Tensor:
    """Standard normal fp32 tensor, drawn in row chunks to bound temporaries."""
    g = _gen(seed, device)
    out = torch.empty(shape, dtype=torch.float32, device=device)
    n = shape[0]
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        out[r0:r1] = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=g,
                                 dtype=torch.float32, device=device)
    return out


def make_x_outlier(n: int, d_in: int, n_outlier_cols: int, outlier_scale: float,
                   seed: int, device="cpu", dtype=torch.float32) -> torch.Tensor:
    """X ~ N(0,1) with `n_outlier_cols` randomly chosen columns multiplied by
    `outlier_scale` (activation outlier channels), cast to `dtype` (RNE)."""
    X = _randn((n, d_in), seed, device)
    g = _gen(seed + 500, "cpu")
    cols = torch.randperm(d_in, generator=g)[:n_outlier_cols].to(device)
    X[:, cols] *= outlier_scale
    return X.to(dtype).contiguous()


def make_x_silu(n: int, d_in: int, seed: int, device="cpu",
                dtype=torch.float32) -> torch.Tensor:
    """Heavy-tailed gated activations a * SiLU(b), a, b ~ N(0,1) (the input of a
    Llama MLP down projection)."""
    a = _randn((n, d_in), seed, device)
    b = _randn((n, d_in), seed + 250, device)
    a.mul_(torch.nn.functional.silu(b))
    del b
    return a.to(dtype).contiguous()


def make_dz(n: int, d_out: int, base_std: float, lognormal_sigma: float,
            seed: int, device="cpu") -> torch.Tensor:
    """dZ[i, :] = base_std * N(0,1) * exp(lognormal_sigma * z_i): fp32 output
    gradients whose magnitude varies strongly from token to token."""
    dZ = _randn((n, d_out), seed, device)
    g = _gen(seed + 500, device)
    z = torch.randn((n, 1), generator=g, dtype=torch.float32, device=device)
    dZ.mul_(base_std * torch.exp(lognormal_sigma * z))
    return dZ.contiguous()


def make_w(d_out: int, d_in: int, seed: int, device="cpu", std: float = 0.02) -> torch.Tensor:
    """W[d_out, d_in] ~ N(0, std): row j holds output channel j."""
    return (_randn((d_out, d_in), seed, device) * std).contiguous()


def quantize_uniform_per_row(W: torch.Tensor, levels: int = 16) -> torch.Tensor:
    """Round every row of W to its own uniform grid of `levels` points spanning
    [row min, row max] (round-to-nearest)."""
    lo = W.min(dim=1, keepdim=True).values
    hi = W.max(dim=1, keepdim=True).values
    step = (hi - lo) / (levels - 1)
    step = torch.where(step > 0, step, torch.ones_like(step))
    q = torch.round((W - lo) / step)
    return (lo + q * step).to(torch.float32).contiguous()


def quantize_codebook_per_row(W: torch.Tensor, bits: int = 3, iters: int = 5, return_codebook: bool = False):
    """Assign every entry of a row to the nearest of 2**bits per-row codebook
    values: codebook initialised at the (2q+1)/2^(bits+1) quantiles of the row
    and refined by `iters` unweighted 1-D Lloyd iterations (ties -> lower index).
    With return_codebook also returns that codebook, [d_out, 2**bits] fp32."""
    m = 1 << bits
    d_out, d_in = W.shape
    qs = (2 * torch.arange(m, device=W.device, dtype=torch.float32) + 1) / (2 * m)
    Ws, _ = torch.sort(W, dim=1)
    pos = (qs * (d_in - 1)).round().long()
    code = Ws[:, pos].contiguous()                      # [d_out, m]
    out = torch.empty_like(W)
    rows_per = max(1, (1 << 24) // max(1, d_in * m))
    for r0 in range(0, d_out, rows_per):
        r1 = min(d_out, r0 + rows_per)
        w = W[r0:r1]
        c = code[r0:r1]
        for _ in range(iters):
            idx = torch.argmin((w[:, :, None] - c[:, None, :]).abs(), dim=2)
            onehot = torch.nn.functional.one_hot(idx, m).to(w.dtype)
            cnt = onehot.sum(dim=1)
            tot = (onehot * w[:, :, None]).sum(dim=1)
            c = torch.where(cnt > 0, tot / cnt.clamp(min=1), c)
        idx = torch.argmin((w[:, :, None] - c[:, None, :]).abs(), dim=2)
        out[r0:r1] = torch.gather(c, 1, idx)
        code[r0:r1] = c
    out = out.to(torch.float32).contiguous()
    return (out, code.to(torch.float32).contiguous()) if return_codebook else out


@dataclass
class LayerSpec:
    """One linear layer's worth of synthetic calibration tensors."""
    name: str
    n: int
    d_in: int
    d_out: int
    G: int
    x_kind: str                 # "outlier" | "silu"
    x_dtype: str                # "f32" | "bf16"
    outlier_frac: float = 0.0   # fraction of columns, or absolute count if >= 1
    outlier_scale: float = 1.0
    dz_std: float = 1.0
    dz_sigma: float = 1.0
    what: str = "codebook3"     # "uniform16" | "codebook3"
    chunks: int = 1
    cfg: int = 0
    extra: dict = field(default_factory=dict)


# The five workload configurations this build is measured and tested on.
CONFIGS = {
    "tiny_f32": LayerSpec("tiny_f32", 2048, 256, 512, 2, "outlier", "f32", 4, 20.0,
                          1.0, 1.0, "uniform16", 1, 1),
    "llama2_7b_attn": LayerSpec("llama2_7b_attn", 65536, 4096, 4096, 4, "outlier", "bf16",
                                0.01, 30.0, 1e-4, 1.5, "codebook3", 1, 2),
    "llama2_7b_down": LayerSpec("llama2_7b_down", 65536, 11008, 4096, 4, "silu", "bf16",
                                0.0, 1.0, 1e-4, 1.5, "codebook3", 8, 3),
    "llama2_13b_attn": LayerSpec("llama2_13b_attn", 65536, 5120, 5120, 4, "outlier", "bf16",
                                 0.01, 30.0, 1e-4, 1.5, "codebook3", 1, 4),
    "llama2_13b_up": LayerSpec("llama2_13b_up", 65536, 5120, 13824, 4, "outlier", "bf16",
                               0.01, 30.0, 1e-4, 1.5, "codebook3", 1, 4),
    "llama2_13b_down": LayerSpec("llama2_13b_down", 65536, 13824, 5120, 4, "silu", "bf16",
                                 0.0, 1.0, 1e-4, 1.5, "codebook3", 1, 4),
    "llama2_70b_attn": LayerSpec("llama2_70b_attn", 32768, 8192, 8192, 4, "outlier", "bf16",
                                 0.01, 30.0, 1e-4, 1.5, "codebook3", 1, 5),
    "llama2_70b_up": LayerSpec("llama2_70b_up", 32768, 8192, 28672, 4, "outlier", "bf16",
                               0.01, 30.0, 1e-4, 1.5, "codebook3", 1, 5),
    "llama2_70b_down": LayerSpec("llama2_70b_down", 32768, 28672, 8192, 4, "silu", "bf16",
                                 0.0, 1.0, 1e-4, 1.5, "codebook3", 1, 5),
}


def _seed(spec: LayerSpec, tensor_index: int) -> int:
    return BASE_SEED + 1000 * spec.cfg + 17 * (sum(map(ord, spec.name)) % 53) + tensor_index


def make_x(spec: LayerSpec, device="cpu", n: Optional[int] = None) -> torch.Tensor:
    n = spec.n if n is None else n
    dtype = torch.bfloat16 if spec.x_dtype == "bf16" else torch.float32
    if spec.x_kind == "outlier":
        k = spec.outlier_frac
        n_cols = int(k) if k >= 1 else int(round(k * spec.d_in))
        return make_x_outlier(n, spec.d_in, n_cols, spec.outlier_scale, _seed(spec, 0), device, dtype)
    if spec.x_kind == "silu":
        return make_x_silu(n, spec.d_in, _seed(spec, 0), device, dtype)
    raise ValueError(spec.x_kind)


def make_dz_for(spec: LayerSpec, device="cpu", n: Optional[int] = None) -> torch.Tensor:
    n = spec.n if n is None else n
    return make_dz(n, spec.d_out, spec.dz_std, spec.dz_sigma, _seed(spec, 1), device)


def make_weights(spec: LayerSpec, device="cpu", d_out: Optional[int] = None):
    """Returns (W, What), both fp32 [d_out, d_in]."""
    d_out = spec.d_out if d_out is None else d_out
    W = make_w(d_out, spec.d_in, _seed(spec, 2), device)
    if spec.what == "uniform16":
        What = quantize_uniform_per_row(W, 16)
    elif spec.what == "codebook3":
        What = quantize_codebook_per_row(W, 3, 5)
    else:
        raise ValueError(spec.what)
    return W, What


def scaled(spec: LayerSpec, **overrides) -> LayerSpec:
    """Copy of a spec with some sizes replaced (smaller parity-test versions of
    the full shapes keep the same value recipe)."""
    d = dict(spec.__dict__)
    d.update(overrides)
    return LayerSpec(**d)
