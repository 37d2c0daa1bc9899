"""Thin ctypes binding of libgq's C ABI (include/gq.h).

Argument marshalling only: torch supplies device memory and the current HIP
stream; every step of the computation runs inside libgq's kernels.  There is no
CPU or PyTorch fallback: a missing library or a non-GPU tensor raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libgq.so")

GQ_F32, GQ_BF16 = 0, 1
GQ_ACCUMULATE, GQ_MIRROR, GQ_TWO_TERMS, GQ_HEAVY_TWO_TERMS = 1, 2, 4, 8

_lib = None


class GQError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {status_string(status)} (gq_status {status})")
        self.status = status


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Load libgq.so, building it first only if no built library exists."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(p)
    c = ctypes
    lib.gq_version.restype = c.c_int
    lib.gq_version.argtypes = []
    lib.gq_status_string.restype = c.c_char_p
    lib.gq_status_string.argtypes = [c.c_int]
    lib.gq_group_weights.restype = c.c_int
    lib.gq_group_weights.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int64, c.c_int64, c.c_int32,
                                     c.c_float, c.c_void_p, c.c_void_p]
    lib.gq_group_weights_strided.restype = c.c_int
    lib.gq_group_weights_strided.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int64, c.c_int64, c.c_int32,
                                             c.c_float, c.c_void_p, c.c_int64, c.c_void_p]
    lib.gq_fisher_gram_workspace_bytes.restype = c.c_size_t
    lib.gq_fisher_gram_workspace_bytes.argtypes = [c.c_int, c.c_int64, c.c_int64, c.c_int32]
    lib.gq_fisher_gram.restype = c.c_int
    lib.gq_fisher_gram.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int64, c.c_int64, c.c_void_p,
                                   c.c_int32, c.c_void_p, c.c_uint32, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.gq_fisher_gram_noalloc.restype = c.c_int
    lib.gq_fisher_gram_noalloc.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int64, c.c_int64, c.c_void_p,
                                           c.c_int32, c.c_void_p, c.c_uint32, c.c_void_p]
    lib.gq_fisher_gram_set_xcd_speeds.restype = c.c_int
    lib.gq_fisher_gram_set_xcd_speeds.argtypes = [c.c_void_p]
    lib.gq_fisher_gram_measured_xcd_speeds.restype = c.c_int
    lib.gq_fisher_gram_measured_xcd_speeds.argtypes = [c.c_int64, c.c_int64, c.c_int32, c.c_void_p, c.c_void_p]
    lib.gq_fisher_gram_heavy_pool_bytes.restype = c.c_size_t
    lib.gq_fisher_gram_heavy_pool_bytes.argtypes = [c.c_int64, c.c_int32, c.c_int64]
    lib.gq_fisher_gram_heavy_deferred.restype = c.c_int
    lib.gq_fisher_gram_heavy_deferred.argtypes = [c.c_void_p, c.c_int, c.c_int64, c.c_int64, c.c_int64, c.c_void_p,
                                                  c.c_int32, c.c_void_p, c.c_uint32, c.c_void_p, c.c_size_t,
                                                  c.c_void_p, c.c_int64, c.c_void_p]
    lib.gq_fisher_gram_heavy_flush.restype = c.c_int
    lib.gq_fisher_gram_heavy_flush.argtypes = [c.c_void_p, c.c_int64, c.c_int64, c.c_int32, c.c_void_p, c.c_uint32,
                                               c.c_void_p, c.c_size_t, c.c_void_p]
    lib.gq_fisher_gram_noalloc_max_scratch_bytes.restype = c.c_size_t
    lib.gq_fisher_gram_noalloc_max_scratch_bytes.argtypes = []
    lib.gq_fisher_mirror.restype = c.c_int
    lib.gq_fisher_mirror.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_void_p]
    lib.gq_objective_workspace_bytes.restype = c.c_size_t
    lib.gq_objective_workspace_bytes.argtypes = [c.c_int64, c.c_int64, c.c_int32]
    lib.gq_objective.restype = c.c_int
    lib.gq_objective.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64, c.c_void_p,
                                 c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.gq_cd_workspace_bytes.restype = c.c_size_t
    lib.gq_cd_workspace_bytes.argtypes = [c.c_int64, c.c_int64, c.c_int32]
    lib.gq_cholesky_workspace_bytes.restype = c.c_size_t
    lib.gq_cholesky_workspace_bytes.argtypes = [c.c_int64, c.c_int32]
    lib.gq_damped_cholesky.restype = c.c_int
    lib.gq_damped_cholesky.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_double, c.c_double, c.c_uint32, c.c_void_p,
                                       c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.gq_damp_diagonal.restype = c.c_int
    lib.gq_damp_diagonal.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_double, c.c_double, c.c_void_p]
    lib.gq_lnq_workspace_bytes.restype = c.c_size_t
    lib.gq_lnq_workspace_bytes.argtypes = [c.c_int64, c.c_int64, c.c_int32, c.c_int32]
    lib.gq_lnq.restype = c.c_int
    lib.gq_lnq.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int64, c.c_int64, c.c_int64,
                           c.c_void_p, c.c_int32, c.c_int32, c.c_int32, c.c_double, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.gq_ldlq_assign.restype = c.c_int
    lib.gq_ldlq_assign.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int64, c.c_int64, c.c_int64,
                                   c.c_void_p, c.c_int32, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.gq_lnq_codebook_workspace_bytes.restype = c.c_size_t
    lib.gq_lnq_codebook_workspace_bytes.argtypes = [c.c_int64, c.c_int64, c.c_int32, c.c_int32]
    lib.gq_lnq_codebook.restype = c.c_int
    lib.gq_lnq_codebook.argtypes = [c.c_void_p, c.c_int64, c.c_int64, c.c_int64, c.c_void_p, c.c_void_p, c.c_int32,
                                    c.c_int32, c.c_double, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.gq_cd_assign.restype = c.c_int
    lib.gq_cd_assign.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int64, c.c_int64, c.c_int64,
                                 c.c_void_p, c.c_int32, c.c_int32, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    if path is None:
        _lib = lib
    return lib


def gq_version() -> int:
    return int(load_library().gq_version())


def status_string(status: int) -> str:
    return load_library().gq_status_string(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise GQError(status, what)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return GQ_F32
    if t.dtype == torch.bfloat16:
        return GQ_BF16
    raise TypeError(f"unsupported dtype {t.dtype}: libgq takes float32 or bfloat16")


def _require_gpu(*tensors: torch.Tensor) -> None:
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise RuntimeError("libgq runs on the GPU only: got a tensor on %s" % t.device)


def _rows(t: torch.Tensor) -> int:
    """Row pitch in elements of a 2-D tensor whose rows are contiguous."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("expected a 2-D tensor with contiguous rows")
    return int(t.stride(0)) if t.shape[0] > 1 else int(max(t.stride(0), t.shape[1]))


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _workspace(nbytes: int, device) -> Tuple[Optional[torch.Tensor], int]:
    if nbytes == 0:
        return None, 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return ws, ws.data_ptr()


def gq_group_weights(dZ: torch.Tensor, G: int, grad_scale: float = 1.0,
                     out: Optional[torch.Tensor] = None, out_col: int = 0) -> torch.Tensor:
    """s[i,k] = grad_scale^2/(d_out/G) * sum_{j in J_k} dZ[i,j]^2 -> fp32 [n, G].
    With a wider contiguous `out` [n, G_total] the G columns starting at `out_col` are written
    (layers that share their input X stack their weights for one gq_fisher_gram call)."""
    _require_gpu(dZ, out)
    n, d_out = dZ.shape
    s = out if out is not None else torch.empty((n, G), dtype=torch.float32, device=dZ.device)
    assert s.dtype == torch.float32 and s.is_contiguous() and s.shape[0] == n and 0 <= out_col and out_col + G <= s.shape[1]
    lib = load_library()
    if s.shape[1] == G:
        st = lib.gq_group_weights(dZ.data_ptr(), _dtype_code(dZ), n, d_out, _rows(dZ), G,
                                  float(grad_scale), s.data_ptr(), _stream())
    else:
        st = lib.gq_group_weights_strided(dZ.data_ptr(), _dtype_code(dZ), n, d_out, _rows(dZ), G, float(grad_scale),
                                          s.data_ptr() + 4 * out_col, int(s.shape[1]), _stream())
    _check(st, "gq_group_weights")
    return s


def gq_fisher_gram_workspace_bytes(x_dtype: torch.dtype, n: int, d_in: int, G: int) -> int:
    code = GQ_BF16 if x_dtype == torch.bfloat16 else GQ_F32
    return int(load_library().gq_fisher_gram_workspace_bytes(code, n, d_in, G))


def gq_fisher_gram(X: torch.Tensor, s: torch.Tensor, H: Optional[torch.Tensor] = None,
                   accumulate: bool = False, mirror: bool = False, two_terms: bool = False,
                   workspace: Optional[torch.Tensor] = None, heavy_two_terms: bool = False) -> torch.Tensor:
    """H[k] (+)= X^T Diag(s[:,k]) X on the upper triangle -> fp32 [G, d_in, d_in].
    two_terms (bf16 X only): the scaled operand as two bf16 terms, twice the work, fp32-grade products.
    heavy_two_terms (bf16 X only): two terms only for the tokens with the largest weights (GQ_HEAVY_TWO_TERMS)."""
    _require_gpu(X, s, H, workspace)
    n, d_in = X.shape
    G = int(s.shape[1])
    assert s.dtype == torch.float32 and s.is_contiguous() and s.shape[0] == n
    if H is None:
        if accumulate:
            raise ValueError("accumulate=True needs an existing H")
        H = torch.empty((G, d_in, d_in), dtype=torch.float32, device=X.device)
    assert H.dtype == torch.float32 and H.is_contiguous() and tuple(H.shape) == (G, d_in, d_in)
    lib = load_library()
    need = int(lib.gq_fisher_gram_workspace_bytes(_dtype_code(X), n, d_in, G))
    if workspace is None:
        workspace, ws_ptr = _workspace(need, X.device)
        ws_bytes = need
    else:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    flags = ((GQ_ACCUMULATE if accumulate else 0) | (GQ_MIRROR if mirror else 0) | (GQ_TWO_TERMS if two_terms else 0)
             | (GQ_HEAVY_TWO_TERMS if heavy_two_terms else 0))
    st = lib.gq_fisher_gram(X.data_ptr(), _dtype_code(X), n, d_in, _rows(X) if n > 0 else d_in,
                            s.data_ptr(), G, H.data_ptr(), flags, ws_ptr, ws_bytes, _stream())
    _check(st, "gq_fisher_gram")
    return H


def gq_fisher_gram_heavy_pool(d_in: int, G: int, pool_rows: int, device) -> torch.Tensor:
    """An empty pool (zero bytes) for gq_fisher_gram_heavy_deferred / gq_fisher_gram_heavy_flush."""
    need = int(load_library().gq_fisher_gram_heavy_pool_bytes(d_in, G, pool_rows))
    if need == 0:
        raise ValueError("pool_rows must be a multiple of 32, at least 32")
    return torch.zeros(need, dtype=torch.uint8, device=device)


def gq_fisher_gram_heavy_deferred(X: torch.Tensor, s: torch.Tensor, pool: torch.Tensor, pool_rows: int,
                                  H: Optional[torch.Tensor] = None, accumulate: bool = False,
                                  workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """gq_fisher_gram with heavy_two_terms for chunked callers: the heavy rows go to `pool`, their two-term pass
    runs in gq_fisher_gram_heavy_flush."""
    _require_gpu(X, s, H, workspace, pool)
    n, d_in = X.shape
    G = int(s.shape[1])
    assert s.dtype == torch.float32 and s.is_contiguous() and s.shape[0] == n
    if H is None:
        if accumulate:
            raise ValueError("accumulate=True needs an existing H")
        H = torch.empty((G, d_in, d_in), dtype=torch.float32, device=X.device)
    assert H.dtype == torch.float32 and H.is_contiguous() and tuple(H.shape) == (G, d_in, d_in)
    lib = load_library()
    need = int(lib.gq_fisher_gram_workspace_bytes(_dtype_code(X), n, d_in, G))
    if workspace is None:
        workspace, ws_ptr = _workspace(need, X.device)
        ws_bytes = need
    else:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    st = lib.gq_fisher_gram_heavy_deferred(X.data_ptr(), _dtype_code(X), n, d_in, _rows(X) if n > 0 else d_in,
                                           s.data_ptr(), G, H.data_ptr(), GQ_ACCUMULATE if accumulate else 0,
                                           ws_ptr, ws_bytes, pool.data_ptr(), pool_rows, _stream())
    _check(st, "gq_fisher_gram_heavy_deferred")
    return H


def gq_fisher_gram_heavy_flush(pool: torch.Tensor, pool_rows: int, H: torch.Tensor, mirror: bool = False,
                               workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Adds the two-term products of the rows gathered in `pool` to H and empties the pool."""
    _require_gpu(H, workspace, pool)
    G, d_in = int(H.shape[0]), int(H.shape[1])
    assert H.dtype == torch.float32 and H.is_contiguous() and tuple(H.shape) == (G, d_in, d_in)
    lib = load_library()
    need = int(lib.gq_fisher_gram_workspace_bytes(GQ_BF16, pool_rows, d_in, G))
    if workspace is None:
        workspace, ws_ptr = _workspace(need, H.device)
        ws_bytes = need
    else:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    st = lib.gq_fisher_gram_heavy_flush(pool.data_ptr(), pool_rows, d_in, G, H.data_ptr(), GQ_MIRROR if mirror else 0,
                                        ws_ptr, ws_bytes, _stream())
    _check(st, "gq_fisher_gram_heavy_flush")
    return H


def gq_fisher_gram_set_xcd_speeds(speeds=None) -> None:
    """Relative speeds of the 8 XCDs for the schedule of the bf16 Gram kernel on the current device (None: equal)."""
    if speeds is None:
        st = load_library().gq_fisher_gram_set_xcd_speeds(None)
    else:
        arr = (ctypes.c_float * 8)(*[float(v) for v in speeds])
        st = load_library().gq_fisher_gram_set_xcd_speeds(ctypes.cast(arr, ctypes.c_void_p))
    _check(st, "gq_fisher_gram_set_xcd_speeds")


def gq_fisher_gram_measured_xcd_speeds(n: int, d_in: int, G: int, workspace: torch.Tensor):
    """The relative XCD speeds recorded by the last plain one-term bf16 gq_fisher_gram call with these sizes and
    this workspace (waits for the device); a list of 8 floats with mean 1."""
    _require_gpu(workspace)
    arr = (ctypes.c_float * 8)()
    st = load_library().gq_fisher_gram_measured_xcd_speeds(n, d_in, G, workspace.data_ptr(),
                                                           ctypes.cast(arr, ctypes.c_void_p))
    _check(st, "gq_fisher_gram_measured_xcd_speeds")
    return [float(v) for v in arr]


def gq_fisher_gram_noalloc(X: torch.Tensor, s: torch.Tensor, H: torch.Tensor, accumulate: bool = False,
                           mirror: bool = False, two_terms: bool = False) -> torch.Tensor:
    """gq_fisher_gram without a workspace: the call allocates nothing (H must exist); raises GQError with
    GQ_ERR_WORKSPACE when the repacked weights do not fit the library's fixed scratch array."""
    _require_gpu(X, s, H)
    n, d_in = X.shape
    G = int(s.shape[1])
    assert s.dtype == torch.float32 and s.is_contiguous() and s.shape[0] == n
    assert H.dtype == torch.float32 and H.is_contiguous() and tuple(H.shape) == (G, d_in, d_in)
    flags = (GQ_ACCUMULATE if accumulate else 0) | (GQ_MIRROR if mirror else 0) | (GQ_TWO_TERMS if two_terms else 0)
    st = load_library().gq_fisher_gram_noalloc(X.data_ptr(), _dtype_code(X), n, d_in, _rows(X) if n > 0 else d_in,
                                               s.data_ptr(), G, H.data_ptr(), flags, _stream())
    _check(st, "gq_fisher_gram_noalloc")
    return H


def gq_fisher_mirror(H: torch.Tensor) -> torch.Tensor:
    """Fill the strictly lower triangle of every H[k] from the upper one, in place."""
    _require_gpu(H)
    assert H.dtype == torch.float32 and H.is_contiguous() and H.dim() == 3 and H.shape[1] == H.shape[2]
    st = load_library().gq_fisher_mirror(H.data_ptr(), int(H.shape[1]), int(H.shape[0]), _stream())
    _check(st, "gq_fisher_mirror")
    return H


def gq_objective(W: torch.Tensor, What: torch.Tensor, H: torch.Tensor, want_rows: bool = False,
                 workspace: Optional[torch.Tensor] = None):
    """obj[k] = sum_{j in J_k} (W[j]-What[j])^T H[k] (W[j]-What[j]) -> fp64 [G]
    (and the per-channel terms, fp32 [d_out], if want_rows)."""
    _require_gpu(W, What, H, workspace)
    d_out, d_in = W.shape
    G = int(H.shape[0])
    assert W.dtype == torch.float32 and What.dtype == torch.float32 and H.dtype == torch.float32
    assert What.shape == W.shape and _rows(W) == _rows(What) and H.is_contiguous()
    lib = load_library()
    need = int(lib.gq_objective_workspace_bytes(d_out, d_in, G))
    if workspace is None:
        workspace, ws_ptr = _workspace(max(need, 1), W.device)
        ws_bytes = need
    else:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    obj = torch.empty(G, dtype=torch.float64, device=W.device)
    rows = torch.empty(d_out, dtype=torch.float32, device=W.device) if want_rows else None
    st = lib.gq_objective(W.data_ptr(), What.data_ptr(), d_out, d_in, _rows(W), H.data_ptr(), G,
                          obj.data_ptr(), rows.data_ptr() if want_rows else None, ws_ptr, ws_bytes, _stream())
    _check(st, "gq_objective")
    return (obj, rows) if want_rows else obj


def gq_cd_assign(W: torch.Tensor, What: torch.Tensor, codebook: torch.Tensor, H: torch.Tensor, n_cycles: int = 1,
                 want_codes: bool = True, workspace: Optional[torch.Tensor] = None):
    """Cyclic coordinate descent on the assignments against H[k] (Section 4.2, Eq. "cd_closed").
    `What` [d_out, d_in] (every entry a point of its row's grid `codebook` [d_out, m]) is updated
    IN PLACE; returns the grid indices [d_out, d_in] uint8 of the last update (or None)."""
    _require_gpu(W, What, codebook, H, workspace)
    d_out, d_in = W.shape
    G = int(H.shape[0])
    assert W.dtype == torch.float32 and What.dtype == torch.float32 and H.dtype == torch.float32
    assert codebook.dtype == torch.float32 and codebook.is_contiguous() and codebook.shape[0] == d_out
    assert What.shape == W.shape and _rows(W) == _rows(What) and H.is_contiguous()
    lib = load_library()
    need = int(lib.gq_cd_workspace_bytes(d_out, d_in, G))
    if workspace is None:
        workspace, ws_ptr = _workspace(max(need, 1), W.device)
        ws_bytes = need
    else:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    Q = torch.empty((d_out, d_in), dtype=torch.uint8, device=W.device) if want_codes else None
    st = lib.gq_cd_assign(W.data_ptr(), What.data_ptr(), codebook.data_ptr(), int(codebook.shape[1]), d_out, d_in,
                          _rows(W), H.data_ptr(), G, int(n_cycles), Q.data_ptr() if want_codes else None,
                          ws_ptr, ws_bytes, _stream())
    _check(st, "gq_cd_assign")
    return Q


def gq_lnq_codebook(W: torch.Tensor, Q: torch.Tensor, H: torch.Tensor, n_levels: int, lam: float = 1e-7,
                    What: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """Closed-form grids for fixed assignments against H[k] (Section 4.2, Eq. "conti-sol").
    `Q` [d_out, d_in] uint8; returns the codebook [d_out, n_levels] fp32.  If `What` (same shape and
    pitch as W) is given it is overwritten with codebook[j, Q[j, i]]."""
    _require_gpu(W, Q, H, What, workspace)
    d_out, d_in = W.shape
    G = int(H.shape[0])
    assert W.dtype == torch.float32 and H.dtype == torch.float32 and H.is_contiguous()
    assert Q.dtype == torch.uint8 and Q.is_contiguous() and tuple(Q.shape) == (d_out, d_in)
    if What is not None:
        assert What.dtype == torch.float32 and What.shape == W.shape and _rows(W) == _rows(What)
    lib = load_library()
    need = int(lib.gq_lnq_codebook_workspace_bytes(d_out, d_in, G, int(n_levels)))
    if workspace is None:
        workspace, ws_ptr = _workspace(max(need, 1), W.device)
        ws_bytes = need
    else:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    codebook = torch.empty((d_out, int(n_levels)), dtype=torch.float32, device=W.device)
    st = lib.gq_lnq_codebook(W.data_ptr(), d_out, d_in, _rows(W), Q.data_ptr(), H.data_ptr(), G, int(n_levels),
                             float(lam), codebook.data_ptr(), What.data_ptr() if What is not None else None,
                             ws_ptr, ws_bytes, _stream())
    _check(st, "gq_lnq_codebook")
    return codebook


def gq_ldlq_assign(W: torch.Tensor, codebook: torch.Tensor, R: torch.Tensor, What: Optional[torch.Tensor] = None,
                   want_codes: bool = True, workspace: Optional[torch.Tensor] = None):
    """Sequential rounding with error feedback (GPTQ / LDLQ) from the upper triangular factor `R`
    [G, d_in, d_in] of the damped group Hessians, H + eps I = R R^T.  Returns (What, Q)."""
    _require_gpu(W, codebook, R, What, workspace)
    d_out, d_in = W.shape
    G = int(R.shape[0])
    assert W.dtype == torch.float32 and R.dtype == torch.float32 and R.is_contiguous()
    assert codebook.dtype == torch.float32 and codebook.is_contiguous() and codebook.shape[0] == d_out
    if What is None:
        What = torch.empty_strided(W.shape, W.stride(), dtype=W.dtype, device=W.device)
    assert What.dtype == torch.float32 and What.shape == W.shape and _rows(W) == _rows(What)
    lib = load_library()
    need = int(lib.gq_cd_workspace_bytes(d_out, d_in, G))
    if workspace is None:
        workspace, ws_ptr = _workspace(max(need, 1), W.device)
        ws_bytes = need
    else:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    Q = torch.empty((d_out, d_in), dtype=torch.uint8, device=W.device) if want_codes else None
    st = lib.gq_ldlq_assign(W.data_ptr(), What.data_ptr(), codebook.data_ptr(), int(codebook.shape[1]), d_out, d_in,
                            _rows(W), R.data_ptr(), G, Q.data_ptr() if want_codes else None, ws_ptr, ws_bytes, _stream())
    _check(st, "gq_ldlq_assign")
    return What, Q


GQ_CHOL_REVERSE = 1


def gq_damped_cholesky(H: torch.Tensor, damp_rel: float = 0.01, damp_abs: float = 0.0, reverse: bool = False,
                       workspace: Optional[torch.Tensor] = None):
    """H[k] + eps_k I = L L^T (L lower) or, with reverse=True, = R R^T (R upper), eps_k = damp_abs +
    damp_rel * mean diag H[k] (Algorithm 2, line 1).  Returns (F [G, d, d] fp32, info [G] int32)."""
    _require_gpu(H, workspace)
    assert H.dtype == torch.float32 and H.is_contiguous() and H.dim() == 3 and H.shape[1] == H.shape[2]
    G, d = int(H.shape[0]), int(H.shape[1])
    lib = load_library()
    need = int(lib.gq_cholesky_workspace_bytes(d, G))
    if workspace is None:
        workspace, ws_ptr = _workspace(max(need, 1), H.device)
        ws_bytes = need
    else:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    F = torch.empty_like(H)
    info = torch.empty(G, dtype=torch.int32, device=H.device)
    st = lib.gq_damped_cholesky(H.data_ptr(), d, G, float(damp_rel), float(damp_abs), GQ_CHOL_REVERSE if reverse else 0,
                                F.data_ptr(), info.data_ptr(), ws_ptr, ws_bytes, _stream())
    _check(st, "gq_damped_cholesky")
    return F, info


def gq_lnq(W: torch.Tensor, Q: torch.Tensor, H: torch.Tensor, n_levels: int, n_iters: int = 2, n_cycles: int = 4,
           lam: float = 1e-7, What: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """Algorithm 2 (LNQ) against H[k]: n_iters x (closed-form grids, n_cycles CD cycles), then the grids once
    more.  `Q` [d_out, d_in] uint8 holds the initial assignments and is updated IN PLACE.
    Returns (What, codebook [d_out, n_levels])."""
    _require_gpu(W, Q, H, What, workspace)
    d_out, d_in = W.shape
    G = int(H.shape[0])
    assert W.dtype == torch.float32 and H.dtype == torch.float32 and H.is_contiguous()
    assert Q.dtype == torch.uint8 and Q.is_contiguous() and tuple(Q.shape) == (d_out, d_in)
    if What is None:
        What = torch.empty_strided(W.shape, W.stride(), dtype=W.dtype, device=W.device)
    assert What.dtype == torch.float32 and What.shape == W.shape and _rows(W) == _rows(What)
    lib = load_library()
    need = int(lib.gq_lnq_workspace_bytes(d_out, d_in, G, int(n_levels)))
    if workspace is None:
        workspace, ws_ptr = _workspace(max(need, 1), W.device)
        ws_bytes = need
    else:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    codebook = torch.empty((d_out, int(n_levels)), dtype=torch.float32, device=W.device)
    st = lib.gq_lnq(W.data_ptr(), What.data_ptr(), Q.data_ptr(), codebook.data_ptr(), int(n_levels), d_out, d_in, _rows(W),
                    H.data_ptr(), G, int(n_iters), int(n_cycles), float(lam), ws_ptr, ws_bytes, _stream())
    _check(st, "gq_lnq")
    return What, codebook


def gq_damp_diagonal(H: torch.Tensor, damp_rel: float = 0.01, damp_abs: float = 0.0) -> torch.Tensor:
    """H[k][i,i] += damp_abs + damp_rel * mean diag H[k], in place."""
    _require_gpu(H)
    assert H.dtype == torch.float32 and H.is_contiguous() and H.dim() == 3 and H.shape[1] == H.shape[2]
    st = load_library().gq_damp_diagonal(H.data_ptr(), int(H.shape[1]), int(H.shape[0]), float(damp_rel), float(damp_abs),
                                         _stream())
    _check(st, "gq_damp_diagonal")
    return H
