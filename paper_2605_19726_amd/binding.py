"""ctypes binding of libbasa.so: argument marshalling only.

Each function has the name of the C entry point it calls (include/basa.h).  torch is
used to allocate device buffers and to supply the current HIP stream; every
computation runs in the library's kernels.  If the library is missing or cannot be
loaded the first call raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

# BASA_LIB_PATH overrides the in-tree library (e.g. to try a differently built libbasa.so)
_LIB_PATH = os.environ.get("BASA_LIB_PATH") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libbasa.so")
_lib = None

BASA_OK = 0
SORT_NONE, SORT_Q, SORT_K, SORT_QK = 0, 1, 2, 3
F32, BF16 = 0, 1

EXPORTS = (
    "basa_kappa", "basa_select_workspace_size", "basa_attn_workspace_size",
    "basa_sort_workspace_size", "basa_norm_sort", "basa_downsample", "basa_select",
    "basa_sparse_attn", "basa_dense_attn", "basa_status_string", "basa_last_error",
    "basa_version", "basa_profile_enable", "basa_profile_kernel_count", "basa_profile_kernel_name",
    "basa_profile_read", "basa_calibrate_mfma", "basa_calibrate_read", "basa_block_mass_workspace_size", "basa_block_mass",
    "basa_block_radius", "basa_deviation_bound", "basa_selection_fidelity", "basa_pearson_sums",
    "basa_static_scratch_size", "basa_static_init", "basa_norm_sort_static",
)


class BasaTensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("dtype", C.c_int32), ("batch", C.c_int32),
                ("heads", C.c_int32), ("L", C.c_int32), ("d", C.c_int32),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_l", C.c_int64)]


class BasaParams(C.Structure):
    _fields_ = [("block", C.c_int32), ("sort", C.c_int32), ("window", C.c_int32),
                ("beta", C.c_float), ("sparsity", C.c_double), ("mass_target", C.c_double),
                ("min_keep", C.c_int32), ("attn_shape", C.c_int32),
                ("n_segments", C.c_int32), ("budget_total", C.c_int32),
                ("segment_starts", C.POINTER(C.c_int32)), ("causal", C.c_int32),
                ("select_path", C.c_int32)]


class BasaError(RuntimeError):
    def __init__(self, status: int, name: str, reason: str):
        super().__init__(f"{name}: {reason}")
        self.status = status
        self.status_name = name


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Open libbasa.so (once) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} not found: build it with "
                           "`python -m paper_2605_19726_amd.build` (no fallback path exists)")
    lib = C.CDLL(_LIB_PATH)
    T, P, V = C.POINTER(BasaTensor), C.POINTER(BasaParams), C.c_void_p
    lib.basa_kappa.restype = C.c_int32
    lib.basa_kappa.argtypes = [C.c_int32, C.c_double]
    for n in ("basa_select_workspace_size", "basa_attn_workspace_size"):
        getattr(lib, n).restype = C.c_size_t
        getattr(lib, n).argtypes = [T, T, P]
    lib.basa_sort_workspace_size.restype = C.c_size_t
    lib.basa_sort_workspace_size.argtypes = [T, P]
    lib.basa_norm_sort.restype = C.c_int
    lib.basa_norm_sort.argtypes = [T, P, V, V, V, C.c_size_t, V]
    lib.basa_static_scratch_size.restype = C.c_size_t
    lib.basa_static_scratch_size.argtypes = []
    lib.basa_static_init.restype = C.c_int
    lib.basa_static_init.argtypes = []
    lib.basa_norm_sort_static.restype = C.c_int
    lib.basa_norm_sort_static.argtypes = [T, P, V, V, V]
    lib.basa_downsample.restype = C.c_int
    lib.basa_downsample.argtypes = [T, V, P, V, V, V, V]
    lib.basa_select.restype = C.c_int
    lib.basa_select.argtypes = [T, T, P, V, V, V, V, V, V, V, V, C.c_size_t, V]
    lib.basa_sparse_attn.restype = C.c_int
    S3 = C.POINTER(C.c_int64)
    lib.basa_sparse_attn.argtypes = [T, T, T, V, V, C.c_int32, V, V, P, V, S3, V, V, C.c_size_t, V]
    lib.basa_dense_attn.restype = C.c_int
    lib.basa_dense_attn.argtypes = [T, T, T, P, V, S3, V, V, C.c_size_t, V]
    lib.basa_status_string.restype = C.c_char_p
    lib.basa_status_string.argtypes = [C.c_int]
    lib.basa_last_error.restype = C.c_char_p
    lib.basa_last_error.argtypes = []
    lib.basa_version.restype = C.c_char_p
    lib.basa_version.argtypes = []
    lib.basa_profile_enable.restype = C.c_int
    lib.basa_profile_enable.argtypes = [C.c_int]
    lib.basa_profile_kernel_count.restype = C.c_int32
    lib.basa_profile_kernel_count.argtypes = []
    lib.basa_profile_kernel_name.restype = C.c_char_p
    lib.basa_profile_kernel_name.argtypes = [C.c_int32]
    lib.basa_profile_read.restype = C.c_int
    lib.basa_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int32), C.c_int32]
    lib.basa_block_mass_workspace_size.restype = C.c_size_t
    lib.basa_block_mass_workspace_size.argtypes = [T, T]
    lib.basa_block_mass.restype = C.c_int
    lib.basa_block_mass.argtypes = [T, T, V, V, P, V, V, V, V, V, C.c_size_t, V]
    lib.basa_block_radius.restype = C.c_int
    lib.basa_block_radius.argtypes = [T, V, P, V, V, V]
    lib.basa_deviation_bound.restype = C.c_int
    lib.basa_deviation_bound.argtypes = [V, V, V, V, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, V, V]
    lib.basa_selection_fidelity.restype = C.c_int
    lib.basa_selection_fidelity.argtypes = [V, V, V, C.c_int64, C.c_int32, V, V, V]
    lib.basa_pearson_sums.restype = C.c_int
    lib.basa_pearson_sums.argtypes = [V, V, C.c_int64, V, V]
    lib.basa_calibrate_read.restype = C.c_int
    lib.basa_calibrate_read.argtypes = [V, C.c_size_t, V, V]
    lib.basa_calibrate_mfma.restype = C.c_int
    lib.basa_calibrate_mfma.argtypes = [C.c_int32, C.c_int32, V, C.c_size_t, C.POINTER(C.c_double), V]
    _lib = lib
    return lib


def _check(status: int):
    if status != BASA_OK:
        lib = load()
        raise BasaError(status, lib.basa_status_string(status).decode(),
                        lib.basa_last_error().decode())


def tensor_desc(x: torch.Tensor) -> BasaTensor:
    """Descriptor of a [batch, heads, L, d] tensor (no copy; d must be contiguous)."""
    if x.dim() != 4:
        raise ValueError("expected a [batch, heads, L, d] tensor")
    if x.stride(3) != 1:
        raise ValueError("the head dimension must be contiguous")
    if x.dtype == torch.float32:
        dt = F32
    elif x.dtype == torch.bfloat16:
        dt = BF16
    else:
        raise ValueError(f"unsupported dtype {x.dtype}")
    return BasaTensor(x.data_ptr(), dt, x.shape[0], x.shape[1], x.shape[2], x.shape[3],
                      x.stride(0), x.stride(1), x.stride(2))


def params(block: int, sparsity: float = 0.0, beta: float = 1.0, sort: int = SORT_QK,
           window: int = 0, mass_target: float = 0.0, min_keep: int = 0, attn_shape: int = 0,
           segments=None, budget_total: int = 0, causal: bool = False, select_path: int = 0) -> BasaParams:
    """segments: host sequence of segment start tokens ([0, s1, s2, ...]) for a segment-aware sort."""
    p = BasaParams(int(block), int(sort), int(window), float(beta), float(sparsity),
                   float(mass_target), int(min_keep), int(attn_shape), 0, int(budget_total), None,
                   1 if causal else 0, int(select_path))
    if segments is not None:
        arr = (C.c_int32 * len(segments))(*[int(v) for v in segments])
        p.n_segments = len(segments)
        p.segment_starts = C.cast(arr, C.POINTER(C.c_int32))
        p._segments_keepalive = arr          # the struct only borrows the array
    return p


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(x: torch.Tensor):
    return C.c_void_p(torch.cuda.current_stream(x.device).cuda_stream)


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def basa_version() -> str:
    return load().basa_version().decode()


def basa_kappa(n_k: int, sparsity: float) -> int:
    return int(load().basa_kappa(int(n_k), float(sparsity)))


def n_blocks(L: int, block: int) -> int:
    return (L + block - 1) // block


def basa_norm_sort(x: torch.Tensor, block: int, window: int = 0, return_keys: bool = False, ws=None,
                   segments=None):
    lib = load()
    xd, p = tensor_desc(x), params(block, window=window, segments=segments)
    b, h, L, _ = x.shape
    perm = torch.empty((b, h, L), dtype=torch.int32, device=x.device)
    keys = torch.empty((b, h, L), dtype=torch.float32, device=x.device) if return_keys else None
    need = lib.basa_sort_workspace_size(C.byref(xd), C.byref(p))
    ws = _ws(need, x.device) if ws is None else ws
    _check(lib.basa_norm_sort(C.byref(xd), C.byref(p), _ptr(perm), _ptr(keys), _ptr(ws),
                              ws.numel(), _stream(x)))
    return (perm, keys) if return_keys else perm


def basa_static_scratch_size() -> int:
    return int(load().basa_static_scratch_size())


def basa_static_init():
    _check(load().basa_static_init())


def basa_norm_sort_static(x: torch.Tensor, block: int, perm: torch.Tensor, window: int = 0,
                          keys: Optional[torch.Tensor] = None, segments=None):
    """basa_norm_sort on the library's static scratch; `perm` (and `keys`) are caller buffers, nothing is allocated."""
    xd, p = tensor_desc(x), params(block, window=window, segments=segments)
    _check(load().basa_norm_sort_static(C.byref(xd), C.byref(p), _ptr(perm), _ptr(keys), _stream(x)))
    return perm


def basa_downsample(x: torch.Tensor, block: int, perm: Optional[torch.Tensor] = None,
                    want_var: bool = True, want_sorted: bool = False):
    """(mean, var), or (mean, var, x_sorted) with want_sorted."""
    lib = load()
    xd, p = tensor_desc(x), params(block)
    b, h, L, d = x.shape
    N = n_blocks(L, block)
    mean = torch.empty((b, h, N, d), dtype=torch.float32, device=x.device)
    var = torch.empty((b, h, N, d), dtype=torch.float32, device=x.device) if want_var else None
    xs = torch.empty((b, h, L, d), dtype=x.dtype, device=x.device) if want_sorted else None
    _check(lib.basa_downsample(C.byref(xd), _ptr(perm), C.byref(p), _ptr(mean), _ptr(var), _ptr(xs), _stream(x)))
    return (mean, var, xs) if want_sorted else (mean, var)


class Selection:
    """Outputs of basa_select (device tensors)."""
    __slots__ = ("mask_bits", "row_count", "row_cols", "perm_q", "perm_k", "row_mass", "scores",
                 "kappa", "n_q", "n_k")


def select_workspace_size(q, k, p: BasaParams) -> int:
    lib = load()
    qd, kd = tensor_desc(q), tensor_desc(k)
    return int(lib.basa_select_workspace_size(C.byref(qd), C.byref(kd), C.byref(p)))


def attn_workspace_size(q, k, p: BasaParams) -> int:
    lib = load()
    qd, kd = tensor_desc(q), tensor_desc(k)
    return int(lib.basa_attn_workspace_size(C.byref(qd), C.byref(kd), C.byref(p)))


def basa_select(q: torch.Tensor, k: torch.Tensor, block: int, sparsity: float, beta: float = 1.0,
                sort: int = SORT_QK, window: int = 0, want_mask: bool = True,
                want_mass: bool = True, want_scores: bool = False, ws=None, out: Selection = None,
                mass_target: float = 0.0, min_keep: int = 0, segments=None, budget_total: int = 0,
                causal: bool = False, select_path: int = 0):
    lib = load()
    qd, kd = tensor_desc(q), tensor_desc(k)
    p = params(block, sparsity, beta, sort, window, mass_target, min_keep, segments=segments,
               budget_total=budget_total, causal=causal, select_path=select_path)
    b, hq, Lq, _ = q.shape
    hk, Lk = k.shape[1], k.shape[2]
    n_q, n_k = n_blocks(Lq, block), n_blocks(Lk, block)
    kappa = basa_kappa(n_k, sparsity)
    if kappa < 0:
        raise BasaError(1, "BASA_ERR_INVALID_ARG", f"sparsity {sparsity} outside [0, 1)")
    dev = q.device
    s = out
    if s is None:
        s = Selection()
        s.mask_bits = torch.empty((b, hq, n_q, (n_k + 31) // 32), dtype=torch.int32, device=dev) if want_mask else None
        s.row_count = torch.empty((b, hq, n_q), dtype=torch.int32, device=dev)
        s.row_cols = torch.empty((b, hq, n_q, kappa), dtype=torch.int32, device=dev)
        s.perm_q = torch.empty((b, hq, Lq), dtype=torch.int32, device=dev)
        s.perm_k = torch.empty((b, hk, Lk), dtype=torch.int32, device=dev)
        s.row_mass = torch.empty((b, hq, n_q), dtype=torch.float32, device=dev) if want_mass else None
        s.scores = torch.empty((b, hq, n_q, n_k), dtype=torch.float32, device=dev) if want_scores else None
        s.kappa, s.n_q, s.n_k = kappa, n_q, n_k
    if ws is None:
        ws = _ws(lib.basa_select_workspace_size(C.byref(qd), C.byref(kd), C.byref(p)), dev)
    _check(lib.basa_select(C.byref(qd), C.byref(kd), C.byref(p), _ptr(s.mask_bits), _ptr(s.row_count),
                           _ptr(s.row_cols), _ptr(s.perm_q), _ptr(s.perm_k), _ptr(s.row_mass),
                           _ptr(s.scores), _ptr(ws), ws.numel(), _stream(q)))
    return s


def _out_strides(out: torch.Tensor, q: torch.Tensor):
    """out must index as [batch, heads_q, L_q, d] (any view whose last axis has stride 1)."""
    if tuple(out.shape) != tuple(q.shape) or out.dtype != q.dtype or out.device != q.device:
        raise ValueError("out must have the shape, dtype and device of q")
    if out.stride(3) != 1:
        raise ValueError("out: the d axis must have stride 1")
    return (C.c_int64 * 3)(out.stride(0), out.stride(1), out.stride(2))


def basa_sparse_attn(q, k, v, row_count, row_cols, block: int, perm_q=None, perm_k=None,
                     want_lse: bool = False, ws=None, out=None, attn_shape: int = 0, causal: bool = False):
    """out: optional [batch, heads_q, L_q, d] view to write into (strided views are passed as such)."""
    lib = load()
    qd, kd, vd = tensor_desc(q), tensor_desc(k), tensor_desc(v)
    p = params(block, attn_shape=attn_shape, causal=causal)
    b, hq, Lq, d = q.shape
    if out is None:
        out = torch.empty((b, hq, Lq, d), dtype=q.dtype, device=q.device)
    ostr = _out_strides(out, q)
    lse = torch.empty((b, hq, Lq), dtype=torch.float32, device=q.device) if want_lse else None
    if ws is None:
        ws = _ws(lib.basa_attn_workspace_size(C.byref(qd), C.byref(kd), C.byref(p)), q.device)
    stride = 0 if row_cols is None else int(row_cols.shape[-1])
    _check(lib.basa_sparse_attn(C.byref(qd), C.byref(kd), C.byref(vd), _ptr(row_count), _ptr(row_cols),
                                stride, _ptr(perm_q), _ptr(perm_k), C.byref(p), _ptr(out), ostr, _ptr(lse),
                                _ptr(ws), ws.numel(), _stream(q)))
    return (out, lse) if want_lse else out


def basa_dense_attn(q, k, v, block: int = 128, want_lse: bool = False, ws=None, out=None, causal: bool = False):
    lib = load()
    qd, kd, vd = tensor_desc(q), tensor_desc(k), tensor_desc(v)
    p = params(block, causal=causal)
    b, hq, Lq, d = q.shape
    if out is None:
        out = torch.empty((b, hq, Lq, d), dtype=q.dtype, device=q.device)
    ostr = _out_strides(out, q)
    lse = torch.empty((b, hq, Lq), dtype=torch.float32, device=q.device) if want_lse else None
    if ws is None:
        ws = _ws(lib.basa_attn_workspace_size(C.byref(qd), C.byref(kd), C.byref(p)), q.device)
    _check(lib.basa_dense_attn(C.byref(qd), C.byref(kd), C.byref(vd), C.byref(p), _ptr(out), ostr, _ptr(lse),
                               _ptr(ws), ws.numel(), _stream(q)))
    return (out, lse) if want_lse else out


def ba_att(q, k, v, block: int = 128, sparsity: float = 0.5, beta: float = 1.0, sort: int = SORT_QK,
           window: int = 0, mass_target: float = 0.0, min_keep: int = 0, segments=None, out=None,
           causal: bool = False):
    """The whole operator (Alg. 1): basa_select, then basa_sparse_attn on its lists.  Returns (out, Selection)."""
    sel = basa_select(q, k, block, sparsity, beta, sort, window, want_mask=False, want_mass=False,
                      mass_target=mass_target, min_keep=min_keep, segments=segments, causal=causal)
    o = basa_sparse_attn(q, k, v, sel.row_count, sel.row_cols, block, sel.perm_q, sel.perm_k, out=out, causal=causal)
    return o, sel


def ba_att_varlen(q, k, v, cu_seqlens, block: int = 128, sparsity: float = 0.5, **kw):
    """Sequences of different lengths packed token-major: q [T, heads_q, d], k and v [T, heads_kv, d],
    cu_seqlens the host list [0, t_1, ..., T] of sequence boundaries.  Every sequence is its own
    problem (its own sort, block map and kappa) and runs as one pair of library calls on strided
    views of the packed buffers, reading and writing them in place; the long sequences this method
    is for each fill the device on their own.  Returns the packed output [T, heads_q, d]."""
    out = torch.empty_like(q)
    view = lambda x, a, b: x[a:b].permute(1, 0, 2).unsqueeze(0)          # [1, heads, L, d], no copy
    for a, b in zip(cu_seqlens[:-1], cu_seqlens[1:]):
        a, b = int(a), int(b)
        if b > a:
            ba_att(view(q, a, b), view(k, a, b), view(v, a, b), block, sparsity, out=view(out, a, b), **kw)
    return out


def basa_profile_enable(on: bool):
    _check(load().basa_profile_enable(1 if on else 0))


def basa_profile_read() -> dict:
    """{kernel name: (total milliseconds, launches)} since the last read; waits for the events."""
    lib = load()
    n = int(lib.basa_profile_kernel_count())
    ms = (C.c_double * n)()
    cnt = (C.c_int32 * n)()
    _check(lib.basa_profile_read(ms, cnt, n))
    return {lib.basa_profile_kernel_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}


def basa_calibrate_mfma(random_operands: bool, iters: int, out: torch.Tensor) -> float:
    """Enqueue the matrix-core calibration loop on the current stream; returns its flop count."""
    flops = C.c_double(0.0)
    _check(load().basa_calibrate_mfma(1 if random_operands else 0, int(iters), _ptr(out), out.numel(),
                                      C.byref(flops), _stream(out)))
    return float(flops.value)


# ---------------------------------------------------------------- selection-fidelity diagnostics
def basa_block_mass(q, k, block: int, perm_q=None, perm_k=None, base_logits=None, want_dev: bool = False,
                    want_lse: bool = False, ws=None):
    """m_hat [b, Hq, Nq, Nk] (and max_dev, lse when asked) of the ordered sequences."""
    lib = load()
    qd, kd, p = tensor_desc(q), tensor_desc(k), params(block)
    b, hq, Lq, _ = q.shape
    n_q, n_k = n_blocks(Lq, block), n_blocks(k.shape[2], block)
    m_hat = torch.empty((b, hq, n_q, n_k), dtype=torch.float32, device=q.device)
    dev = torch.empty_like(m_hat) if want_dev else None
    lse = torch.empty((b, hq, Lq), dtype=torch.float32, device=q.device) if want_lse else None
    if ws is None:
        ws = _ws(lib.basa_block_mass_workspace_size(C.byref(qd), C.byref(kd)), q.device)
    _check(lib.basa_block_mass(C.byref(qd), C.byref(kd), _ptr(perm_q), _ptr(perm_k), C.byref(p),
                               _ptr(base_logits), _ptr(m_hat), _ptr(dev), _ptr(lse), _ptr(ws), ws.numel(),
                               _stream(q)))
    return m_hat, dev, lse


def basa_block_radius(x, block: int, perm=None):
    lib = load()
    xd, p = tensor_desc(x), params(block)
    b, h, L, _ = x.shape
    radius = torch.empty((b, h, n_blocks(L, block)), dtype=torch.float32, device=x.device)
    max_norm = torch.empty_like(radius)
    _check(lib.basa_block_radius(C.byref(xd), _ptr(perm), C.byref(p), _ptr(radius), _ptr(max_norm), _stream(x)))
    return radius, max_norm


def basa_deviation_bound(radius_q, max_norm_q, radius_k, max_norm_k, d: int):
    b, hq, n_q = radius_q.shape
    hk, n_k = radius_k.shape[1], radius_k.shape[2]
    bound = torch.empty((b, hq, n_q, n_k), dtype=torch.float32, device=radius_q.device)
    _check(load().basa_deviation_bound(_ptr(radius_q), _ptr(max_norm_q), _ptr(radius_k), _ptr(max_norm_k),
                                       b * hq, b * hk, n_q, n_k, int(d), _ptr(bound), _stream(radius_q)))
    return bound


def basa_selection_fidelity(scores, mask_bits, m_hat):
    """(recall, l1), each [b, Hq, Nq]."""
    n_k = scores.shape[-1]
    rows = scores.numel() // n_k
    recall = torch.empty(scores.shape[:-1], dtype=torch.float32, device=scores.device)
    l1 = torch.empty_like(recall)
    _check(load().basa_selection_fidelity(_ptr(scores), _ptr(mask_bits), _ptr(m_hat), rows, n_k, _ptr(recall),
                                          _ptr(l1), _stream(scores)))
    return recall, l1


def basa_pearson_sums(x, y):
    """Device tensor of the six fp64 sums (n, sx, sy, sxx, syy, sxy) over two float tensors."""
    sums = torch.empty(6, dtype=torch.float64, device=x.device)
    _check(load().basa_pearson_sums(_ptr(x), _ptr(y), x.numel(), _ptr(sums), _stream(x)))
    return sums


def basa_calibrate_read(buf: torch.Tensor, out: torch.Tensor) -> int:
    """Enqueue one read-only pass over `buf` on the current stream; returns the bytes it covers."""
    nbytes = buf.numel() * buf.element_size()
    _check(load().basa_calibrate_read(_ptr(buf), nbytes, _ptr(out), _stream(buf)))
    return nbytes
