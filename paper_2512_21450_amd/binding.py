"""Thin Python binding of the C-ABI library (argument marshalling only).

Every step of the computation runs in the HIP kernels behind
``librl_decode_attn.so``; PyTorch is used for device memory and streams.
There is no CPU fallback: importing this module raises if the library has not
been built (``python -m paper_2512_21450_amd.build``).

Function names mirror ``include/rl_decode_attn.h``.
"""
from __future__ import annotations

import ctypes
import os

# torch first: it brings its own HIP runtime (same soname as the system one), and
# the library must bind to the runtime that owns torch's streams and allocations.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librl_decode_attn.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build the HIP library first (python -m paper_2512_21450_amd.build). "
        "There is no fallback path.")

_lib = ctypes.CDLL(LIB_PATH)

RLDA_F32, RLDA_BF16, RLDA_BF16_KV8 = 0, 1, 2
RLDA_ALGO_AUTO, RLDA_ALGO_SIMPLE, RLDA_ALGO_SHARED = 0, 1, 2
RLDA_OK, RLDA_ERR_INVALID, RLDA_ERR_UNSUPPORTED = 0, -1, -2
RLDA_ERR_WORKSPACE, RLDA_ERR_STRUCT_SIZE, RLDA_ERR_LAUNCH = -3, -4, -5


class rlda_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("algo", ctypes.c_int32),
        ("P", ctypes.c_int32), ("G", ctypes.c_int32),
        ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("Lp_cap", ctypes.c_int32), ("Ls_cap", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("q", ctypes.c_void_p),
        ("k_prefix", ctypes.c_void_p), ("v_prefix", ctypes.c_void_p), ("prefix_lens", ctypes.c_void_p),
        ("k_suffix", ctypes.c_void_p), ("v_suffix", ctypes.c_void_p), ("suffix_lens", ctypes.c_void_p),
        ("out", ctypes.c_void_p), ("lse", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
    ]


class rlda_paged_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("algo", ctypes.c_int32),
        ("P", ctypes.c_int32), ("G", ctypes.c_int32),
        ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("Lp_cap", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32), ("n_pages", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("q", ctypes.c_void_p),
        ("k_prefix", ctypes.c_void_p), ("v_prefix", ctypes.c_void_p), ("prefix_lens", ctypes.c_void_p),
        ("k_pages", ctypes.c_void_p), ("v_pages", ctypes.c_void_p), ("block_table", ctypes.c_void_p),
        ("suffix_lens", ctypes.c_void_p), ("seq_active", ctypes.c_void_p),
        ("out", ctypes.c_void_p), ("lse", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
    ]


RLDA_MAX_TREE_LEVELS = 4


class rlda_tree_level(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("lens", ctypes.c_void_p),
                ("group", ctypes.c_int32), ("cap", ctypes.c_int32)]


class rlda_tree_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("B", ctypes.c_int32),
        ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("n_levels", ctypes.c_int32),
        ("Ls_cap", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("levels", rlda_tree_level * RLDA_MAX_TREE_LEVELS),
        ("q", ctypes.c_void_p),
        ("k_suffix", ctypes.c_void_p), ("v_suffix", ctypes.c_void_p), ("suffix_lens", ctypes.c_void_p),
        ("out", ctypes.c_void_p), ("lse", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
    ]


_dp = ctypes.POINTER(rlda_desc)
_tp = ctypes.POINTER(rlda_tree_desc)
_lib.rl_decode_attn_tree.restype = ctypes.c_int
_lib.rl_decode_attn_tree.argtypes = [_tp, ctypes.c_void_p]
_lib.rl_decode_attn_tree_workspace_bytes.restype = ctypes.c_size_t
_lib.rl_decode_attn_tree_workspace_bytes.argtypes = [_tp]
_pp = ctypes.POINTER(rlda_paged_desc)
_lib.rl_decode_attn_paged.restype = ctypes.c_int
_lib.rl_decode_attn_paged.argtypes = [_pp, ctypes.c_void_p, ctypes.c_void_p]
_lib.rl_decode_attn_paged_workspace_bytes.restype = ctypes.c_size_t
_lib.rl_decode_attn_paged_workspace_bytes.argtypes = [_pp]
_lib.rl_decode_attn_paged_plan.restype = ctypes.c_int
_lib.rl_decode_attn_paged_plan.argtypes = [_pp]
_lib.rl_decode_attn.restype = ctypes.c_int
_lib.rl_decode_attn.argtypes = [_dp, ctypes.c_void_p]
_lib.rl_decode_attn_static.restype = ctypes.c_int
_lib.rl_decode_attn_static.argtypes = [_dp, ctypes.c_void_p]
_lib.rl_decode_attn_static_workspace_limit.restype = ctypes.c_size_t
_lib.rl_decode_attn_static_workspace_limit.argtypes = []
_lib.rl_decode_attn_profiled.restype = ctypes.c_int
_lib.rl_decode_attn_profiled.argtypes = [_dp, ctypes.c_void_p, ctypes.c_void_p]
_lib.rl_decode_attn_workspace_bytes.restype = ctypes.c_size_t
_lib.rl_decode_attn_workspace_bytes.argtypes = [_dp]
_lib.rl_decode_attn_plan.restype = ctypes.c_int
_lib.rl_decode_attn_plan.argtypes = [_dp]
_lib.rl_decode_attn_strerror.restype = ctypes.c_char_p
_lib.rl_decode_attn_strerror.argtypes = [ctypes.c_int]
_lib.rl_decode_attn_version.restype = ctypes.c_int
_lib.rl_decode_attn_version.argtypes = []
_lib.rl_decode_attn_last_hip_error.restype = ctypes.c_char_p
_lib.rl_decode_attn_last_hip_error.argtypes = []
_lib.rl_lse_combine.restype = ctypes.c_int
_lib.rl_lse_combine.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                                ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]


class RldaError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        detail = f" ({rl_decode_attn_last_hip_error()})" if code == RLDA_ERR_LAUNCH else ""
        super().__init__(f"rl_decode_attn error {code}: {rl_decode_attn_strerror(code)}{detail}")


def make_desc(dtype, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, scale, algo=RLDA_ALGO_AUTO, **ptrs) -> rlda_desc:
    """Fill a descriptor from plain integers; pointer fields default to NULL."""
    ds = rlda_desc()
    ds.struct_size = ctypes.sizeof(rlda_desc)
    ds.dtype, ds.algo = dtype, algo
    ds.P, ds.G, ds.Hq, ds.Hkv, ds.d, ds.Lp_cap, ds.Ls_cap = P, G, Hq, Hkv, d, Lp_cap, Ls_cap
    ds.scale = scale
    for k, v in ptrs.items():
        setattr(ds, k, v)
    return ds


def rl_decode_attn_version() -> int:
    return _lib.rl_decode_attn_version()


def rl_decode_attn_strerror(code: int) -> str:
    return _lib.rl_decode_attn_strerror(code).decode()


def rl_decode_attn_last_hip_error() -> str:
    return _lib.rl_decode_attn_last_hip_error().decode()


def rl_decode_attn_workspace_bytes(desc: rlda_desc) -> int:
    return _lib.rl_decode_attn_workspace_bytes(ctypes.byref(desc))


def rl_decode_attn_plan(desc: rlda_desc) -> int:
    return _lib.rl_decode_attn_plan(ctypes.byref(desc))


def rl_decode_attn_raw(desc: rlda_desc, stream_handle=None) -> int:
    """Direct call; returns the C return code."""
    return _lib.rl_decode_attn(ctypes.byref(desc), stream_handle)


def rl_decode_attn_profiled(desc: rlda_desc, stream_handle, mid_event_handle) -> int:
    """Direct call that also records ``mid_event_handle`` after the K/V-streaming kernel."""
    return _lib.rl_decode_attn_profiled(ctypes.byref(desc), stream_handle, mid_event_handle)


def rl_decode_attn_static_raw(desc: rlda_desc, stream_handle=None) -> int:
    """Direct call of the entry point that uses the library's own scratch array; returns the C return code."""
    return _lib.rl_decode_attn_static(ctypes.byref(desc), stream_handle)


def rl_decode_attn_static_workspace_limit() -> int:
    return _lib.rl_decode_attn_static_workspace_limit()


def _torch_dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return RLDA_F32
    if t.dtype == torch.bfloat16:
        return RLDA_BF16
    raise TypeError(f"q/k/v must be float32 or bfloat16, got {t.dtype}")


def _kv_dtype_code(q, stores, k_scale, v_scale):
    """Descriptor dtype for q and its K/V stores; e4m3 stores are uint8 (or torch.float8_e4m3fn) tensors."""
    import torch
    code = _torch_dtype_code(q)
    kv8 = [t.dtype in (torch.uint8, torch.float8_e4m3fn) for t in stores]
    if all(kv8):
        if code != RLDA_BF16:
            raise TypeError("e4m3 K/V stores go with a bfloat16 q")
        for sc in (k_scale, v_scale):
            if sc is not None and (sc.dtype != torch.float32 or sc.numel() != stores[0].shape[1] or not sc.is_contiguous()):
                raise TypeError("k_scale / v_scale must be contiguous float32 [Hkv]")
        return RLDA_BF16_KV8
    if any(kv8) or any(_torch_dtype_code(t) != code for t in stores):
        raise TypeError("q/k/v dtypes differ")
    if k_scale is not None or v_scale is not None:
        raise TypeError("k_scale / v_scale belong to e4m3 K/V stores")
    return code


def _check_lens(t, n, name, like):
    """A length array as the kernels read it: int32, n entries, contiguous, on q's device."""
    import torch
    if t.dtype != torch.int32:
        raise TypeError(f"{name} must be int32 (got {t.dtype}): the kernels read 4-byte lengths")
    if t.numel() != n or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous array of {n} lengths (got shape {tuple(t.shape)})")
    if t.device != like.device:
        raise ValueError(f"{name} is on {t.device}, q on {like.device}")


def _check_outputs(q, out, lse):
    """out [B, Hq, d] and lse [B, Hq] (optional) as the kernels write them: float32, contiguous, on q's device."""
    import torch
    B, Hq, d = q.shape
    for t, shape, name in ((out, (B, Hq, d), "out"), (lse, (B, Hq), "lse")):
        if t is None:
            if name == "out":
                raise ValueError("out is required")
            continue
        if t.dtype != torch.float32:
            raise TypeError(f"{name} must be float32 (got {t.dtype})")
        if tuple(t.shape) != shape or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous tensor of shape {shape} (got {tuple(t.shape)})")
        if t.device != q.device:
            raise ValueError(f"{name} is on {t.device}, q on {q.device}")


def _check_stores(q, pairs):
    """every (K store, V store) pair: equal shapes, contiguous, on q's device"""
    for k, v, name in pairs:
        if k.shape != v.shape:
            raise ValueError(f"v_{name} has shape {tuple(v.shape)}, k_{name} {tuple(k.shape)}")
        for t in (k, v):
            if not t.is_contiguous():
                raise ValueError("tensors must be contiguous")
            if t.device != q.device:
                raise ValueError(f"a {name} store is on {t.device}, q on {q.device}")


def desc_from_tensors(q, k_prefix, v_prefix, prefix_lens, k_suffix, v_suffix, suffix_lens, scale, G,
                      out, lse=None, workspace=None, algo=RLDA_ALGO_AUTO, k_scale=None, v_scale=None) -> rlda_desc:
    """Descriptor over torch device tensors (shapes as in the header)."""
    B, Hq, d = q.shape
    P, Hkv, Lp_cap, _ = k_prefix.shape
    Ls_cap = k_suffix.shape[2]
    if B != P * G or k_suffix.shape[0] != B or k_suffix.shape[1] != Hkv:
        raise ValueError("inconsistent shapes")
    if not q.is_contiguous():
        raise ValueError("tensors must be contiguous")
    _check_stores(q, ((k_prefix, v_prefix, "prefix"), (k_suffix, v_suffix, "suffix")))
    _check_lens(prefix_lens, P, "prefix_lens", q)
    _check_lens(suffix_lens, B, "suffix_lens", q)
    _check_outputs(q, out, lse)
    code = _kv_dtype_code(q, (k_prefix, v_prefix, k_suffix, v_suffix), k_scale, v_scale)
    ptr = lambda t: None if t is None or t.numel() == 0 else t.data_ptr()
    return make_desc(code, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, float(scale), algo,
                     q=ptr(q), k_prefix=ptr(k_prefix), v_prefix=ptr(v_prefix), prefix_lens=ptr(prefix_lens),
                     k_suffix=ptr(k_suffix), v_suffix=ptr(v_suffix), suffix_lens=ptr(suffix_lens),
                     out=ptr(out), lse=ptr(lse), workspace=ptr(workspace),
                     workspace_bytes=0 if workspace is None else workspace.numel() * workspace.element_size(),
                     k_scale=ptr(k_scale), v_scale=ptr(v_scale))


def rl_decode_attn(q, k_prefix, v_prefix, prefix_lens, k_suffix, v_suffix, suffix_lens, scale, G,
                   out=None, lse=None, workspace=None, algo=RLDA_ALGO_AUTO, stream=None, k_scale=None, v_scale=None):
    """One decode-attention step on torch device tensors; returns (out, lse).

    Allocates out/lse/workspace with torch when they are not passed in.  The
    call is asynchronous on ``stream`` (default: torch's current stream).
    """
    import torch
    if not q.is_cuda:
        raise RuntimeError("rl_decode_attn needs device tensors; there is no CPU path")
    B, Hq, d = q.shape
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty((B, Hq), dtype=torch.float32, device=q.device)
    ds = desc_from_tensors(q, k_prefix, v_prefix, prefix_lens, k_suffix, v_suffix, suffix_lens, scale, G,
                           out, lse, workspace, algo, k_scale, v_scale)
    if workspace is None:
        need = rl_decode_attn_workspace_bytes(ds)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
            ds.workspace, ds.workspace_bytes = workspace.data_ptr(), need
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    rc = _lib.rl_decode_attn(ctypes.byref(ds), ctypes.c_void_p(s.cuda_stream))
    if rc != RLDA_OK:
        raise RldaError(rc)
    return out, lse


def rl_decode_attn_static(q, k_prefix, v_prefix, prefix_lens, k_suffix, v_suffix, suffix_lens, scale, G,
                          out, lse=None, algo=RLDA_ALGO_AUTO, stream=None, k_scale=None, v_scale=None):
    """rl_decode_attn without any allocation: ``out`` (and ``lse``) are the caller's, the scratch is the library's."""
    import torch
    if not q.is_cuda:
        raise RuntimeError("rl_decode_attn_static needs device tensors; there is no CPU path")
    ds = desc_from_tensors(q, k_prefix, v_prefix, prefix_lens, k_suffix, v_suffix, suffix_lens, scale, G,
                           out, lse, None, algo, k_scale, v_scale)
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    rc = _lib.rl_decode_attn_static(ctypes.byref(ds), ctypes.c_void_p(s.cuda_stream))
    if rc != RLDA_OK:
        raise RldaError(rc)
    return out, lse


def make_tree_desc(dtype, B, Hq, Hkv, d, Ls_cap, scale, levels=(), **ptrs) -> rlda_tree_desc:
    """Fill a tree descriptor from plain integers; ``levels``: (k_ptr, v_ptr, lens_ptr, group, cap) per level."""
    ds = rlda_tree_desc()
    ds.struct_size = ctypes.sizeof(rlda_tree_desc)
    ds.dtype, ds.B, ds.Hq, ds.Hkv, ds.d, ds.Ls_cap, ds.scale = dtype, B, Hq, Hkv, d, Ls_cap, scale
    ds.n_levels = len(levels)
    for i, (k, v, lens, group, cap) in enumerate(levels[:RLDA_MAX_TREE_LEVELS]):
        ds.levels[i].k, ds.levels[i].v, ds.levels[i].lens = k, v, lens
        ds.levels[i].group, ds.levels[i].cap = group, cap
    for k, v in ptrs.items():
        setattr(ds, k, v)
    return ds


def rl_decode_attn_tree_workspace_bytes(desc: rlda_tree_desc) -> int:
    return _lib.rl_decode_attn_tree_workspace_bytes(ctypes.byref(desc))


def rl_decode_attn_tree_raw(desc: rlda_tree_desc, stream_handle=None) -> int:
    """Direct call; returns the C return code."""
    return _lib.rl_decode_attn_tree(ctypes.byref(desc), stream_handle)


def tree_desc_from_tensors(q, levels, k_suffix, v_suffix, suffix_lens, scale, out, lse=None, workspace=None) -> rlda_tree_desc:
    """Tree descriptor over torch device tensors.  ``levels``: list of (k [n_seg, Hkv, cap, d], v, lens [n_seg],
    group) with n_seg * group == B."""
    B, Hq, d = q.shape
    Hkv, Ls_cap = k_suffix.shape[1], k_suffix.shape[2]
    if len(levels) > RLDA_MAX_TREE_LEVELS:
        raise ValueError(f"at most {RLDA_MAX_TREE_LEVELS} shared levels")
    if k_suffix.shape[0] != B or not q.is_contiguous():
        raise ValueError("inconsistent shapes")
    pairs = [(k_suffix, v_suffix, "suffix")]
    lv = []
    ptr = lambda t: None if t is None or t.numel() == 0 else t.data_ptr()
    for i, (k, v, lens, group) in enumerate(levels):
        if group < 1 or B % group or k.shape[0] * group != B or k.shape[1] != Hkv or k.shape[3] != d:
            raise ValueError(f"level {i}: {tuple(k.shape)} stores with groups of {group} do not cover {B} sequences")
        pairs.append((k, v, f"level {i}"))
        _check_lens(lens, B // group, f"lens of level {i}", q)
        lv.append((ptr(k), ptr(v), ptr(lens), int(group), int(k.shape[2])))
    _check_stores(q, pairs)
    _check_lens(suffix_lens, B, "suffix_lens", q)
    _check_outputs(q, out, lse)
    code = _kv_dtype_code(q, [t for k, v, _ in pairs for t in (k, v)], None, None)
    return make_tree_desc(code, B, Hq, Hkv, d, Ls_cap, float(scale), lv, q=ptr(q), k_suffix=ptr(k_suffix),
                          v_suffix=ptr(v_suffix), suffix_lens=ptr(suffix_lens), out=ptr(out), lse=ptr(lse),
                          workspace=ptr(workspace),
                          workspace_bytes=0 if workspace is None else workspace.numel() * workspace.element_size())


def rl_decode_attn_tree(q, levels, k_suffix, v_suffix, suffix_lens, scale, out=None, lse=None, workspace=None, stream=None):
    """One decode step over a tree of shared prefix segments plus the own suffixes; returns (out, lse)."""
    import torch
    if not q.is_cuda:
        raise RuntimeError("rl_decode_attn_tree needs device tensors; there is no CPU path")
    B, Hq, d = q.shape
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty((B, Hq), dtype=torch.float32, device=q.device)
    ds = tree_desc_from_tensors(q, levels, k_suffix, v_suffix, suffix_lens, scale, out, lse, workspace)
    if workspace is None:
        need = rl_decode_attn_tree_workspace_bytes(ds)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
        ds.workspace, ds.workspace_bytes = workspace.data_ptr(), workspace.numel()
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    rc = _lib.rl_decode_attn_tree(ctypes.byref(ds), ctypes.c_void_p(s.cuda_stream))
    if rc != RLDA_OK:
        raise RldaError(rc)
    return out, lse


def make_paged_desc(dtype, P, G, Hq, Hkv, d, Lp_cap, page_size, max_pages, n_pages, scale,
                    algo=RLDA_ALGO_AUTO, **ptrs) -> rlda_paged_desc:
    """Fill a paged descriptor from plain integers; pointer fields default to NULL."""
    ds = rlda_paged_desc()
    ds.struct_size = ctypes.sizeof(rlda_paged_desc)
    ds.dtype, ds.algo = dtype, algo
    ds.P, ds.G, ds.Hq, ds.Hkv, ds.d, ds.Lp_cap = P, G, Hq, Hkv, d, Lp_cap
    ds.page_size, ds.max_pages, ds.n_pages = page_size, max_pages, n_pages
    ds.scale = scale
    for k, v in ptrs.items():
        setattr(ds, k, v)
    return ds


def rl_decode_attn_paged_workspace_bytes(desc: rlda_paged_desc) -> int:
    return _lib.rl_decode_attn_paged_workspace_bytes(ctypes.byref(desc))


def rl_decode_attn_paged_plan(desc: rlda_paged_desc) -> int:
    return _lib.rl_decode_attn_paged_plan(ctypes.byref(desc))


def rl_decode_attn_paged_raw(desc: rlda_paged_desc, stream_handle=None, mid_event_handle=None) -> int:
    """Direct call; returns the C return code."""
    return _lib.rl_decode_attn_paged(ctypes.byref(desc), stream_handle, mid_event_handle)


def paged_desc_from_tensors(q, k_prefix, v_prefix, prefix_lens, k_pages, v_pages, block_table, suffix_lens,
                            scale, G, out, lse=None, seq_active=None, workspace=None,
                            algo=RLDA_ALGO_AUTO, k_scale=None, v_scale=None) -> rlda_paged_desc:
    """Paged descriptor over torch device tensors (shapes as in the header)."""
    import torch
    B, Hq, d = q.shape
    P, Hkv, Lp_cap, _ = k_prefix.shape
    n_pages, Hkv2, page_size, _ = k_pages.shape
    if B != P * G or Hkv2 != Hkv or block_table.shape[0] != B or k_pages.shape != v_pages.shape:
        raise ValueError("inconsistent shapes")
    if block_table.dtype != torch.int32 or (seq_active is not None and seq_active.dtype != torch.uint8):
        raise TypeError("block_table must be int32 and seq_active uint8")
    if seq_active is not None and (seq_active.numel() != B or not seq_active.is_contiguous()):
        raise ValueError(f"seq_active must hold one byte per sequence ({B})")
    for t in (q, block_table):
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")
    _check_stores(q, ((k_prefix, v_prefix, "prefix"), (k_pages, v_pages, "pages")))
    _check_lens(prefix_lens, P, "prefix_lens", q)
    _check_lens(suffix_lens, B, "suffix_lens", q)
    _check_outputs(q, out, lse)
    code = _kv_dtype_code(q, (k_prefix, v_prefix, k_pages, v_pages), k_scale, v_scale)
    ptr = lambda t: None if t is None or t.numel() == 0 else t.data_ptr()
    return make_paged_desc(code, P, G, Hq, Hkv, d, Lp_cap, page_size, block_table.shape[1], n_pages, float(scale),
                           algo, q=ptr(q), k_prefix=ptr(k_prefix), v_prefix=ptr(v_prefix),
                           prefix_lens=ptr(prefix_lens), k_pages=ptr(k_pages), v_pages=ptr(v_pages),
                           block_table=ptr(block_table), suffix_lens=ptr(suffix_lens), seq_active=ptr(seq_active),
                           out=ptr(out), lse=ptr(lse), workspace=ptr(workspace),
                           workspace_bytes=0 if workspace is None else workspace.numel() * workspace.element_size(),
                           k_scale=ptr(k_scale), v_scale=ptr(v_scale))


def rl_decode_attn_paged(q, k_prefix, v_prefix, prefix_lens, k_pages, v_pages, block_table, suffix_lens, scale, G,
                         seq_active=None, out=None, lse=None, workspace=None, algo=RLDA_ALGO_AUTO, stream=None,
                         k_scale=None, v_scale=None):
    """One decode step over a paged suffix store; returns (out, lse).  Asynchronous on ``stream``."""
    import torch
    if not q.is_cuda:
        raise RuntimeError("rl_decode_attn_paged needs device tensors; there is no CPU path")
    B, Hq, d = q.shape
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty((B, Hq), dtype=torch.float32, device=q.device)
    ds = paged_desc_from_tensors(q, k_prefix, v_prefix, prefix_lens, k_pages, v_pages, block_table, suffix_lens,
                                 scale, G, out, lse, seq_active, workspace, algo, k_scale, v_scale)
    if workspace is None:
        need = rl_decode_attn_paged_workspace_bytes(ds)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
            ds.workspace, ds.workspace_bytes = workspace.data_ptr(), need
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    rc = _lib.rl_decode_attn_paged(ctypes.byref(ds), ctypes.c_void_p(s.cuda_stream), None)
    if rc != RLDA_OK:
        raise RldaError(rc)
    return out, lse


def rl_lse_combine(o_parts, lse_parts, out=None, lse=None, stream=None):
    """Merge partials o_parts [n_parts, n_rows, d], lse_parts [n_parts, n_rows] (fp32 device tensors)."""
    import torch
    n_parts, n_rows, d = o_parts.shape
    if out is None:
        out = torch.empty((n_rows, d), dtype=torch.float32, device=o_parts.device)
    if lse is None:
        lse = torch.empty((n_rows,), dtype=torch.float32, device=o_parts.device)
    s = stream if stream is not None else torch.cuda.current_stream(o_parts.device)
    rc = _lib.rl_lse_combine(o_parts.data_ptr(), lse_parts.data_ptr(), n_parts, n_rows, d,
                             out.data_ptr(), lse.data_ptr(), ctypes.c_void_p(s.cuda_stream))
    if rc != RLDA_OK:
        raise RldaError(rc)
    return out, lse


# ---------------------------------------------------------------- rl_token_logprob.h
class rl_token_logprob_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("n_rows", ctypes.c_int64),
        ("row_stride", ctypes.c_int64),
        ("vocab", ctypes.c_int32),
        ("inv_temperature", ctypes.c_float),
        ("logits", ctypes.c_void_p), ("ref_logits", ctypes.c_void_p), ("token_ids", ctypes.c_void_p),
        ("logprob", ctypes.c_void_p), ("lse", ctypes.c_void_p), ("entropy", ctypes.c_void_p),
        ("ref_logprob", ctypes.c_void_p), ("kl", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
    ]


_tp = ctypes.POINTER(rl_token_logprob_desc)
_lib.rl_token_logprob.restype = ctypes.c_int
_lib.rl_token_logprob.argtypes = [_tp, ctypes.c_void_p]
_lib.rl_token_logprob_workspace_bytes.restype = ctypes.c_size_t
_lib.rl_token_logprob_workspace_bytes.argtypes = [_tp]


def make_token_logprob_desc(dtype, n_rows, vocab, row_stride, inv_temperature=1.0, **ptrs) -> rl_token_logprob_desc:
    ds = rl_token_logprob_desc()
    ds.struct_size = ctypes.sizeof(rl_token_logprob_desc)
    ds.dtype, ds.n_rows, ds.vocab, ds.row_stride, ds.inv_temperature = dtype, n_rows, vocab, row_stride, inv_temperature
    for k, v in ptrs.items():
        setattr(ds, k, v)
    return ds


def rl_token_logprob_workspace_bytes(desc: rl_token_logprob_desc) -> int:
    return _lib.rl_token_logprob_workspace_bytes(ctypes.byref(desc))


def rl_token_logprob_raw(desc: rl_token_logprob_desc, stream_handle=None) -> int:
    return _lib.rl_token_logprob(ctypes.byref(desc), stream_handle)


_TOKEN_OUTPUTS = ("logprob", "lse", "entropy", "ref_logprob", "kl")


def token_logprob_desc_from_tensors(logits, token_ids, inv_temperature=1.0, ref_logits=None, outputs=None,
                                    workspace=None) -> rl_token_logprob_desc:
    """Descriptor over torch device tensors: logits [n_rows, vocab] (a row-strided view is fine),
    token_ids [n_rows] int32, outputs: dict name -> fp32 tensor [n_rows]."""
    import torch
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be [n_rows, vocab] with unit stride along the vocabulary")
    if token_ids.dtype != torch.int32 or not token_ids.is_contiguous():
        raise TypeError("token_ids must be contiguous int32")
    code = _torch_dtype_code(logits)
    if ref_logits is not None and (ref_logits.shape != logits.shape or ref_logits.stride() != logits.stride()
                                   or ref_logits.dtype != logits.dtype):
        raise ValueError("ref_logits must match logits in shape, strides and dtype")
    n, V = logits.shape
    ptr = lambda t: None if t is None or t.numel() == 0 else t.data_ptr()
    outs = {k: ptr(v) for k, v in (outputs or {}).items()}
    unknown = set(outs) - set(_TOKEN_OUTPUTS)
    if unknown:
        raise KeyError(f"unknown outputs {sorted(unknown)}")
    return make_token_logprob_desc(code, n, V, logits.stride(0) if n > 1 else max(logits.stride(0), V),
                                   float(inv_temperature), logits=ptr(logits), ref_logits=ptr(ref_logits),
                                   token_ids=ptr(token_ids), workspace=ptr(workspace),
                                   workspace_bytes=0 if workspace is None else workspace.numel(), **outs)


def rl_token_logprob(logits, token_ids, inv_temperature=1.0, ref_logits=None, want=None, workspace=None,
                     stream=None) -> dict:
    """Per-token log-prob / lse / entropy (and ref_logprob / kl with ``ref_logits``); returns a dict of
    fp32 device tensors [n_rows].  Asynchronous on ``stream``."""
    import torch
    if not logits.is_cuda:
        raise RuntimeError("rl_token_logprob needs device tensors; there is no CPU path")
    names = want or (_TOKEN_OUTPUTS if ref_logits is not None else _TOKEN_OUTPUTS[:3])
    outs = {k: torch.empty(logits.shape[0], dtype=torch.float32, device=logits.device) for k in names}
    ds = token_logprob_desc_from_tensors(logits, token_ids, inv_temperature, ref_logits, outs, workspace)
    if workspace is None:
        need = rl_token_logprob_workspace_bytes(ds)
        if need:
            workspace = torch.empty(need, dtype=torch.uint8, device=logits.device)
            ds.workspace, ds.workspace_bytes = workspace.data_ptr(), need
    s = stream if stream is not None else torch.cuda.current_stream(logits.device)
    rc = _lib.rl_token_logprob(ctypes.byref(ds), ctypes.c_void_p(s.cuda_stream))
    if rc != RLDA_OK:
        raise RldaError(rc)
    return outs


# ---------------------------------------------------------------- rl_kv_append.h
class rl_kv_append_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("Ls_cap", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32), ("n_pages", ctypes.c_int32),
        ("sections", ctypes.c_int32 * 3),
        ("q", ctypes.c_void_p), ("k_new", ctypes.c_void_p), ("v_new", ctypes.c_void_p),
        ("positions", ctypes.c_void_p), ("inv_freq", ctypes.c_void_p),
        ("k_store", ctypes.c_void_p), ("v_store", ctypes.c_void_p),
        ("block_table", ctypes.c_void_p), ("suffix_lens", ctypes.c_void_p), ("seq_active", ctypes.c_void_p),
        ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
    ]


_lib.rl_kv_append_rope.restype = ctypes.c_int
_lib.rl_kv_append_rope.argtypes = [ctypes.POINTER(rl_kv_append_desc), ctypes.c_void_p]


def make_kv_append_desc(dtype, B, Hq, Hkv, d, sections, Ls_cap=0, page_size=0, max_pages=0, n_pages=0,
                        **ptrs) -> rl_kv_append_desc:
    ds = rl_kv_append_desc()
    ds.struct_size = ctypes.sizeof(rl_kv_append_desc)
    ds.dtype, ds.B, ds.Hq, ds.Hkv, ds.d, ds.Ls_cap = dtype, B, Hq, Hkv, d, Ls_cap
    ds.page_size, ds.max_pages, ds.n_pages = page_size, max_pages, n_pages
    ds.sections[:] = list(sections)
    for k, v in ptrs.items():
        setattr(ds, k, v)
    return ds


def rl_kv_append_rope_raw(desc: rl_kv_append_desc, stream_handle=None) -> int:
    return _lib.rl_kv_append_rope(ctypes.byref(desc), stream_handle)


def kv_append_desc_from_tensors(q, k_new, v_new, positions, inv_freq, sections, k_store, v_store, suffix_lens,
                                block_table=None, seq_active=None, k_scale=None, v_scale=None) -> rl_kv_append_desc:
    """Descriptor over torch device tensors.  ``k_store`` / ``v_store`` are [B, Hkv, Ls_cap, d], or with
    ``block_table`` the page pools [n_pages, Hkv, page_size, d]; uint8 / float8_e4m3fn stores take e4m3
    bytes quantised with the factors ``k_scale`` / ``v_scale`` (float32 [Hkv])."""
    import torch
    B, Hq, d = q.shape
    Hkv = k_new.shape[1]
    code = _torch_dtype_code(q)
    for t in (k_new, v_new):
        if _torch_dtype_code(t) != code:
            raise TypeError("q, k_new and v_new must share one element type")
    if _kv_dtype_code(q, (k_store, v_store), k_scale, v_scale) == RLDA_BF16_KV8:
        code = 2
    if positions.dtype != torch.int32 or tuple(positions.shape) != (3, B) or inv_freq.dtype != torch.float32:
        raise TypeError("positions must be int32 [3, B] and inv_freq float32 [d/2]")
    if suffix_lens.dtype != torch.int32 or (block_table is not None and block_table.dtype != torch.int32):
        raise TypeError("suffix_lens / block_table must be int32")
    for t in (q, k_new, v_new, positions, inv_freq, k_store, v_store, suffix_lens):
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")
    ptr = lambda t: None if t is None or t.numel() == 0 else t.data_ptr()
    kw = dict(q=ptr(q), k_new=ptr(k_new), v_new=ptr(v_new), positions=ptr(positions), inv_freq=ptr(inv_freq),
              k_store=ptr(k_store), v_store=ptr(v_store), block_table=ptr(block_table),
              suffix_lens=ptr(suffix_lens), seq_active=ptr(seq_active), k_scale=ptr(k_scale), v_scale=ptr(v_scale))
    if block_table is None:
        if tuple(k_store.shape[:2]) != (B, Hkv):
            raise ValueError("contiguous store must be [B, Hkv, Ls_cap, d]")
        return make_kv_append_desc(code, B, Hq, Hkv, d, sections, Ls_cap=k_store.shape[2], **kw)
    return make_kv_append_desc(code, B, Hq, Hkv, d, sections, page_size=k_store.shape[2],
                               max_pages=block_table.shape[1], n_pages=k_store.shape[0], **kw)


def rl_kv_append_rope(q, k_new, v_new, positions, inv_freq, sections, k_store, v_store, suffix_lens,
                      block_table=None, seq_active=None, stream=None, k_scale=None, v_scale=None) -> None:
    """Rotate q (in place) and k_new, append k / v to the store, increment suffix_lens.  Asynchronous."""
    import torch
    if not q.is_cuda:
        raise RuntimeError("rl_kv_append_rope needs device tensors; there is no CPU path")
    ds = kv_append_desc_from_tensors(q, k_new, v_new, positions, inv_freq, sections, k_store, v_store, suffix_lens,
                                     block_table, seq_active, k_scale, v_scale)
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    rc = _lib.rl_kv_append_rope(ctypes.byref(ds), ctypes.c_void_p(s.cuda_stream))
    if rc != RLDA_OK:
        raise RldaError(rc)


# ---------------------------------------------------------------- rl_policy_loss.h
RL_ADV_GROUP_NORM, RL_ADV_GROUP_CENTER, RL_ADV_LEAVE_ONE_OUT = 0, 1, 2
RL_PG_PPO_CLIP, RL_PG_AS_PRINTED = 0, 1
RL_AGG_TOKEN_MEAN, RL_AGG_SEQ_MEAN = 0, 1
POLICY_LOSS_STATS = ("loss", "pg", "kl", "entropy", "clip_frac", "ratio_mean", "approx_kl", "n_tokens")


class rl_group_advantage_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("mode", ctypes.c_int32),
        ("P", ctypes.c_int32), ("G", ctypes.c_int32),
        ("n_metrics", ctypes.c_int32),
        ("unbiased", ctypes.c_int32),
        ("eps", ctypes.c_float),
        ("metrics", ctypes.c_void_p), ("weights", ctypes.c_void_p),
        ("rewards", ctypes.c_void_p), ("advantages", ctypes.c_void_p),
    ]


class rl_policy_loss_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("form", ctypes.c_int32), ("agg", ctypes.c_int32),
        ("B", ctypes.c_int32), ("T", ctypes.c_int32),
        ("row_stride", ctypes.c_int64),
        ("clip_low", ctypes.c_float), ("clip_high", ctypes.c_float),
        ("beta_kl", ctypes.c_float), ("beta_ent", ctypes.c_float),
        ("logprob", ctypes.c_void_p), ("old_logprob", ctypes.c_void_p), ("advantages", ctypes.c_void_p),
        ("kl", ctypes.c_void_p), ("entropy", ctypes.c_void_p), ("lens", ctypes.c_void_p),
        ("grad_logprob", ctypes.c_void_p), ("stats", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
    ]


_lib.rl_group_advantage.restype = ctypes.c_int
_lib.rl_group_advantage.argtypes = [ctypes.POINTER(rl_group_advantage_desc), ctypes.c_void_p]
_lib.rl_policy_loss.restype = ctypes.c_int
_lib.rl_policy_loss.argtypes = [ctypes.POINTER(rl_policy_loss_desc), ctypes.c_void_p]
_lib.rl_policy_loss_workspace_bytes.restype = ctypes.c_size_t
_lib.rl_policy_loss_workspace_bytes.argtypes = [ctypes.POINTER(rl_policy_loss_desc)]


def make_group_advantage_desc(P, G, n_metrics, mode=RL_ADV_GROUP_NORM, eps=1e-6, unbiased=1, **ptrs):
    ds = rl_group_advantage_desc()
    ds.struct_size = ctypes.sizeof(rl_group_advantage_desc)
    ds.mode, ds.P, ds.G, ds.n_metrics, ds.unbiased, ds.eps = mode, P, G, n_metrics, unbiased, eps
    for k, v in ptrs.items():
        setattr(ds, k, v)
    return ds


def rl_group_advantage_raw(desc: rl_group_advantage_desc, stream_handle=None) -> int:
    return _lib.rl_group_advantage(ctypes.byref(desc), stream_handle)


def rl_group_advantage(metrics, weights, G, mode=RL_ADV_GROUP_NORM, eps=1e-6, unbiased=True, stream=None):
    """metrics [M, B], weights [M] (float32 device tensors) -> (rewards [B], advantages [B]).  Asynchronous."""
    import torch
    if not metrics.is_cuda:
        raise RuntimeError("rl_group_advantage needs device tensors; there is no CPU path")
    if metrics.dtype != torch.float32 or weights.dtype != torch.float32 or not metrics.is_contiguous():
        raise TypeError("metrics / weights must be contiguous float32")
    M, Bn = metrics.shape
    if Bn % G or weights.numel() != M:
        raise ValueError("inconsistent shapes")
    rewards = torch.empty(Bn, dtype=torch.float32, device=metrics.device)
    adv = torch.empty(Bn, dtype=torch.float32, device=metrics.device)
    ds = make_group_advantage_desc(Bn // G, G, M, mode, float(eps), int(bool(unbiased)), metrics=metrics.data_ptr(),
                                   weights=weights.data_ptr(), rewards=rewards.data_ptr(), advantages=adv.data_ptr())
    s = stream if stream is not None else torch.cuda.current_stream(metrics.device)
    rc = _lib.rl_group_advantage(ctypes.byref(ds), ctypes.c_void_p(s.cuda_stream))
    if rc != RLDA_OK:
        raise RldaError(rc)
    return rewards, adv


def make_policy_loss_desc(B, T, row_stride, clip_low, clip_high, beta_kl=0.0, beta_ent=0.0, form=RL_PG_PPO_CLIP,
                          agg=RL_AGG_TOKEN_MEAN, **ptrs) -> rl_policy_loss_desc:
    ds = rl_policy_loss_desc()
    ds.struct_size = ctypes.sizeof(rl_policy_loss_desc)
    ds.form, ds.agg, ds.B, ds.T, ds.row_stride = form, agg, B, T, row_stride
    ds.clip_low, ds.clip_high, ds.beta_kl, ds.beta_ent = clip_low, clip_high, beta_kl, beta_ent
    for k, v in ptrs.items():
        setattr(ds, k, v)
    return ds


def rl_policy_loss_workspace_bytes(desc: rl_policy_loss_desc) -> int:
    return _lib.rl_policy_loss_workspace_bytes(ctypes.byref(desc))


def rl_policy_loss_raw(desc: rl_policy_loss_desc, stream_handle=None) -> int:
    return _lib.rl_policy_loss(ctypes.byref(desc), stream_handle)


def policy_loss_desc_from_tensors(logprob, old_logprob, advantages, lens, clip_low, clip_high, stats, kl=None,
                                  entropy=None, grad=None, beta_kl=0.0, beta_ent=0.0, form=RL_PG_PPO_CLIP,
                                  agg=RL_AGG_TOKEN_MEAN, workspace=None) -> rl_policy_loss_desc:
    """Descriptor over torch device tensors; the [B, T] tensors may be row-strided views sharing one stride."""
    import torch
    Bn, T = logprob.shape
    stride = logprob.stride(0) if Bn > 1 else max(T, 1)
    for t in (logprob, old_logprob, kl, entropy, grad):
        if t is None:
            continue
        if t.dtype != torch.float32 or tuple(t.shape) != (Bn, T) or (T > 1 and t.stride(1) != 1) or \
                (Bn > 1 and t.stride(0) != stride):
            raise TypeError("the [B, T] tensors must be float32 with unit column stride and one common row stride")
    if advantages.dtype != torch.float32 or lens.dtype != torch.int32 or stats.dtype != torch.float32 or stats.numel() < 8:
        raise TypeError("advantages float32 [B], lens int32 [B], stats float32 [8]")
    ptr = lambda t: None if t is None or t.numel() == 0 else t.data_ptr()
    return make_policy_loss_desc(Bn, T, stride, float(clip_low), float(clip_high), float(beta_kl), float(beta_ent), form,
                                 agg, logprob=ptr(logprob), old_logprob=ptr(old_logprob), advantages=ptr(advantages),
                                 kl=ptr(kl), entropy=ptr(entropy), lens=ptr(lens), grad_logprob=ptr(grad),
                                 stats=ptr(stats), workspace=ptr(workspace),
                                 workspace_bytes=0 if workspace is None else workspace.numel() * workspace.element_size())


def rl_policy_loss(logprob, old_logprob, advantages, lens, clip_low, clip_high, kl=None, entropy=None, beta_kl=0.0,
                   beta_ent=0.0, form=RL_PG_PPO_CLIP, agg=RL_AGG_TOKEN_MEAN, want_grad=True, workspace=None, stream=None):
    """Clipped policy loss over [B, T] per-token tensors; returns (stats [8] device tensor in the order of
    POLICY_LOSS_STATS, grad_logprob [B, T] or None).  Asynchronous."""
    import torch
    if not logprob.is_cuda:
        raise RuntimeError("rl_policy_loss needs device tensors; there is no CPU path")
    stats = torch.empty(8, dtype=torch.float32, device=logprob.device)
    grad = torch.empty_like(logprob) if want_grad else None
    ds = policy_loss_desc_from_tensors(logprob, old_logprob, advantages, lens, clip_low, clip_high, stats, kl, entropy,
                                       grad, beta_kl, beta_ent, form, agg, workspace)
    if workspace is None:
        need = rl_policy_loss_workspace_bytes(ds)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=logprob.device)
        ds.workspace, ds.workspace_bytes = workspace.data_ptr(), workspace.numel()
    s = stream if stream is not None else torch.cuda.current_stream(logprob.device)
    rc = _lib.rl_policy_loss(ctypes.byref(ds), ctypes.c_void_p(s.cuda_stream))
    if rc != RLDA_OK:
        raise RldaError(rc)
    return stats, grad


# ---------------------------------------------------------------- rl_prefill_attn.h
class rl_prefill_desc(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("dtype", ctypes.c_int32),
        ("P", ctypes.c_int32),
        ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("d", ctypes.c_int32),
        ("Lp_cap", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("lens", ctypes.c_void_p),
        ("out", ctypes.c_void_p), ("lse", ctypes.c_void_p),
    ]


_lib.rl_prefill_attn.restype = ctypes.c_int
_lib.rl_prefill_attn.argtypes = [ctypes.POINTER(rl_prefill_desc), ctypes.c_void_p]


def make_prefill_desc(dtype, P, Hq, Hkv, d, Lp_cap, scale, **ptrs) -> rl_prefill_desc:
    ds = rl_prefill_desc()
    ds.struct_size = ctypes.sizeof(rl_prefill_desc)
    ds.dtype, ds.P, ds.Hq, ds.Hkv, ds.d, ds.Lp_cap, ds.scale = dtype, P, Hq, Hkv, d, Lp_cap, scale
    for k, v in ptrs.items():
        setattr(ds, k, v)
    return ds


def rl_prefill_attn_raw(desc: rl_prefill_desc, stream_handle=None) -> int:
    return _lib.rl_prefill_attn(ctypes.byref(desc), stream_handle)


def prefill_desc_from_tensors(q, k, v, lens, scale, out, lse=None) -> rl_prefill_desc:
    import torch
    P, Lc, Hq, d = q.shape
    Hkv = k.shape[1]
    if tuple(k.shape) != (P, Hkv, Lc, d) or k.shape != v.shape or tuple(out.shape) != (P, Lc, Hq, d):
        raise ValueError("q / out are [P, L_cap, Hq, d], k / v are [P, Hkv, L_cap, d]")
    if lens.dtype != torch.int32 or out.dtype != torch.float32 or (lse is not None and lse.dtype != torch.float32):
        raise TypeError("lens int32, out / lse float32")
    for t in (q, k, v, lens, out):
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")
    code = _torch_dtype_code(q)
    if _torch_dtype_code(k) != code or _torch_dtype_code(v) != code:
        raise TypeError("q/k/v dtypes differ")
    ptr = lambda t: None if t is None or t.numel() == 0 else t.data_ptr()
    return make_prefill_desc(code, P, Hq, Hkv, d, Lc, float(scale), q=ptr(q), k=ptr(k), v=ptr(v), lens=ptr(lens),
                             out=ptr(out), lse=ptr(lse))


def rl_prefill_attn(q, k, v, lens, scale, out=None, lse=None, stream=None):
    """Causal attention of every prompt over itself; returns (out [P, L_cap, Hq, d], lse [P, L_cap, Hq]) fp32.
    Rows at positions >= lens[p] are left as they were (zero when the outputs are allocated here)."""
    import torch
    if not q.is_cuda:
        raise RuntimeError("rl_prefill_attn needs device tensors; there is no CPU path")
    P, Lc, Hq, d = q.shape
    if out is None:
        out = torch.zeros((P, Lc, Hq, d), dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.zeros((P, Lc, Hq), dtype=torch.float32, device=q.device)
    ds = prefill_desc_from_tensors(q, k, v, lens, scale, out, lse)
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    rc = _lib.rl_prefill_attn(ctypes.byref(ds), ctypes.c_void_p(s.cuda_stream))
    if rc != RLDA_OK:
        raise RldaError(rc)
    return out, lse
