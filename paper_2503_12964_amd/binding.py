"""Thin ctypes binding over libvfm.so: argument marshalling only.

Every step of the path runs in the HIP kernels of the library; this module
turns torch tensors (device memory) and host int32 arrays into the pointers and
sizes the C ABI takes (include/vfm.h).  There is no fallback: if the library
is not built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# VFM_LIB may point at another build of the library (same C ABI).
LIB_PATH = os.environ.get("VFM_LIB") or os.path.join(_HERE, "libvfm.so")

VFM_BF16 = 0
VFM_F32 = 1
VFM_MAX_SEQS = 256

EXPORTS = ("vfm_rope3d", "vfm_qknorm_rope3d", "vfm_qknorm_rope3d_bwd", "vfm_attn_fwd", "vfm_attn_bwd_workspace_size", "vfm_attn_bwd", "vfm_attn_bwd_noalloc", "vfm_xattn_fwd", "vfm_xattn_bwd_workspace_size", "vfm_xattn_bwd", "vfm_tattn_fwd", "vfm_tattn_bwd",
           "vfm_fp8_pack_sizes", "vfm_fp8_pack", "vfm_attn_fwd_fp8", "vfm_strerror", "vfm_last_hip_error", "vfm_schedule_units",
           "vfm_attn_fwd_tile_rows")

_lib = None


class VfmError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libvfm status {status}: {message}")
        self.status = status


def load_library(path: str = LIB_PATH) -> ctypes.CDLL:
    """dlopen libvfm.so and declare the C signatures.  Raises if it is missing."""
    global _lib
    if _lib is not None and path == LIB_PATH:
        return _lib
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build it first (python -m paper_2503_12964_amd.build); "
            "there is no CPU fallback")
    # The library and PyTorch must share ONE HIP runtime: the tensors and streams handed over
    # belong to PyTorch's.  libvfm.so asks for the runtime by its soname; with PyTorch (which
    # ships its own copy under that soname) loaded first, the dynamic linker gives the library
    # that copy.  Loaded the other way round, the library would bring in the system's copy as a
    # second runtime in the process, and a second runtime finds no device.
    import torch  # noqa: F401
    lib = ctypes.CDLL(path)
    c_int, c_float, c_void_p, c_size_t = ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
    p_i32 = ctypes.POINTER(ctypes.c_int32)
    lib.vfm_rope3d.restype = c_int
    lib.vfm_rope3d.argtypes = [c_void_p, p_i32, p_i32, c_int, c_int, c_int, c_int, c_int, c_int, c_int,
                               c_float, c_int, c_int, c_void_p]
    lib.vfm_qknorm_rope3d.restype = c_int
    lib.vfm_qknorm_rope3d.argtypes = [c_void_p, c_void_p, c_float, c_void_p, p_i32, p_i32, c_int, c_int, c_int,
                                      c_int, c_int, c_int, c_int, c_float, c_int, c_void_p]
    lib.vfm_qknorm_rope3d_bwd.restype = c_int
    lib.vfm_qknorm_rope3d_bwd.argtypes = [c_void_p, c_void_p, c_float, c_void_p, c_void_p, c_void_p, p_i32, p_i32,
                                          c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_float, c_int,
                                          c_void_p]
    lib.vfm_attn_fwd.restype = c_int
    lib.vfm_attn_fwd.argtypes = [c_void_p, c_void_p, c_void_p, p_i32, c_int, c_int, c_int, c_int, c_float,
                                 c_void_p, c_void_p, c_int, c_void_p]
    lib.vfm_attn_bwd_workspace_size.restype = c_size_t
    lib.vfm_attn_bwd_workspace_size.argtypes = [c_int, c_int, c_int]
    lib.vfm_attn_bwd.restype = c_int
    lib.vfm_attn_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, p_i32, c_int,
                                 c_int, c_int, c_int, c_float, c_void_p, c_void_p, c_void_p, c_void_p,
                                 c_size_t, c_int, c_void_p]
    lib.vfm_attn_bwd_noalloc.restype = c_int
    lib.vfm_attn_bwd_noalloc.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, p_i32, c_int,
                                         c_int, c_int, c_int, c_float, c_void_p, c_void_p, c_void_p, c_int,
                                         c_void_p]
    lib.vfm_xattn_fwd.restype = c_int
    lib.vfm_xattn_fwd.argtypes = [c_void_p, c_void_p, c_void_p, p_i32, p_i32, c_int, c_int, c_int, c_int, c_int,
                                  c_float, c_void_p, c_void_p, c_int, c_void_p]
    lib.vfm_xattn_bwd_workspace_size.restype = c_size_t
    lib.vfm_xattn_bwd_workspace_size.argtypes = [c_int, c_int, c_int, c_int]
    lib.vfm_xattn_bwd.restype = c_int
    lib.vfm_xattn_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, p_i32, p_i32, c_int,
                                  c_int, c_int, c_int, c_int, c_float, c_void_p, c_void_p, c_void_p, c_void_p,
                                  c_size_t, c_int, c_void_p]
    lib.vfm_tattn_fwd.restype = c_int
    lib.vfm_tattn_fwd.argtypes = [c_void_p, c_void_p, c_void_p, p_i32, p_i32, c_int, c_int, c_int, c_int, c_float,
                                  c_void_p, c_int, c_void_p]
    lib.vfm_tattn_bwd.restype = c_int
    lib.vfm_tattn_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, p_i32, p_i32, c_int, c_int, c_int, c_int,
                                  c_float, c_void_p, c_void_p, c_void_p, c_int, c_void_p]
    p_size = ctypes.POINTER(c_size_t)
    lib.vfm_fp8_pack_sizes.restype = c_int
    lib.vfm_fp8_pack_sizes.argtypes = [p_i32, c_int, c_int, c_int, c_int, p_size, p_size, p_size, p_size]
    lib.vfm_fp8_pack.restype = c_int
    lib.vfm_fp8_pack.argtypes = [c_void_p, c_void_p, c_void_p, p_i32, c_int, c_int, c_int, c_int, c_float,
                                 c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p]
    lib.vfm_attn_fwd_fp8.restype = c_int
    lib.vfm_attn_fwd_fp8.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, p_i32, c_int, c_int, c_int, c_int,
                                     c_void_p, c_void_p, c_void_p]
    lib.vfm_strerror.restype = ctypes.c_char_p
    lib.vfm_strerror.argtypes = [c_int]
    lib.vfm_schedule_units.restype = c_int
    lib.vfm_schedule_units.argtypes = [p_i32, c_int, c_int, c_int, c_int, p_i32, c_int, ctypes.POINTER(c_int)]
    lib.vfm_attn_fwd_tile_rows.restype = c_int
    lib.vfm_attn_fwd_tile_rows.argtypes = [p_i32, c_int, c_int, c_int, c_int, ctypes.POINTER(c_int)]
    lib.vfm_last_hip_error.restype = ctypes.c_char_p
    lib.vfm_last_hip_error.argtypes = []
    if path == LIB_PATH:
        _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().vfm_strerror(int(status)).decode()


def vfm_last_hip_error() -> str:
    return load_library().vfm_last_hip_error().decode()


VFM_ERR_LAUNCH = 8


def _check(status: int) -> None:
    if status != 0:
        text = strerror(status)
        if status == VFM_ERR_LAUNCH:
            text += " (" + vfm_last_hip_error() + ")"
        raise VfmError(status, text)


def vfm_schedule_units(cu_seqlens, n_heads: int, rows_per_tile: int) -> np.ndarray:
    """(head, first packed row, rows) of every workgroup of a launch that cuts rows_per_tile-row
    tiles from the clips; head -1 marks grid padding.  Host only."""
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    n = ctypes.c_int(0)
    st = lib.vfm_schedule_units(_i32_ptr(cu), int(cu.size - 1), int(cu[-1]), int(n_heads), int(rows_per_tile),
                                None, 0, ctypes.byref(n))
    if st not in (0, 2):          # SHAPE only says "capacity too small" here
        _check(st)
    units = np.zeros((max(n.value, 1), 3), dtype=np.int32)
    _check(lib.vfm_schedule_units(_i32_ptr(cu), int(cu.size - 1), int(cu[-1]), int(n_heads), int(rows_per_tile),
                                  _i32_ptr(units), int(units.shape[0]), ctypes.byref(n)))
    return units[:n.value]


def vfm_attn_fwd_tile_rows(cu_seqlens, head_dim: int, run: int = 0) -> int:
    """Query rows per workgroup the forward uses for run `run` of these clips.  Host only."""
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    rows = ctypes.c_int(0)
    _check(lib.vfm_attn_fwd_tile_rows(_i32_ptr(cu), int(cu.size - 1), int(cu[-1]), int(head_dim), int(run),
                                      ctypes.byref(rows)))
    return rows.value


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _i32_ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(int(getattr(stream, "cuda_stream", stream)))


def _dev(t, name: str) -> ctypes.c_void_p:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return VFM_BF16
    if t.dtype == torch.float32:
        return VFM_F32
    raise ValueError(f"unsupported dtype {t.dtype}")


def vfm_rope3d(x, thw, cu_seqlens, dims: Sequence[int], theta: float = 10000.0,
               inverse: bool = False, stream=None):
    """In-place 3D RoPE on x[total, heads, head_dim] (device, bf16).  Returns x."""
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    g = _host_i32(thw).reshape(-1)
    total, heads, hd = x.shape
    _check(lib.vfm_rope3d(_dev(x, "x"), _i32_ptr(g), _i32_ptr(cu), int(cu.size - 1), int(total), int(heads),
                          int(hd), int(dims[0]), int(dims[1]), int(dims[2]), float(theta), int(bool(inverse)),
                          _dtype_code(x), _stream_ptr(stream)))
    return x


def vfm_qknorm_rope3d(x, gain, eps: float, thw, cu_seqlens, dims: Sequence[int], theta: float = 10000.0,
                      y=None, stream=None):
    """y = RoPE3D(gain * x / sqrt(mean_d x^2 + eps)) per (token, head); y=None works in place on x."""
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    g = _host_i32(thw).reshape(-1)
    total, heads, hd = x.shape
    y = x if y is None else y
    _check(lib.vfm_qknorm_rope3d(_dev(x, "x"), _dev(gain, "gain"), float(eps), _dev(y, "y"), _i32_ptr(g),
                                 _i32_ptr(cu), int(cu.size - 1), int(total), int(heads), int(hd),
                                 int(dims[0]), int(dims[1]), int(dims[2]), float(theta), _dtype_code(x),
                                 _stream_ptr(stream)))
    return y


def vfm_qknorm_rope3d_bwd(x, gain, eps: float, dy, thw, cu_seqlens, dims: Sequence[int],
                          theta: float = 10000.0, dx=None, dgain=None, stream=None) -> Tuple:
    """dx (bf16, shape of x; may be dy itself) and dgain (fp32 [head_dim]) given the forward's input x."""
    import torch
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    g = _host_i32(thw).reshape(-1)
    total, heads, hd = x.shape
    dx = torch.empty_like(x) if dx is None else dx
    dgain = torch.empty(hd, dtype=torch.float32, device=x.device) if dgain is None else dgain
    _check(lib.vfm_qknorm_rope3d_bwd(_dev(x, "x"), _dev(gain, "gain"), float(eps), _dev(dy, "dy"), _dev(dx, "dx"),
                                     _dev(dgain, "dgain"), _i32_ptr(g), _i32_ptr(cu), int(cu.size - 1),
                                     int(total), int(heads), int(hd), int(dims[0]), int(dims[1]), int(dims[2]),
                                     float(theta), _dtype_code(x), _stream_ptr(stream)))
    return dx, dgain


def vfm_attn_fwd(q, k, v, cu_seqlens, scale: float, out=None, lse=None, stream=None) -> Tuple:
    """out[total, heads, head_dim] (bf16) and lse[heads, total] (fp32) for packed q, k, v."""
    import torch
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    total, heads, hd = q.shape
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((heads, total), dtype=torch.float32, device=q.device)
    _check(lib.vfm_attn_fwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _i32_ptr(cu), int(cu.size - 1), int(total),
                            int(heads), int(hd), float(scale), _dev(out, "out"), _dev(lse, "lse"),
                            _dtype_code(q), _stream_ptr(stream)))
    return out, lse


def vfm_attn_bwd_workspace_size(total_tokens: int, n_heads: int, head_dim: int) -> int:
    return int(load_library().vfm_attn_bwd_workspace_size(int(total_tokens), int(n_heads), int(head_dim)))


def vfm_attn_bwd(q, k, v, out, lse, dout, cu_seqlens, scale: float, dq=None, dk=None, dv=None,
                 workspace=None, stream=None) -> Tuple:
    """dq, dk, dv (bf16, shape of q) given the forward's out and lse."""
    import torch
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    total, heads, hd = q.shape
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    need = vfm_attn_bwd_workspace_size(total, heads, hd)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(lib.vfm_attn_bwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"), _dev(lse, "lse"),
                            _dev(dout, "dout"), _i32_ptr(cu), int(cu.size - 1), int(total), int(heads), int(hd),
                            float(scale), _dev(dq, "dq"), _dev(dk, "dk"), _dev(dv, "dv"),
                            _dev(workspace, "workspace"), int(workspace.numel() * workspace.element_size()),
                            _dtype_code(q), _stream_ptr(stream)))
    return dq, dk, dv


def vfm_attn_bwd_noalloc(q, k, v, out, lse, dout, cu_seqlens, scale: float, dq, dk, dv, stream=None) -> Tuple:
    """vfm_attn_bwd without a workspace (the library's built-in scratch holds the statistics).
    The caller passes every output; nothing is allocated here or in the library."""
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    total, heads, hd = q.shape
    _check(lib.vfm_attn_bwd_noalloc(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"), _dev(lse, "lse"),
                                    _dev(dout, "dout"), _i32_ptr(cu), int(cu.size - 1), int(total), int(heads),
                                    int(hd), float(scale), _dev(dq, "dq"), _dev(dk, "dk"), _dev(dv, "dv"),
                                    _dtype_code(q), _stream_ptr(stream)))
    return dq, dk, dv


def vfm_xattn_fwd(q, k, v, cu_seqlens_q, cu_seqlens_kv, scale: float, out=None, lse=None, stream=None) -> Tuple:
    """Cross-attention: out[total_q, heads, head_dim] (bf16), lse[heads, total_q] (fp32)."""
    import torch
    lib = load_library()
    cq, ck = _host_i32(cu_seqlens_q), _host_i32(cu_seqlens_kv)
    if cq.size != ck.size:
        raise ValueError("cu_seqlens_q and cu_seqlens_kv must have the same length")
    total_q, heads, hd = q.shape
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((heads, total_q), dtype=torch.float32, device=q.device)
    _check(lib.vfm_xattn_fwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _i32_ptr(cq), _i32_ptr(ck), int(cq.size - 1),
                             int(total_q), int(k.shape[0]), int(heads), int(hd), float(scale), _dev(out, "out"),
                             _dev(lse, "lse"), _dtype_code(q), _stream_ptr(stream)))
    return out, lse


def vfm_xattn_bwd_workspace_size(total_q: int, total_kv: int, n_heads: int, head_dim: int) -> int:
    return int(load_library().vfm_xattn_bwd_workspace_size(int(total_q), int(total_kv), int(n_heads), int(head_dim)))


def vfm_xattn_bwd(q, k, v, out, lse, dout, cu_seqlens_q, cu_seqlens_kv, scale: float, dq=None, dk=None,
                  dv=None, workspace=None, stream=None) -> Tuple:
    """Cross-attention gradients: dq (shape of q), dk, dv (shape of k)."""
    import torch
    lib = load_library()
    cq, ck = _host_i32(cu_seqlens_q), _host_i32(cu_seqlens_kv)
    if cq.size != ck.size:
        raise ValueError("cu_seqlens_q and cu_seqlens_kv must have the same length")
    total_q, heads, hd = q.shape
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    need = vfm_xattn_bwd_workspace_size(total_q, int(k.shape[0]), heads, hd)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(lib.vfm_xattn_bwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"), _dev(lse, "lse"),
                             _dev(dout, "dout"), _i32_ptr(cq), _i32_ptr(ck), int(cq.size - 1), int(total_q),
                             int(k.shape[0]), int(heads), int(hd), float(scale), _dev(dq, "dq"), _dev(dk, "dk"),
                             _dev(dv, "dv"), _dev(workspace, "workspace"),
                             int(workspace.numel() * workspace.element_size()), _dtype_code(q),
                             _stream_ptr(stream)))
    return dq, dk, dv


def vfm_tattn_fwd(q, k, v, thw, cu_seqlens, scale: float, out=None, stream=None):
    """Temporal attention (one sequence per pixel across a clip's frames): out, shape of q."""
    import torch
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    g = _host_i32(thw).reshape(-1)
    total, heads, hd = q.shape
    out = torch.empty_like(q) if out is None else out
    _check(lib.vfm_tattn_fwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _i32_ptr(g), _i32_ptr(cu), int(cu.size - 1),
                             int(total), int(heads), int(hd), float(scale), _dev(out, "out"), _dtype_code(q),
                             _stream_ptr(stream)))
    return out


def vfm_tattn_bwd(q, k, v, dout, thw, cu_seqlens, scale: float, dq=None, dk=None, dv=None, stream=None) -> Tuple:
    """Temporal attention gradients dq, dk, dv (shape of q)."""
    import torch
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    g = _host_i32(thw).reshape(-1)
    total, heads, hd = q.shape
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    _check(lib.vfm_tattn_bwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(dout, "dout"), _i32_ptr(g), _i32_ptr(cu),
                             int(cu.size - 1), int(total), int(heads), int(hd), float(scale), _dev(dq, "dq"),
                             _dev(dk, "dk"), _dev(dv, "dv"), _dtype_code(q), _stream_ptr(stream)))
    return dq, dk, dv


def vfm_fp8_pack_sizes(cu_seqlens, n_heads: int, head_dim: int) -> Tuple[int, int, int, int]:
    """Bytes of the packed q8, k8, vT8 and scales buffers for these clips."""
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    a, b, c, d = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.vfm_fp8_pack_sizes(_i32_ptr(cu), int(cu.size - 1), int(cu[-1]), int(n_heads), int(head_dim),
                                  ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d)))
    return int(a.value), int(b.value), int(c.value), int(d.value)


def vfm_fp8_pack(q, k, v, cu_seqlens, scale: float, q8=None, k8=None, vT8=None, scales=None, stream=None) -> Tuple:
    """Quantise bf16 q, k, v to E4M3 tiles with power-of-two scales, in the packed layout
    vfm_attn_fwd_fp8 reads (uint8 device buffers q8, k8, vT8 and the scales buffer).  q also
    carries scale * log2(e) (scale = softmax scale)."""
    import torch
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    total, heads, hd = q.shape
    nq, nk, nv, ns = vfm_fp8_pack_sizes(cu, heads, hd)
    q8 = torch.empty(max(nq, 16), dtype=torch.uint8, device=q.device) if q8 is None else q8
    k8 = torch.empty(max(nk, 16), dtype=torch.uint8, device=q.device) if k8 is None else k8
    vT8 = torch.empty(max(nv, 16), dtype=torch.uint8, device=q.device) if vT8 is None else vT8
    scales = torch.empty(max(ns, 16), dtype=torch.uint8, device=q.device) if scales is None else scales
    _check(lib.vfm_fp8_pack(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _i32_ptr(cu), int(cu.size - 1), int(total),
                            int(heads), int(hd), float(scale), _dev(q8, "q8"), _dev(k8, "k8"), _dev(vT8, "vT8"),
                            _dev(scales, "scales"), _dtype_code(q), _stream_ptr(stream)))
    return q8, k8, vT8, scales


def vfm_attn_fwd_fp8(q8, k8, vT8, scales, cu_seqlens, n_heads: int, head_dim: int, out=None, lse=None,
                     stream=None) -> Tuple:
    """FP8 attention forward on packed operands: out (bf16 [total, heads, head_dim]) and lse (fp32)."""
    import torch
    lib = load_library()
    cu = _host_i32(cu_seqlens)
    total = int(cu[-1])
    if out is None:
        out = torch.empty((total, n_heads, head_dim), dtype=torch.bfloat16, device=q8.device)
    if lse is None:
        lse = torch.empty((n_heads, total), dtype=torch.float32, device=q8.device)
    _check(lib.vfm_attn_fwd_fp8(_dev(q8, "q8"), _dev(k8, "k8"), _dev(vT8, "vT8"), _dev(scales, "scales"), _i32_ptr(cu),
                                int(cu.size - 1), total, int(n_heads), int(head_dim), _dev(out, "out"),
                                _dev(lse, "lse"), _stream_ptr(stream)))
    return out, lse
