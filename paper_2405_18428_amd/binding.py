"""ctypes binding of ``include/gla.h`` (argument marshalling only).

Tensors are torch tensors on an AMD GPU; torch is used for device memory and
the current stream, nothing else.  Every arithmetic step runs inside
``libgla.so``; if that library has not been built the calls raise.
"""
from __future__ import annotations

import ctypes
import os
import re
from typing import List, Optional

SCAN_ROW_FWD, SCAN_ROW_REV, SCAN_COL_FWD, SCAN_COL_REV = 0, 1, 2, 3
DT_F32, DT_BF16 = 0, 1
OPT_CHUNKS_PER_SPAN, OPT_ENGINE, OPT_CARRY, OPT_BWD_SPLIT, OPT_RANGE_FALLBACK = 0, 1, 2, 3, 4
CARRY_AUTO, CARRY_KERNEL, CARRY_IN_OUTPUT_PASS = 0, 1, 2
LAYOUT_BHTD, LAYOUT_BTHD = 0, 1
ENGINE_AUTO, ENGINE_RECURRENT, ENGINE_MFMA, ENGINE_MFMA_FP16 = 0, 1, 2, 3

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "csrc", "libgla.so")
_HEADER = os.path.join(os.path.dirname(_PKG), "include", "gla.h")
_lib = None


class GlaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"gla status {status}: {message}")
        self.status = status


def library_path() -> str:
    return _LIB_PATH


def lib_symbols() -> List[str]:
    """Names of the functions that include/gla.h declares."""
    text = open(_HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gla_[a-z_]+)\s*\(", text)))


def load_library():
    """Load libgla.so (built by ``__graft_entry__.build()`` / ``csrc/build.py``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build the HIP library first "
            "(python -c 'import __graft_entry__ as g; g.build()'). There is no fallback path.")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i, fp, sz = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.c_size_t
    shape = [i] * 8
    lib.gla_fwd.restype = i
    lib.gla_fwd.argtypes = [vp, vp, vp, vp] + shape + [vp, vp, vp]
    lib.gla_fwd_static.restype = i
    lib.gla_fwd_static.argtypes = [vp, vp, vp, vp] + shape + [vp, vp, vp]
    lib.gla_fwd_ex.restype = i
    lib.gla_fwd_ex.argtypes = [vp, vp, vp, vp] + shape + [i, i, vp, vp, vp, sz, vp]
    lib.gla_fwd_layout.restype = i
    lib.gla_fwd_layout.argtypes = [vp, vp, vp, vp] + shape + [i, i, i, vp, vp, vp, vp, sz, vp]
    lib.gla_fwd_gates.restype = i
    lib.gla_fwd_gates.argtypes = [vp, vp, vp, vp, vp] + shape + [i, i, i, vp, vp, vp, vp, sz, vp]
    lib.gla_bwd.restype = i
    lib.gla_bwd.argtypes = [vp] * 5 + shape + [i] + [vp] * 4 + [vp, sz, vp]
    lib.gla_bwd_layout.restype = i
    lib.gla_bwd_layout.argtypes = [vp] * 5 + shape + [i, i] + [vp, sz] + [vp] * 4 + [vp, sz, vp]
    lib.gla_bwd_reuse.restype = i
    lib.gla_bwd_reuse.argtypes = [vp] * 5 + shape + [i] + [vp, sz] + [vp] * 4 + [vp, sz, vp]
    lib.gla_srem_dwconv.restype = i
    lib.gla_srem_dwconv.argtypes = [vp, vp, vp] + [i] * 7 + [vp, vp]
    lib.gla_fwd_multi.restype = i
    lib.gla_fwd_multi.argtypes = [vp, vp, vp, vp] + [i] * 7 + [ctypes.c_uint, i, vp, vp, sz, vp]
    lib.gla_fwd_fused.restype = i
    lib.gla_fwd_fused.argtypes = [vp, vp, vp, vp, ctypes.c_float, vp, vp, vp, ctypes.c_float] + shape + \
        [i, i, vp, vp, vp, sz, vp]
    lib.gla_fwd_fused_gates.restype = i
    lib.gla_fwd_fused_gates.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, vp, ctypes.c_float] + shape + \
        [i, i, vp, vp, vp, sz, vp]
    lib.gla_bwd_gates.restype = i
    lib.gla_bwd_gates.argtypes = [vp] * 7 + shape + [i] + [vp] * 5 + [vp, sz, vp]
    lib.gla_bwd_gates_workspace_bytes.restype = sz
    lib.gla_bwd_gates_workspace_bytes.argtypes = [i] * 6
    lib.gla_bwd_workspace_bytes.restype = sz
    lib.gla_bwd_workspace_bytes.argtypes = [i] * 6
    lib.gla_calibrate_mfma.restype = i
    lib.gla_calibrate_mfma.argtypes = [ctypes.POINTER(ctypes.c_double), vp]
    lib.gla_fwd_timed.restype = i
    lib.gla_fwd_timed.argtypes = [vp, vp, vp, vp] + shape + [i, i, vp, vp, vp, sz, vp, i, fp]
    lib.gla_fwd_workspace_bytes.restype = sz
    lib.gla_fwd_workspace_bytes.argtypes = [i] * 6
    lib.gla_set_option.restype = i
    lib.gla_set_option.argtypes = [i, i]
    lib.gla_get_option.restype = i
    lib.gla_get_option.argtypes = [i]
    lib.gla_status_string.restype = ctypes.c_char_p
    lib.gla_status_string.argtypes = [i]
    lib.gla_version.restype = i
    lib.gla_version.argtypes = []
    lib.gla_block_scan_dir.restype = i
    lib.gla_block_scan_dir.argtypes = [i, i]
    _lib = lib
    return lib


def gla_status_string(status: int) -> str:
    return load_library().gla_status_string(int(status)).decode()


def gla_version() -> int:
    return int(load_library().gla_version())


SCHEDULE_BLOCK_PROCESS, SCHEDULE_BLOCK_SCAN = 0, 1


def gla_block_scan_dir(block: int, schedule: int = SCHEDULE_BLOCK_PROCESS) -> int:
    """Scan order of DiG block `block` (1-based) under Algorithm 1's (or Algorithm 4's) transposes and flips."""
    d = int(load_library().gla_block_scan_dir(int(block), int(schedule)))
    if d < 0:
        raise GlaError(2, gla_status_string(2))
    return d


def gla_set_option(option: int, value: int) -> None:
    _check(load_library().gla_set_option(int(option), int(value)))


def gla_get_option(option: int) -> int:
    return int(load_library().gla_get_option(int(option)))


def gla_fwd_workspace_bytes(B, H, T, dk, dv, qkv_dtype=DT_BF16) -> int:
    return int(load_library().gla_fwd_workspace_bytes(B, H, T, dk, dv, qkv_dtype))


def _check(status: int) -> None:
    if status != 0:
        raise GlaError(status, gla_status_string(status))


def _torch():
    import torch
    return torch


def _dt(t) -> int:
    torch = _torch()
    if t.dtype == torch.bfloat16:
        return DT_BF16
    if t.dtype == torch.float32:
        return DT_F32
    raise TypeError(f"unsupported element type {t.dtype}")


def _prep(q, k, v, log_alpha, grid_h, grid_w):
    torch = _torch()
    for name, t in (("q", q), ("k", k), ("v", v), ("log_alpha", log_alpha)):
        if not t.is_cuda:
            raise ValueError(f"{name} must live on the GPU")
        if not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous")
    if q.dim() != 4 or q.shape != k.shape or q.shape != log_alpha.shape:
        raise ValueError("q, k, log_alpha must be [B,H,T,dk] with equal shapes")
    if v.dim() != 4 or v.shape[:3] != q.shape[:3]:
        raise ValueError("v must be [B,H,T,dv]")
    if q.dtype != k.dtype or q.dtype != v.dtype:
        raise TypeError("q, k, v must share one element type")
    if log_alpha.dtype != torch.float32:
        raise TypeError("log_alpha must be fp32")
    B, H, T, dk = q.shape
    return B, H, T, dk, v.shape[3]


def _stream_ptr(stream) -> int:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def gla_fwd(q, k, v, log_alpha, grid_h, grid_w, scan_dir=SCAN_ROW_FWD,
            want_final_state=True, out=None, final_state=None, stream=None):
    """bf16 q/k/v -> fp32 out (and fp32 final state); library-owned scratch."""
    torch = _torch()
    lib = load_library()
    B, H, T, dk, dv = _prep(q, k, v, log_alpha, grid_h, grid_w)
    if q.dtype != torch.bfloat16:
        raise TypeError("gla_fwd takes bf16 q/k/v; use gla_fwd_ex for fp32")
    if out is None:
        out = torch.empty((B, H, T, dv), dtype=torch.float32, device=q.device)
    if final_state is None and want_final_state:
        final_state = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device)
    with torch.cuda.device(q.device):
        _check(lib.gla_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(),
                           B, H, T, dk, dv, grid_h, grid_w, scan_dir,
                           out.data_ptr(), final_state.data_ptr() if final_state is not None else None,
                           _stream_ptr(stream)))
    return out, final_state


def gla_fwd_static(q, k, v, log_alpha, grid_h, grid_w, scan_dir=SCAN_ROW_FWD, out=None, final_state=None,
                   stream=None):
    """gla_fwd with the span states in the library's static device array (no allocation inside the call):
    the caller passes ``out`` (fp32 [B,H,T,dv]) and, if wanted, ``final_state`` (fp32 [B,H,dk,dv])."""
    torch = _torch()
    lib = load_library()
    B, H, T, dk, dv = _prep(q, k, v, log_alpha, grid_h, grid_w)
    if q.dtype != torch.bfloat16:
        raise TypeError("gla_fwd_static takes bf16 q/k/v")
    if out is None or out.dtype != torch.float32 or tuple(out.shape) != (B, H, T, dv) or not out.is_contiguous():
        raise ValueError("out must be a contiguous fp32 GPU tensor [B,H,T,dv]")
    with torch.cuda.device(q.device):
        _check(lib.gla_fwd_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(),
                                  B, H, T, dk, dv, grid_h, grid_w, scan_dir,
                                  out.data_ptr(), final_state.data_ptr() if final_state is not None else None,
                                  _stream_ptr(stream)))
    return out, final_state


def gla_fwd_ex(q, k, v, log_alpha, grid_h, grid_w, scan_dir=SCAN_ROW_FWD,
               out_dtype=None, want_final_state=True, out=None, final_state=None,
               workspace=None, stream=None):
    """Explicit element types and caller-owned workspace (a uint8 GPU tensor)."""
    torch = _torch()
    lib = load_library()
    B, H, T, dk, dv = _prep(q, k, v, log_alpha, grid_h, grid_w)
    qdt = _dt(q)
    if out is None:
        odt = torch.float32 if out_dtype is None else out_dtype
        out = torch.empty((B, H, T, dv), dtype=odt, device=q.device)
    if final_state is None and want_final_state:
        final_state = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device)
    if workspace is None:
        nbytes = gla_fwd_workspace_bytes(B, H, T, dk, dv, qdt)
        workspace = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=q.device)
    with torch.cuda.device(q.device):
        _check(lib.gla_fwd_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(),
                              B, H, T, dk, dv, grid_h, grid_w, scan_dir, qdt, _dt(out),
                              out.data_ptr(), final_state.data_ptr() if final_state is not None else None,
                              workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return out, final_state


def gla_fwd_layout(q, k, v, log_alpha, grid_h, grid_w, scan_dir=SCAN_ROW_FWD, layout=LAYOUT_BHTD,
                   initial_state=None, out_dtype=None, want_final_state=True, out=None, final_state=None,
                   workspace=None, stream=None):
    """gla_fwd_ex for [B,H,T,d] (LAYOUT_BHTD) or [B,T,H,d] (LAYOUT_BTHD) tensors, starting from
    ``initial_state`` ([B,H,dk,dv] fp32, or None for zero)."""
    torch = _torch()
    lib = load_library()
    if layout not in (LAYOUT_BHTD, LAYOUT_BTHD):
        raise ValueError("unknown layout")
    for name, t in (("q", q), ("k", k), ("v", v), ("log_alpha", log_alpha)):
        if not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous 4-d GPU tensor")
    if q.shape != k.shape or q.shape != log_alpha.shape or v.shape[:3] != q.shape[:3]:
        raise ValueError("q, k, log_alpha must share one shape and v its first three sizes")
    if q.dtype != k.dtype or q.dtype != v.dtype or log_alpha.dtype != torch.float32:
        raise TypeError("q, k, v must share one element type and log_alpha must be fp32")
    if layout == LAYOUT_BHTD:
        B, H, T, dk = q.shape
    else:
        B, T, H, dk = q.shape
    dv = v.shape[3]
    qdt = _dt(q)
    if initial_state is not None:
        if (initial_state.dtype != torch.float32 or tuple(initial_state.shape) != (B, H, dk, dv)
                or not initial_state.is_contiguous() or not initial_state.is_cuda):
            raise ValueError("initial_state must be a contiguous fp32 GPU tensor [B,H,dk,dv]")
    if out is None:
        odt = torch.float32 if out_dtype is None else out_dtype
        out = torch.empty(tuple(v.shape), dtype=odt, device=q.device)
    if final_state is None and want_final_state:
        final_state = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device)
    if workspace is None:
        nbytes = gla_fwd_workspace_bytes(B, H, T, dk, dv, qdt)
        workspace = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=q.device)
    with torch.cuda.device(q.device):
        _check(lib.gla_fwd_layout(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(),
                                  B, H, T, dk, dv, grid_h, grid_w, scan_dir, qdt, _dt(out), layout,
                                  initial_state.data_ptr() if initial_state is not None else None,
                                  out.data_ptr(), final_state.data_ptr() if final_state is not None else None,
                                  workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return out, final_state


def gla_fwd_gates(q, k, v, log_alpha, log_beta, grid_h, grid_w, scan_dir=SCAN_ROW_FWD, layout=LAYOUT_BHTD,
                  initial_state=None, out_dtype=None, want_final_state=True, out=None, final_state=None,
                  workspace=None, stream=None):
    """The recurrence with the two-sided gate alpha_t^T beta_t; ``log_beta`` is fp32, shaped like v."""
    torch = _torch()
    lib = load_library()
    if layout not in (LAYOUT_BHTD, LAYOUT_BTHD):
        raise ValueError("unknown layout")
    for name, t in (("q", q), ("k", k), ("v", v), ("log_alpha", log_alpha), ("log_beta", log_beta)):
        if not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous 4-d GPU tensor")
    if q.shape != k.shape or q.shape != log_alpha.shape or v.shape[:3] != q.shape[:3] or log_beta.shape != v.shape:
        raise ValueError("q, k, log_alpha must share one shape, v and log_beta another with the same first three sizes")
    if q.dtype != k.dtype or q.dtype != v.dtype or log_alpha.dtype != torch.float32 or log_beta.dtype != torch.float32:
        raise TypeError("q, k, v must share one element type and the gates must be fp32")
    if layout == LAYOUT_BHTD:
        B, H, T, dk = q.shape
    else:
        B, T, H, dk = q.shape
    dv = v.shape[3]
    qdt = _dt(q)
    if initial_state is not None:
        if (initial_state.dtype != torch.float32 or tuple(initial_state.shape) != (B, H, dk, dv)
                or not initial_state.is_contiguous() or not initial_state.is_cuda):
            raise ValueError("initial_state must be a contiguous fp32 GPU tensor [B,H,dk,dv]")
    if out is None:
        out = torch.empty(tuple(v.shape), dtype=torch.float32 if out_dtype is None else out_dtype, device=q.device)
    if final_state is None and want_final_state:
        final_state = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device)
    if workspace is None:
        nbytes = gla_fwd_workspace_bytes(B, H, T, dk, dv, qdt)
        workspace = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=q.device)
    with torch.cuda.device(q.device):
        _check(lib.gla_fwd_gates(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(), log_beta.data_ptr(),
                                 B, H, T, dk, dv, grid_h, grid_w, scan_dir, qdt, _dt(out), layout,
                                 initial_state.data_ptr() if initial_state is not None else None,
                                 out.data_ptr(), final_state.data_ptr() if final_state is not None else None,
                                 workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return out, final_state


def gla_srem_dwconv(x, weight, bias, grid_h, grid_w, orient=0, out_dtype=None, out=None, stream=None):
    """3x3 depth-wise convolution of the SREM on tokens x [B, T, D] (canonical order); weight fp32 [D,3,3], bias
    fp32 [D] or None; ``orient`` = the scan order the paper's sequence would be in at this block."""
    torch = _torch()
    lib = load_library()
    if not x.is_cuda or not x.is_contiguous() or x.dim() != 3:
        raise ValueError("x must be a contiguous 3-d GPU tensor [B,T,D]")
    B, T, D = x.shape
    if T != grid_h * grid_w:
        raise ValueError("T != grid_h * grid_w")
    if weight.dtype != torch.float32 or tuple(weight.shape) != (D, 3, 3) or not weight.is_contiguous() or not weight.is_cuda:
        raise ValueError("weight must be a contiguous fp32 GPU tensor [D,3,3]")
    if bias is not None and (bias.dtype != torch.float32 or tuple(bias.shape) != (D,) or not bias.is_cuda):
        raise ValueError("bias must be a contiguous fp32 GPU tensor [D]")
    if out is None:
        out = torch.empty_like(x, dtype=x.dtype if out_dtype is None else out_dtype)
    with torch.cuda.device(x.device):
        _check(lib.gla_srem_dwconv(x.data_ptr(), weight.data_ptr(), bias.data_ptr() if bias is not None else None,
                                   B, grid_h, grid_w, D, orient, _dt(x), _dt(out), out.data_ptr(), _stream_ptr(stream)))
    return out


def gla_fwd_multi(q, k, v, log_alpha, grid_h, grid_w, scan_dirs=(SCAN_ROW_FWD, SCAN_ROW_REV), out=None,
                  workspace=None, stream=None):
    """Sum over the scan orders in ``scan_dirs`` of the forward outputs (fp32, canonical token order)."""
    torch = _torch()
    lib = load_library()
    for name, t in (("q", q), ("k", k), ("v", v), ("log_alpha", log_alpha)):
        if not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous 4-d GPU tensor")
    if q.shape != k.shape or q.shape != log_alpha.shape or v.shape[:3] != q.shape[:3]:
        raise ValueError("q, k, log_alpha must share one shape and v its first three sizes")
    if q.dtype != k.dtype or q.dtype != v.dtype or log_alpha.dtype != torch.float32:
        raise TypeError("q, k, v must share one element type and log_alpha must be fp32")
    mask = 0
    for d in scan_dirs:
        if d not in (0, 1, 2, 3):
            raise ValueError("scan orders are 0..3")
        mask |= 1 << d
    B, H, T, dk = q.shape
    dv = v.shape[3]
    qdt = _dt(q)
    if out is None:
        out = torch.empty(tuple(v.shape), dtype=torch.float32, device=q.device)
    if workspace is None:
        nbytes = gla_fwd_workspace_bytes(B, H, T, dk, dv, qdt)
        workspace = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=q.device)
    with torch.cuda.device(q.device):
        _check(lib.gla_fwd_multi(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(),
                                 B, H, T, dk, dv, grid_h, grid_w, mask, qdt, out.data_ptr(),
                                 workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return out


def gla_fwd_fused(q, k, v, z_alpha, tau, grid_h, grid_w, scan_dir=SCAN_ROW_FWD, r_pre=None, ln_weight=None,
                  ln_bias=None, ln_eps=1e-5, out_dtype=None, want_final_state=True, out=None, final_state=None,
                  workspace=None, stream=None, _z_beta=None):
    """Forward pass with the gates taken from their pre-activations (``log_alpha = logsigmoid(z_alpha) / tau``) and,
    if ``r_pre`` is given, ``Swish(r_pre) * LayerNorm_head(o)`` stored instead of ``o``.  q, k, v, z_alpha, r_pre
    share one element type; ln_weight / ln_bias are fp32 [H, dv] or None."""
    torch = _torch()
    lib = load_library()
    tensors = [("q", q), ("k", k), ("v", v), ("z_alpha", z_alpha)] + ([("r_pre", r_pre)] if r_pre is not None else [])
    if _z_beta is not None:
        tensors.append(("z_beta", _z_beta))
        if _z_beta.shape != v.shape:
            raise ValueError("z_beta must have the shape of v")
    for name, t in tensors:
        if not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous 4-d GPU tensor")
        if t.dtype != q.dtype:
            raise TypeError("q, k, v, z_alpha and r_pre must share one element type")
    if q.shape != k.shape or q.shape != z_alpha.shape or v.shape[:3] != q.shape[:3]:
        raise ValueError("q, k, z_alpha must share one shape and v its first three sizes")
    if r_pre is not None and r_pre.shape != v.shape:
        raise ValueError("r_pre must have the shape of v")
    B, H, T, dk = q.shape
    dv = v.shape[3]
    for name, t in (("ln_weight", ln_weight), ("ln_bias", ln_bias)):
        if t is not None and (t.dtype != torch.float32 or tuple(t.shape) != (H, dv) or not t.is_contiguous()
                              or not t.is_cuda):
            raise ValueError(f"{name} must be a contiguous fp32 GPU tensor [H,dv]")
    qdt = _dt(q)
    if out is None:
        odt = torch.float32 if out_dtype is None else out_dtype
        out = torch.empty(tuple(v.shape), dtype=odt, device=q.device)
    if final_state is None and want_final_state:
        final_state = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device)
    if workspace is None:
        nbytes = gla_fwd_workspace_bytes(B, H, T, dk, dv, qdt)
        workspace = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=q.device)
    ptr = lambda t: t.data_ptr() if t is not None else None
    tail = (ptr(r_pre), ptr(ln_weight), ptr(ln_bias), float(ln_eps), B, H, T, dk, dv, grid_h, grid_w, scan_dir, qdt,
            _dt(out), out.data_ptr(), ptr(final_state), workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    with torch.cuda.device(q.device):
        if _z_beta is not None:
            _check(lib.gla_fwd_fused_gates(q.data_ptr(), k.data_ptr(), v.data_ptr(), z_alpha.data_ptr(),
                                           _z_beta.data_ptr(), float(tau), *tail))
        else:
            _check(lib.gla_fwd_fused(q.data_ptr(), k.data_ptr(), v.data_ptr(), z_alpha.data_ptr(), float(tau), *tail))
    return out, final_state


def gla_fwd_fused_gates(q, k, v, z_alpha, z_beta, tau, grid_h, grid_w, scan_dir=SCAN_ROW_FWD, **kwargs):
    """gla_fwd_fused with the value-side gate as well: ``log_beta = logsigmoid(z_beta) / tau``, z_beta shaped like v
    and of the element type of q, k, v.  Keyword arguments as gla_fwd_fused."""
    if z_beta is None:
        raise ValueError("z_beta is required")
    return gla_fwd_fused(q, k, v, z_alpha, tau, grid_h, grid_w, scan_dir, _z_beta=z_beta, **kwargs)


def gla_bwd_gates(q, k, v, log_alpha, log_beta, d_out, grid_h, grid_w, scan_dir=SCAN_ROW_FWD, out_fwd=None,
                  workspace=None, stream=None):
    """Gradients of the two-sided-gate recurrence: returns (dq, dk, dv, dlog_alpha, dlog_beta), all fp32.
    ``out_fwd``: the fp32 outputs of gla_fwd_gates on the same inputs, if the caller still holds them."""
    torch = _torch()
    lib = load_library()
    for name, t in (("q", q), ("k", k), ("v", v), ("log_alpha", log_alpha), ("log_beta", log_beta), ("d_out", d_out)):
        if not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous 4-d GPU tensor")
    if (q.shape != k.shape or q.shape != log_alpha.shape or v.shape[:3] != q.shape[:3] or log_beta.shape != v.shape
            or d_out.shape != v.shape):
        raise ValueError("q, k, log_alpha must share one shape; v, log_beta, d_out another with the same first three sizes")
    if q.dtype != k.dtype or q.dtype != v.dtype or d_out.dtype != q.dtype:
        raise TypeError("q, k, v, d_out must share one element type")
    if log_alpha.dtype != torch.float32 or log_beta.dtype != torch.float32:
        raise TypeError("the gates must be fp32")
    B, H, T, dk = q.shape
    dv = v.shape[3]
    qdt = _dt(q)
    if out_fwd is not None and (out_fwd.dtype != torch.float32 or out_fwd.shape != v.shape or not out_fwd.is_cuda
                                or not out_fwd.is_contiguous()):
        raise ValueError("out_fwd must be a contiguous fp32 GPU tensor shaped like v")
    f32 = dict(dtype=torch.float32, device=q.device)
    dq, dk_g, dla = (torch.empty((B, H, T, dk), **f32) for _ in range(3))
    dv_g, dlb = (torch.empty((B, H, T, dv), **f32) for _ in range(2))
    if workspace is None:
        nbytes = int(lib.gla_bwd_gates_workspace_bytes(B, H, T, dk, dv, qdt))
        workspace = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=q.device)
    with torch.cuda.device(q.device):
        _check(lib.gla_bwd_gates(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(), log_beta.data_ptr(),
                                 d_out.data_ptr(), out_fwd.data_ptr() if out_fwd is not None else None,
                                 B, H, T, dk, dv, grid_h, grid_w, scan_dir, qdt,
                                 dq.data_ptr(), dk_g.data_ptr(), dv_g.data_ptr(), dla.data_ptr(), dlb.data_ptr(),
                                 workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return dq, dk_g, dv_g, dla, dlb


def gla_bwd_gates_workspace_bytes(B, H, T, dk, dv, qkv_dtype=DT_BF16) -> int:
    return int(load_library().gla_bwd_gates_workspace_bytes(B, H, T, dk, dv, qkv_dtype))


def gla_bwd_workspace_bytes(B, H, T, dk, dv, qkv_dtype=DT_BF16) -> int:
    return int(load_library().gla_bwd_workspace_bytes(B, H, T, dk, dv, qkv_dtype))


def gla_bwd_layout(q, k, v, log_alpha, d_out, grid_h, grid_w, scan_dir=SCAN_ROW_FWD, layout=LAYOUT_BHTD,
                   fwd_workspace=None, workspace=None, stream=None):
    """gla_bwd for [B,H,T,d] (LAYOUT_BHTD) or [B,T,H,d] (LAYOUT_BTHD) tensors; the gradients come in the same order."""
    torch = _torch()
    lib = load_library()
    if layout not in (LAYOUT_BHTD, LAYOUT_BTHD):
        raise ValueError("unknown layout")
    for name, t in (("q", q), ("k", k), ("v", v), ("log_alpha", log_alpha), ("d_out", d_out)):
        if not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous 4-d GPU tensor")
    if q.shape != k.shape or q.shape != log_alpha.shape or v.shape[:3] != q.shape[:3] or d_out.shape != v.shape:
        raise ValueError("q, k, log_alpha must share one shape, v its first three sizes, d_out the shape of v")
    if q.dtype != k.dtype or q.dtype != v.dtype or q.dtype != d_out.dtype or log_alpha.dtype != torch.float32:
        raise TypeError("q, k, v, d_out must share one element type and log_alpha must be fp32")
    if layout == LAYOUT_BHTD:
        B, H, T, dk = q.shape
    else:
        B, T, H, dk = q.shape
    dv = v.shape[3]
    qdt = _dt(q)
    f32 = dict(dtype=torch.float32, device=q.device)
    dq, dk_, dg = (torch.empty(tuple(q.shape), **f32) for _ in range(3))
    dv_ = torch.empty(tuple(v.shape), **f32)
    if workspace is None:
        nbytes = gla_bwd_workspace_bytes(B, H, T, dk, dv, qdt)
        workspace = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=q.device)
    with torch.cuda.device(q.device):
        _check(lib.gla_bwd_layout(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(), d_out.data_ptr(),
                                  B, H, T, dk, dv, grid_h, grid_w, scan_dir, qdt, layout,
                                  fwd_workspace.data_ptr() if fwd_workspace is not None else None,
                                  fwd_workspace.numel() if fwd_workspace is not None else 0,
                                  dq.data_ptr(), dk_.data_ptr(), dv_.data_ptr(), dg.data_ptr(),
                                  workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return dq, dk_, dv_, dg


def gla_bwd(q, k, v, log_alpha, d_out, grid_h, grid_w, scan_dir=SCAN_ROW_FWD, workspace=None, stream=None,
            fwd_workspace=None):
    """Gradients (dq, dk, dv, dlog_alpha), all fp32, of a loss with upstream gradient ``d_out`` = dL/d out.
    q, k, v, d_out share one element type (bf16 or fp32); [B,H,T,d] order.  ``fwd_workspace``: the workspace
    tensor of the gla_fwd_ex call on the same tensors and scan order (untouched since, same options): its span
    states are reused instead of recomputed (gla_bwd_reuse)."""
    torch = _torch()
    lib = load_library()
    B, H, T, dk, dv = _prep(q, k, v, log_alpha, grid_h, grid_w)
    if d_out.shape != v.shape or d_out.dtype != v.dtype or not d_out.is_cuda or not d_out.is_contiguous():
        raise ValueError("d_out must be a contiguous GPU tensor shaped and typed like v")
    qdt = _dt(q)
    f32 = dict(dtype=torch.float32, device=q.device)
    dq, dk_ = torch.empty((B, H, T, dk), **f32), torch.empty((B, H, T, dk), **f32)
    dg, dv_ = torch.empty((B, H, T, dk), **f32), torch.empty((B, H, T, dv), **f32)
    if workspace is None:
        nbytes = gla_bwd_workspace_bytes(B, H, T, dk, dv, qdt)
        workspace = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device=q.device)
    with torch.cuda.device(q.device):
        if fwd_workspace is None:
            _check(lib.gla_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(), d_out.data_ptr(),
                               B, H, T, dk, dv, grid_h, grid_w, scan_dir, qdt,
                               dq.data_ptr(), dk_.data_ptr(), dv_.data_ptr(), dg.data_ptr(),
                               workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
        else:
            _check(lib.gla_bwd_reuse(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(), d_out.data_ptr(),
                                     B, H, T, dk, dv, grid_h, grid_w, scan_dir, qdt,
                                     fwd_workspace.data_ptr(), fwd_workspace.numel(),
                                     dq.data_ptr(), dk_.data_ptr(), dv_.data_ptr(), dg.data_ptr(),
                                     workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return dq, dk_, dv_, dg


def gla_calibrate_mfma(stream=None):
    """TFLOP/s of a register-resident v_mfma_f32_16x16x32_bf16 loop on the current device."""
    lib = load_library()
    x = ctypes.c_double(0.0)
    _check(lib.gla_calibrate_mfma(ctypes.byref(x), _stream_ptr(stream)))
    return float(x.value)


def gla_fwd_timed(q, k, v, log_alpha, grid_h, grid_w, scan_dir, out, final_state,
                  workspace, iters=10, stream=None):
    """Mean milliseconds per call: [span-state kernel, carry kernel, output kernel, whole call]."""
    torch = _torch()
    lib = load_library()
    B, H, T, dk, dv = _prep(q, k, v, log_alpha, grid_h, grid_w)
    ms = (ctypes.c_float * 4)()
    with torch.cuda.device(q.device):
        _check(lib.gla_fwd_timed(q.data_ptr(), k.data_ptr(), v.data_ptr(), log_alpha.data_ptr(),
                                 B, H, T, dk, dv, grid_h, grid_w, scan_dir, _dt(q), _dt(out),
                                 out.data_ptr(), final_state.data_ptr() if final_state is not None else None,
                                 workspace.data_ptr(), workspace.numel(), _stream_ptr(stream),
                                 int(iters), ms))
    return [float(x) for x in ms]
