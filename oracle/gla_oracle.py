"""CPU fp64 oracle for the GLA token mixer of DiG (forward pass, and its reverse-mode derivative).

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the
``cpu_baseline`` leg of the benchmark may import this module; the product
package never does, and this module never imports the product package.

Two renderings of the same definition live here:

* :func:`gla_fwd` calls the plain-C fp64 loop nest of ``gla_oracle.c`` (built
  by :func:`build` into ``libgla_oracle.so`` next to this file);
* :func:`gla_fwd_numpy` is the same token-by-token recurrence in numpy, kept
  so that the two can be checked against each other and so that an
  ``initial_state`` experiment needs no compiler.

Both follow the recurrence of Sec. 3.1 (Eq. (attn_gla), rows 1-3) with the gate
G_t reduced to its key-side factor alpha_t (beta_t = 1):

    S_t = diag(alpha_t) S_{t-1} + k_t^T v_t ,   o_t = q_t S_t ,   S_0 = 0,

run along a scan order of the token grid (Sec. 3.3 / Algorithm 1: transpose and
flip alternate between blocks, giving row-major, column-major and their two
reversals).  ``log_alpha`` holds log(alpha_t) <= 0.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

SCAN_ROW_FWD, SCAN_ROW_REV, SCAN_COL_FWD, SCAN_COL_REV = 0, 1, 2, 3
SCAN_NAMES = {0: "row_fwd", 1: "row_rev", 2: "col_fwd", 3: "col_rev"}

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gla_oracle.c")
_SRC_BWD = os.path.join(_HERE, "gla_oracle_bwd.c")
_LIB = os.path.join(_HERE, "libgla_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile gla_oracle.c and gla_oracle_bwd.c with gcc (-O2, no fast-math, OpenMP over b*h)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_BWD))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp",
               "-o", _LIB, _SRC, _SRC_BWD, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.gla_oracle_fwd.restype = ctypes.c_int
        lib.gla_oracle_fwd.argtypes = [dp, dp, dp, dp, dp] + [ctypes.c_int] * 8 + [dp, dp, ctypes.c_int]
        lib.gla_oracle_bwd.restype = ctypes.c_int
        lib.gla_oracle_bwd.argtypes = [dp] * 5 + [ctypes.c_int] * 8 + [dp] * 4 + [ctypes.c_int]
        lib.gla_oracle_scan_index.restype = ctypes.c_long
        lib.gla_oracle_scan_index.argtypes = [ctypes.c_int, ctypes.c_long, ctypes.c_int, ctypes.c_int]
        lib.gla_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def scan_index(scan_dir: int, s: int, grid_h: int, grid_w: int) -> int:
    """Canonical token index visited at scan step s (C implementation)."""
    return int(_load().gla_oracle_scan_index(scan_dir, s, grid_h, grid_w))


def scan_order(scan_dir: int, grid_h: int, grid_w: int) -> np.ndarray:
    """pi[s] = canonical (row-major) token index visited at scan step s.

    Written with numpy reshapes, the way the paper's operators are named:
    row-major order is the flattened grid; column-major order is the flattened
    transposed grid; the reversed orders are those sequences flipped.
    """
    T = grid_h * grid_w
    grid = np.arange(T, dtype=np.int64).reshape(grid_h, grid_w)
    if scan_dir in (SCAN_ROW_FWD, SCAN_ROW_REV):
        seq = grid.reshape(-1)
    elif scan_dir in (SCAN_COL_FWD, SCAN_COL_REV):
        seq = grid.T.reshape(-1)
    else:
        raise ValueError("scan_dir")
    if scan_dir in (SCAN_ROW_REV, SCAN_COL_REV):
        seq = seq[::-1]
    return np.ascontiguousarray(seq)


SCHEDULE_BLOCK_PROCESS = 0   # Algorithm 1: transpose after blocks with even index, flip after odd ones
SCHEDULE_BLOCK_SCAN = 1      # Algorithm 4 (supplement): flip after even, transpose after odd


def block_scan_dir(block: int, schedule: int = SCHEDULE_BLOCK_PROCESS, grid: int = 4) -> int:
    """Scan order in which DiG block ``block`` (1-based, the paper's l) sees the tokens when the transposes and flips
    that the paper applies to the sequence after every block (Algorithm 1; Algorithm 4 with the parities swapped)
    are left out and the sequence stays in canonical row-major order.

    Done the paper's way on an index array of a ``grid`` x ``grid`` token matrix: start from the row-major
    sequence, after every block before ``block`` apply its operator (reshape2d, transpose, flatten; or flip), and
    name the resulting order by comparing it with the four scan orders.
    """
    if block < 1 or schedule not in (SCHEDULE_BLOCK_PROCESS, SCHEDULE_BLOCK_SCAN) or grid < 2:
        raise ValueError("block / schedule / grid")
    seq = np.arange(grid * grid, dtype=np.int64)
    for l in range(1, block):
        transpose = (l % 2 == 0) if schedule == SCHEDULE_BLOCK_PROCESS else (l % 2 == 1)
        if transpose:
            seq = np.ascontiguousarray(seq.reshape(grid, grid).T).reshape(-1)
        else:
            seq = seq[::-1].copy()
    for d in (SCAN_ROW_FWD, SCAN_ROW_REV, SCAN_COL_FWD, SCAN_COL_REV):
        if np.array_equal(seq, scan_order(d, grid, grid)):
            return d
    raise AssertionError("the sequence left the four scan orders")


def _as_f64(x, shape):
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    if a.shape != tuple(shape):
        raise ValueError(f"shape {a.shape} != {tuple(shape)}")
    return a


def gla_fwd(q, k, v, log_alpha, grid_h, grid_w, scan_dir=SCAN_ROW_FWD,
            initial_state=None, nthreads=0):
    """fp64 token-by-token GLA forward (C loop nest).

    q, k, log_alpha: [B,H,T,dk]; v: [B,H,T,dv].  Returns (out [B,H,T,dv],
    final_state [B,H,dk,dv]) as float64 arrays.
    """
    q = np.asarray(q)
    B, H, T, dk = q.shape
    dv = np.asarray(v).shape[-1]
    q = _as_f64(q, (B, H, T, dk))
    k = _as_f64(k, (B, H, T, dk))
    g = _as_f64(log_alpha, (B, H, T, dk))
    v = _as_f64(v, (B, H, T, dv))
    s0 = None if initial_state is None else _as_f64(initial_state, (B, H, dk, dv))
    out = np.empty((B, H, T, dv), dtype=np.float64)
    fin = np.empty((B, H, dk, dv), dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    p = lambda a: a.ctypes.data_as(dp)
    rc = _load().gla_oracle_fwd(p(q), p(k), p(v), p(g),
                                p(s0) if s0 is not None else None,
                                B, H, T, dk, dv, grid_h, grid_w, scan_dir,
                                p(out), p(fin), int(nthreads))
    if rc != 0:
        raise ValueError("gla_oracle_fwd rejected its arguments")
    return out, fin


def gla_fwd_multi(q, k, v, log_alpha, grid_h, grid_w, scan_dirs, nthreads=0):
    """Multi-directional scanning (supplement, Algorithms 2 and 3): the same mixer applied along several scan
    orders of the token grid, every result brought back to canonical token order, and the results added.
    ``scan_dirs`` is an iterable of scan orders, e.g. (0, 1) for the bidirectional and (0, 1, 2, 3) for the
    4-directional variant.  Returns the sum [B,H,T,dv] in float64."""
    total = None
    for d in scan_dirs:
        o, _ = gla_fwd(q, k, v, log_alpha, grid_h, grid_w, d, nthreads=nthreads)
        total = o if total is None else total + o
    if total is None:
        raise ValueError("no scan order given")
    return total


def gla_bwd(q, k, v, log_alpha, d_out, grid_h, grid_w, scan_dir=SCAN_ROW_FWD, nthreads=0):
    """fp64 reverse-mode derivative of :func:`gla_fwd` (zero initial state, loss depending on ``out`` only),
    one scan step at a time (C loop nest of ``gla_oracle_bwd.c``).

    d_out: [B,H,T,dv] = dL/d out.  Returns (dq, dk, dv, dlog_alpha) as float64 arrays shaped like the inputs.
    """
    q = np.asarray(q)
    B, H, T, dk = q.shape
    dv = np.asarray(v).shape[-1]
    q = _as_f64(q, (B, H, T, dk))
    k = _as_f64(k, (B, H, T, dk))
    g = _as_f64(log_alpha, (B, H, T, dk))
    v = _as_f64(v, (B, H, T, dv))
    do = _as_f64(d_out, (B, H, T, dv))
    dq = np.empty((B, H, T, dk), dtype=np.float64)
    dk_ = np.empty((B, H, T, dk), dtype=np.float64)
    dg = np.empty((B, H, T, dk), dtype=np.float64)
    dv_ = np.empty((B, H, T, dv), dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    p = lambda a: a.ctypes.data_as(dp)
    rc = _load().gla_oracle_bwd(p(q), p(k), p(v), p(g), p(do), B, H, T, dk, dv, grid_h, grid_w, scan_dir,
                                p(dq), p(dk_), p(dv_), p(dg), int(nthreads))
    if rc != 0:
        raise ValueError("gla_oracle_bwd rejected its arguments")
    return dq, dk_, dv_, dg


def threads() -> int:
    return int(_load().gla_oracle_threads())


def gla_fwd_numpy(q, k, v, log_alpha, grid_h, grid_w, scan_dir=SCAN_ROW_FWD,
                  initial_state=None):
    """The same recurrence, one token at a time, in numpy fp64."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g = np.asarray(log_alpha, dtype=np.float64)
    B, H, T, dk = q.shape
    dv = v.shape[-1]
    if grid_h * grid_w != T:
        raise ValueError("grid")
    pi = scan_order(scan_dir, grid_h, grid_w)
    out = np.zeros((B, H, T, dv))
    S = np.zeros((B, H, dk, dv)) if initial_state is None else np.array(initial_state, dtype=np.float64)
    for s in range(T):
        n = pi[s]
        alpha = np.exp(g[:, :, n, :])                                   # [B,H,dk]
        S = alpha[..., None] * S + k[:, :, n, :, None] * v[:, :, n, None, :]
        out[:, :, n, :] = np.einsum("bhc,bhcj->bhj", q[:, :, n, :], S)
    return out, S
