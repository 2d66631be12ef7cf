"""CPU fp64 oracle for the convolution of the spatial reorient & enhancement module (SREM) of DiG.

TEST INFRASTRUCTURE ONLY (same rules as ``gla_oracle.py``).

Algorithm 1 reshapes the block's token sequence to the 2-D token matrix, applies a 3x3 depth-wise convolution
(DWConv2d: every channel has its own 3x3 kernel, zero padding of one token, stride one, optional bias; Sec. 3.3)
and then transposes or flips the sequence for the next block.  The paper permutes the sequence physically, so
from the second block on the 2-D matrix that the convolution sees is the transposed and / or reversed one.
Here tensors stay in canonical (row-major) token order and ``orient`` names the order the paper's sequence
would be in (0 row-major, 1 reversed, 2 column-major, 3 column-major reversed); the oracle does what the paper
does, literally: permute, reshape2d, convolve, flatten, un-permute.
"""
from __future__ import annotations

import numpy as np

from . import gla_oracle


def identity_weights(D):
    """The paper's initialisation: kernel centre one, surroundings zero."""
    w = np.zeros((D, 3, 3))
    w[:, 1, 1] = 1.0
    return w


def dwconv2d(img, w, bias=None):
    """img [B, Hh, Ww, D], w [D, 3, 3]: y[r, c] = bias + sum_{dy,dx in -1..1} w[dy+1, dx+1] img[r+dy, c+dx],
    terms outside the matrix dropped (zero padding).  Plain loops over the nine taps."""
    img = np.asarray(img, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    B, Hh, Ww, D = img.shape
    y = np.zeros_like(img)
    for dy in (-1, 0, 1):
        for dx in (-1, 0, 1):
            r0, r1 = max(0, -dy), min(Hh, Hh - dy)
            c0, c1 = max(0, -dx), min(Ww, Ww - dx)
            if r0 < r1 and c0 < c1:
                y[:, r0:r1, c0:c1] += img[:, r0 + dy:r1 + dy, c0 + dx:c1 + dx] * w[:, dy + 1, dx + 1]
    if bias is not None:
        y += np.asarray(bias, dtype=np.float64)
    return y


def srem_dwconv(x, w, bias, grid_h, grid_w, orient=0):
    """x [B, T, D] in canonical token order; returns DWConv2d applied to the token matrix of the sequence
    ordered by ``orient``, brought back to canonical order, float64 [B, T, D]."""
    x = np.asarray(x, dtype=np.float64)
    B, T, D = x.shape
    if T != grid_h * grid_w:
        raise ValueError("T != grid_h * grid_w")
    perm = gla_oracle.scan_order(orient, grid_h, grid_w)       # sequence position -> canonical token
    rows, cols = (grid_h, grid_w) if orient < 2 else (grid_w, grid_h)
    seq = x[:, perm]                                           # the sequence as the paper holds it
    y_seq = dwconv2d(seq.reshape(B, rows, cols, D), w, bias).reshape(B, T, D)
    y = np.empty_like(y_seq)
    y[:, perm] = y_seq
    return y
