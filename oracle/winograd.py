"""float64 Winograd convolution, one step at a time.  TEST INFRASTRUCTURE ONLY.

Takes Section 3.3.1 in its own order and notation:

    Y = A^T [ sum_channel (G W G^T) (.) (B^T X B) ] A          (Winograd formula)

  1. block division from the output side: the output plane is cut into n x n
     blocks; each block reads the (n+k-1) x (n+k-1) input tile X whose origin is
     (block_row*n - pad, block_col*n - pad) in the zero-extended input
     (ragged blocks at the right/bottom edge are computed in full and clipped:
     ceil, not floor, of o/n -- the floor in the block-count formula would drop
     them);
  2. U = G W G^T per (output channel, input channel);
  3. V = B^T X B per (input channel, tile);
  4. the channel sum of Hadamard products is, for every position (i,j) of the
     transformed tile, a matrix product  M_ij[K, P] = U_ij[K, C] @ V_ij[C, P]
     (item (2) of that section: "Hadamard product -> matrix multiplication");
  5. Y = A^T M A per (output channel, tile), plus the bias, clipped to H_o x W_o.

Stride 1, dilation 1 only (the paper gives no Winograd form for anything
else).  The matrices come from oracle.cook_toom and are widened to float64.
The intermediate tensors are returned too so that each device stage can be
compared on its own.
"""
from __future__ import annotations

from fractions import Fraction
from typing import Dict, Optional

import numpy as np

from . import cook_toom


def winograd_conv2d(x: np.ndarray, w: np.ndarray, b: Optional[np.ndarray], n: int, pad=0,
                    f: Fraction = Fraction(1, 2), return_stages: bool = False):
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    N, C, H, W = x.shape
    K, C2, kh, kw = w.shape
    assert C == C2 and kh == kw, "square kernels only"
    k = kh
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    alpha = n + k - 1
    AT_q, G_q, BT_q = cook_toom.matrices(n, k, f)
    AT, G, BT = (cook_toom.to_float(m) for m in (AT_q, G_q, BT_q))

    Ho, Wo = H + 2 * ph - k + 1, W + 2 * pw - k + 1
    th, tw = -(-Ho // n), -(-Wo // n)
    P = N * th * tw

    # step 2: filter transform  U[i,j,K,C]
    U = np.einsum("ir,kcrs,js->ijkc", G, w, G)

    # steps 1+3: gather tiles from the zero-extended input, transform
    Hp, Wp = (th - 1) * n + alpha, (tw - 1) * n + alpha
    xp = np.zeros((N, C, max(Hp, H + 2 * ph), max(Wp, W + 2 * pw)), dtype=np.float64)
    xp[:, :, ph:ph + H, pw:pw + W] = x
    V = np.empty((alpha, alpha, C, P), dtype=np.float64)
    for img in range(N):
        for ty in range(th):
            for tx in range(tw):
                p = (img * th + ty) * tw + tx
                d = xp[img, :, ty * n:ty * n + alpha, tx * n:tx * n + alpha]      # [C, a, a]
                V[:, :, :, p] = np.einsum("ia,cab,jb->ijc", BT, d, BT)

    # step 4: one matrix product per transformed position
    M = np.einsum("ijkc,ijcp->ijkp", U, V)

    # step 5: inverse transform, bias, clip
    y = np.zeros((N, K, th * n, tw * n), dtype=np.float64)
    for img in range(N):
        for ty in range(th):
            for tx in range(tw):
                p = (img * th + ty) * tw + tx
                m = M[:, :, :, p]                                                  # [a, a, K]
                yt = np.einsum("ia,abk,jb->kij", AT, m, AT)
                y[img, :, ty * n:(ty + 1) * n, tx * n:(tx + 1) * n] = yt
    y = y[:, :, :Ho, :Wo]
    if b is not None:
        y = y + np.asarray(b, dtype=np.float64)[None, :, None, None]
    y = np.ascontiguousarray(y)
    if return_stages:
        stages: Dict[str, np.ndarray] = {"AT": AT, "G": G, "BT": BT, "U": U, "V": V, "M": M}
        return y, stages
    return y
