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

A kernel that is not square takes the same formula with one matrix set per axis, U = G_h W G_w^T,
V = B_h^T X B_w, Y = A_h^T M A_w with n_h x n_w output blocks: along a side with k > 1 taps the generated
F(n, k) matrices, along a side with one tap (1 x k, k x 1 kernels) the trivial F(1, 1), whose three matrices
are the 1 x 1 identity.

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
    assert C == C2
    assert kh > 1 or kw > 1, "a 1 x 1 kernel has no Winograd form"
    ph, pw = (pad, pad) if np.isscalar(pad) else pad

    def axis(k_axis):
        """(n, alpha, A^T, G, B^T) of one axis: F(n, k) along a side with k > 1 taps, the identity for one tap."""
        if k_axis == 1:
            one = np.ones((1, 1), dtype=np.float64)
            return 1, 1, one, one, one
        mats = cook_toom.matrices(n, k_axis, f)
        return (n, n + k_axis - 1) + tuple(cook_toom.to_float(m) for m in mats)

    nh, ah, ATh, Gh, BTh = axis(kh)
    nw, aw, ATw, Gw, BTw = axis(kw)

    Ho, Wo = H + 2 * ph - kh + 1, W + 2 * pw - kw + 1
    th, tw = -(-Ho // nh), -(-Wo // nw)
    P = N * th * tw

    # step 2: filter transform  U[i,j,K,C]
    U = np.einsum("ir,kcrs,js->ijkc", Gh, w, Gw)

    # steps 1+3: gather tiles from the zero-extended input, transform
    Hp, Wp = (th - 1) * nh + ah, (tw - 1) * nw + aw
    xp = np.zeros((N, C, max(Hp, H + 2 * ph), max(Wp, W + 2 * pw)), dtype=np.float64)
    xp[:, :, ph:ph + H, pw:pw + W] = x
    V = np.empty((ah, aw, C, P), dtype=np.float64)
    for img in range(N):
        for ty in range(th):
            for tx in range(tw):
                p = (img * th + ty) * tw + tx
                d = xp[img, :, ty * nh:ty * nh + ah, tx * nw:tx * nw + aw]        # [C, a_h, a_w]
                V[:, :, :, p] = np.einsum("ia,cab,jb->ijc", BTh, d, BTw)

    # step 4: one matrix product per transformed position
    M = np.einsum("ijkc,ijcp->ijkp", U, V)

    # step 5: inverse transform, bias, clip
    y = np.zeros((N, K, th * nh, tw * nw), dtype=np.float64)
    for img in range(N):
        for ty in range(th):
            for tx in range(tw):
                p = (img * th + ty) * tw + tx
                m = M[:, :, :, p]                                                  # [a_h, a_w, K]
                yt = np.einsum("ia,abk,jb->kij", ATh, m, ATw)
                y[img, :, ty * nh:(ty + 1) * nh, tx * nw:(tx + 1) * nw] = yt
    y = y[:, :, :Ho, :Wo]
    if b is not None:
        y = y + np.asarray(b, dtype=np.float64)[None, :, None, None]
    y = np.ascontiguousarray(y)
    if return_stages:
        stages: Dict[str, np.ndarray] = {"AT": ATh, "G": Gh, "BT": BTh, "AT_w": ATw, "G_w": Gw, "BT_w": BTw,
                                         "U": U, "V": V, "M": M}
        return y, stages
    return y
