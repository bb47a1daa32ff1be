"""Step 5 of the method: local rejection and expansion (Sec. 3.3, Eq. 6-7).
Test infrastructure.

R_T is the set of rejected positions of the block, t_0 the first of them.
N(t, l) = { u : |i_u - i_t| <= l, |j_u - j_t| <= l, u >= t_0 } on the true 2-D
coordinates (no wrap across rows), R_X the union of N(t, l) over t in R_T.
Positions outside the drafted block do not exist yet (Alg. 1 advances n by L
afterwards), so R_X is cut to the block.  `expand` dilation steps of radius l
are one dilation of Chebyshev radius expand * l; expand = 1 is Eq. 6-7 as
printed, expand = 0 is the "naive local verification" of the ablation
(R_X = R_T).  radius = -1 selects the raster-scan rule of standard speculative
decoding (everything from t_0 on), kept for comparison.
"""
import numpy as np


def local_mask(accept, W, n0, radius, expand=1):
    """accept: bool/uint8 [L] for block positions n0 .. n0+L-1 of a grid with
    W columns (raster order).  Returns (mask uint8 [L], t0 int); t0 = L when
    nothing was rejected."""
    accept = np.asarray(accept).astype(bool)
    L = accept.shape[0]
    mask = np.zeros(L, dtype=np.uint8)
    R_T = np.flatnonzero(~accept)
    if R_T.size == 0:
        return mask, L
    t0 = int(R_T[0])
    u = np.arange(L)
    if radius < 0:
        mask[u >= t0] = 1
        return mask, t0
    rho = int(radius) * int(expand)
    iu, ju = (n0 + u) // W, (n0 + u) % W
    for t in R_T:
        it, jt = (n0 + t) // W, (n0 + t) % W
        inside = (np.abs(iu - it) <= rho) & (np.abs(ju - jt) <= rho) & (u >= t0)
        mask[inside] = 1
    return mask, t0
