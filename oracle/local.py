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


def rejection_islands(mask, W, n0):
    """Rejection islands (Sec. 3.4, Eq. 8): the 8-connected components of R_X on the 2-D token grid.

    mask: bool/uint8 [L] for block positions n0 .. n0+L-1 of a grid with W columns.  Two marked positions
    are neighbours when their rows and their columns each differ by at most one (columns do not wrap).
    Returns (island int32 [L], rank int32 [L], n_islands, largest):
      island[t] = 0 for an unmarked position, else 1 + the smallest block position of its island (a label
                  that does not depend on the order in which the components are found);
      rank[t]   = number of positions of the same island before t in raster order (-1 if unmarked): islands
                  are re-sampled concurrently, the positions inside one in this order, so pass r handles
                  every position of rank r and `largest` passes finish the block.
    Plain flood fill, one island at a time."""
    mask = np.asarray(mask).astype(bool)
    L = mask.shape[0]
    island = np.zeros(L, dtype=np.int32)
    rank = np.full(L, -1, dtype=np.int32)
    n_islands, largest = 0, 0
    for start in range(L):
        if not mask[start] or island[start]:
            continue
        n_islands += 1
        members, stack = [], [start]
        island[start] = start + 1
        while stack:
            t = stack.pop()
            members.append(t)
            g = n0 + t
            i, j = g // W, g % W
            for di in (-1, 0, 1):
                for dj in (-1, 0, 1):
                    jj = j + dj
                    if (di == 0 and dj == 0) or jj < 0 or jj >= W:
                        continue
                    u = (i + di) * W + jj - n0
                    if 0 <= u < L and mask[u] and not island[u]:
                        island[u] = start + 1
                        stack.append(u)
        for r, t in enumerate(sorted(members)):
            rank[t] = r
        largest = max(largest, len(members))
    return island, rank, n_islands, largest
