"""Plain fp64 CPU oracle for the GSPN line-scan propagation.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its
Python binding) may import, call or link this module; only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` do.
It shares no code with the GPU path and imports nothing from it.

What is computed (GSPN-2 paper, Sec. 3.2 Eq. 1-2, Sec. 4.2 shared-weight
recurrence and Eq. 3):

    h_i = T_i h_{i-1} + lambda_i (.) x_i        (Eq. 1; T_i tridiagonal)
    y_i = u_i (.) h_i                           (Eq. 2)

swept line by line over the feature map in up to four scan directions
(top->bottom, bottom->top, left->right, right->left; Sec. 3.2), the
per-direction outputs merged by a plain sum.  The three weights of T_i are
shared by the channels of one weight group (Sec. 4.2: one ``w_i`` for all
channels; ``G = C`` gives the per-channel weights of Eq. 1).

Every function takes and returns float64 numpy arrays.  Storage-precision
rounding (bf16 / fp32) is applied to the *inputs* by the caller before they
reach this module; nothing here rounds.

Readings of points the paper leaves open (each is pinned by a test):
  * state before the first line is zero, so h_0 = lambda_0 (.) x_0 (first
    block row of Eq. 3 is just Lambda_1);
  * a neighbour outside the line contributes 0, whatever weight is passed;
  * weight plane k (k = 0, 1, 2) multiplies the neighbour at offset k-1 along
    the orthogonal axis *in image coordinates* (column index for the vertical
    scans, row index for the horizontal scans), not mirrored for the reversed
    directions;
  * w, lambda, u carry a leading direction axis of 4 (one parameter set per
    direction); x is shared;
  * channel c belongs to group c // (C // G).

Backward: the paper gives no algorithm for it (only timings, Sec. 5.1); the
formulas here are the chain rule applied to Eq. 1-2 with the sum merge.

Parity pins (tests/test_oracle_*.py): dense solve of (I - A) h = lambda*x with
A assembled in image coordinates per direction, the explicit block
lower-triangular product form of Eq. 3, the width-1 scalar recurrence closed
form, identity weights -> cumulative sum, the row-stochastic constant
invariant, group replication, linearity, central finite differences, the
adjoint identity and the dense transposed operator for the backward.
GSPN-local (scan_fwd_local / scan_bwd_local, tests/test_oracle_local.py): the
dense solve with the links between stretches removed, kchunk = 1 (no
propagation: y = sum_d u_d lam_d x) and kchunk >= scan length (the global
scan), confinement of a perturbation to its stretch, central finite
differences and the adjoint identity for the backward.
Weights as logits (weights_from_logits, scan_*_logits, tests/test_oracle_logits.py):
scipy's softmax on the taps that exist, rows of the assembled T_i summing to
1, shift invariance, indifference to what a masked logit holds, central finite
differences through the logits.
Proxy projections (proxy_project, tests/test_oracle_proxy.py): explicit loops,
identity and selection matrices, composition of two projections.
"""
from __future__ import annotations

import numpy as np

DIR_TB, DIR_BT, DIR_LR, DIR_RL = 0, 1, 2, 3
ALL_DIRS = (DIR_TB, DIR_BT, DIR_LR, DIR_RL)


def _dirs_of(dir_mask: int):
    if not (1 <= dir_mask <= 15):
        raise ValueError("dir_mask must be in 1..15")
    return [d for d in ALL_DIRS if (dir_mask >> d) & 1]


# --------------------------------------------------------------------------
# view transforms: bring direction d into canonical form (scan along axis -2
# from index 0 upward, line along axis -1) and back.  Only axis swaps and flips
# of the scan axis; the orthogonal axis is never reversed, which is what makes
# weight plane k mean "offset k-1 in image coordinates" for every direction.
# --------------------------------------------------------------------------
def _to_canonical(a: np.ndarray, d: int) -> np.ndarray:
    if d == DIR_TB:
        return a
    if d == DIR_BT:
        return a[..., ::-1, :]
    if d == DIR_LR:
        return np.swapaxes(a, -1, -2)
    if d == DIR_RL:
        return np.swapaxes(a, -1, -2)[..., ::-1, :]
    raise ValueError(d)


def _from_canonical(a: np.ndarray, d: int) -> np.ndarray:
    if d == DIR_TB:
        return a
    if d == DIR_BT:
        return a[..., ::-1, :]
    if d == DIR_LR:
        return np.swapaxes(a, -1, -2)
    if d == DIR_RL:
        return np.swapaxes(a[..., ::-1, :], -1, -2)
    raise ValueError(d)


def _shift_from_left(a: np.ndarray) -> np.ndarray:
    """out[..., j] = a[..., j-1], 0 at j = 0."""
    out = np.zeros_like(a)
    out[..., 1:] = a[..., :-1]
    return out


def _shift_from_right(a: np.ndarray) -> np.ndarray:
    """out[..., j] = a[..., j+1], 0 at j = L-1."""
    out = np.zeros_like(a)
    out[..., :-1] = a[..., 1:]
    return out


def _expand_groups(wline: np.ndarray, cpg: int) -> np.ndarray:
    """[B, G, L] -> [B, C, L]: channel c reads group c // cpg (Sec. 4.2)."""
    return np.repeat(wline, cpg, axis=1)


# --------------------------------------------------------------------------
# forward
# --------------------------------------------------------------------------
def scan_canonical(x, w, lam):
    """Hidden state of Eq. 1 for the canonical direction.

    x, lam : [B, C, S, L]   scan axis S (serial), line axis L (parallel)
    w      : [B, G, 3, S, L]
    returns h : [B, C, S, L]
    """
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    B, C, S, L = x.shape
    G = w.shape[1]
    if C % G != 0 or w.shape != (B, G, 3, S, L) or lam.shape != x.shape:
        raise ValueError("shape mismatch")
    cpg = C // G
    h = np.empty_like(x)
    prev = np.zeros((B, C, L))
    for i in range(S):
        w0 = _expand_groups(w[:, :, 0, i, :], cpg)
        w1 = _expand_groups(w[:, :, 1, i, :], cpg)
        w2 = _expand_groups(w[:, :, 2, i, :], cpg)
        cur = (w0 * _shift_from_left(prev) + w1 * prev + w2 * _shift_from_right(prev)
               + lam[:, :, i, :] * x[:, :, i, :])
        h[:, :, i, :] = cur
        prev = cur
    return h


def scan_fwd(x, w, lam, u, dir_mask=15):
    """Merged output and per-direction hidden states (Eq. 1, Eq. 2, sum merge).

    x        : [B, C, H, W]
    w        : [4, B, G, 3, H, W]   normalised weights, image coordinates
    lam, u   : [4, B, C, H, W]
    returns  y [B, C, H, W]  and  h [4, B, C, H, W] (zeros for unmasked dirs)
    """
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    y = np.zeros_like(x)
    h_all = np.zeros((4,) + x.shape)
    for d in _dirs_of(dir_mask):
        hc = scan_canonical(_to_canonical(x, d), _to_canonical(w[d], d), _to_canonical(lam[d], d))
        h = _from_canonical(hc, d)
        h_all[d] = h
        y += u[d] * h
    return y, h_all


# --------------------------------------------------------------------------
# backward (chain rule on Eq. 1-2; the paper states no backward algorithm)
# --------------------------------------------------------------------------
def scan_canonical_bwd(gy, x, w, lam, u, h):
    """Gradients for one direction in canonical coordinates.

    With e_i = dL/dh_i:   e_i = u_i*gy_i + T_{i+1}^T e_{i+1},  e past the last line = 0
      gu_i   = gy_i * h_i
      glam_i = x_i * e_i
      gx_i   = lam_i * e_i
      gw_i[k][j] = sum_{c in group} e_i[j] * h_{i-1}[j+k-1]   (0 on the first line / outside)
    returns gx, gw, glam, gu
    """
    gy = np.asarray(gy, dtype=np.float64)
    B, C, S, L = x.shape
    G = w.shape[1]
    cpg = C // G
    gx = np.empty_like(x)
    glam = np.empty_like(x)
    gu = gy * h
    gw = np.zeros_like(w)
    e_next = np.zeros((B, C, L))       # e_{i+1}
    for i in range(S - 1, -1, -1):
        e = u[:, :, i, :] * gy[:, :, i, :]
        if i + 1 < S:
            w0 = _expand_groups(w[:, :, 0, i + 1, :], cpg)
            w1 = _expand_groups(w[:, :, 1, i + 1, :], cpg)
            w2 = _expand_groups(w[:, :, 2, i + 1, :], cpg)
            # (T^T e)[j] = w2[j-1] e[j-1] + w1[j] e[j] + w0[j+1] e[j+1]
            e = e + _shift_from_left(w2 * e_next) + w1 * e_next + _shift_from_right(w0 * e_next)
        glam[:, :, i, :] = x[:, :, i, :] * e
        gx[:, :, i, :] = lam[:, :, i, :] * e
        if i > 0:
            hp = h[:, :, i - 1, :]
            per_c = np.stack([e * _shift_from_left(hp), e * hp, e * _shift_from_right(hp)], axis=2)
            gw[:, :, :, i, :] = per_c.reshape(B, G, cpg, 3, L).sum(axis=2)
        e_next = e
    return gx, gw, glam, gu


def scan_bwd(gy, x, w, lam, u, h_all, dir_mask=15):
    """Gradients of L w.r.t. x, w, lam, u given gy = dL/dy (sum merge).

    returns gx [B,C,H,W], gw [4,B,G,3,H,W], glam [4,B,C,H,W], gu [4,B,C,H,W]
    (slots of unmasked directions are zero).
    """
    gy = np.asarray(gy, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    h_all = np.asarray(h_all, dtype=np.float64)
    gx = np.zeros_like(x)
    gw = np.zeros_like(w)
    glam = np.zeros_like(lam)
    gu = np.zeros_like(u)
    for d in _dirs_of(dir_mask):
        c = lambda a: np.ascontiguousarray(_to_canonical(a, d))
        gxd, gwd, glamd, gud = scan_canonical_bwd(c(gy), c(x), c(w[d]), c(lam[d]), c(u[d]), c(h_all[d]))
        gx += _from_canonical(gxd, d)
        gw[d] = _from_canonical(gwd, d)
        glam[d] = _from_canonical(glamd, d)
        gu[d] = _from_canonical(gud, d)
    return gx, gw, glam, gu


# --------------------------------------------------------------------------
# GSPN-local (Sec. 3.2): propagation confined to stretches of `kchunk` lines
# --------------------------------------------------------------------------
def _stretches(S: int, kchunk: int):
    """The scan axis [0, S) cut into stretches of kchunk lines, the last one shorter when kchunk does
    not divide S.  The cut is made in image coordinates, so it is the same for a direction and its
    reverse (reading: the paper only says that each row or column is split into fixed-length segments)."""
    if kchunk < 1:
        raise ValueError("kchunk must be >= 1")
    return [(a, min(a + kchunk, S)) for a in range(0, S, kchunk)]


def _cut(a, d, lo, hi):
    """Lines lo..hi-1 of the scan axis of direction d (rows for the vertical scans, columns otherwise)."""
    return a[..., lo:hi, :] if d < 2 else a[..., :, lo:hi]


def scan_fwd_local(x, w, lam, u, kchunk, dir_mask=15):
    """GSPN-local forward: every stretch of kchunk lines along the scan axis is a scan of its own (Eq. 1-2
    on the sub-image, state zero before the stretch's first line in scan order), written out as exactly
    that: one call of the global scan per (direction, stretch).  Shapes as in scan_fwd."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    H, W = x.shape[-2:]
    y = np.zeros_like(x)
    h_all = np.zeros((4,) + x.shape)
    for d in _dirs_of(dir_mask):
        for lo, hi in _stretches(H if d < 2 else W, kchunk):
            ys, hs = scan_fwd(_cut(x, d, lo, hi), _cut(w, d, lo, hi), _cut(lam, d, lo, hi), _cut(u, d, lo, hi), 1 << d)
            _cut(y, d, lo, hi)[...] += ys
            _cut(h_all[d], d, lo, hi)[...] = hs[d]
    return y, h_all


def scan_bwd_local(gy, x, w, lam, u, h_all, kchunk, dir_mask=15):
    """GSPN-local backward: the gradients of every (direction, stretch) scan on its own sub-image; gx is
    summed over the directions, gw of a stretch's first line in scan order is zero.  Shapes as in scan_bwd."""
    gy = np.asarray(gy, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    lam = np.asarray(lam, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    h_all = np.asarray(h_all, dtype=np.float64)
    H, W = x.shape[-2:]
    gx = np.zeros_like(x)
    gw = np.zeros_like(w)
    glam = np.zeros_like(lam)
    gu = np.zeros_like(u)
    for d in _dirs_of(dir_mask):
        for lo, hi in _stretches(H if d < 2 else W, kchunk):
            c = lambda a: _cut(a, d, lo, hi)
            gxs, gws, gls, gus = scan_bwd(c(gy), c(x), c(w), c(lam), c(u), c(h_all), 1 << d)
            c(gx)[...] += gxs
            c(gw[d])[...] = gws[d]
            c(glam[d])[...] = gls[d]
            c(gu[d])[...] = gus[d]
    return gx, gw, glam, gu


# --------------------------------------------------------------------------
# weights given as raw logits (the normalisation of Sec. 3.2 done on the way in)
# --------------------------------------------------------------------------
def _outside_taps(d, H, W):
    """[3, H, W] bool: tap k at (r, c) addresses a neighbour outside the line (column c+k-1 for the vertical
    scans, row r+k-1 for the horizontal ones, image coordinates)."""
    out = np.zeros((3, H, W), dtype=bool)
    if d < 2:
        out[0, :, 0] = True
        out[2, :, W - 1] = True
    else:
        out[0, 0, :] = True
        out[2, H - 1, :] = True
    return out


def weights_from_logits(z):
    """Row-stochastic tridiagonal weights from raw logits (Sec. 3.2: the weights are "learned and normalized"
    so that every row of T_i sums to 1; the normaliser taken here is the softmax over the three taps).
    A tap whose neighbour lies outside the line gets weight 0 and takes no part in the normalisation, whatever
    its logit holds -- so the rows at the ends of a line are stochastic over the two neighbours that exist.

    z : [4, B, G, 3, H, W] -> w of the same shape
    """
    z = np.asarray(z, dtype=np.float64)
    H, W = z.shape[-2:]
    w = np.zeros_like(z)
    for d in ALL_DIRS:
        out = _outside_taps(d, H, W)
        zd = np.where(out, -np.inf, z[d])                 # what a masked logit holds (NaN included) is never used
        m = zd.max(axis=-3, keepdims=True)
        e = np.exp(zd - m)
        w[d] = e / e.sum(axis=-3, keepdims=True)
    return w


def logits_grad_from_weights_grad(gw, w):
    """Gradient w.r.t. the logits given the gradient w.r.t. the normalised weights (softmax over the taps,
    per position): gz_k = w_k (gw_k - sum_j w_j gw_j).  Taps outside the line have w = 0, hence gz = 0."""
    gw = np.asarray(gw, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    return w * (gw - (w * gw).sum(axis=-3, keepdims=True))


def scan_fwd_logits(x, z, lam, u, dir_mask=15, kchunk=None):
    """Forward scan with the weights given as logits z [4, B, G, 3, H, W]; otherwise as scan_fwd
    (scan_fwd_local with kchunk)."""
    w = weights_from_logits(z)
    if kchunk is None:
        return scan_fwd(x, w, lam, u, dir_mask)
    return scan_fwd_local(x, w, lam, u, kchunk, dir_mask)


def scan_bwd_logits(gy, x, z, lam, u, h_all, dir_mask=15, kchunk=None):
    """Backward scan with the weights given as logits: returns gx, gz, glam, gu (gz in place of gw)."""
    w = weights_from_logits(z)
    if kchunk is None:
        gx, gw, glam, gu = scan_bwd(gy, x, w, lam, u, h_all, dir_mask)
    else:
        gx, gw, glam, gu = scan_bwd_local(gy, x, w, lam, u, h_all, kchunk, dir_mask)
    return gx, logits_grad_from_weights_grad(gw, w), glam, gu


# --------------------------------------------------------------------------
# compressive proxy projections (Sec. 4.2): 1x1 convolutions over the channel axis
# --------------------------------------------------------------------------
def proxy_project(inp, P):
    """out[b, m, h, w] = sum_k P[m, k] * inp[b, k, h, w]: the projection of Sec. 4.2 that takes x from C
    channels to C_proxy before the scan (P: [C_proxy, C]) and the learned 1x1 projection back (P: [C, C_proxy])."""
    inp = np.asarray(inp, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    if P.ndim != 2 or inp.ndim != 4 or P.shape[1] != inp.shape[1]:
        raise ValueError("shape mismatch")
    return np.einsum("mk,bkhw->bmhw", P, inp)


def proxy_project_bwd(gout, inp, P):
    """Gradients of out = proxy_project(inp, P) for a loss L with gout = dL/dout (chain rule on the sum above):
        gin[b, k, h, w] = sum_m P[m, k] * gout[b, m, h, w]
        gP[m, k]        = sum over b, h, w of gout[b, m, h, w] * inp[b, k, h, w]
    Returns (gin, gP)."""
    gout = np.asarray(gout, dtype=np.float64)
    inp = np.asarray(inp, dtype=np.float64)
    P = np.asarray(P, dtype=np.float64)
    if P.ndim != 2 or inp.ndim != 4 or gout.ndim != 4 or P.shape[1] != inp.shape[1] or P.shape[0] != gout.shape[1]:
        raise ValueError("shape mismatch")
    if gout.shape[0] != inp.shape[0] or gout.shape[2:] != inp.shape[2:]:
        raise ValueError("shape mismatch")
    gin = np.einsum("mk,bmhw->bkhw", P, gout)
    gP = np.einsum("bmhw,bkhw->mk", gout, inp)
    return gin, gP


def proxy_scan_fwd(x, Pd, w, lam, u, Pu, dir_mask=15):
    """The scan wrapped in the compressive proxy (Sec. 4.2): project down, propagate in the proxy space with the
    shared weights, project back.  x [B,C,H,W]; Pd [Cp,C]; w [4,B,G,3,H,W]; lam, u [4,B,Cp,H,W]; Pu [C,Cp]."""
    yp, _ = scan_fwd(proxy_project(x, Pd), w, lam, u, dir_mask)
    return proxy_project(yp, Pu)


def proxy_scan_bwd(gy, x, Pd, w, lam, u, Pu, dir_mask=15):
    """Gradients through the wrapped scan (chain rule over its three stages, each with its own definition above):
    returns (gx, gPd, gw, glam, gu, gPu) for y = proxy_scan_fwd(x, Pd, w, lam, u, Pu) and gy = dL/dy."""
    xp = proxy_project(x, Pd)
    yp, h = scan_fwd(xp, w, lam, u, dir_mask)
    gyp, gPu = proxy_project_bwd(gy, yp, Pu)
    gxp, gw, glam, gu = scan_bwd(gyp, xp, w, lam, u, h, dir_mask)
    gx, gPd = proxy_project_bwd(gxp, x, Pd)
    return gx, gPd, gw, glam, gu, gPu


# --------------------------------------------------------------------------
# dense forms used only to pin the scans on tiny inputs
# --------------------------------------------------------------------------
def tridiagonal(w_line):
    """Dense L x L matrix T with T[j, j+k-1] = w_line[k, j] (Sec. 3.2: each
    element of a line connects to three neighbours of the previous line)."""
    w_line = np.asarray(w_line, dtype=np.float64)
    L = w_line.shape[-1]
    T = np.zeros((L, L))
    for j in range(L):
        for k in range(3):
            jj = j + k - 1
            if 0 <= jj < L:
                T[j, jj] = w_line[k, j]
    return T


def eq3_block_matrix(w_bg, lam_bc):
    """The block lower-triangular matrix of Eq. 3 for one (batch, channel) in
    canonical coordinates: block (i, j) = T_i T_{i-1} ... T_{j+1} Lambda_j for
    j <= i (empty product = identity), zero above the diagonal.

    w_bg : [3, S, L]   lam_bc : [S, L]   returns [S*L, S*L]
    """
    w_bg = np.asarray(w_bg, dtype=np.float64)
    lam_bc = np.asarray(lam_bc, dtype=np.float64)
    S, L = lam_bc.shape
    T = [tridiagonal(w_bg[:, i, :]) for i in range(S)]
    M = np.zeros((S * L, S * L))
    for i in range(S):
        for j in range(i + 1):
            P = np.eye(L)
            for k in range(j + 1, i + 1):      # later index on the left
                P = T[k] @ P
            M[i * L:(i + 1) * L, j * L:(j + 1) * L] = P @ np.diag(lam_bc[j])
    return M


def one_step_matrix_image(w_dbg, d, H, W, kchunk=None):
    """A [H*W, H*W] with A[p, q] = weight with which pixel q (on the previous
    line of direction d) feeds pixel p, written directly in image coordinates
    (row-major pixel index r*W + c) without any view transform.  With kchunk
    (GSPN-local) a pixel is fed only from its own stretch of kchunk lines.

    w_dbg : [3, H, W] weights of direction d for one (batch, group)
    """
    w_dbg = np.asarray(w_dbg, dtype=np.float64)
    A = np.zeros((H * W, H * W))
    for r in range(H):
        for c in range(W):
            for k in range(3):
                if d == DIR_TB:
                    rr, cc = r - 1, c + k - 1
                elif d == DIR_BT:
                    rr, cc = r + 1, c + k - 1
                elif d == DIR_LR:
                    rr, cc = r + k - 1, c - 1
                else:
                    rr, cc = r + k - 1, c + 1
                if kchunk is not None and (r // kchunk != rr // kchunk if d < 2 else c // kchunk != cc // kchunk):
                    continue
                if 0 <= rr < H and 0 <= cc < W:
                    A[r * W + c, rr * W + cc] = w_dbg[k, r, c]
    return A


def dense_fwd(x, w, lam, u, dir_mask=15, kchunk=None):
    """y and h by solving (I - A_d) h_d = lam_d * x per (direction, batch,
    channel): the recurrence h = A h + lam*x with A strictly "previous line"
    (nilpotent), which is Eq. 3 written without choosing a line order.  With
    kchunk the links that leave a stretch of kchunk lines are absent."""
    x = np.asarray(x, dtype=np.float64)
    B, C, H, W = x.shape
    G = w.shape[2]
    cpg = C // G
    y = np.zeros_like(x)
    h_all = np.zeros((4,) + x.shape)
    eye = np.eye(H * W)
    for d in _dirs_of(dir_mask):
        for b in range(B):
            for c in range(C):
                A = one_step_matrix_image(w[d, b, c // cpg], d, H, W, kchunk)
                rhs = (np.asarray(lam[d, b, c], dtype=np.float64) * x[b, c]).reshape(-1)
                h = np.linalg.solve(eye - A, rhs).reshape(H, W)
                h_all[d, b, c] = h
                y[b, c] += np.asarray(u[d, b, c], dtype=np.float64) * h
    return y, h_all
