"""Small, independent statements of the paper's algorithms used to pin the C++ oracle.

Nothing here is shared with the oracle or with the GPU path: these are numpy float64 (or exact
`fractions.Fraction`) re-codings of the algorithm boxes and of textbook routines, written for
tiny sizes.  The only thing they take from the oracle is the list of chosen blocks, which the
selector tests pin separately.
"""
from fractions import Fraction

import numpy as np


def column_mask(block_mask, d, block):
    """Expand a per-block 0/1 mask to per-column booleans for a flat d-vector cut into blocks."""
    return np.repeat(np.asarray(block_mask, dtype=bool), block)[:d]


def psync_np(V, cols):
    """Algorithm PSync on V[W][d] with a GRBS compressor keeping the columns in `cols`."""
    Vc = np.where(cols[None, :], V, 0.0)          # v'_i = C(v_i)
    Rres = V - Vc                                   # r_i = v_i - v'_i
    vbar = Vc.mean(axis=0)                          # (1/n) sum_i v'_i
    return vbar[None, :] + Rres, Rres               # v'_i = vbar' + r_i ; r_i


def nesterov_sgd(x0, grads, lr, beta):
    """Sutskever form of Nesterov momentum (Section 3.2): m = beta m + g; x -= lr (beta m + g)."""
    x = np.array(x0, dtype=np.float64)
    m = np.zeros_like(x)
    for g in grads:
        m = beta * m + g
        x = x - lr * (beta * m + g)
    return x, m


def alg2_cser(x0, grads, step_masks, reset_masks, H, lr, block):
    """Algorithm 2 (CSER without momentum), written out: grads[t] is [W][d]."""
    W, d = grads[0].shape
    x = np.tile(np.asarray(x0, dtype=np.float64), (W, 1))
    e = np.zeros((W, d))
    for t, g in enumerate(grads, start=1):
        gp, r = psync_np(g, column_mask(step_masks[t], d, block))
        x = x - lr * gp
        e = e - lr * r
        if t % H == 0:
            ep, enew = psync_np(e, column_mask(reset_masks[t], d, block))
            x = x - e + ep
            e = enew
    return x, e


def csea_impl1(x0, grads, reset_masks, lr, block):
    """CSEA, implementation I (Appendix A.1.1): p = e - lr g; e', e = PSync(p, C1); x += e' - e_old."""
    W, d = grads[0].shape
    x = np.tile(np.asarray(x0, dtype=np.float64), (W, 1))
    e = np.zeros((W, d))
    for t, g in enumerate(grads, start=1):
        p = e - lr * g
        ep, enew = psync_np(p, column_mask(reset_masks[t], d, block))
        x = x + ep - e
        e = enew
    return x, e


def cser_pl_impl1(x0, grads, reset_masks, H, lr, block):
    """CSER-PL, implementation I (Appendix A.1.2): plain local steps, PSync of e every H."""
    W, d = grads[0].shape
    x = np.tile(np.asarray(x0, dtype=np.float64), (W, 1))
    e = np.zeros((W, d))
    for t, g in enumerate(grads, start=1):
        x = x - lr * g
        e = e - lr * g
        if t % H == 0:
            ep, enew = psync_np(e, column_mask(reset_masks[t], d, block))
            x = x + ep - e
            e = enew
    return x, e


def local_sgd(x0, grads, H, lr):
    """Local SGD with synchronisation interval H: local steps, full model average every H."""
    W, d = grads[0].shape
    x = np.tile(np.asarray(x0, dtype=np.float64), (W, 1))
    for t, g in enumerate(grads, start=1):
        x = x - lr * g
        if t % H == 0:
            x = np.tile(x.mean(axis=0), (W, 1))
    return x


def mcser_exact(x0, grads, step_masks, reset_masks, H, lr, beta, block):
    """Algorithm 3 in exact rational arithmetic (python Fractions), element by element.

    x0: list of d Fractions; grads[t-1][i][j] Fractions; masks: dict t -> per-block 0/1.
    Returns x, e, m as nested lists [W][d] of Fractions.
    """
    W = len(grads[0])
    d = len(x0)
    lr, beta = Fraction(lr), Fraction(beta)
    x = [[Fraction(v) for v in x0] for _ in range(W)]
    e = [[Fraction(0)] * d for _ in range(W)]
    m = [[Fraction(0)] * d for _ in range(W)]

    def psync(v, bmask):
        vp = [[v[i][j] if bmask[j // block] else Fraction(0) for j in range(d)] for i in range(W)]
        r = [[v[i][j] - vp[i][j] for j in range(d)] for i in range(W)]
        vbar = [sum(vp[i][j] for i in range(W)) / W for j in range(d)]
        return [[vbar[j] + r[i][j] for j in range(d)] for i in range(W)], r

    for t, g in enumerate(grads, start=1):
        p = [[None] * d for _ in range(W)]
        for i in range(W):
            for j in range(d):
                m[i][j] = beta * m[i][j] + g[i][j]
                p[i][j] = lr * (beta * m[i][j] + g[i][j])
        pp, r = psync(p, step_masks[t])
        for i in range(W):
            for j in range(d):
                x[i][j] -= pp[i][j]
                e[i][j] -= r[i][j]
        if H > 0 and t % H == 0:
            ep, enew = psync(e, reset_masks[t])
            for i in range(W):
                for j in range(d):
                    x[i][j] = x[i][j] - e[i][j] + ep[i][j]
            e = enew
    return x, e, m
