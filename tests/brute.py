"""Independent brute-force enumerators used to pin the oracle (tests only).

Structurally different from the oracle on purpose: every output first
materialises ALL K candidate sums in an array (padded taps hold the semiring
identity, -inf for max-plus and +inf for min-plus, paper Sec. 3.1), then numpy's
argmax / argmin (first occurrence = lowest tap index) picks the winner.  Nothing
here imports the oracle or the HIP binding.
"""
import numpy as np


def out_hw(H, W, KH, KW, stride, pad, dil):
    return ((H + 2 * pad - dil * (KH - 1) - 1) // stride + 1,
            (W + 2 * pad - dil * (KW - 1) - 1) // stride + 1)


def candidates(x, w, n, co, oh, ow, stride, pad, dil, fill, dtype=np.float32):
    """All K sums for one output, in flattened tap order k = (c*KH + i)*KW + j."""
    _, C, H, W = x.shape
    _, _, KH, KW = w.shape
    out = np.full(C * KH * KW, fill, dtype=dtype)
    for c in range(C):
        for i in range(KH):
            for j in range(KW):
                ih, iw = oh * stride - pad + i * dil, ow * stride - pad + j * dil
                if 0 <= ih < H and 0 <= iw < W:
                    out[(c * KH + i) * KW + j] = dtype(x[n, c, ih, iw]) + dtype(w[co, c, i, j])
    return out


def forward(x, w, want_max, stride=1, pad=0, dil=1, dtype=np.float32):
    """(y, idx) of one branch by enumeration."""
    N, C, H, W = x.shape
    CO, _, KH, KW = w.shape
    ho, wo = out_hw(H, W, KH, KW, stride, pad, dil)
    y = np.empty((N, CO, ho, wo), dtype)
    idx = np.empty((N, CO, ho, wo), np.int32)
    fill = -np.inf if want_max else np.inf
    for n in range(N):
        for co in range(CO):
            for oh in range(ho):
                for ow in range(wo):
                    s = candidates(x, w, n, co, oh, ow, stride, pad, dil, fill, dtype)
                    k = int(np.argmax(s)) if want_max else int(np.argmin(s))
                    y[n, co, oh, ow], idx[n, co, oh, ow] = s[k], k
    return y, idx


def combine(y_min, y_max, alpha, beta):
    """fl(fl(alpha*y_min) + fl(beta*y_max)) per output channel, fp32, no fused multiply-add."""
    a = np.ones(y_min.shape[1], np.float32) if alpha is None else alpha.astype(np.float32)
    b = np.ones(y_min.shape[1], np.float32) if beta is None else beta.astype(np.float32)
    pa = (a[None, :, None, None] * y_min.astype(np.float32)).astype(np.float32)
    pb = (b[None, :, None, None] * y_max.astype(np.float32)).astype(np.float32)
    return (pa + pb).astype(np.float32)


def scatter_backward(xshape, wshape, idx, g, stride, pad, dil):
    """grad_x, grad_w (float64) from one branch's indices and per-output gradients g."""
    N, C, H, W = xshape
    CO, _, KH, KW = wshape
    gx = np.zeros(xshape, np.float64)
    gw = np.zeros(wshape, np.float64)
    _, _, ho, wo = idx.shape
    for n in range(N):
        for co in range(CO):
            for oh in range(ho):
                for ow in range(wo):
                    k = int(idx[n, co, oh, ow])
                    c, r = divmod(k, KH * KW)
                    i, j = divmod(r, KW)
                    gx[n, c, oh * stride - pad + i * dil, ow * stride - pad + j * dil] += g[n, co, oh, ow]
                    gw[co, c, i, j] += g[n, co, oh, ow]
    return gx, gw


def forward_mixed(x, w, outer_max, stride=1, pad=0, dil=1, dtype=np.float32):
    """(y, idx) of the mixed layers of paper Sec. 3.1 by enumeration: every output's K candidate sums are
    laid out as [C_in, KH*KW]; the inner operator reduces each row (min-plus under an outer max = layer
    (iii), max-plus under an outer min = layer (vi)), the outer one the column of row results.  numpy's
    argmin / argmax return the first occurrence, i.e. the lowest tap and the lowest channel."""
    N, C, H, W = x.shape
    CO, _, KH, KW = w.shape
    ho, wo = out_hw(H, W, KH, KW, stride, pad, dil)
    y = np.empty((N, CO, ho, wo), dtype)
    idx = np.empty((N, CO, ho, wo), np.int32)
    fill = np.inf if outer_max else -np.inf          # identity of the INNER operator
    for n in range(N):
        for co in range(CO):
            for oh in range(ho):
                for ow in range(wo):
                    s = candidates(x, w, n, co, oh, ow, stride, pad, dil, fill, dtype).reshape(C, KH * KW)
                    t = np.argmin(s, axis=1) if outer_max else np.argmax(s, axis=1)
                    v = s[np.arange(C), t]
                    c = int(np.argmax(v)) if outer_max else int(np.argmin(v))
                    y[n, co, oh, ow], idx[n, co, oh, ow] = v[c], c * KH * KW + int(t[c])
    return y, idx
