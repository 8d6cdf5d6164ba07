"""Brute-force definitions in pure Python (lists, math.exp, explicit loops).

Used only on tiny inputs to pin the C oracle.  Written directly from the
textbook statements: softmax attention (Sec. 3.1 Eq. (1) with the exponential
similarity of Sec. 3.2), average pooling over windows, a 3x3 depthwise
cross-correlation with zero padding, and bilinear interpolation with
half-pixel centres.  No numpy arithmetic is used on purpose.
"""
import math


def attention(Q, K, V, scale, bias=None):
    M, L = len(Q), len(K)
    d, dv = len(Q[0]), len(V[0])
    out = []
    for i in range(M):
        sims = []
        for j in range(L):
            s = 0.0
            for c in range(d):
                s += Q[i][c] * K[j][c]
            s = s * scale
            if bias is not None:
                s += bias[i][j]
            sims.append(math.exp(s))          # no max subtraction: tiny inputs only
        tot = sum(sims)
        row = []
        for c in range(dv):
            acc = 0.0
            for j in range(L):
                acc += sims[j] / tot * V[j][c]
            row.append(acc)
        out.append(row)
    return out


def pool(Q, gh, gw, ah, aw):
    """Adaptive average pooling of tokens t = y*gw+x onto the ah x aw agent grid."""
    d = len(Q[0])
    A = []
    for ay in range(ah):
        for ax in range(aw):
            ys = [y for y in range(gh) if (ay * gh) // ah <= y < -((-(ay + 1) * gh) // ah)]
            xs = [x for x in range(gw) if (ax * gw) // aw <= x < -((-(ax + 1) * gw) // aw)]
            row = []
            for c in range(d):
                tot = 0.0
                for y in ys:
                    for x in xs:
                        tot += Q[y * gw + x][c]
                row.append(tot / (len(ys) * len(xs)))
            A.append(row)
    return A


def dwc(V, wgt, b, gh, gw):
    d = len(V[0])
    out = [[0.0] * d for _ in range(gh * gw)]
    for y in range(gh):
        for x in range(gw):
            for c in range(d):
                acc = b[c] if b is not None else 0.0
                for ky in range(3):
                    for kx in range(3):
                        yy, xx = y + ky - 1, x + kx - 1
                        if 0 <= yy < gh and 0 <= xx < gw:
                            acc += wgt[c][ky][kx] * V[yy * gw + xx][c]
                out[y * gw + x][c] = acc
    return out


def bilinear(plane, h, w):
    h0, w0 = len(plane), len(plane[0])

    def coord(dst, L, L0):
        s = max((dst + 0.5) * L0 / L - 0.5, 0.0)
        lo = min(int(math.floor(s)), L0 - 1)
        hi = min(lo + 1, L0 - 1)
        return lo, hi, s - lo

    out = [[0.0] * w for _ in range(h)]
    for y in range(h):
        y0, y1, fy = coord(y, h, h0)
        for x in range(w):
            x0, x1, fx = coord(x, w, w0)
            out[y][x] = ((1 - fy) * ((1 - fx) * plane[y0][x0] + fx * plane[y0][x1])
                         + fy * ((1 - fx) * plane[y1][x0] + fx * plane[y1][x1]))
    return out


def agent_attention(Q, K, V, A, scale1, scale2, B1=None, B2=None):
    """Sec. 4.1 Eq. (3): Attn^S(Q, A, Attn^S(A, K, V))."""
    VA = attention(A, K, V, scale1, B1)
    return attention(Q, A, VA, scale2, B2)
