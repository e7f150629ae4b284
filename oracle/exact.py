"""Winograd and direct convolution in exact rational arithmetic (test oracle).

Test infrastructure only; see the package docstring.  Pure-Python loops over
`fractions.Fraction`: meant for inputs of a few tiles and a few channels.

The 2D algorithm is the nesting of the 1D one (App. "2D Extension via Kronecker
Products" and the reconstruction formula in "Exact Zero with Rational
Arithmetic"):  Y = A^T [ (G g G^T) * (B^T d B) ] A  for one n x n input tile d
and one 3 x 3 filter g, summed over input channels before the output transform.
"""
from fractions import Fraction


def _matmul(a, b):
    return [[sum((a[i][k] * b[k][j] for k in range(len(b))), Fraction(0))
             for j in range(len(b[0]))] for i in range(len(a))]


def _transpose(a):
    return [list(col) for col in zip(*a)]


def direct_conv2d(x, g):
    """y[n][k][h][w] = sum_{c,a,b} g[k][c][a][b] * xpad[n][c][h+a][w+b], xpad = x with a
    zero border of (r-1)/2 pixels: stride 1, no kernel flip (Sec. 2.1, y_i = sum_k g_k x_{i+k}).
    x: [N][C][H][W], g: [K][C][r][r] (r odd; 3 in the paper's experiments), nested lists of
    ints or Fractions."""
    N, C, H, W = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0])
    K = len(g)
    r = len(g[0][0])
    pad = (r - 1) // 2
    y = [[[[Fraction(0)] * W for _ in range(H)] for _ in range(K)] for _ in range(N)]
    for n in range(N):
        for k in range(K):
            for h in range(H):
                for w in range(W):
                    acc = Fraction(0)
                    for c in range(C):
                        for a in range(r):
                            for b in range(r):
                                hh, ww = h + a - pad, w + b - pad
                                if 0 <= hh < H and 0 <= ww < W:
                                    acc += Fraction(g[k][c][a][b]) * Fraction(x[n][c][hh][ww])
                    y[n][k][h][w] = acc
    return y


def winograd_conv2d(x, g, A, BT, G):
    """Same result through F(m x m, r x r) tiles with the exact matrices A, B^T, G.
    The padded image is cut into n x n tiles at stride m (n = m + r - 1); positions outside
    the image, including those of a ragged last tile row / column, read as zero and the
    outputs beyond H x W are dropped."""
    N, C, H, W = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0])
    K = len(g)
    n, m = len(A), len(A[0])
    pad = (n - m) // 2                       # (r - 1) / 2
    B = _transpose(BT)
    GT = _transpose(G)
    AT = _transpose(A)
    U = [[_matmul(_matmul(G, [[Fraction(v) for v in row] for row in g[k][c]]), GT)
          for c in range(C)] for k in range(K)]
    y = [[[[Fraction(0)] * W for _ in range(H)] for _ in range(K)] for _ in range(N)]
    for img in range(N):
        for h0 in range(0, H, m):
            for w0 in range(0, W, m):
                V = []
                for c in range(C):
                    d = [[Fraction(x[img][c][h0 - pad + a][w0 - pad + b])
                          if 0 <= h0 - pad + a < H and 0 <= w0 - pad + b < W else Fraction(0)
                          for b in range(n)] for a in range(n)]
                    V.append(_matmul(_matmul(BT, d), B))
                for k in range(K):
                    Mk = [[sum((U[k][c][i][j] * V[c][i][j] for c in range(C)), Fraction(0))
                           for j in range(n)] for i in range(n)]
                    Y = _matmul(_matmul(AT, Mk), A)
                    for p in range(m):
                        for q in range(m):
                            if h0 + p < H and w0 + q < W:
                                y[img][k][h0 + p][w0 + q] = Y[p][q]
    return y


def winograd_1d(x, g, A, BT, G):
    """y = A^T [ (G g) * (B^T x) ] for one length-n input (Sec. 2.1 steps 1-4)."""
    n, m = len(A), len(A[0])
    gt = [sum((G[p][k] * Fraction(g[k]) for k in range(len(g))), Fraction(0)) for p in range(n)]
    xt = [sum((BT[p][j] * Fraction(x[j]) for j in range(n)), Fraction(0)) for p in range(n)]
    return [sum((A[p][i] * gt[p] * xt[p] for p in range(n)), Fraction(0)) for i in range(m)]
