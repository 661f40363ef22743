"""Pure-python, scalar-loop recomputation of the sparse block, patch by patch.

An independent pin for the oracle on tiny inputs: it follows the *gather ->
compute -> scatter* schedule (Sec. 3.1) literally -- cut the (S+2)x(S+2) window
around one active patch, run the three convolutions on it with python floats,
write the S x S result back -- whereas the oracle computes the dense block and
masks its output.  The two agree only if halo handling, padding, tap geometry,
weight layout and the residual add are all right.
"""
import numpy as np


def brute_index_list(mask):
    out = []
    N, G, GW = mask.shape
    for n in range(N):
        for gy in range(G):
            for gx in range(GW):
                if mask[n, gy, gx]:
                    out.append(n * G * GW + gy * GW + gx)
    return out


def brute_logits(x, Wm, bm, S):
    N, H, W, C = x.shape
    G, GW = H // S, W // S
    out = np.zeros((N, G, GW))
    for n in range(N):
        for gy in range(G):
            for gx in range(GW):
                acc = 0.0
                for c in range(C):
                    p = 0.0
                    for i in range(S):
                        for j in range(S):
                            p += float(x[n, gy * S + i, gx * S + j, c])
                    acc += float(Wm[c]) * (p / (S * S))
                out[n, gy, gx] = acc + bm
    return out


def brute_sparse_block(x, idx, S, W1, b1, W2, b2, W3, b3):
    x = np.asarray(x, dtype=np.float64)
    N, H, W, C = x.shape
    M = W1.shape[0]
    G, GW = H // S, W // S
    out = x.copy()
    T = S + 2
    for cell in idx:
        n, rem = divmod(int(cell), G * GW)
        gy, gx = divmod(rem, GW)
        # gather: window with one pixel of neighbours; conv1 on it
        y1 = [[[0.0] * M for _ in range(T)] for _ in range(T)]
        for wy in range(T):
            for wx in range(T):
                h, w = gy * S + wy - 1, gx * S + wx - 1
                if 0 <= h < H and 0 <= w < W:
                    for m in range(M):
                        a = float(b1[m])
                        for c in range(C):
                            a += float(x[n, h, w, c]) * float(W1[m, c])
                        y1[wy][wx][m] = a if a > 0.0 else 0.0
                # outside the image y1 stays 0 (zero padding of conv1's output)
        for i in range(S):
            for j in range(S):
                y2 = [0.0] * M
                for o in range(M):
                    a = float(b2[o])
                    for ky in range(3):
                        for kx in range(3):
                            src = y1[i + ky][j + kx]
                            for m in range(M):
                                a += src[m] * float(W2[o, ky, kx, m])
                    y2[o] = a if a > 0.0 else 0.0
                h, w = gy * S + i, gx * S + j
                for c in range(C):
                    a = float(b3[c])
                    for o in range(M):
                        a += y2[o] * float(W3[c, o])
                    out[n, h, w, c] = x[n, h, w, c] + a      # scatter + add
    return out
