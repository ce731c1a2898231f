"""Dense-matrix brute force of the sampling framework, for graphs of a few dozen vertices.

Every step is the matrix expression of the paper written out with dense numpy arrays:
P = Q A as a dense product, inverse-transform sampling as a literal prefix sum over a
dense row of P followed by a linear scan, extraction as dense row/column selection.
The only thing taken from the oracle is the random stream (key, draw, range reduction),
which is an input of the method, not part of what is being checked.
"""
import numpy as np

from oracle import bms_oracle as O


def dense_adjacency(rowptr, col):
    n = len(rowptr) - 1
    A = np.zeros((n, n), dtype=np.int64)
    for v in range(n):
        A[v, col[rowptr[v]:rowptr[v + 1]]] = 1
    return A


def its_literal(weights, r):
    """Smallest t with inclusive prefix sum of `weights` > r (linear scan)."""
    acc = 0
    for t, w in enumerate(weights):
        acc += int(w)
        if acc > r:
            return t
    raise AssertionError("draw outside the total weight")


def distinct_positions_literal(key, deg, s):
    """s distinct positions of a row of deg unit weights: each draw is ITS on the weight
    vector whose already chosen entries are zero (Sec. 4.1.2, sampling without replacement)."""
    w = [1] * deg
    out = []
    for j in range(s):
        total = sum(w)
        r = O.bounded32(O.draw32(key, j), total)
        t = its_literal(w, r)
        out.append(t)
        w[t] = 0
    return sorted(out)


def nodewise(A, batches, fanouts, seed, mb_base=0, union_dst=False, replace=False):
    """Alg. 1 for GraphSAGE with dense matrices. Returns per minibatch, per hop:
    (frontier ids, dense sampled adjacency A^l (rows x kept columns), kept column ids).

    replace: every draw is ITS on the untouched unit weights of the row (independent draws), the picks are the
    nonzeros of Q'.  union_dst: the columns of the frontier's own vertices are kept even when empty."""
    n = A.shape[0]
    out = []
    for i, batch in enumerate(batches):
        F = [int(v) for v in batch]
        hops = []
        for h, s in enumerate(fanouts):
            Q = np.zeros((len(F), n), dtype=np.int64)
            for r, v in enumerate(F):
                Q[r, v] = 1                       # one nonzero per row, in column v_r
            P = Q @ A                             # row r = neighbourhood of v_r
            Qnext = np.zeros_like(P)
            for r, v in enumerate(F):
                w = P[r].copy()
                key = O.rowkey(seed, h, mb_base + i, v)
                if replace:
                    if w.sum() > 0:
                        for j in range(s):
                            Qnext[r, its_literal(w, O.bounded32(O.draw32(key, j), int(w.sum())))] = 1
                    continue
                if w.sum() <= s:
                    Qnext[r] = (w > 0)
                    continue
                for j in range(s):
                    rr = O.bounded32(O.draw32(key, j), int(w.sum()))
                    t = its_literal(w, rr)
                    Qnext[r, t] = 1
                    w[t] = 0
            nonempty = Qnext.sum(axis=0) > 0              # remove empty columns
            if union_dst:
                nonempty = nonempty | (Q.sum(axis=0) > 0)
            kept = np.nonzero(nonempty)[0]
            hops.append((list(F), Qnext[:, kept], kept))
            F = [int(v) for v in kept]
        out.append(hops)
    return out


def ladies(A, batches, s_per_layer, seed, mb_base=0, squared=False):
    """Alg. 1 for LADIES with dense matrices. Returns per minibatch, per hop:
    (frontier ids, dense row of P (length n), sampled ids ascending, dense A_S)."""
    n = A.shape[0]
    out = []
    for i, batch in enumerate(batches):
        F = [int(v) for v in batch]
        hops = []
        for h, s in enumerate(s_per_layer):
            Q = np.zeros((1, n), dtype=np.int64)
            Q[0, F] = 1                           # one row, a nonzero per frontier vertex
            P = (Q @ A)[0]                        # e_v
            w = P * P if squared else P
            W = int(w.sum())
            picks = set()
            if W > 0:
                key = O.rowkey(seed, h, mb_base + i, O.NOVERTEX)
                for j in range(s):
                    r = O.bounded64(O.draw64(key, j), W)
                    picks.add(its_literal(w, r))
            S = sorted(picks)
            QR = np.zeros((len(F), n), dtype=np.int64)
            for r, v in enumerate(F):
                QR[r, v] = 1                      # row extraction matrix
            QC = np.zeros((n, len(S)), dtype=np.int64)
            for c, v in enumerate(S):
                QC[v, c] = 1                      # column extraction matrix
            AS = QR @ A @ QC
            hops.append((list(F), P, S, AS))
            F = S
        out.append(hops)
    return out


def hop_block_dense(hop, i):
    """Dense (rows x cols) 0/1 block of minibatch i from a stacked CSR hop (oracle or library)."""
    r0, r1 = int(hop.mb_rowoff[i]), int(hop.mb_rowoff[i + 1])
    c0, c1 = int(hop.mb_coloff[i]), int(hop.mb_coloff[i + 1])
    M = np.zeros((r1 - r0, c1 - c0), dtype=np.int64)
    for r in range(r0, r1):
        cols = hop.col[hop.rowptr[r]:hop.rowptr[r + 1]]
        assert (np.diff(cols) > 0).all(), "columns must ascend inside a row"
        M[r - r0, cols] += 1
    return M
