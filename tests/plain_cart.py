"""Plaintext reference used to pin the oracle: level-wise Gini CART on binary
candidate columns with the same rules the secure protocol follows (Sec. II-A and
Sec. V-B of the paper): complete tree of depth H, node types 0/1/2 =
internal/leaf/dummy, a real leaf that holds more than one class is split on the
unused candidate with the largest score sum_j S_j/Q_j (= 1 - Gini index), lowest
index on ties, the quotients taken as floor(S * 2^tau / Q).  Pure Python integers;
no code shared with the oracle or the GPU library."""
from fractions import Fraction

import numpy as np


def scores_fixed(n1, tot, tau):
    """n1[k][c], tot[c] -> list of floor-quotient scores per candidate k."""
    n = int(sum(tot))
    out = []
    for k in range(len(n1)):
        s = 0
        for j in (0, 1):
            njc = [int(n1[k][c]) if j else int(tot[c]) - int(n1[k][c]) for c in range(len(tot))]
            nj = sum(njc)
            S, Q = sum(v * v for v in njc), nj * n
            s += (S << tau) // (Q if Q else 1)
        out.append(s)
    return out


def scores_exact(n1, tot):
    n = int(sum(tot))
    out = []
    for k in range(len(n1)):
        s = Fraction(0)
        for j in (0, 1):
            njc = [int(n1[k][c]) if j else int(tot[c]) - int(n1[k][c]) for c in range(len(tot))]
            nj = sum(njc)
            if nj * n:
                s += Fraction(sum(v * v for v in njc), nj * n)
        out.append(s)
    return out


def gini_real(n1, tot):
    """Weighted Gini index of the definition in Sec. II-A, in floating point."""
    n = float(sum(tot))
    out = []
    for k in range(len(n1)):
        g = 0.0
        for j in (0, 1):
            njc = np.array([float(n1[k][c]) if j else float(tot[c]) - float(n1[k][c]) for c in range(len(tot))])
            nj = njc.sum()
            if nj > 0:
                g += nj / n * (1.0 - ((njc / nj) ** 2).sum())
        out.append(g)
    return out


def train(X, y, K, H, tau):
    X = np.asarray(X).astype(np.int64)
    y = np.asarray(y).astype(np.int64)
    N, d = X.shape
    nn = (2 << H) - 1
    T = np.zeros(nn, dtype=np.int64)
    F = np.zeros(nn, dtype=np.int64)
    F[0] = 1
    M = np.zeros(N, dtype=np.int64)
    Cn1 = {0: np.zeros((d, K), dtype=np.int64)}
    Ctot = {0: np.zeros(K, dtype=np.int64)}
    gam = {0: np.ones(d, dtype=np.int64)}
    levels = []
    for h in range(H + 1):
        nh, base = 1 << h, (1 << h) - 1
        if h > 0:
            M = 2 * M + X[np.arange(N), T[M]] + 1
        rec = dict(M=M.copy(), n1=[], tot=[], score=[], SD=[], gamma=[], split=[])
        nCn1, nCtot, ngam = {}, {}, {}
        for r in range(nh):
            node = base + r
            n1, tot = Cn1[r].copy(), Ctot[r].copy()
            if F[node] == 1:
                sel = M == node
                for c in range(K):
                    tot[c] += int((sel & (y == c)).sum())
                    if h < H:
                        n1[:, c] += X[sel & (y == c)].sum(axis=0)
            rec["n1"].append(n1); rec["tot"].append(tot)
            if h == H:
                T[node] = int(np.argmax(tot))            # first maximum
                continue
            sc = [s * int(g) for s, g in zip(scores_fixed(n1, tot, tau), gam[r])]
            sd = int(np.argmax(sc))
            g2 = gam[r].copy(); g2[sd] = 0
            n = int(tot.sum())
            pure = n * n - int((tot * tot).sum()) == 0
            split = int(F[node] == 1 and not pure)
            F[node] = F[node] * (1 - split)
            F[2 * node + 1] = F[2 * node + 2] = 2 - split
            T[node] = sd
            for ch in (0, 1):
                nCn1[2 * r + ch] = n1 * (1 - split)
                nCtot[2 * r + ch] = tot * (1 - split)
                ngam[2 * r + ch] = g2.copy()
            rec["score"].append(sc); rec["SD"].append(sd); rec["gamma"].append(g2); rec["split"].append(split)
        levels.append(rec)
        Cn1, Ctot, gam = nCn1, nCtot, ngam
    return dict(T=T, F=F, M=M, levels=levels)


def predict(T, H, X, thr=None):
    """Walk the complete tree: feature ids at levels < H, labels at level H."""
    X = np.asarray(X).astype(np.int64)
    N = X.shape[0]
    idx = np.zeros(N, dtype=np.int64)
    for _ in range(H):
        v = X[np.arange(N), T[idx]]
        bit = v if thr is None else (v > np.asarray(thr).astype(np.int64)[idx]).astype(np.int64)
        idx = 2 * idx + 1 + bit
    return T[idx]
