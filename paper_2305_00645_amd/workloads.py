"""Seeded synthetic inputs shaped like the paper's workloads.

Input generation only: nothing here shares, multiplies, compares or trains.
Every function returns plain numpy arrays; callers secret-share them.  The five
recipes stand in for the experiments of the paper's evaluation (its UCI data sets
are not available and are not reproduced): C1 a unit-scale check, C2 the shape of
the 267 x 22 heart data, C3 the shape of the 48,842 x 14 census data after
discretisation, C4 the 10^4-instance depth-7 inference batch, C5 a scale test.
"""
import numpy as np

PROTOCOL_SEED = [
    [0x243F6A8885A308D3, 0x13198A2E03707344, 0xA4093822299F31D0, 0x082EFA98EC4E6C89],
    [0x452821E638D01377, 0xBE5466CF34E90C6C, 0xC0AC29B7C97C50DD, 0x3F84D5B5B5470917],
    [0x9216D5D98979FB1B, 0xD1310BA698DFB5AC, 0x2FFD72DBD01ADFB7, 0xB8E1AFED6A267E96],
    [0xBA7C9045F12C7F99, 0x24A19947B3916CF7, 0x0801F2E2858EFC16, 0x636920D871574E69],
    [0xA458FEA3F4933D7E, 0x0D95748F728EB658, 0x718BCD5882154AEE, 0x7B54A41DC25A59B5],
]


def _onehot(y, K):
    Y = np.zeros((y.size, K), dtype=np.uint64)
    Y[np.arange(y.size), y] = 1
    return Y


def c1_train(N=256, d=16, depth=3, seed=1001):
    """Bernoulli(0.5) columns; labels from a random depth-`depth` tree, 5% flipped."""
    rng = np.random.default_rng(seed)
    X = (rng.random((N, d)) < 0.5).astype(np.uint64)
    nint = (1 << depth) - 1
    feat = np.zeros(nint, dtype=np.int64)
    for node in range(nint):                     # distinct features along each path
        used, a = set(), node
        while a > 0:
            a = (a - 1) // 2
            used.add(int(feat[a]))
        feat[node] = rng.choice([k for k in range(d) if k not in used])
    leaf = rng.integers(0, 2, size=1 << depth)
    idx = np.zeros(N, dtype=np.int64)
    for _ in range(depth):
        idx = 2 * idx + 1 + X[np.arange(N), feat[idx]].astype(np.int64)
    y = leaf[idx - nint]
    flip = rng.random(N) < 0.05
    y = np.where(flip, 1 - y, y)
    return dict(X=X, Y=_onehot(y, 2), y=y, N=N, d=d, K=2, H=depth)


def c2_train(N=267, d=22, H=7, seed=1002):
    """Column k ~ Bernoulli(p_k), p_k ~ U[0.2, 0.8]; 21% positives driven by 5 columns."""
    rng = np.random.default_rng(seed)
    p = rng.uniform(0.2, 0.8, size=d)
    X = (rng.random((N, d)) < p).astype(np.uint64)
    inf = rng.choice(d, size=5, replace=False)
    w = rng.normal(0.0, 1.5, size=5)
    logit = X[:, inf].astype(np.float64) @ w + rng.normal(0.0, 0.7, size=N)
    y = (logit > np.quantile(logit, 0.79)).astype(np.int64)
    return dict(X=X, Y=_onehot(y, 2), y=y, N=N, d=d, K=2, H=H)


C3_CARD = (2, 5, 6, 7, 9, 15, 16, 42)


def c3_train(N=48842, H=7, n_thr=32, seed=1003):
    """6 continuous features cut at `n_thr` quantiles each (columns [x > t]) and 8
    Zipf-distributed categorical features one-hot encoded: 6*n_thr + 102 columns."""
    rng = np.random.default_rng(seed)
    cont = np.concatenate([rng.lognormal(0.0, 1.0, size=(N, 3)), rng.uniform(0.0, 1.0, size=(N, 3))], axis=1)
    cols = []
    for f in range(6):
        qs = np.quantile(cont[:, f], (np.arange(n_thr) + 1.0) / (n_thr + 1.0))
        cols.append((cont[:, f][:, None] > qs[None, :]).astype(np.uint64))
    cats = []
    for card in C3_CARD:
        pz = 1.0 / np.arange(1, card + 1) ** 1.2
        pz /= pz.sum()
        cvals = rng.choice(card, size=N, p=pz)
        cats.append(cvals)
        oh = np.zeros((N, card), dtype=np.uint64)
        oh[np.arange(N), cvals] = 1
        cols.append(oh)
    X = np.ascontiguousarray(np.concatenate(cols, axis=1))
    z = (0.9 * np.log(cont[:, 0]) + 1.2 * (cont[:, 3] - 0.5) + 0.8 * (cats[2] == 0) - 0.6 * (cats[5] > 3)
         + 0.5 * (cats[0] == 1) + rng.normal(0.0, 0.8, size=N))
    y = (z > np.quantile(z, 0.76)).astype(np.int64)
    return dict(X=X, Y=_onehot(y, 2), y=y, N=N, d=X.shape[1], K=2, H=H)


def random_tree(H, d, rng, thresholds=False, n_labels=2):
    nint = (1 << H) - 1
    feat = rng.integers(0, d, size=nint).astype(np.uint64)
    thr = rng.integers(0, 1 << 16, size=nint).astype(np.uint64) if thresholds else None
    leaf = rng.integers(0, n_labels, size=1 << H).astype(np.uint64)
    return feat, thr, leaf


def c4_infer(NI=10000, d=16, H=7, seed=1004, binary=False):
    """Uniform 16-bit features (int16 offset by 2^15, so in [0, 2^16)) and a random
    complete tree with feature ids, thresholds and binary leaf labels.  With
    binary=True the features' low bit is used and thresholds are dropped."""
    rng = np.random.default_rng(seed)
    I = rng.integers(0, 1 << 16, size=(NI, d)).astype(np.uint64)
    feat, thr, leaf = random_tree(H, d, rng, thresholds=True)
    if binary:
        I, thr = I & np.uint64(1), None
    return dict(I=I, feat=feat, thr=thr, leaf=leaf, NI=NI, d=d, H=H)


def c5_level(N=1000000, d=64, K=4, h=7, seed=1005):
    """One split-scoring level at scale: Bernoulli(0.5) columns, Dirichlet(1) class mix,
    samples spread uniformly over the 2^(h-1) nodes of level h-1, each of which was just
    split on a random column, so that level h has 2^h real leaves."""
    rng = np.random.default_rng(seed)
    X = (rng.random((N, d)) < 0.5).astype(np.uint64)
    mix = rng.dirichlet(np.ones(K))
    y = rng.choice(K, size=N, p=mix)
    nprev = 1 << (h - 1)
    M = (nprev - 1 + rng.integers(0, nprev, size=N)).astype(np.uint64)
    Tprev = rng.integers(0, d, size=nprev).astype(np.uint64)
    return dict(X=X, Y=_onehot(y, K), y=y, N=N, d=d, K=K, h=h, M=M, Tprev=Tprev,
                F=np.ones(1 << h, dtype=np.uint64), gamma=np.ones((1 << h, d), dtype=np.uint64))


def c5_infer(NI=1000000, d=64, H=10, K=4, seed=1005):
    rng = np.random.default_rng(seed + 1)
    I = (rng.random((NI, d)) < 0.5).astype(np.uint64)
    feat, _, leaf = random_tree(H, d, rng, thresholds=False, n_labels=K)
    return dict(I=I, feat=feat, thr=None, leaf=leaf, NI=NI, d=d, H=H)
