"""GPU library against the CPU oracle: every share plane bit for bit, plus the
round and wire-byte counters.  All calls go through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

M64 = (1 << 64) - 1


def u64(vals):
    return np.array([int(v) & M64 for v in vals], dtype=np.uint64)


@pytest.fixture(scope="module")
def mods():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from oracle import Oracle
    from paper_2305_00645_amd import gtree
    gtree.load()
    return Oracle, gtree


def pair(mods, seed, tau=16, K=2):
    Oracle, gtree = mods
    return Oracle(seed, tau=tau, K=K), gtree.GTree(seed, tau=tau, K=K)


def same(gs, oc, what=""):
    """gs: gtree.Shares, oc: oracle components (3, n)."""
    comp = gs.components()
    assert comp.shape == oc.shape, (what, comp.shape, oc.shape)
    if not np.array_equal(comp, oc):
        bad = np.argwhere(comp != oc)
        raise AssertionError("%s: %d of %d words differ, first at %s" % (what, len(bad), comp.size, bad[0]))


def same_stats(o, g):
    ro, wo = o.stats()
    rg, wg, _ = g.stats()
    assert ro == rg and np.array_equal(wo, wg), (ro, rg, wo.tolist(), wg.tolist())
    assert o.op_counter() == g.op_counter()
    # what the kernels counted at their message stores (payload bits per directed pair)
    # against what the oracle's protocol steps sent
    bo, bg = o.wire_bits(), g.wire_bits_dev()
    assert np.array_equal(bo, bg), (bo.tolist(), bg.tolist())


@pytest.mark.parametrize("n", [1, 7, 8, 63, 64, 65, 1000, 4099])
def test_share_reconstruct(mods, seed, n):
    o, g = pair(mods, seed)
    rng = np.random.default_rng(n)
    x = rng.integers(0, M64, size=n, dtype=np.uint64)
    so, sg = o.share(x), g.share_a(x)
    same(sg, so, "share")
    assert np.array_equal(g.rec(sg), x)


def test_empty_vectors(mods, seed):
    o, g = pair(mods, seed)
    sg = g.share_a(np.zeros(0, dtype=np.uint64))
    o.share(np.zeros(0, dtype=np.uint64))
    assert g.mult(sg, sg).n == 0
    o.mult(np.zeros((3, 0), dtype=np.uint64), np.zeros((3, 0), dtype=np.uint64))
    assert o.op_counter() == g.op_counter()


@pytest.mark.parametrize("n", [1, 9, 512, 1531])
def test_mult(mods, seed, n):
    o, g = pair(mods, seed)
    rng = np.random.default_rng(10 + n)
    x = rng.integers(0, M64, size=n, dtype=np.uint64)
    y = rng.integers(0, M64, size=n, dtype=np.uint64)
    xo, yo = o.share(x), o.share(y)
    xg, yg = g.share_a(x), g.share_a(y)
    zo, zg = o.mult(xo, yo), g.mult(xg, yg)
    same(zg, zo, "mult")
    assert np.array_equal(g.rec(zg), x * y)
    same_stats(o, g)


def test_eq_public_and_shared(mods, seed):
    o, g = pair(mods, seed)
    rng = np.random.default_rng(3)
    xs, ys = [], []
    for b in range(64):
        v = int(rng.integers(0, M64, dtype=np.uint64))
        xs.append(v); ys.append(v ^ (1 << b))
    for v in [0, 1, M64, 1 << 63, (1 << 63) - 1]:
        xs += [v, v, v]; ys += [v, v + 1, v - 1]
    for _ in range(150):
        v = int(rng.integers(0, M64, dtype=np.uint64))
        xs.append(v); ys.append(v if rng.random() < 0.5 else int(rng.integers(0, M64, dtype=np.uint64)))
    x, y = u64(xs), u64(ys)
    xo, xg = o.share(x), g.share_a(x)
    eo, eg = o.eq_a(xo, y), g.eq_a(xg, y)
    same(eg, eo, "eq_a public")
    assert np.array_equal(g.rec(eg), (x == y).astype(np.uint64))
    yo, yg = o.share(y), g.share_a(y)
    do = xo - yo
    dg = g.new(x.size); dg.t.copy_(xg.t - yg.t)
    eo, eg = o.eq_a(do, None), g.eq_a(dg, None)
    same(eg, eo, "eq_a shared")
    same_stats(o, g)


def test_ge(mods, seed):
    o, g = pair(mods, seed)
    rng = np.random.default_rng(4)
    xs, ys = [], []
    smalls = [0, 1, 2, 5, 1 << 16, (1 << 40) - 1, 1 << 40, 1 << 62, (1 << 63) - 1]
    for a in smalls:
        for b in smalls:
            xs.append(a); ys.append(b)
    for b in range(63):
        v = int(rng.integers(0, 1 << 62))
        xs.append(v | (1 << b)); ys.append(v & ~(1 << b))
        xs.append(v & ~(1 << b)); ys.append(v | (1 << b))
    for _ in range(300):
        xs.append(int(rng.integers(0, 1 << 62))); ys.append(int(rng.integers(0, 1 << 62)))
    for a, b in [(-5, 3), (3, -5), (-1, -1), (-7, -8)]:
        xs.append(a); ys.append(b)
    x, y = u64(xs), u64(ys)
    zo = o.ge_a(o.share(x), o.share(y))
    zg = g.ge_a(g.share_a(x), g.share_a(y))
    same(zg, zo, "ge_a")
    want = u64([1 if a >= b else 0 for a, b in zip(xs, ys)])
    assert np.array_equal(g.rec(zg), want)
    same_stats(o, g)


@pytest.mark.parametrize("w,n", [(1, 5), (2, 64), (5, 100), (16, 513), (64, 1025), (37, 777)])
def test_oaa(mods, seed, w, n):
    o, g = pair(mods, seed)
    rng = np.random.default_rng(w * 1000 + n)
    Wp = rng.integers(0, M64, size=w, dtype=np.uint64)
    u = rng.integers(0, w + 2, size=n).astype(np.uint64)
    zo = o.oaa(o.share(Wp), o.share(u))
    zg = g.oaa(g.share_a(Wp), g.share_a(u))
    same(zg, zo, "oaa")
    want = np.array([Wp[int(i)] if int(i) < w else 0 for i in u], dtype=np.uint64)
    assert np.array_equal(g.rec(zg), want)
    same_stats(o, g)


@pytest.mark.parametrize("tau", [5, 16])
def test_div(mods, seed, tau):
    o, g = pair(mods, seed, tau=tau)
    rng = np.random.default_rng(6)
    Q = [1, 2, 3, 7, 1000, (1 << 40) - 1] + [int(rng.integers(1, 1 << 40)) for _ in range(200)]
    S = [int(rng.integers(0, q + 1)) for q in Q]
    S[0], S[1], S[2] = 1, 0, 3
    qo = o.div(o.share(u64(S)), o.share(u64(Q)))
    qg = g.div(g.share_a(u64(S)), g.share_a(u64(Q)))
    same(qg, qo, "div")
    assert np.array_equal(g.rec(qg), u64([(s << tau) // q for s, q in zip(S, Q)]))
    same_stats(o, g)


# ------------------------------------------------------------------ training
def run_train_pair(mods, seed, w, tau=16, H=None, every_level=True):
    from oracle import X_T, X_F, X_M, X_C, X_GAMMA, X_SD, X_L, X_SCORE, X_C_PAPER
    H = w["H"] if H is None else H
    N, d, K = w["N"], w["d"], w["K"]
    o, g = pair(mods, seed, tau=tau, K=K)
    xo, yo = o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1))
    xg, yg = g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1))
    o.train_create(xo, yo, N, d, H)
    g.train_create(xg, yg, N, d, H)
    names = dict(M=X_M, L=X_L, C=X_C, SCORE=X_SCORE, SD=X_SD, GAMMA=X_GAMMA, F=X_F, T=X_T, CP=X_C_PAPER)
    for h in range(H):
        o.train_level(h)
        g.train_level(h)
        if every_level or h == H - 1:
            for nm, what in names.items():
                same(g.train_export(what), o.train_export(what), "level %d %s" % (h, nm))
        same_stats(o, g)
    fo, lo = o.train_finish()
    tree = g.train_finish()
    fg, lg = tree.export()
    same(fg, fo, "tree features")
    same(lg, lo, "tree labels")
    for nm in ("M", "L", "C", "F", "T"):
        same(g.train_export(names[nm]), o.train_export(names[nm]), "finish %s" % nm)
    same_stats(o, g)
    return o, g, tree, (fo, lo)


def test_train_c1(mods, seed):
    import plain_cart
    from paper_2305_00645_amd import workloads as wl
    w = wl.c1_train()
    o, g, tree, (fo, lo) = run_train_pair(mods, seed, w)
    ref = plain_cart.train(w["X"], w["y"], w["K"], w["H"], 16)
    fg, lg = tree.export()
    assert np.array_equal(g.rec(fg).astype(np.int64), ref["T"][:7])
    assert np.array_equal(g.rec(lg).astype(np.int64), ref["T"][7:])
    # inference with the trained tree, binary mode, against plaintext prediction
    rng = np.random.default_rng(5)
    I = (rng.random((333, w["d"])) < 0.5).astype(np.uint64)
    Ro = o.infer(fo, None, lo, w["H"], o.share(I.reshape(-1)), 333, w["d"])
    Rg = g.infer_batch(tree, g.share_a(I.reshape(-1)), 333, w["d"])
    same(Rg, Ro, "inference on trained tree")
    assert np.array_equal(g.rec(Rg).astype(np.int64), plain_cart.predict(ref["T"], w["H"], I))
    same_stats(o, g)


@pytest.mark.parametrize("keyseed", [1, 2])
def test_other_protocol_keys(mods, keyseed):
    """Fresh keys for all five roles: training, then inference with the trained tree."""
    from paper_2305_00645_amd import workloads as wl
    keys = np.random.default_rng(1000 + keyseed).integers(0, 1 << 63, size=(5, 4), dtype=np.uint64) * np.uint64(2) + np.uint64(keyseed & 1)
    w = wl.c1_train(N=300, d=10, depth=3)
    o, g, tree, (fo, lo) = run_train_pair(mods, keys, w, every_level=False)
    I = (np.random.default_rng(keyseed).random((129, w["d"])) < 0.5).astype(np.uint64)
    Ro = o.infer(fo, None, lo, w["H"], o.share(I.reshape(-1)), 129, w["d"])
    Rg = g.infer_batch(tree, g.share_a(I.reshape(-1)), 129, w["d"])
    same(Rg, Ro, "inference with other keys")
    same_stats(o, g)


def test_train_c2_depth7(mods, seed):
    from paper_2305_00645_amd import workloads as wl
    run_train_pair(mods, seed, wl.c2_train(), H=7, every_level=False)


def test_train_multiclass_ragged(mods, seed):
    rng = np.random.default_rng(77)
    N, d, K = 203, 9, 4
    X = (rng.random((N, d)) < 0.4).astype(np.uint64)
    y = (X[:, 0].astype(np.int64) * 2 + X[:, 3].astype(np.int64) + (rng.random(N) < 0.1)) % K
    Y = np.zeros((N, K), dtype=np.uint64); Y[np.arange(N), y] = 1
    run_train_pair(mods, seed, dict(X=X, Y=Y, y=y, N=N, d=d, K=K, H=3), tau=10)


def test_train_c3_shape_reduced(mods, seed):
    from paper_2305_00645_amd import workloads as wl
    w = wl.c3_train(N=3000, H=4, n_thr=8)
    run_train_pair(mods, seed, w, every_level=False)


def test_train_degenerate(mods, seed):
    X = np.array([[0, 1], [1, 1], [1, 0], [0, 0], [1, 1]], dtype=np.uint64)
    y = np.ones(5, dtype=np.int64)
    Y = np.zeros((5, 2), dtype=np.uint64); Y[:, 1] = 1
    run_train_pair(mods, seed, dict(X=X, Y=Y, y=y, N=5, d=2, K=2, H=2))
    run_train_pair(mods, seed, dict(X=X, Y=Y, y=y, N=5, d=2, K=2, H=0))
    X1 = np.array([[0], [1], [1], [0]], dtype=np.uint64)
    y1 = np.array([0, 1, 1, 0])
    Y1 = np.zeros((4, 2), dtype=np.uint64); Y1[np.arange(4), y1] = 1
    run_train_pair(mods, seed, dict(X=X1, Y=Y1, y=y1, N=4, d=1, K=2, H=2))


def test_train_limits_of_classes_and_precision(mods, seed):
    """Largest class count and largest number of fractional bits the library accepts."""
    rng = np.random.default_rng(99)
    N, d, K = 130, 5, 16
    X = (rng.random((N, d)) < 0.5).astype(np.uint64)
    y = (X[:, 0].astype(np.int64) * 8 + X[:, 2].astype(np.int64) * 4 + rng.integers(0, 4, N)) % K
    Y = np.zeros((N, K), dtype=np.uint64); Y[np.arange(N), y] = 1
    run_train_pair(mods, seed, dict(X=X, Y=Y, y=y, N=N, d=d, K=K, H=3), tau=20)


@pytest.mark.parametrize("N,d,K,H", [(600, 4, 16, 3), (300, 3, 12, 2), (700, 5, 2, 3), (900, 21, 3, 3), (500, 40, 2, 4)])
def test_train_column_group_remainders(mods, seed, N, d, K, H):
    """The statistics contraction splits its d*K+K columns into groups of 64 and a remainder that
    takes its own path: 16 columns beside a full group (two passes of the packed 16-wide tile), 12
    class columns alone at the label level, 12 columns with no full group at all, 2 beside a full
    group, and a remainder of 18 (a launch of its own)."""
    rng = np.random.default_rng(1000 * d + K)
    X = (rng.random((N, d)) < 0.45).astype(np.uint64)
    y = (X[:, 0].astype(np.int64) * 3 + X[:, d - 1].astype(np.int64) + rng.integers(0, 2, N)) % K
    Y = np.zeros((N, K), dtype=np.uint64); Y[np.arange(N), y] = 1
    run_train_pair(mods, seed, dict(X=X, Y=Y, y=y, N=N, d=d, K=K, H=H), tau=12)


def test_train_deep_tree_few_samples(mods, seed):
    """Far more nodes than samples: 2^11 leaves for 40 samples, most nodes empty."""
    rng = np.random.default_rng(98)
    N, d, K, H = 40, 12, 2, 11
    X = (rng.random((N, d)) < 0.5).astype(np.uint64)
    y = (X[:, 1] ^ X[:, 4] ^ X[:, 7]).astype(np.int64)
    Y = np.zeros((N, K), dtype=np.uint64); Y[np.arange(N), y] = 1
    run_train_pair(mods, seed, dict(X=X, Y=Y, y=y, N=N, d=d, K=K, H=H), every_level=False)


def test_train_reset_starts_an_equal_job(mods, seed):
    """gt_train_reset reuses every buffer of the object (limb tiles, partial sums, tree):
    a second job on different data must equal an oracle run started at the same operation
    counter, share by share, and give the plaintext tree."""
    import plain_cart
    from oracle import X_T, X_F, X_M, X_C, X_SD, X_GAMMA
    from paper_2305_00645_amd import workloads as wl
    N, d, H = 300, 11, 3
    wa, wb = wl.c1_train(N=N, d=d, depth=H, seed=31), wl.c1_train(N=N, d=d, depth=H, seed=32)
    o, g = pair(mods, seed)
    xa, ya = g.share_a(wa["X"].reshape(-1)), g.share_a(wa["Y"].reshape(-1))
    oxa, oya = o.share(wa["X"].reshape(-1)), o.share(wa["Y"].reshape(-1))
    g.train_create(xa, ya, N, d, H)
    o.train_create(oxa, oya, N, d, H)
    for h in range(H):
        g.train_level(h); o.train_level(h)
    t1 = g.train_finish(); o.train_finish()
    same(g.train_export(X_T), o.train_export(X_T), "first job T")
    t1.close()
    xb, yb = g.share_a(wb["X"].reshape(-1)), g.share_a(wb["Y"].reshape(-1))
    oxb, oyb = o.share(wb["X"].reshape(-1)), o.share(wb["Y"].reshape(-1))
    g.train_reset(xb, yb)
    o.train_create(oxb, oyb, N, d, H)          # the oracle has no reset: a new object, same operation counter
    assert o.op_counter() == g.op_counter()
    for h in range(H):
        g.train_level(h); o.train_level(h)
        for nm, what in (("M", X_M), ("C", X_C), ("SD", X_SD), ("GAMMA", X_GAMMA), ("F", X_F)):
            same(g.train_export(what), o.train_export(what), "second job level %d %s" % (h, nm))
    t2 = g.train_finish()
    fo, lo = o.train_finish()
    fg, lg = t2.export()
    same(fg, fo, "second job features"); same(lg, lo, "second job labels")
    ref = plain_cart.train(wb["X"], wb["y"], 2, H, 16)
    assert np.array_equal(g.rec(g.train_export(X_T)).astype(np.int64), ref["T"])
    same_stats(o, g)
    # a tree that is still alive when the object finishes again gets buffers of its own
    g.train_reset(xa, ya)
    for h in range(H):
        g.train_level(h)
    t3 = g.train_finish()
    assert np.array_equal(g.rec(t2.export()[0]).astype(np.int64), ref["T"][:(1 << H) - 1])
    ref_a = plain_cart.train(wa["X"], wa["y"], 2, H, 16)
    assert np.array_equal(g.rec(t3.export()[0]).astype(np.int64), ref_a["T"][:(1 << H) - 1])
    t2.close(); t3.close()


def test_export_after_import_needs_a_level(mods, seed):
    Oracle, gtree = mods
    from oracle import X_C, X_M
    from paper_2305_00645_amd import workloads as wl
    w = wl.c5_level(N=100, d=5, K=2, h=2)
    g = gtree.GTree(seed, K=2)
    g.train_create(g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1)), 100, 5, 3)
    st = [w["M"], w["Tprev"], w["F"], np.zeros(4 * 12, dtype=np.uint64), w["gamma"].reshape(-1)]
    g.train_import(2, *[g.share_a(a) for a in st])
    assert np.array_equal(g.rec(g.train_export(X_M)), w["M"])
    with pytest.raises(gtree.GtError) as e:
        g.train_export(X_C)
    assert e.value.code == gtree.GT_ESTATE
    g.train_level(2)
    assert g.train_export(X_C).n == 4 * 12


@pytest.mark.parametrize("case", ["c1", "c2", "multi", "degenerate"])
def test_heuristic_by_reconstruction(mods, seed, case):
    """Reconstruct-and-score heuristic (host analogue of the TEE-based protocol): share by
    share against the oracle in the same mode, and the reconstructed tree against the
    plaintext CART (hence equal to the MPC heuristic's)."""
    import plain_cart
    from oracle import X_T, X_F, X_M, X_C, X_GAMMA, X_SD, X_SCORE
    from paper_2305_00645_amd import workloads as wl
    tau = 16
    if case == "c1":
        w = wl.c1_train()
    elif case == "c2":
        w = wl.c2_train(H=5)
    elif case == "multi":
        rng = np.random.default_rng(77)
        N, d, K = 203, 9, 4
        X = (rng.random((N, d)) < 0.4).astype(np.uint64)
        y = (X[:, 0].astype(np.int64) * 2 + X[:, 3].astype(np.int64) + (rng.random(N) < 0.1)) % K
        Y = np.zeros((N, K), dtype=np.uint64); Y[np.arange(N), y] = 1
        w, tau = dict(X=X, Y=Y, y=y, N=N, d=d, K=K, H=3), 10
    else:
        X = np.array([[0, 1], [1, 1], [1, 0], [0, 0], [1, 1]], dtype=np.uint64)
        y = np.ones(5, dtype=np.int64)
        Y = np.zeros((5, 2), dtype=np.uint64); Y[:, 1] = 1
        w = dict(X=X, Y=Y, y=y, N=5, d=2, K=2, H=2)
    N, d, K, H = w["N"], w["d"], w["K"], w["H"]
    o, g = pair(mods, seed, tau=tau, K=K)
    o.train_create(o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1)), N, d, H)
    g.train_create(g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1)), N, d, H)
    o.train_set_heuristic(True); g.train_set_heuristic(True)
    for h in range(H):
        o.train_level(h); g.train_level(h)
        for nm, what in (("M", X_M), ("C", X_C), ("SCORE", X_SCORE), ("SD", X_SD), ("GAMMA", X_GAMMA), ("F", X_F), ("T", X_T)):
            same(g.train_export(what), o.train_export(what), "level %d %s" % (h, nm))
    fo, lo = o.train_finish()
    tree = g.train_finish()
    fg, lg = tree.export()
    same(fg, fo, "features"); same(lg, lo, "labels")
    ref = plain_cart.train(w["X"], w["y"], K, H, tau)
    assert np.array_equal(g.rec(g.train_export(X_T)).astype(np.int64), ref["T"])
    assert np.array_equal(g.rec(g.train_export(X_F)).astype(np.int64), ref["F"])
    same_stats(o, g)
    assert o.scorer_bytes() == g.scorer_bytes()
    tree.close(); g.close()


@pytest.mark.parametrize("w,n", [(1, 5), (16, 513), (37, 100)])
def test_oaa_as_printed(mods, seed, w, n):
    """Array access element by element as the paper prints it: oracle's shares, W[u], and
    exactly N(4l-1) bits per party counted by the kernels."""
    o, g = pair(mods, seed)
    rng = np.random.default_rng(w * 1000 + n)
    Wp = rng.integers(0, M64, size=w, dtype=np.uint64)
    u = rng.integers(0, w + 2, size=n).astype(np.uint64)
    so, sg = (o.share(Wp), o.share(u)), (g.share_a(Wp), g.share_a(u))
    o.stats_reset(); g.stats_reset()
    zo, zg = o.oaa_literal(*so), g.oaa_literal(*sg)
    same(zg, zo, "oaa as printed")
    assert np.array_equal(g.rec(zg), np.array([Wp[int(i)] if int(i) < w else 0 for i in u], dtype=np.uint64))
    same_stats(o, g)
    assert int(g.wire_bits_dev()[0].sum()) == w * n * (4 * 64 - 1) and g.stats()[0] == 9
    same(g.oaa(*sg), o.oaa(*so), "fused access after the literal one (shared scratch left clean)")


@pytest.mark.parametrize("case", ["c1", "c2"])
def test_learning_as_printed(mods, seed, case):
    """Training with the learning protocol as printed (whole-tree scans, per-element
    SelectShare, local accumulation): share by share against the oracle in the same mode, the
    tree against the plaintext CART, the message volume against the fused mode."""
    import plain_cart
    from oracle import X_T, X_F, X_M, X_C, X_GAMMA, X_SD, X_SCORE
    from paper_2305_00645_amd import workloads as wl
    w = wl.c1_train(N=200, d=8, depth=3) if case == "c1" else wl.c2_train(H=4)
    N, d, K, H = w["N"], w["d"], w["K"], w["H"]
    o, g = pair(mods, seed, K=K)
    o.train_create(o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1)), N, d, H)
    g.train_create(g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1)), N, d, H)
    o.train_set_literal(True); g.train_set_literal(True)
    for h in range(H):
        o.train_level(h); g.train_level(h)
        for nm, what in (("M", X_M), ("C", X_C), ("SCORE", X_SCORE), ("SD", X_SD), ("GAMMA", X_GAMMA), ("F", X_F)):
            same(g.train_export(what), o.train_export(what), "level %d %s" % (h, nm))
    fo, lo = o.train_finish()
    tree = g.train_finish()
    fg, lg = tree.export()
    same(fg, fo, "features"); same(lg, lo, "labels")
    ref = plain_cart.train(w["X"], w["y"], K, H, 16)
    assert np.array_equal(g.rec(g.train_export(X_T)).astype(np.int64), ref["T"])
    same_stats(o, g)
    g2 = mods[1].GTree(seed, K=K)
    g2.train_create(g2.share_a(w["X"].reshape(-1)), g2.share_a(w["Y"].reshape(-1)), N, d, H)
    for h in range(H):
        g2.train_level(h)
    g2.train_finish().close()
    assert int(g.stats()[1][0].sum()) > 5 * int(g2.stats()[1][0].sum())      # what the fusion into inner products saves
    tree.close(); g.close(); g2.close()


@pytest.mark.parametrize("case", ["c1", "c2", "multi", "c3small"])
def test_partition_by_products(mods, seed, case):
    """Data partition by products with the previous level's leaf one-hot: share by share
    against the oracle in the same mode at every level, the tree against the plaintext CART."""
    import plain_cart
    from oracle import X_T, X_F, X_M, X_C, X_GAMMA, X_SD, X_SCORE, X_L
    from paper_2305_00645_amd import workloads as wl
    tau = 16
    if case == "c1":
        w = wl.c1_train()
    elif case == "c2":
        w = wl.c2_train(H=6)
    elif case == "c3small":
        w = wl.c3_train(N=3000, H=4, n_thr=8)
    else:
        rng = np.random.default_rng(77)
        N, d, K = 203, 9, 4
        X = (rng.random((N, d)) < 0.4).astype(np.uint64)
        y = (X[:, 0].astype(np.int64) * 2 + X[:, 3].astype(np.int64) + (rng.random(N) < 0.1)) % K
        Y = np.zeros((N, K), dtype=np.uint64); Y[np.arange(N), y] = 1
        w, tau = dict(X=X, Y=Y, y=y, N=N, d=d, K=K, H=3), 10
    N, d, K, H = w["N"], w["d"], w["K"], w["H"]
    o, g = pair(mods, seed, tau=tau, K=K)
    o.train_create(o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1)), N, d, H)
    g.train_create(g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1)), N, d, H)
    o.train_set_partition(True); g.train_set_partition(True)
    for h in range(H):
        o.train_level(h); g.train_level(h)
        for nm, what in (("M", X_M), ("L", X_L), ("C", X_C), ("SCORE", X_SCORE), ("SD", X_SD), ("GAMMA", X_GAMMA), ("F", X_F)):
            same(g.train_export(what), o.train_export(what), "level %d %s" % (h, nm))
    fo, lo = o.train_finish()
    tree = g.train_finish()
    fg, lg = tree.export()
    same(fg, fo, "features"); same(lg, lo, "labels")
    same(g.train_export(X_M), o.train_export(X_M), "M at the label level")
    ref = plain_cart.train(w["X"], w["y"], K, H, tau)
    assert np.array_equal(g.rec(g.train_export(X_T)).astype(np.int64), ref["T"])
    same_stats(o, g)
    tree.close(); g.close()


def test_train_errors(mods, seed):
    Oracle, gtree = mods
    from paper_2305_00645_amd import workloads as wl
    w = wl.c1_train(N=32, d=4, depth=2)
    g = gtree.GTree(seed)
    xg, yg = g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1))
    g.train_create(xg, yg, 32, 4, 2)
    with pytest.raises(gtree.GtError) as e:
        g.train_level(1)                       # out of order
    assert e.value.code == gtree.GT_ESTATE
    with pytest.raises(gtree.GtError) as e:
        g.train_create(xg, yg, 33, 4, 2)       # buffers too small
    assert e.value.code == gtree.GT_EINVAL
    with pytest.raises(gtree.GtError):
        g.train_create(xg, yg, 32, 4, 99)      # depth over the limit


# ------------------------------------------------------------------ inference
@pytest.mark.parametrize("binary,NI,H", [(False, 1000, 7), (True, 1000, 7), (False, 77, 3), (True, 1, 2), (True, 5, 16), (False, 9, 13)])
def test_infer(mods, seed, binary, NI, H):
    import plain_cart
    from paper_2305_00645_amd import workloads as wl
    w = wl.c4_infer(NI=NI, H=H, binary=binary)
    o, g = pair(mods, seed)
    fo, lo = o.share(w["feat"]), o.share(w["leaf"])
    fg, lg = g.share_a(w["feat"]), g.share_a(w["leaf"])
    to = tg = None
    if not binary:
        to, tg = o.share(w["thr"]), g.share_a(w["thr"])
    Io, Ig = o.share(w["I"].reshape(-1)), g.share_a(w["I"].reshape(-1))
    tree = g.tree_import(fg, tg, lg, H)
    Ro = o.infer(fo, to, lo, H, Io, NI, w["d"])
    Rg = g.infer_batch(tree, Ig, NI, w["d"])
    same(Rg, Ro, "inference")
    T = np.concatenate([w["feat"], w["leaf"]]).astype(np.int64)
    thr = None if binary else np.concatenate([w["thr"], np.zeros(1 << H, dtype=np.uint64)])
    assert np.array_equal(g.rec(Rg).astype(np.int64), plain_cart.predict(T, H, w["I"], thr))
    same_stats(o, g)


@pytest.mark.parametrize("how", ["levelwise", 16, 32, 64])
@pytest.mark.parametrize("binary,NI,H,d", [(False, 333, 5, 16), (True, 1000, 7, 16), (True, 70, 9, 3), (False, 129, 3, 37), (True, 17, 0, 5)])
def test_infer_paths_agree(mods, seed, how, binary, NI, H, d):
    """The level-by-level path and the one-launch path with each of its three tile shapes
    (16, 32, 64 instances per workgroup; 32, 16, 8 columns per step, so column counts that
    are not a multiple of the step and instance counts that leave a ragged tile) all give the
    oracle's shares, rounds, bytes and bits."""
    import plain_cart
    Oracle, gtree = mods
    from paper_2305_00645_amd import workloads as wl
    w = wl.c4_infer(NI=NI, H=H, d=d, binary=binary, seed=4000 + H)
    flags = gtree.GT_FLAG_LEVELWISE_INFER if how == "levelwise" else gtree.GT_FLAG_INFER_TILE[how]
    o, g = Oracle(seed), gtree.GTree(seed, flags=flags)
    fo, lo = o.share(w["feat"]), o.share(w["leaf"])
    fg, lg = g.share_a(w["feat"]), g.share_a(w["leaf"])
    to = tg = None
    if not binary:
        to, tg = o.share(w["thr"]), g.share_a(w["thr"])
    Io, Ig = o.share(w["I"].reshape(-1)), g.share_a(w["I"].reshape(-1))
    tree = g.tree_import(fg, tg, lg, H)
    Ro = o.infer(fo, to, lo, H, Io, NI, d)
    Rg = g.infer_batch(tree, Ig, NI, d)
    same(Rg, Ro, "inference (%s)" % how)
    T = np.concatenate([w["feat"], w["leaf"]]).astype(np.int64)
    thr = None if binary else np.concatenate([w["thr"], np.zeros(1 << H, dtype=np.uint64)])
    assert np.array_equal(g.rec(Rg).astype(np.int64), plain_cart.predict(T, H, w["I"], thr))
    same_stats(o, g)
    tree.close(); g.close()


@pytest.mark.parametrize("binary,ntrees,NI,H,d", [(True, 7, 150, 3, 9), (False, 3, 77, 4, 16), (True, 40, 1000, 2, 5)])
def test_forest_in_one_launch(mods, seed, binary, ntrees, NI, H, d):
    """Many shallow trees on one batch in one launch: shares, operation ids, rounds, bytes
    and bits are those of the oracle's single-tree inference called tree after tree."""
    import plain_cart
    Oracle, gtree = mods
    from paper_2305_00645_amd import workloads as wl
    o, g = pair(mods, seed)
    rng = np.random.default_rng(500 + ntrees)
    I = rng.integers(0, 1 << 16, size=(NI, d)).astype(np.uint64)
    if binary:
        I &= np.uint64(1)
    Io, Ig = o.share(I.reshape(-1)), g.share_a(I.reshape(-1))
    plain = [wl.random_tree(H, d, rng, thresholds=not binary) for _ in range(ntrees)]
    so = [(o.share(f), None if t is None else o.share(t), o.share(l)) for f, t, l in plain]
    trees = []
    for f, t, l in plain:
        trees.append(g.tree_import(g.share_a(f), None if t is None else g.share_a(t), g.share_a(l), H))
    assert o.op_counter() == g.op_counter()
    forest = g.forest_create(trees)
    for tr in trees:
        tr.close()                               # the forest holds copies
    Rg = g.infer_forest(forest, Ig, NI, d).components()
    for t, (f, th, l) in enumerate(plain):
        Ro = o.infer(so[t][0], so[t][1], so[t][2], H, Io, NI, d)
        assert np.array_equal(Rg[:, t * NI:(t + 1) * NI], Ro), t
        T = np.concatenate([f, l]).astype(np.int64)
        thr = None if binary else np.concatenate([th, np.zeros(1 << H, dtype=np.uint64)])
        got = (Rg[0, t * NI:(t + 1) * NI] + Rg[1, t * NI:(t + 1) * NI] + Rg[2, t * NI:(t + 1) * NI]).astype(np.int64)
        assert np.array_equal(got, plain_cart.predict(T, H, I, thr))
    same_stats(o, g)
    forest.close(); g.close()


def test_infer_depth0(mods, seed):
    o, g = pair(mods, seed)
    lo, lg = o.share(u64([3])), g.share_a(u64([3]))
    Io, Ig = o.share(u64([1, 0, 1, 1])), g.share_a(u64([1, 0, 1, 1]))
    tree = g.tree_import(g.new(0), None, lg, 0)
    Ro = o.infer(np.zeros((3, 0), dtype=np.uint64), None, lo, 0, Io, 2, 2)
    Rg = g.infer_batch(tree, Ig, 2, 2)
    same(Rg, Ro, "depth 0")
    assert g.rec(Rg).tolist() == [3, 3]


# the shapes reach the variants of the statistics contraction: few nodes; 128 nodes with a
# remainder of 4 columns beside a full group of 64; 256 nodes with a remainder of 18 columns;
# exactly 64 columns; 64 nodes (two row tiles per workgroup) with a remainder above 32
# columns; 32 nodes (one row tile per workgroup) with exactly 64 columns
@pytest.mark.parametrize("N,d,K,h", [(5000, 12, 4, 3), (1500, 16, 4, 7), (700, 40, 2, 8),
                                     (900, 15, 4, 7), (900, 24, 4, 6), (600, 31, 2, 5)])
def test_single_level_from_imported_state(mods, seed, N, d, K, h):
    """One split-scoring level started from a synthetic state (reduced C5 recipe)."""
    from oracle import X_M, X_C, X_SD, X_SCORE, X_F
    from paper_2305_00645_amd import workloads as wl
    w = wl.c5_level(N=N, d=d, K=K, h=h)
    N, d, K, h = w["N"], w["d"], w["K"], w["h"]
    o, g = pair(mods, seed, K=K)
    xo, yo = o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1))
    xg, yg = g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1))
    o.train_create(xo, yo, N, d, h + 1)
    g.train_create(xg, yg, N, d, h + 1)
    CW = d * K + K
    st = [w["M"], w["Tprev"], w["F"], np.zeros((1 << h) * CW, dtype=np.uint64), w["gamma"].reshape(-1)]
    so = [o.share(a) for a in st]
    sg = [g.share_a(a) for a in st]
    o.train_import(h, *so)
    g.train_import(h, *sg)
    o.train_level(h)
    g.train_level(h)
    for what in (X_M, X_C, X_SCORE, X_SD, X_F):
        same(g.train_export(what), o.train_export(what), "import level, export %d" % what)
    # counts equal the plaintext histogram of the routed samples
    X, y = w["X"].astype(np.int64), w["y"]
    M = 2 * w["M"].astype(np.int64) + 1 + X[np.arange(N), w["Tprev"].astype(np.int64)[w["M"].astype(np.int64) - ((1 << (h - 1)) - 1)]]
    assert np.array_equal(g.rec(g.train_export(X_M)).astype(np.int64), M)
    C = g.rec(g.train_export(X_C)).astype(np.int64).reshape(1 << h, CW)
    for r in range(1 << h):
        sel = M == (1 << h) - 1 + r
        for c in range(K):
            assert C[r, d * K + c] == (sel & (y == c)).sum()
            assert np.array_equal(C[r, :d * K].reshape(d, K)[:, c], X[sel & (y == c)].sum(axis=0))
    same_stats(o, g)


def test_launch_and_message_pattern_is_data_independent(mods, seed):
    """Only sizes and depth may show (Sec. I, goals): two data sets of the same shape give
    the same operation count, rounds, wire bytes and kernel launches per class."""
    Oracle, gtree = mods
    from paper_2305_00645_amd import workloads as wl
    seen = []
    for s in (21, 22):
        w = wl.c1_train(N=300, d=7, depth=3, seed=s)
        g = gtree.GTree(seed, K=2, profile=True)
        g.train_create(g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1)), 300, 7, 3)
        for h in range(3):
            g.train_level(h)
        tree = g.train_finish()
        g.infer_batch(tree, g.share_a(w["X"].reshape(-1)), 300, 7)
        rounds, wire, _ = g.stats()
        seen.append((g.op_counter(), rounds, wire.tolist(), {k: v[1] for k, v in g.prof().items()}))
        tree.close(); g.close()
    assert seen[0] == seen[1]
    assert seen[0][3]["eqgrid"] > 0 and seen[0][3]["count"] > 0


def test_calls_return_before_the_stream_drains(mods, seed):
    """Calls only enqueue: with a long kernel ahead of it on the context's stream a whole
    training level returns to the host while that kernel is still running, and the results
    still equal the oracle's."""
    import torch
    from oracle import X_C, X_SD, X_M
    Oracle, gtree = mods
    from paper_2305_00645_amd import workloads as wl
    w = wl.c1_train(N=500, d=9, depth=2)
    N, d, H = w["N"], w["d"], w["H"]
    o = Oracle(seed)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        g = gtree.GTree(seed, stream=st)
        xg, yg = g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1))
        g.train_create(xg, yg, N, d, H)
        g.train_level(0)
        st.synchronize()
        torch.cuda._sleep(int(2.0e9))            # about a second of GPU time on this stream
        g.train_level(1)
        tree = g.train_finish()
        pending = not st.query()                 # the sleep kernel (and everything behind it) has not finished
        st.synchronize()
        assert pending, "gt_train_level/gt_train_finish waited for the stream"
        o.train_create(o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1)), N, d, H)
        o.train_level(0); o.train_level(1)
        fo, lo = o.train_finish()
        fg, lg = tree.export()
        same(fg, fo, "features"); same(lg, lo, "labels")
        same(g.train_export(X_M), o.train_export(X_M), "M")
        same_stats(o, g)
        tree.close(); g.close()


def test_context_on_a_side_stream(mods, seed):
    """The library enqueues on the stream it is given (default priority)."""
    import torch
    Oracle, gtree = mods
    o = Oracle(seed)
    st = torch.cuda.Stream()
    rng = np.random.default_rng(9)
    x = rng.integers(0, M64, size=3000, dtype=np.uint64)
    y = rng.integers(0, M64, size=3000, dtype=np.uint64)
    with torch.cuda.stream(st):
        g = gtree.GTree(seed, stream=st)
        xg, yg = g.share_a(x), g.share_a(y)
        zg = g.mult(xg, yg)
        ug = g.oaa(g.share_a(x[:37]), g.share_a(np.arange(500, dtype=np.uint64) % 40))
        st.synchronize()
        zo = o.mult(o.share(x), o.share(y))
        uo = o.oaa(o.share(x[:37]), o.share(np.arange(500, dtype=np.uint64) % 40))
        same(zg, zo, "mult on side stream")
        same(ug, uo, "oaa on side stream")
        g.close()
