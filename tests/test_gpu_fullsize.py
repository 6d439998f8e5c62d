"""Parity at the full size of the scale workload (C5), in the launch configuration that
bench.py times: 10^6 samples x 64 columns, 4 classes, one split-scoring level over 128 nodes,
and depth-10 inference on 10^6 instances.  Training is compared share by share with a full
oracle run (about a minute of host time); inference, too large to simulate in full, is
checked on sampled rows that the oracle computes one by one, and on all rows against
plaintext traversal."""
import numpy as np
import pytest

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def _same(gs, oc, what):
    comp = gs.components()
    assert comp.shape == oc.shape, (what, comp.shape, oc.shape)
    if not np.array_equal(comp, oc):
        bad = np.argwhere(comp != oc)
        raise AssertionError("%s: %d of %d words differ, first at %s" % (what, len(bad), comp.size, bad[0]))


def test_c5_level_full_size(seed):
    import torch
    from oracle import Oracle, X_M, X_C, X_SD, X_SCORE, X_F, X_GAMMA, X_L
    from paper_2305_00645_amd import gtree, workloads as wl
    w = wl.c5_level()
    N, d, K, h = w["N"], w["d"], w["K"], w["h"]
    assert (N, d, K, h) == (1000000, 64, 4, 7)
    CW = d * K + K
    o, g = Oracle(seed, K=K), gtree.GTree(seed, K=K)
    state = [w["M"], w["Tprev"], w["F"], np.zeros((1 << h) * CW, dtype=np.uint64), w["gamma"].reshape(-1)]
    xg, yg = g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1))
    sg = [g.share_a(a) for a in state]
    g.train_create(xg, yg, N, d, h + 1)
    g.train_import(h, *sg)
    g.train_level(h)
    xo, yo = o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1))
    so = [o.share(a) for a in state]
    o.train_create(xo, yo, N, d, h + 1)
    o.train_import(h, *so)
    o.train_level(h)
    for what, name in ((X_M, "M"), (X_C, "C"), (X_SCORE, "score"), (X_SD, "SD"), (X_F, "F"), (X_GAMMA, "gamma")):
        _same(g.train_export(what), o.train_export(what), name)
    # the per-sample leaf one-hot is 128 x 10^6 shares: every party's two planes of every node,
    # one node slab at a time
    Lg = g.train_export(X_L)
    Lo = o.train_export(X_L)
    N8 = (N + 7) // 8 * 8
    pl = Lg.t.view(3, 2, 1 << h, N8)
    for r in range(1 << h):
        got = pl[:, :, r, :].cpu().numpy().view(np.uint64)
        for p in range(3):
            assert np.array_equal(got[p, 0], Lo[p].reshape(1 << h, N8)[r]), ("L own", r, p)
            assert np.array_equal(got[p, 1], Lo[(p + 1) % 3].reshape(1 << h, N8)[r]), ("L next", r, p)
    ro, wo = o.stats()
    rg, wg, _ = g.stats()
    assert ro == rg and np.array_equal(wo, wg)
    assert np.array_equal(o.wire_bits(), g.wire_bits_dev())      # counted by the kernels at their message stores
    # and the reconstructed counts are the plaintext histogram of the routed samples
    X, y = w["X"].astype(np.int64), w["y"]
    Mi = w["M"].astype(np.int64)
    M = 2 * Mi + 1 + X[np.arange(N), w["Tprev"].astype(np.int64)[Mi - ((1 << (h - 1)) - 1)]]
    assert np.array_equal(g.rec(g.train_export(X_M)).astype(np.int64), M)
    C = g.rec(g.train_export(X_C)).astype(np.int64).reshape(1 << h, CW)
    node = M - ((1 << h) - 1)
    for c in range(K):
        sel = y == c
        assert np.array_equal(C[:, d * K + c], np.bincount(node[sel], minlength=1 << h))
        H2 = np.zeros((1 << h, d), dtype=np.int64)
        np.add.at(H2, node[sel], X[sel])
        assert np.array_equal(C[:, :d * K].reshape(1 << h, d, K)[:, :, c], H2)
    del Lg, pl
    g.close(); o.close()
    torch.cuda.empty_cache()


def test_c5_inference_full_size(seed):
    import torch
    import plain_cart
    from oracle import Oracle
    from paper_2305_00645_amd import gtree, workloads as wl
    w = wl.c5_infer()
    NI, d, H = w["NI"], w["d"], w["H"]
    assert (NI, d, H) == (1000000, 64, 10)
    o, g = Oracle(seed, K=4), gtree.GTree(seed, K=4)
    fg, lg = g.share_a(w["feat"]), g.share_a(w["leaf"])
    Ig = g.share_a(w["I"].reshape(-1))
    tree = g.tree_import(fg, None, lg, H)
    R = g.infer_batch(tree, Ig, NI, d)
    comp = R.components()                                   # also checks the replicated copies
    T = np.concatenate([w["feat"], w["leaf"]]).astype(np.int64)
    assert np.array_equal(g.rec(R).astype(np.int64), plain_cart.predict(T, H, w["I"]))
    # share by share on more than 2*10^4 rows: whole tiles of 512 rows (what one workgroup
    # carries) - the first ones, the last full one, the ragged last one, tiles on both sides of
    # the point where the launch's grid-stride loop starts its second pass (the launch has at
    # most 4096 workgroups for 1954 tiles x 3 column ranges) - and random rows
    rng = np.random.default_rng(3)
    ntile = (NI + 511) // 512
    tiles = sorted(set([0, 1, 2, ntile // 3, 1364, 1365, 1366, 1367, ntile - 3, ntile - 2, ntile - 1]
                       + rng.integers(0, ntile, size=30).tolist()))
    rows = np.concatenate([np.arange(t * 512, min(NI, (t + 1) * 512)) for t in tiles] + [rng.integers(0, NI, size=1500)])
    rows = np.unique(rows)
    assert rows.size >= 20000
    fo, lo = o.share(w["feat"]), o.share(w["leaf"])
    Io = o.share(w["I"].reshape(-1)).reshape(3, NI, d)[:, rows, :].reshape(3, -1)
    Ro = o.infer_rows(fo, None, lo, H, Io, NI, d, rows)
    assert np.array_equal(comp[:, rows], Ro)
    assert o.op_counter() == g.op_counter()
    tree.close(); g.close(); o.close()
    torch.cuda.empty_cache()


def test_c5_inference_levelwise_equals_one_launch(seed):
    """At full size (10^6 instances, depth 10) the level-by-level path and the one-launch path
    give the same six planes of R; together with the sampled-row test above this ties both to
    the oracle."""
    import torch
    from paper_2305_00645_amd import gtree, workloads as wl
    w = wl.c5_infer()
    NI, d, H = w["NI"], w["d"], w["H"]
    res = []
    for flags in (0, gtree.GT_FLAG_LEVELWISE_INFER):
        g = gtree.GTree(seed, K=4, flags=flags)
        tree = g.tree_import(g.share_a(w["feat"]), None, g.share_a(w["leaf"]), H)
        R = g.infer_batch(tree, g.share_a(w["I"].reshape(-1)), NI, d)
        res.append((R.planes(), g.stats()[0], g.stats()[1], g.wire_bits_dev(), g.op_counter()))
        tree.close(); g.close()
        torch.cuda.empty_cache()
    assert np.array_equal(res[0][0], res[1][0])
    assert res[0][1] == res[1][1] and np.array_equal(res[0][2], res[1][2]) and np.array_equal(res[0][3], res[1][3])
    assert res[0][4] == res[1][4]


def test_c3_full_training(seed):
    """Census-shaped workload at full size: 48,842 samples x 294 candidate columns, depth 7,
    every exported share of the last level and of the finished tree against the oracle."""
    import torch
    from oracle import Oracle, X_M, X_C, X_SD, X_SCORE, X_F, X_T, X_GAMMA
    from paper_2305_00645_amd import gtree, workloads as wl
    w = wl.c3_train()
    N, d, K, H = w["N"], w["d"], w["K"], w["H"]
    assert (N, d, H) == (48842, 294, 7)
    o, g = Oracle(seed, K=K), gtree.GTree(seed, K=K)
    xg, yg = g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1))
    g.train_create(xg, yg, N, d, H)
    xo, yo = o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1))
    o.train_create(xo, yo, N, d, H)
    for h in range(H):
        g.train_level(h)
        o.train_level(h)
        for what, name in ((X_SD, "SD"), (X_C, "C")):
            _same(g.train_export(what), o.train_export(what), "level %d %s" % (h, name))
    for what, name in ((X_M, "M"), (X_SCORE, "score"), (X_F, "F"), (X_GAMMA, "gamma")):
        _same(g.train_export(what), o.train_export(what), name)
    fo, lo = o.train_finish()
    tree = g.train_finish()
    fg, lg = tree.export()
    _same(fg, fo, "tree features")
    _same(lg, lo, "tree labels")
    _same(g.train_export(X_T), o.train_export(X_T), "T")
    ro, wo = o.stats()
    rg, wg, _ = g.stats()
    assert ro == rg and np.array_equal(wo, wg) and o.op_counter() == g.op_counter()
    assert np.array_equal(o.wire_bits(), g.wire_bits_dev())
    # the tree is the plaintext fixed-point Gini CART of the same data
    import plain_cart
    ref = plain_cart.train(w["X"], w["y"], K, H, 16)
    assert np.array_equal(g.rec(g.train_export(X_T)).astype(np.int64), ref["T"])
    tree.close(); g.close(); o.close()
    torch.cuda.empty_cache()


def test_c4_full_inference(seed):
    """The 10^4-instance depth-7 batch with thresholds, every share against the oracle."""
    import plain_cart
    from oracle import Oracle
    from paper_2305_00645_amd import gtree, workloads as wl
    w = wl.c4_infer()
    NI, d, H = w["NI"], w["d"], w["H"]
    assert (NI, d, H) == (10000, 16, 7)
    o, g = Oracle(seed), gtree.GTree(seed)
    fo, to, lo = o.share(w["feat"]), o.share(w["thr"]), o.share(w["leaf"])
    fg, tg, lg = g.share_a(w["feat"]), g.share_a(w["thr"]), g.share_a(w["leaf"])
    Io, Ig = o.share(w["I"].reshape(-1)), g.share_a(w["I"].reshape(-1))
    tree = g.tree_import(fg, tg, lg, H)
    Ro = o.infer(fo, to, lo, H, Io, NI, d)
    Rg = g.infer_batch(tree, Ig, NI, d)
    _same(Rg, Ro, "inference")
    T = np.concatenate([w["feat"], w["leaf"]]).astype(np.int64)
    thr = np.concatenate([w["thr"], np.zeros(1 << H, dtype=np.uint64)])
    assert np.array_equal(g.rec(Rg).astype(np.int64), plain_cart.predict(T, H, w["I"], thr))
    ro, wo = o.stats()
    rg, wg, _ = g.stats()
    assert ro == rg and np.array_equal(wo, wg)
    assert np.array_equal(o.wire_bits(), g.wire_bits_dev())
    tree.close(); g.close(); o.close()


def test_maximum_sample_count(seed):
    """GT_MAX_N = 2^20 samples (the bound that keeps the Gini terms below 2^40): a level and the
    label level on 2 columns, every share against the oracle, the split and the statistics
    against plain integer arithmetic; one sample more is refused."""
    import torch
    from oracle import Oracle, X_M, X_C, X_SD, X_SCORE, X_T
    from paper_2305_00645_amd import gtree
    N, d, K, H = 1 << 20, 2, 2, 1
    rng = np.random.default_rng(2020)
    X = (rng.random((N, d)) < np.array([0.5, 0.3])).astype(np.uint64)
    y = (X[:, 1] ^ (rng.random(N) < 0.05)).astype(np.int64)          # column 1 decides the class, 5 % flipped
    Y = np.zeros((N, K), dtype=np.uint64); Y[np.arange(N), y] = 1
    o, g = Oracle(seed, K=K), gtree.GTree(seed, K=K)
    xg, yg = g.share_a(X.reshape(-1)), g.share_a(Y.reshape(-1))
    g.train_create(xg, yg, N, d, H)
    o.train_create(o.share(X.reshape(-1)), o.share(Y.reshape(-1)), N, d, H)
    g.train_level(0); o.train_level(0)
    for what, name in ((X_SD, "SD"), (X_C, "C"), (X_SCORE, "score"), (X_M, "M")):
        _same(g.train_export(what), o.train_export(what), name)
    C = g.rec(g.train_export(X_C)).astype(np.int64)
    want = [int(((X[:, k] == 1) & (y == c)).sum()) for k in range(d) for c in range(K)] + [int((y == c).sum()) for c in range(K)]
    assert C.tolist() == want
    assert g.rec(g.train_export(X_SD)).tolist() == [1]
    fo, lo = o.train_finish()
    tree = g.train_finish()
    fg, lg = tree.export()
    _same(fg, fo, "tree features"); _same(lg, lo, "tree labels")
    _same(g.train_export(X_M), o.train_export(X_M), "M after the label level")
    assert g.rec(lg).tolist() == [0, 1]
    ro, wo = o.stats(); rg, wg, _ = g.stats()
    assert ro == rg and np.array_equal(wo, wg) and np.array_equal(o.wire_bits(), g.wire_bits_dev())
    tree.close()
    big = g.new((N + 1) * d)
    with pytest.raises(gtree.GtError) as e:
        g.train_create(big, g.new((N + 1) * K), N + 1, d, H)
    assert e.value.code == gtree.GT_EINVAL
    g.close(); o.close()
    torch.cuda.empty_cache()


def test_maximum_depth(seed):
    """GT_MAX_DEPTH = 16 decision levels: inference through a random complete tree of 2^16 - 1
    nodes and 2^16 leaves (the last array access scans 65,536 labels per instance), every share
    against the oracle and the labels against plaintext traversal; depth 17 is refused."""
    import torch
    from oracle import Oracle
    from paper_2305_00645_amd import gtree
    H, d, NI = 16, 5, 21
    rng = np.random.default_rng(1616)
    feat = rng.integers(0, d, size=(1 << H) - 1).astype(np.uint64)
    leaf = rng.integers(0, 3, size=1 << H).astype(np.uint64)
    I = (rng.random((NI, d)) < 0.5).astype(np.uint64)
    o, g = Oracle(seed), gtree.GTree(seed)
    tree = g.tree_import(g.share_a(feat), None, g.share_a(leaf), H)
    fo, lo = o.share(feat), o.share(leaf)
    Rg = g.infer_batch(tree, g.share_a(I.reshape(-1)), NI, d)
    Ro = o.infer(fo, None, lo, H, o.share(I.reshape(-1)), NI, d)
    _same(Rg, Ro, "labels")
    T = np.concatenate([feat, leaf]).astype(np.int64)
    idx = np.zeros(NI, dtype=np.int64)
    for _ in range(H):
        idx = 2 * idx + 1 + I[np.arange(NI), T[idx]].astype(np.int64)
    assert np.array_equal(g.rec(Rg).astype(np.int64), T[idx])
    ro, wo = o.stats(); rg, wg, _ = g.stats()
    assert ro == rg and np.array_equal(wo, wg) and np.array_equal(o.wire_bits(), g.wire_bits_dev())
    tree.close()
    with pytest.raises(gtree.GtError) as e:
        g.tree_import(g.new((1 << 17) - 1), None, g.new(1 << 17), 17)
    assert e.value.code == gtree.GT_EINVAL
    g.close(); o.close()
    torch.cuda.empty_cache()
