"""Pins for the oracle's training and inference against plaintext references."""
from fractions import Fraction

import numpy as np
import pytest

import plain_cart
from oracle import Oracle, X_T, X_F, X_M, X_C, X_GAMMA, X_SD, X_L, X_SCORE, X_C_PAPER
from paper_2305_00645_amd import workloads as wl

M64 = (1 << 64) - 1


def expected_M_by_products(ref, w, H):
    """M per level when the partition uses the previous level's leaf one-hot: a sample moves by
    its feature value only while it sits in a real leaf; below a node that stopped being one it
    keeps going left."""
    X = np.asarray(w["X"]).astype(np.int64)
    N = X.shape[0]
    M = np.zeros(N, dtype=np.int64)
    out = [M.copy()]
    for h in range(1, H + 1):
        prev = M - ((1 << (h - 1)) - 1)
        real = np.array([_was_leaf(ref, h - 1, int(r)) for r in prev])
        M = 2 * M + 1 + np.where(real, X[np.arange(N), ref["T"][M]], 0)
        out.append(M.copy())
    return out


def run_oracle_train(seed, w, tau=16, H=None, check_levels=True, by_reconstruction=False, literal=False, by_products=False):
    H = w["H"] if H is None else H
    N, d, K = w["N"], w["d"], w["K"]
    o = Oracle(seed, tau=tau, K=K)
    sx, sy = o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1))
    o.train_create(sx, sy, N, d, H)
    o.train_set_heuristic(by_reconstruction)
    o.train_set_literal(literal)
    o.train_set_partition(by_products)
    ref = plain_cart.train(w["X"], w["y"], K, H, tau)
    Mexp = expected_M_by_products(ref, w, H) if by_products else [ref["levels"][h]["M"] for h in range(H + 1)]
    CW = d * K + K
    for h in range(H):
        o.train_level(h)
        if not check_levels:
            continue
        nh = 1 << h
        L = ref["levels"][h]
        assert np.array_equal(Oracle.rec(o.train_export(X_M)).astype(np.int64), Mexp[h])
        C = Oracle.rec(o.train_export(X_C)).astype(np.int64).reshape(nh, CW)
        for r in range(nh):
            assert np.array_equal(C[r, :d * K].reshape(d, K), L["n1"][r]), (h, r)
            assert np.array_equal(C[r, d * K:], L["tot"][r]), (h, r)
        S = Oracle.rec(o.train_export(X_SCORE)).astype(np.int64).reshape(nh, d)
        assert np.array_equal(S, np.array(L["score"]))
        assert np.array_equal(Oracle.rec(o.train_export(X_SD)).astype(np.int64), np.array(L["SD"]))
        G = Oracle.rec(o.train_export(X_GAMMA)).astype(np.int64).reshape(nh, d)
        assert np.array_equal(G, np.array(L["gamma"]))
        if literal:
            continue                           # no arithmetic one-hot exists in this mode
        # per-sample leaf one-hot: 1 exactly at the sample's node when that node is a real leaf
        LT = Oracle.rec(o.train_export(X_L)).astype(np.int64).reshape(nh, -1)[:, :N]
        Fbefore = np.array([1 if (L["split"][r] or _was_leaf(ref, h, r)) else 0 for r in range(nh)])
        want = ((Mexp[h][None, :] - (nh - 1)) == np.arange(nh)[:, None]) & (Fbefore[:, None] == 1)
        assert np.array_equal(LT, want.astype(np.int64))
    feat, leaf = o.train_finish()
    T = Oracle.rec(o.train_export(X_T)).astype(np.int64)
    F = Oracle.rec(o.train_export(X_F)).astype(np.int64)
    assert np.array_equal(T, ref["T"])
    assert np.array_equal(F, ref["F"])
    assert np.array_equal(Oracle.rec(feat).astype(np.int64), ref["T"][:(1 << H) - 1])
    assert np.array_equal(Oracle.rec(leaf).astype(np.int64), ref["T"][(1 << H) - 1:])
    assert np.array_equal(Oracle.rec(o.train_export(X_M)).astype(np.int64), Mexp[H])
    return o, ref, (feat, leaf)


def _was_leaf(ref, h, r):
    """Node type before this level's update: a node is a real leaf iff it is the
    root or its parent was split."""
    if h == 0:
        return True
    return bool(ref["levels"][h - 1]["split"][r // 2])


def check_tree_encoding(F, H):
    """Every root-to-bottom path reads 0..0, then at most one 1, then 2..2 (Sec. IV)."""
    for leafpos in range(1 << H):
        node = (1 << H) - 1 + leafpos
        path = []
        while True:
            path.append(int(F[node]))
            if node == 0:
                break
            node = (node - 1) // 2
        path = path[::-1]
        s = "".join(map(str, path))
        assert s.lstrip("0").lstrip("1").strip("2") == "" and s.count("1") <= 1, s
        assert set(path) <= {0, 1, 2}


def test_c1_full_training_matches_plaintext_cart(seed):
    w = wl.c1_train()
    o, ref, _ = run_oracle_train(seed, w)
    check_tree_encoding(ref["F"], w["H"])
    # the learned tree fits the (noisy) training labels far better than chance
    acc = (plain_cart.predict(ref["T"], w["H"], w["X"]) == w["y"]).mean()
    assert acc > 0.85


@pytest.mark.parametrize("H", [1, 4])
def test_c2_training_matches_plaintext_cart(seed, H):
    w = wl.c2_train()
    run_oracle_train(seed, w, H=H)


def test_c2_depth7_tree_and_structure(seed):
    w = wl.c2_train()
    o, ref, _ = run_oracle_train(seed, w, H=7, check_levels=False)
    check_tree_encoding(ref["F"], 7)
    assert (ref["F"] == 2).sum() > 0 and (ref["F"] == 0).sum() > 5


def test_multiclass_and_other_tau(seed):
    rng = np.random.default_rng(77)
    N, d, K = 150, 9, 4
    X = (rng.random((N, d)) < 0.4).astype(np.uint64)
    y = (X[:, 0].astype(np.int64) * 2 + X[:, 3].astype(np.int64) + (rng.random(N) < 0.1)) % K
    Y = np.zeros((N, K), dtype=np.uint64); Y[np.arange(N), y] = 1
    w = dict(X=X, Y=Y, y=y, N=N, d=d, K=K, H=3)
    run_oracle_train(seed, w, tau=10)


def test_small_c3_shape_matches_plaintext_cart(seed):
    w = wl.c3_train(N=600, H=3, n_thr=4)
    assert w["d"] == 6 * 4 + 102
    run_oracle_train(seed, w, check_levels=False)


def test_degenerate_inputs(seed):
    # one class only: the root is pure, everything below is a dummy, all labels equal
    X = np.array([[0, 1], [1, 1], [1, 0], [0, 0], [1, 1]], dtype=np.uint64)
    y = np.ones(5, dtype=np.int64)
    Y = np.zeros((5, 2), dtype=np.uint64); Y[:, 1] = 1
    o, ref, (feat, leaf) = run_oracle_train(seed, dict(X=X, Y=Y, y=y, N=5, d=2, K=2, H=2))
    assert list(ref["F"]) == [1, 2, 2, 2, 2, 2, 2]
    assert set(Oracle.rec(leaf).tolist()) == {1}
    # depth 0: only a label
    o, ref, (feat, leaf) = run_oracle_train(seed, dict(X=X, Y=Y, y=y, N=5, d=2, K=2, H=0))
    assert feat.shape[1] == 0 and Oracle.rec(leaf).tolist() == [1]
    # a single candidate column, more levels than candidates
    X1 = np.array([[0], [1], [1], [0]], dtype=np.uint64)
    y1 = np.array([0, 1, 1, 0])
    Y1 = np.zeros((4, 2), dtype=np.uint64); Y1[np.arange(4), y1] = 1
    run_oracle_train(seed, dict(X=X1, Y=Y1, y=y1, N=4, d=1, K=2, H=2))


def test_heuristic_by_reconstruction_matches_plaintext_cart(seed):
    """The reconstruct-and-score heuristic (host analogue of the TEE-based protocol, Sec. V-B)
    gives, level by level, the same M, statistics, masked scores, split decisions, gamma, node
    types and tree as the plaintext CART - hence the same as the MPC heuristic, which the
    tests above pin to the same reference - on two-class, multi-class, ragged and degenerate
    inputs; its sharings are fresh (components differ from the MPC run) and it needs far fewer
    rounds."""
    w = wl.c1_train()
    o, ref, _ = run_oracle_train(seed, w, by_reconstruction=True)
    o2, _, _ = run_oracle_train(seed, w)
    assert o.stats()[0] < o2.stats()[0] / 5
    assert not np.array_equal(o.train_export(X_T), o2.train_export(X_T))
    assert np.array_equal(Oracle.rec(o.train_export(X_T)), Oracle.rec(o2.train_export(X_T)))
    sin, sout = o.scorer_bytes()
    CW = w["d"] * w["K"] + w["K"]
    nn = sum(1 << h for h in range(w["H"]))
    assert sin == 3 * 8 * nn * (CW + w["d"] + 1) and sout == 3 * 16 * nn * (2 * w["d"] + 4)
    run_oracle_train(seed, wl.c2_train(), H=5, by_reconstruction=True)
    rng = np.random.default_rng(77)
    N, d, K = 150, 9, 4
    X = (rng.random((N, d)) < 0.4).astype(np.uint64)
    y = (X[:, 0].astype(np.int64) * 2 + X[:, 3].astype(np.int64) + (rng.random(N) < 0.1)) % K
    Y = np.zeros((N, K), dtype=np.uint64); Y[np.arange(N), y] = 1
    run_oracle_train(seed, dict(X=X, Y=Y, y=y, N=N, d=d, K=K, H=3), tau=10, by_reconstruction=True)
    X = np.array([[0, 1], [1, 1], [1, 0], [0, 0], [1, 1]], dtype=np.uint64)
    y = np.ones(5, dtype=np.int64)
    Y = np.zeros((5, 2), dtype=np.uint64); Y[:, 1] = 1
    run_oracle_train(seed, dict(X=X, Y=Y, y=y, N=5, d=2, K=2, H=2), by_reconstruction=True)


def test_learning_protocol_as_printed_matches_plaintext_and_cost_formula(seed):
    """The learning protocol run as the paper prints it (array access over the whole tree
    array, a SelectShare per element of the per-sample counter arrays, local accumulation)
    gives the plaintext CART level by level - hence the same reconstructed state as the fused
    protocol - and costs what the formulas of Sec. V-A say: per level h >= 1 and party,
    (N*|T| + N*d)(4l-1) bits for the two array accesses, n_h(2l-1) for the leaf flags,
    N*n_h*2l for the per-sample flags (test and AND), N*n_h*(1+K)*2d*2l for the selects."""
    w = wl.c1_train(N=60, d=5, depth=3)
    N, d, K, H, l = w["N"], w["d"], w["K"], w["H"], 64
    o, ref, _ = run_oracle_train(seed, w, literal=True)
    o2, _, _ = run_oracle_train(seed, w)
    for what in (X_T, X_F, X_M, X_C):
        assert np.array_equal(Oracle.rec(o.train_export(what)), Oracle.rec(o2.train_export(what)))
    # learning part of the cost, separated from heuristic and node split by differencing two modes:
    # both runs share the heuristic, so the difference of their bits is (literal - fused) learning
    nT = (2 << H) - 1
    lit = 0
    for h in range(H + 1):
        nh = 1 << h
        cols = (1 + K) * 2 * (1 if h == H else d)
        lit += (N * nT + N * d) * (4 * l - 1) if h > 0 else 0
        lit += nh * (2 * l - 1) + N * nh * 2 * l + N * nh * cols * 2 * l
    fused = 0
    CW = d * K + K
    for h in range(H + 1):
        nh = 1 << h
        if h > 0:       # two array accesses: opening per sample, 63 + 1 bits per test, reshare per sample
            fused += (N * l + N * (nh // 2) * l + N * l) + (N * l + N * d * l + N * l)
        # leaf flags (per node), leaf grid (opening per sample; 63 + AND 1 + conversion 1 per test), count reshare
        fused += nh * (2 * l - 1) + N * l + N * nh * (l + 1) + nh * (K if h == H else CW) * l
    assert int(o.wire_bits()[0].sum()) - int(o2.wire_bits()[0].sum()) == lit - fused
    run_oracle_train(seed, wl.c2_train(N=80, d=7, H=3), literal=True)


def test_partition_by_products_matches_plaintext_cart(seed):
    """Data partition by products with the previous level's leaf one-hot: statistics, scores,
    split decisions, node types, tree and labels equal the plaintext CART level by level; M
    equals the paper's recurrence for every sample in a real leaf (and goes left below a node
    that stopped being one); the partition costs N*d*l + N*l bits plus n_{h-1}*d equality tests
    with conversion instead of N*(n_{h-1} + d)*l + 4*N*l (two array accesses, each with one
    opening and one reshare per sample and l bits per test)."""
    w = wl.c1_train()
    N, d, K, H, l = w["N"], w["d"], w["K"], w["H"], 64
    o, ref, _ = run_oracle_train(seed, w, by_products=True)
    o2, _, _ = run_oracle_train(seed, w)
    assert np.array_equal(Oracle.rec(o.train_export(X_T)), Oracle.rec(o2.train_export(X_T)))
    saved = 0
    for h in range(1, H + 1):
        npv = 1 << (h - 1)
        saved += (N * (npv + d) * l + 4 * N * l) - (npv * d * 2 * l + N * d * l + N * l)
    assert int(o2.wire_bits()[0].sum()) - int(o.wire_bits()[0].sum()) == saved
    assert o.stats()[0] == o2.stats()[0] - H * (18 - 10)           # two array accesses of 9 rounds against 7 + 1 + 1 + 1
    run_oracle_train(seed, wl.c2_train(), H=5, by_products=True)          # has nodes that stop early
    rng = np.random.default_rng(77)
    N, d, K = 150, 9, 4
    X = (rng.random((N, d)) < 0.4).astype(np.uint64)
    y = (X[:, 0].astype(np.int64) * 2 + X[:, 3].astype(np.int64) + (rng.random(N) < 0.1)) % K
    Y = np.zeros((N, K), dtype=np.uint64); Y[np.arange(N), y] = 1
    run_oracle_train(seed, dict(X=X, Y=Y, y=y, N=N, d=d, K=K, H=3), tau=10, by_products=True)
    X = np.array([[0, 1], [1, 1], [1, 0], [0, 0], [1, 1]], dtype=np.uint64)
    y = np.ones(5, dtype=np.int64)
    Y = np.zeros((5, 2), dtype=np.uint64); Y[:, 1] = 1
    run_oracle_train(seed, dict(X=X, Y=Y, y=y, N=5, d=2, K=2, H=2), by_products=True)
    # a state that was imported has no one-hot of the previous level: the level is refused
    wi = wl.c5_level(N=50, d=4, K=2, h=2)
    oi = Oracle(seed, K=2)
    oi.train_create(oi.share(wi["X"].reshape(-1)), oi.share(wi["Y"].reshape(-1)), 50, 4, 3)
    oi.train_set_partition(True)
    oi.train_import(2, *[oi.share(a) for a in (wi["M"], wi["Tprev"], wi["F"], np.zeros(4 * 10, dtype=np.uint64), wi["gamma"].reshape(-1))])
    with pytest.raises(RuntimeError):
        oi.train_level(2)


def test_counter_array_paper_layout(seed):
    """Row/column relations of the counter array (Sec. V-B, statistics counting)."""
    w = wl.c1_train()
    N, d, K = w["N"], w["d"], w["K"]
    o = Oracle(seed, K=K)
    o.train_create(o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1)), N, d, 2)
    o.train_level(0)
    C = Oracle.rec(o.train_export(X_C_PAPER)).astype(np.int64).reshape(1 + K, 2 * d)
    X, y = w["X"].astype(np.int64), w["y"]
    for k in range(d):
        for v in (0, 1):
            assert C[0, 2 * k + v] == (X[:, k] == v).sum()
            for c in range(K):
                assert C[c + 1, 2 * k + v] == ((X[:, k] == v) & (y == c)).sum()
    assert np.array_equal(C[0], C[1:].sum(axis=0))


def test_choice_close_to_real_valued_gini_and_exact_rational(seed):
    """The chosen candidate's Gini index (definition of Sec. II-A) is within 2^(2-tau)
    of the minimum over unused candidates, and by exact rational comparison
    (cross-multiplication, valid here since N <= 8192) it is within two floor errors."""
    for w, H, tau in ((wl.c1_train(), 3, 16), (wl.c2_train(), 5, 16), (wl.c2_train(), 3, 6)):
        ref = plain_cart.train(w["X"], w["y"], w["K"], H, tau)
        N, d, K = w["N"], w["d"], w["K"]
        o = Oracle(seed, tau=tau, K=K)
        o.train_create(o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1)), N, d, H)
        gam = {0: np.ones(d, dtype=np.int64)}
        for h in range(H):
            o.train_level(h)
            SD = Oracle.rec(o.train_export(X_SD)).astype(np.int64)
            L = ref["levels"][h]
            ngam = {}
            for r in range(1 << h):
                g = gam[r]
                if L["split"][r] and g.sum() > 0:
                    gr = plain_cart.gini_real(L["n1"][r], L["tot"][r])
                    ex = plain_cart.scores_exact(L["n1"][r], L["tot"][r])
                    free = [k for k in range(d) if g[k]]
                    k = int(SD[r])
                    assert g[k] == 1
                    assert gr[k] <= min(gr[q] for q in free) + 2.0 ** (2 - tau)
                    assert ex[k] >= max(ex[q] for q in free) - Fraction(2, 1 << tau)
                g2 = g.copy(); g2[int(SD[r])] = 0
                ngam[2 * r] = ngam[2 * r + 1] = g2
            gam = ngam


@pytest.mark.parametrize("N,d,K,h", [(700, 12, 4, 3), (300, 7, 2, 5)])
def test_level_from_imported_state_matches_plaintext_histogram(seed, N, d, K, h):
    """The import call (used to start a single level from a synthetic state) holds no
    arithmetic of its own: after it, one level must route every sample as the plaintext
    recurrence M <- 2M + X[i][T[M]] + 1 says (Sec. V-B, data partition) and count exactly the
    plaintext histogram of the routed samples (statistics counting); inherited statistics
    that are imported are added to, not replaced."""
    w = wl.c5_level(N=N, d=d, K=K, h=h)
    CW = d * K + K
    rng = np.random.default_rng(N)
    C0 = rng.integers(0, 50, size=(1 << h) * CW).astype(np.uint64)       # inherited statistics
    o = Oracle(seed, K=K)
    o.train_create(o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1)), N, d, h + 1)
    st = [w["M"], w["Tprev"], w["F"], C0, w["gamma"].reshape(-1)]
    o.train_import(h, *[o.share(a) for a in st])
    with pytest.raises(RuntimeError):
        o.train_export(X_C)                    # nothing of a "last level" exists before a level has run
    assert np.array_equal(Oracle.rec(o.train_export(X_M)), w["M"])       # the state itself is there
    o.train_level(h)
    X, y, Mi = w["X"].astype(np.int64), w["y"], w["M"].astype(np.int64)
    M = 2 * Mi + 1 + X[np.arange(N), w["Tprev"].astype(np.int64)[Mi - ((1 << (h - 1)) - 1)]]
    assert np.array_equal(Oracle.rec(o.train_export(X_M)).astype(np.int64), M)
    C = Oracle.rec(o.train_export(X_C)).astype(np.int64).reshape(1 << h, CW)
    C0 = C0.astype(np.int64).reshape(1 << h, CW)
    for r in range(1 << h):
        sel = M == (1 << h) - 1 + r
        for c in range(K):
            assert C[r, d * K + c] == C0[r, d * K + c] + (sel & (y == c)).sum()
            assert np.array_equal(C[r, :d * K].reshape(d, K)[:, c],
                                  C0[r, :d * K].reshape(d, K)[:, c] + X[sel & (y == c)].sum(axis=0))
    # all nodes were imported as real leaves: the one-hot of a sample is 1 exactly at its node
    LT = Oracle.rec(o.train_export(X_L)).astype(np.int64).reshape(1 << h, -1)[:, :N]
    assert np.array_equal(LT, ((M[None, :] - ((1 << h) - 1)) == np.arange(1 << h)[:, None]).astype(np.int64))
    # a level started by import consumes the same operations and messages as the same level
    # reached by training: partition 2 array accesses, leaf flags, grid, count, ...
    o2 = Oracle(seed, K=K)
    o2.train_create(o2.share(w["X"].reshape(-1)), o2.share(w["Y"].reshape(-1)), N, d, h + 1)
    for hh in range(h):
        o2.train_level(hh)
    ops0, (r0, w0) = o2.op_counter(), o2.stats()
    o2.train_level(h)
    o3 = Oracle(seed, K=K)
    o3.train_create(o3.share(w["X"].reshape(-1)), o3.share(w["Y"].reshape(-1)), N, d, h + 1)
    o3.train_import(h, *[o3.share(a) for a in st])
    ops1, (r1, w1) = o3.op_counter(), o3.stats()
    o3.train_level(h)
    assert o2.op_counter() - ops0 == o3.op_counter() - ops1
    assert o2.stats()[0] - r0 == o3.stats()[0] - r1
    assert np.array_equal(o2.stats()[1] - w0, o3.stats()[1] - w1)


def test_wire_and_rounds_do_not_depend_on_data(seed):
    """Only sizes and depth may show in the message pattern (Sec. I, goals)."""
    res = []
    for s in (11, 12):
        w = wl.c1_train(N=64, d=6, depth=2, seed=s)
        o = Oracle(seed, K=2)
        o.train_create(o.share(w["X"].reshape(-1)), o.share(w["Y"].reshape(-1)), 64, 6, 2)
        o.train_level(0); o.train_level(1); o.train_finish()
        res.append((o.stats()[0], o.stats()[1].tolist(), o.op_counter()))
    assert res[0] == res[1]


# ---------------------------------------------------------------- inference
@pytest.mark.parametrize("binary", [False, True])
def test_inference_matches_plaintext_traversal(seed, binary):
    w = wl.c4_infer(NI=300, H=5, binary=binary)
    o = Oracle(seed)
    sf, sl = o.share(w["feat"]), o.share(w["leaf"])
    st = None if w["thr"] is None else o.share(w["thr"])
    sI = o.share(w["I"].reshape(-1))
    o.stats_reset()
    R = o.infer(sf, st, sl, w["H"], sI, w["NI"], w["d"])
    T = np.concatenate([w["feat"], w["leaf"]]).astype(np.int64)
    thr = None if w["thr"] is None else np.concatenate([w["thr"], np.zeros(1 << w["H"], dtype=np.uint64)])
    want = plain_cart.predict(T, w["H"], w["I"], thr)
    assert np.array_equal(Oracle.rec(R).astype(np.int64), want)
    rounds, _ = o.stats()
    per_level = 9 + 9 + (0 if binary else 8)
    assert rounds == w["H"] * per_level + 9


def test_inference_on_trained_tree_equals_plaintext_prediction(seed):
    w = wl.c1_train()
    o, ref, (feat, leaf) = run_oracle_train(seed, w, check_levels=False)
    rng = np.random.default_rng(5)
    I = (rng.random((200, w["d"])) < 0.5).astype(np.uint64)
    R = o.infer(feat, None, leaf, w["H"], o.share(I.reshape(-1)), 200, w["d"])
    assert np.array_equal(Oracle.rec(R).astype(np.int64), plain_cart.predict(ref["T"], w["H"], I))


def test_inference_depth0_and_single_instance(seed):
    o = Oracle(seed)
    leaf = o.share(np.array([3], dtype=np.uint64))
    feat = np.zeros((3, 0), dtype=np.uint64)
    I = o.share(np.array([1, 0], dtype=np.uint64))
    R = o.infer(feat, None, leaf, 0, I, 1, 2)
    assert Oracle.rec(R).tolist() == [3]


@pytest.mark.parametrize("binary", [False, True])
def test_sampled_rows_equal_full_inference(seed, binary):
    """The row-subset mode used for spot checks of large batches gives the same shares."""
    w = wl.c4_infer(NI=203, H=4, binary=binary)
    oa, ob = Oracle(seed), Oracle(seed)
    parts = [w["feat"], w["leaf"]] + ([] if binary else [w["thr"]])
    sa = [oa.share(a) for a in parts]
    sb = [ob.share(a) for a in parts]
    Ia, Ib = oa.share(w["I"].reshape(-1)), ob.share(w["I"].reshape(-1))
    full = oa.infer(sa[0], None if binary else sa[2], sa[1], w["H"], Ia, w["NI"], w["d"])
    rows = np.array([0, 7, 8, 100, 202])
    Irows = Ib.reshape(3, w["NI"], w["d"])[:, rows, :].reshape(3, -1)
    part = ob.infer_rows(sb[0], None if binary else sb[2], sb[1], w["H"], Irows, w["NI"], w["d"], rows)
    assert np.array_equal(part, full[:, rows])
    assert oa.op_counter() == ob.op_counter()
