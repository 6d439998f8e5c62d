"""Pins for the oracle's building blocks against plain integer arithmetic and the
paper's cost formulas (Sec. II-B, Sec. V-A)."""
import numpy as np
import pytest

from oracle import Oracle

M64 = (1 << 64) - 1
U = np.uint64


def u64(vals):
    return np.array([int(v) & M64 for v in vals], dtype=np.uint64)


EDGE = [0, 1, 2, 3, (1 << 63), (1 << 63) - 1, M64, M64 - 1, 1 << 32, (1 << 32) - 1, 0xDEADBEEFCAFEF00D]


def test_share_reconstruct_and_replication(seed):
    o = Oracle(seed)
    x = u64(EDGE + list(range(50)))
    s = o.share(x)
    assert s.shape == (3, x.size)
    assert np.array_equal(Oracle.rec(s), x)
    # fresh randomness per call, and components look random
    s2 = o.share(x)
    assert not np.array_equal(s[0], s2[0])
    assert len(set(s[0].tolist())) == x.size
    # component 3 is determined by the other two
    assert np.array_equal(s[2], x - s[0] - s[1])


def test_linear_ops_are_local(seed):
    o = Oracle(seed)
    rng = np.random.default_rng(1)
    x = rng.integers(0, M64, size=100, dtype=np.uint64)
    s = o.share(x)
    t = s * U(5)
    t[0] += U(7)                      # public constant goes to component 1 only
    assert np.array_equal(Oracle.rec(t), x * U(5) + U(7))


def test_mult_matches_ring_product(seed):
    o = Oracle(seed)
    rng = np.random.default_rng(2)
    x = np.concatenate([u64(EDGE), rng.integers(0, M64, size=200, dtype=np.uint64)])
    y = np.concatenate([u64(EDGE[::-1]), rng.integers(0, M64, size=200, dtype=np.uint64)])
    sx, sy = o.share(x), o.share(y)
    op0 = o.op_counter()
    z = o.mult(sx, sy)
    assert o.op_counter() == op0 + 1
    assert np.array_equal(Oracle.rec(z), x * y)
    # z_i = x_i y_i + x_{i+1} y_i + x_i y_{i+1} + alpha_i  (Sec. II-B)
    for j in range(3):
        n = (j + 1) % 3
        e = 5
        al = o.zero_sharing(op0, 0, e)
        assert int(z[j][e]) == (int(sx[j][e]) * int(sy[j][e]) + int(sx[n][e]) * int(sy[j][e])
                                + int(sx[j][e]) * int(sy[n][e]) + int(al[j])) & M64


def _eq_cases():
    xs, ys = [], []
    rng = np.random.default_rng(3)
    for b in range(64):                       # single-bit differences at every position
        v = int(rng.integers(0, M64, dtype=np.uint64))
        xs.append(v); ys.append(v ^ (1 << b))
    for v in EDGE:
        xs += [v, v, v, v, v]
        ys += [v, v + 1, v - 1, v + (1 << 62), v - (1 << 62)]
    for _ in range(100):
        v = int(rng.integers(0, M64, dtype=np.uint64))
        xs.append(v); ys.append(v if rng.random() < 0.5 else int(rng.integers(0, M64, dtype=np.uint64)))
    return u64(xs), u64(ys)


def test_eq_brute_force_public_and_shared_operand(seed):
    o = Oracle(seed)
    x, y = _eq_cases()
    want = (x == y).astype(np.uint64)
    sx = o.share(x)
    eb = o.eq_b(sx, y)                               # public second operand
    assert np.array_equal(Oracle.rec_b(eb) , want)
    assert np.all(Oracle.rec_b(eb) <= 1) and np.all(eb <= 1)
    sy = o.share(y)
    ea = o.eq_a(sx - sy, None)                       # both operands shared
    assert np.array_equal(Oracle.rec(ea), want)
    assert want.sum() > 20 and (1 - want).sum() > 100


def test_eq_cost_is_2l_minus_1_bits_in_log_l_plus_1_rounds(seed):
    o = Oracle(seed)
    n = 4096
    sx = o.share(np.arange(n, dtype=np.uint64))
    o.stats_reset()
    o.eq_b(sx, np.arange(n, dtype=np.uint64))
    rounds, wire = o.stats()
    assert rounds == 7                               # log l + 1, l = 64 (Sec. V-A)
    for p in range(3):
        assert int(wire[p].sum()) * 8 == n * (2 * 64 - 1)
        assert wire[p][p] == 0


def _ge_cases():
    rng = np.random.default_rng(4)
    xs, ys = [], []
    smalls = [0, 1, 2, 5, 1 << 16, (1 << 40) - 1, 1 << 40, (1 << 41), (1 << 62), (1 << 63) - 1]
    for a in smalls:
        for b in smalls:
            xs.append(a); ys.append(b)
    for b in range(63):                              # differ exactly in bit b
        v = int(rng.integers(0, 1 << 62))
        xs.append(v | (1 << b)); ys.append(v & ~(1 << b))
        xs.append(v & ~(1 << b)); ys.append(v | (1 << b))
    for _ in range(300):
        a, b = int(rng.integers(0, 1 << 62)), int(rng.integers(0, 1 << 62))
        xs.append(a); ys.append(b)
    # signed operands whose difference stays below 2^63 in magnitude
    for a, b in [(-5, 3), (3, -5), (-1, -1), (-(1 << 61), 1 << 61), (1 << 61, -(1 << 61)), (-7, -8)]:
        xs.append(a); ys.append(b)
    return xs, ys


def test_ge_brute_force(seed):
    o = Oracle(seed)
    xs, ys = _ge_cases()
    want = u64([1 if a >= b else 0 for a, b in zip(xs, ys)])
    g = o.ge_a(o.share(u64(xs)), o.share(u64(ys)))
    assert np.array_equal(Oracle.rec(g), want)


def test_ge_cost(seed):
    o = Oracle(seed)
    n = 1024
    s = o.share(np.arange(n, dtype=np.uint64))
    o.stats_reset()
    o.ge_a(s, s)
    rounds, wire = o.stats()
    assert rounds == 7 + 1
    assert int(wire[0].sum()) * 8 == n * (64 + 125 + 1)


def test_oaa_reads_every_index_and_zero_outside(seed):
    o = Oracle(seed)
    rng = np.random.default_rng(5)
    for w in (1, 2, 5, 8, 13, 64):
        Wp = rng.integers(0, M64, size=w, dtype=np.uint64)
        u = u64(list(range(w)) + [w, w + 1, M64, 1 << 40] + list(rng.integers(0, w, size=11)))
        want = np.array([Wp[int(i)] if int(i) < w else 0 for i in u], dtype=np.uint64)
        o.stats_reset()
        z = o.oaa(o.share(Wp), o.share(u))
        rounds, wire = o.stats()
        assert np.array_equal(Oracle.rec(z), want)
        assert rounds == 9                           # log l + 3 (Sec. V-A)


def test_oaa_rounds_log_l_plus_3(seed):
    o = Oracle(seed)
    W, u = o.share(np.arange(16, dtype=np.uint64)), o.share(np.arange(8, dtype=np.uint64))
    o.stats_reset()
    o.oaa(W, u)
    rounds, wire = o.stats()
    assert rounds == 9
    # per row: ONE opening of the masked index (64 bits) for all w comparisons, per comparison the
    # 63 bits of the AND rounds and 1 bit of conversion, and one 64-bit reshare of the inner product;
    # the paper's unfused select costs (4l-1) bits per array element instead
    assert int(wire[1].sum()) * 8 == 8 * (64 + 16 * 64 + 64)
    assert 8 * (64 + 16 * 64 + 64) < 8 * 16 * (4 * 64 - 1)


@pytest.mark.parametrize("tau", [4, 10, 16])
def test_division_is_exact_floor(seed, tau):
    o = Oracle(seed, tau=tau)
    rng = np.random.default_rng(6)
    S, Q = [], []
    for q in [1, 2, 3, 7, 1000, (1 << 20) + 1, (1 << 40) - 1]:
        for s in [0, 1, q // 2, q - 1, q]:
            S.append(min(s, q)); Q.append(q)
    for _ in range(200):
        q = int(rng.integers(1, 1 << 40)); s = int(rng.integers(0, q + 1))
        S.append(s); Q.append(q)
    want = u64([(s << tau) // q for s, q in zip(S, Q)])
    op0 = o.op_counter()
    quo = o.div(o.share(u64(S)), o.share(u64(Q)))
    assert np.array_equal(Oracle.rec(quo), want)
    assert o.op_counter() - op0 == 2 + tau + 1


def test_payload_bits_follow_the_cost_formulas(seed):
    """The bit counters (no rounding to bytes) reproduce the paper's per-element costs
    exactly: equality test 2l-1 = 127 bits per party, comparison 189, bit conversion 1,
    product l = 64 (Sec. II-B, Sec. V-A)."""
    o = Oracle(seed)
    n = 37
    x = o.share(np.arange(n, dtype=np.uint64))
    o.stats_reset()
    o.eq_b(x, None)
    assert int(o.wire_bits().sum()) == 3 * n * 127
    assert int(o.wire_bits()[0, 1]) == n * 64 and int(o.wire_bits()[0, 2]) == n * 63
    o.stats_reset()
    o.eq_a(x, None)
    assert int(o.wire_bits().sum()) == 3 * n * 128
    o.stats_reset()
    o.ge_a(x, x)
    assert int(o.wire_bits().sum()) == 3 * n * 190
    o.stats_reset()
    o.mult(x, x)
    assert int(o.wire_bits().sum()) == 3 * n * 64
    # bytes are the bits of each message rounded up separately
    o.stats_reset()
    o.eq_b(o.share(np.arange(3, dtype=np.uint64)), None)
    assert int(o.stats()[1][0].sum()) == 24 + 12 + 6 + 3 + 2 + 1 + 1      # 3 elements: 64,32,16,8,4,2,1 bits each
    assert int(o.wire_bits()[0].sum()) == 3 * 127


@pytest.mark.parametrize("w,n", [(1, 3), (5, 40), (16, 9)])
def test_array_access_as_printed_costs_4l_minus_1_bits(seed, w, n):
    """The array access run element by element as the paper prints it (Sec. V-A) returns
    W[u] and costs exactly N(4l-1) bits per party in log l + 3 rounds for N = |W|*|U|; the
    fused access used elsewhere returns the same values for fewer bits."""
    o = Oracle(seed)
    rng = np.random.default_rng(w * 100 + n)
    Wp = rng.integers(0, M64, size=w, dtype=np.uint64)
    u = rng.integers(0, w + 1, size=n).astype(np.uint64)
    sW, su = o.share(Wp), o.share(u)
    o.stats_reset()
    z = o.oaa_literal(sW, su)
    want = np.array([Wp[int(i)] if int(i) < w else 0 for i in u], dtype=np.uint64)
    assert np.array_equal(Oracle.rec(z), want)
    rounds, _ = o.stats()
    assert rounds == 6 + 3
    bits = o.wire_bits()
    for p in range(3):
        assert int(bits[p].sum()) == w * n * (4 * 64 - 1)
    o.stats_reset()
    z2 = o.oaa(sW, su)
    assert np.array_equal(Oracle.rec(z2), want)
    assert int(o.wire_bits()[0].sum()) == n * 64 + w * n * 64 + n * 64 < w * n * 255 + 1


def test_grid_opens_one_masked_index_per_row(seed):
    """In an equality grid the comparisons of a row are all with public constants, so the row's
    masked index is opened once: the array access must still return W[u] for every u (also
    outside the array), its messages must be 64 bits per row + 63 + 1 per test + the reshare,
    and the daBits of the eight tests of a group come from three dealer blocks whose Boolean
    and arithmetic components share the same bit."""
    o = Oracle(seed)
    for e in (0, 1, 2, 3, 7, 8, 1000003):
        d = o.dabit_grid(5, e)
        assert int(d["bB"][0] ^ d["bB"][1] ^ d["bB"][2]) == d["beta"] and d["beta"] in (0, 1)
        assert (int(d["bA"][0]) + int(d["bA"][1]) + int(d["bA"][2])) & M64 == d["beta"]
    # tests 0..2 share a block and differ; tests of different groups use different blocks
    assert len({int(o.dabit_grid(5, e)["bA"][0]) for e in range(16)}) == 16
    rng = np.random.default_rng(8)
    w, n = 11, 29
    Wp = rng.integers(0, M64, size=w, dtype=np.uint64)
    u = np.concatenate([np.arange(w + 3), rng.integers(0, w, size=n - w - 3)]).astype(np.uint64)
    sW, su = o.share(Wp), o.share(u)
    o.stats_reset()
    z = o.oaa(sW, su)
    assert np.array_equal(Oracle.rec(z), np.array([Wp[int(i)] if int(i) < w else 0 for i in u], dtype=np.uint64))
    bits = o.wire_bits()
    assert int(bits[0, 1]) == n * 64 + w * n * 1                  # to the successor: opening per row, conversion bit per test
    assert int(bits[0, 2]) == w * n * 63 + n * 64                 # to the predecessor: AND rounds per test, reshare per row
