"""Pins for the oracle's randomness: RFC 8439 vectors, stream layout, correlated
randomness identities (zero sharings, edaBits, daBits)."""
import os

import numpy as np

from oracle import Oracle
from oracle import orc

M64 = (1 << 64) - 1
GOLD = os.path.join(os.path.dirname(__file__), "golden", "rfc8439_chacha20.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        out[k] = [int(x, 16) for x in v]
    return out


def test_quarter_round_rfc8439():
    g = _gold()
    assert list(orc.chacha_quarter(g["qr_in"])) == g["qr_out"]


def test_block_rfc8439_20_rounds():
    g = _gold()
    out = orc.chacha_block(g["key"], *g["ctr"], 20)
    assert [int(x) for x in out] == g["block"]


def test_prf_word_is_le_pair_of_8_round_block(seed):
    o = Oracle(seed)
    for key_index in range(5):
        key = []
        for w in seed[key_index]:
            key += [w & 0xFFFFFFFF, w >> 32]
        for (op, stream, j) in [(0, 0, 0), (7, 3, 5), (123456, 2, (1 << 35) + 13), (1, 1, 8), (1, 1, 15)]:
            blk = j >> 3
            out = orc.chacha_block(key, blk & 0xFFFFFFFF, blk >> 32, op, stream, 8)
            w = j & 7
            assert o.prf_word(key_index, op, stream, j) == int(out[2 * w]) | (int(out[2 * w + 1]) << 32)


def test_streams_differ(seed):
    o = Oracle(seed)
    words = {o.prf_word(k, op, s, j) for k in range(5) for op in range(3) for s in range(3) for j in range(20)}
    assert len(words) == 5 * 3 * 3 * 20


def test_zero_sharings_cancel(seed):
    o = Oracle(seed)
    for e in [0, 1, 7, 8, 1000003]:
        a = o.zero_sharing(5, 0, e, boolean=False)
        assert (int(a[0]) + int(a[1]) + int(a[2])) & M64 == 0
        b = o.zero_sharing(5, 1, e, boolean=True)
        assert int(b[0]) ^ int(b[1]) ^ int(b[2]) == 0
        assert len({int(x) for x in a}) == 3
        # component j is the word under k_j minus the word under k_{j+1}: party j+1 holds both
        for j in range(3):
            wj, wn = o.prf_word(j, 5, 0, e), o.prf_word((j + 1) % 3, 5, 0, e)
            assert int(a[j]) == (wj - wn) & M64


def test_dealer_material_is_consistent(seed):
    o = Oracle(seed)
    betas = []
    for e in range(64):
        D = o.dealer(9, e)
        assert sum(int(x) for x in D["rA"]) & M64 == D["r"]
        assert int(D["rho"][0]) ^ int(D["rho"][1]) ^ int(D["rho"][2]) == D["r"]
        assert D["beta"] in (0, 1)
        assert int(D["bB"][0]) ^ int(D["bB"][1]) ^ int(D["bB"][2]) == D["beta"]
        assert sum(int(x) for x in D["bA"]) & M64 == D["beta"]
        assert D["r"] == o.prf_word(3, 9, 0, 8 * e)
        betas.append(D["beta"])
    assert 10 < sum(betas) < 54
