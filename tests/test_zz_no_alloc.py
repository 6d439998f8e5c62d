"""The array access that allocates nothing (gt_oaa_static, for callers that cannot call
hipMalloc) against the ordinary entry point gt_oaa: same shares bit for bit, on two calls
in a row, the second with a smaller input (the static scratch array keeps the first call's
contents), through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

M64 = (1 << 64) - 1


def test_static_array_access_equals_gt_oaa(seed):
    import torch
    assert torch.cuda.is_available()
    from oracle import Oracle
    from paper_2305_00645_amd import gtree
    gtree.load()
    ga, gb, o = gtree.GTree(seed), gtree.GTree(seed), Oracle(seed)
    rng = np.random.default_rng(12)
    # sizes that split the columns over several workgroups (the scratch is used), ragged tails
    for call, (w, n) in enumerate(((200, 5003), (37, 777))):
        Wp = rng.integers(0, M64, size=w, dtype=np.uint64)
        u = rng.integers(0, w + 2, size=n).astype(np.uint64)
        Wa, ua = ga.share_a(Wp), ga.share_a(u)
        Wb, ub = gb.share_a(Wp), gb.share_a(u)
        za = ga.oaa(Wa, ua)
        zb = gb.new(n)                                   # output allocated by the caller, before the call
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]       # the driver's view: sees hipMalloc by anyone
        gb.oaa_static(Wb, ub, zb)
        torch.cuda.synchronize()
        if call:                                         # (the first launch of a kernel may load its code)
            assert torch.cuda.mem_get_info()[0] == free_before
        assert np.array_equal(za.planes(), zb.planes()), (w, n)
        zo = o.oaa(o.share(Wp), o.share(u))
        assert np.array_equal(zb.components(), zo)
        want = np.array([Wp[int(i)] if int(i) < w else 0 for i in u], dtype=np.uint64)
        assert np.array_equal(gb.rec(zb), want)
        assert ga.op_counter() == gb.op_counter() == o.op_counter()
    assert np.array_equal(ga.stats()[1], gb.stats()[1]) and ga.stats()[0] == gb.stats()[0]
    assert np.array_equal(ga.wire_bits_dev(), gb.wire_bits_dev())
    # beyond the static array's size the call is refused, nothing is launched
    big = (1 << 18) + 1
    ub = gb.share_a(np.zeros(big, dtype=np.uint64))
    with pytest.raises(gtree.GtError) as e:
        gb.oaa_static(gb.share_a(np.arange(4, dtype=np.uint64)), ub, gb.new(big))
    assert e.value.code == gtree.GT_EINVAL
    ga.close(); gb.close()
