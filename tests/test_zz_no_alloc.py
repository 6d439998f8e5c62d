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


def test_static_array_access_replayed_from_a_hip_graph(seed):
    """gt_oaa_static is what a caller under HIP graph capture can use: captured once on the
    context's stream, replayed three times with eager work of the same program and device
    synchronisations in between, every replay must leave the shares of the eager call (same
    operation id, hence the same randomness) in the caller's output."""
    import torch
    from oracle import Oracle
    from paper_2305_00645_amd import gtree
    gtree.load()
    rng = np.random.default_rng(21)
    w, n = 150, 3001                                     # columns split over workgroups: the scratch array is used
    Wp = rng.integers(0, M64, size=w, dtype=np.uint64)
    u = rng.integers(0, w + 2, size=n).astype(np.uint64)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        g, e, o = gtree.GTree(seed, stream=st), gtree.GTree(seed, stream=st), Oracle(seed)
        Wg, ug, zg = g.share_a(Wp), g.share_a(u), g.new(n)
        We, ue = e.share_a(Wp), e.share_a(u)
        ze = e.oaa(We, ue)
        st.synchronize()
        want = ze.planes()
        assert np.array_equal(ze.components(), o.oaa(o.share(Wp), o.share(u)))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            g.oaa_static(Wg, ug, zg)
        for replay in range(3):
            zg.t.zero_()
            e.mult(We, We)                               # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(zg.planes(), want), replay
        del graph
        g.close(); e.close()
