#!/usr/bin/env python3
"""Benchmark of the GTree hot path on one MI355X.

A step is one pass of the whole hot path at the scale workload (C5 of the workload
list): the one-time products (a0), one full split-scoring level over 128 nodes
(a1-a7: partition, leaf one-hot, class counts, Gini division, arg-max, updates), the
label level (a8) and a depth-10 inference batch (b1-b5), all three parties on one GPU,
inputs resident in device memory.  `value` is split candidates scored per second of
the split-scoring level; the other parts are reported beside it.  One JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
LANE_OPS_PEAK = 256 * 4 * 16 * 2.4e9 / 1e12   # 32-bit vector ALU lane-ops, Tops/s: CUs x SIMDs x lanes x clock
# Algorithmic 32-bit ALU ops per equality test of a grid, three parties together.  A ChaCha8 block
# is 400 ops.  Dealer: 3 blocks per 8 tests (150: the daBits of the tests, offline material that the
# paper's timings exclude but that this simulation derives inside the kernel; the edaBit is one
# block per ROW of the grid, 400/w per test, left out) + 3 mask blocks per 8 tests (150: the zero
# sharings of the AND rounds, online) + protocol steps 3 x 50 on packed fields (online)
EQ_ALU_OPS_DEALER, EQ_ALU_OPS_ONLINE = 150, 300
EQ_ALU_OPS = EQ_ALU_OPS_DEALER + EQ_ALU_OPS_ONLINE
# HBM bytes per equality test of the three grid variants, from rocprofv3 FETCH_SIZE / WRITE_SIZE
# (table in profiles/pmc_traffic_micro.md): inner product against a shared array, against the
# sample's own row, leaf one-hot written as limb tiles
# (the one-launch inference reads every feature of an instance once per level: 10 levels x 48 B x 64
# features over 2687 tests per instance at C5)
EQ_HBM_BYTES = {"eqgrid": 7.4, "eqgrid_rows": 55.4, "eqgrid_store": 24.4, "infer": 15.1}
SHADER_CLOCK_MEASURED_GHZ = 2.1  # under the equality grid's load (profiles/pmc_sq_micro.md); the peak below uses the nominal 2.4


def paper_literal_ol_bytes(N, d, K, h, H, l=64):
    """Per-party bytes of the learning protocol of one level if it were run as printed in the paper
    (Sec. V-A cost formulas: equality test (2l-1) bits, array access (4l-1) bits per array element,
    hence 2l bits per element for the select step): array access over the whole tree array of
    2^H - 1 entries and over the d feature values for every sample, the leaf-flag equality grid, and
    the per-sample select over n_h counter arrays of (1+K) x 2d entries."""
    nh = 1 << h
    bits = 0
    if h > 0:
        bits += N * ((1 << H) - 1) * (4 * l - 1) + N * d * (4 * l - 1)
    bits += nh * (2 * l - 1) + N * nh * (2 * l - 1) + N * nh
    bits += N * nh * (1 + K) * 2 * d * 2 * l
    return bits / 8.0


def paper_shapes(np, torch, gtree, wl):
    """Timings on the two workloads shaped like the paper's headline experiments: C3 (census
    shape, 48,842 x 294 columns, depth 7) full training, and C4 (10^4 instances, depth-7 tree with
    thresholds) inference.  Median of 5 runs after one warm-up; context only, not `value`."""
    res = {}
    w = wl.c3_train()
    N, d, K, H = w["N"], w["d"], w["K"], w["H"]
    g = gtree.GTree(wl.PROTOCOL_SEED, tau=16, K=K)
    X, Y = g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1))
    g.train_create(X, Y, N, d, H)
    times, per_level = [], None
    for it in range(7):
        torch.cuda.synchronize(); t0 = time.perf_counter()
        g.train_reset(X, Y)
        lv = []
        for h in range(H):
            if it == 6:                          # last run only: wait after every level for the per-level figures
                torch.cuda.synchronize(); t1 = time.perf_counter()
            g.train_level(h)
            if it == 6:
                torch.cuda.synchronize(); lv.append(time.perf_counter() - t1)
        g.train_finish().close()
        torch.cuda.synchronize()
        if 0 < it < 6:
            times.append(time.perf_counter() - t0)
        per_level = lv
    tm = sorted(times)[len(times) // 2]
    ncand = sum((1 << h) * d for h in range(H))
    res["c3_train_depth7"] = {"samples": N, "columns": d, "seconds": tm, "candidates_per_s": ncand / tm,
                              "candidates_per_s_per_level": [(1 << h) * d / per_level[h] for h in range(H)]}
    # the same training with the heuristic by reconstruction (host analogue of the TEE-based protocol):
    # what is left when Gini division, arg-max and updates cost two rounds - the bound for steps a4-a7
    g.train_set_heuristic(True)
    times = []
    for it in range(6):
        torch.cuda.synchronize(); t0 = time.perf_counter()
        g.train_reset(X, Y)
        for h in range(H):
            g.train_level(h)
        g.train_finish().close()
        torch.cuda.synchronize()
        if it:
            times.append(time.perf_counter() - t0)
    res["c3_train_depth7"]["seconds_with_heuristic_by_reconstruction"] = sorted(times)[len(times) // 2]
    g.close(); del g, X, Y
    # the learning protocol run as the paper prints it (whole-tree scans, per-element SelectShare) beside
    # the fused one, on the small heart-data-shaped workload (267 x 22, depth 4): counted bytes and time
    w2 = wl.c2_train(H=4)
    lit = {}
    for mode in ("fused", "as_printed"):
        g = gtree.GTree(wl.PROTOCOL_SEED, tau=16, K=w2["K"])
        g.train_create(g.share_a(w2["X"].reshape(-1)), g.share_a(w2["Y"].reshape(-1)), w2["N"], w2["d"], w2["H"])
        g.train_set_literal(mode == "as_printed")
        g.stats_reset()
        torch.cuda.synchronize(); t0 = time.perf_counter()
        for h in range(w2["H"]):
            g.train_level(h)
        g.train_finish().close()
        torch.cuda.synchronize()
        rounds, wire, _ = g.stats()
        lit[mode] = {"seconds": time.perf_counter() - t0, "rounds": rounds, "bytes_sent_per_party": int(wire[0].sum()),
                     "payload_bits_counted_by_the_kernels_per_party": int(g.wire_bits_dev()[0].sum())}
        g.close()
    res["c2_train_depth4_learning_as_printed_vs_fused"] = lit
    wi = wl.c4_infer()
    g = gtree.GTree(wl.PROTOCOL_SEED, tau=16, K=2)
    tree = g.tree_import(g.share_a(wi["feat"]), g.share_a(wi["thr"]), g.share_a(wi["leaf"]), wi["H"])
    I = g.share_a(wi["I"].reshape(-1))
    times = []
    for it in range(6):
        torch.cuda.synchronize(); t0 = time.perf_counter()
        g.infer_batch(tree, I, wi["NI"], wi["d"])
        torch.cuda.synchronize()
        if it:
            times.append(time.perf_counter() - t0)
    tm = sorted(times)[len(times) // 2]
    res["c4_infer_depth7"] = {"instances": wi["NI"], "features": wi["d"], "mode": "threshold", "seconds": tm,
                              "instances_per_s": wi["NI"] / tm}
    tree.close(); g.close()
    torch.cuda.empty_cache()
    return res


def micro(args, np, torch, gtree, wl):
    """Calibration: gt_reconstruct_a on 2^27 words reads 3 GiB and writes 1 GiB exactly.
    Then one array access (equality grid with inner product) over 64 entries for
    --instances rows, one split-scoring level of the C5 recipe at --samples, and one
    depth-10 inference batch of --instances."""
    g = gtree.GTree(wl.PROTOCOL_SEED, tau=16, K=4)
    n = 1 << 27
    s = g.new(n)
    g.reconstruct_a(s)
    del s
    torch.cuda.empty_cache()
    NI = args.instances
    rng = np.random.default_rng(1)
    W = g.share_a(rng.integers(0, 1 << 20, size=64).astype(np.uint64))
    u = g.share_a(rng.integers(0, 64, size=NI).astype(np.uint64))
    g.oaa(W, u)
    N, d, K, h = args.samples, 64, 4, 7
    w = wl.c5_level(N=N, d=d, K=K, h=h)
    CW = d * K + K
    X, Y = g.share_a(w["X"].reshape(-1)), g.share_a(w["Y"].reshape(-1))
    st = [g.share_a(a) for a in (w["M"], w["Tprev"], w["F"], np.zeros((1 << h) * CW, dtype=np.uint64), w["gamma"].reshape(-1))]
    g.train_create(X, Y, N, d, h + 1)
    g.train_import(h, *st)
    g.train_level(h)
    torch.cuda.synchronize()
    del X, Y, st
    torch.cuda.empty_cache()
    # the one-launch inference on the C5 batch (depth 10, 64 binary features)
    wi = wl.c5_infer(NI=NI)
    tree = g.tree_import(g.share_a(wi["feat"]), None, g.share_a(wi["leaf"]), wi["H"])
    g.infer_batch(tree, g.share_a(wi["I"].reshape(-1)), NI, wi["d"])
    torch.cuda.synchronize()
    print(json.dumps({"micro": "done", "calibration_words": n, "oaa_rows": NI, "oaa_entries": 64, "level_samples": N,
                      "inference_instances": NI, "inference_depth": wi["H"]}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--samples", type=int, default=1000000, help="training samples (C5: 10^6)")
    ap.add_argument("--instances", type=int, default=1000000, help="inference batch (C5: 10^6)")
    ap.add_argument("--cpu-samples", type=int, default=1000000, help="oracle samples for cpu_baseline (0 = skip)")
    ap.add_argument("--cpu-single-samples", type=int, default=62500,
                    help="samples of the single-threaded oracle timing (0 = skip)")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--no-paper-shapes", action="store_true", help="skip the C3 training / C4 inference timings")
    ap.add_argument("--only-paper-shapes", action="store_true",
                    help="only the C3 training / C4 inference timings (for a kernel trace of those workloads)")
    ap.add_argument("--micro", action="store_true",
                    help="one launch of each hot kernel plus a calibration kernel of known traffic, for rocprofv3 --pmc")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build simulates the three parties on ONE GPU; --gpus %d is not supported "
              "(no collectives, no second device)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2305_00645_amd import gtree, workloads as wl
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    gtree.load()

    if args.micro:
        return micro(args, np, torch, gtree, wl)
    if args.only_paper_shapes:
        print(json.dumps({"paper_shape_workloads": paper_shapes(np, torch, gtree, wl)}))
        return
    N, NI, d, K, h, Hinf = args.samples, args.instances, 64, 4, 7, 10
    H = h + 1
    CW = d * K + K
    w = wl.c5_level(N=N, d=d, K=K, h=h)
    wi = wl.c5_infer(NI=NI, d=d, H=Hinf, K=K)

    def setup(profile):
        g = gtree.GTree(wl.PROTOCOL_SEED, tau=16, K=K, profile=profile)
        st = dict(
            X=g.share_a(w["X"].reshape(-1)), Y=g.share_a(w["Y"].reshape(-1)),
            M=g.share_a(w["M"]), Tprev=g.share_a(w["Tprev"]), F=g.share_a(w["F"]),
            C=g.share_a(np.zeros((1 << h) * CW, dtype=np.uint64)), gamma=g.share_a(w["gamma"].reshape(-1)),
            I=g.share_a(wi["I"].reshape(-1)),
        )
        st["tree"] = g.tree_import(g.share_a(wi["feat"]), None, g.share_a(wi["leaf"]), Hinf)
        g.train_create(st["X"], st["Y"], N, d, H)
        return g, st

    def step(g, st, t, pc=None):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.train_reset(st["X"], st["Y"])                                   # a0
        torch.cuda.synchronize(); t1 = time.perf_counter()
        g.train_import(h, st["M"], st["Tprev"], st["F"], st["C"], st["gamma"])   # set-up of the level's state (copies)
        torch.cuda.synchronize(); t1b = time.perf_counter()
        c0 = g.prof()["count"][0] if pc is not None else 0.0
        g.train_level(h)                                                  # a1-a7
        torch.cuda.synchronize(); t2 = time.perf_counter()
        if pc is not None:                                                # the level's own contraction, apart from the label level's
            pc["level_count_ms"] = pc.get("level_count_ms", 0.0) + g.prof()["count"][0] - c0
        tree = g.train_finish()                                           # a1, a2, a8 at level H
        torch.cuda.synchronize(); t3 = time.perf_counter()
        R = g.infer_batch(st["tree"], st["I"], NI, d)                     # b1-b5
        torch.cuda.synchronize(); t4 = time.perf_counter()
        tree.close()
        if t is not None:
            t["a0"] += t1 - t0; t["import"] += t1b - t1; t["level"] += t2 - t1b; t["finish"] += t3 - t2; t["infer"] += t4 - t3
        return R

    g, st = setup(False)
    for _ in range(args.warmup):
        step(g, st, None)
    t = dict(a0=0.0, level=0.0, finish=0.0, infer=0.0)
    t["import"] = 0.0
    torch.cuda.synchronize()
    T0 = time.perf_counter()
    for _ in range(args.steps):
        R = step(g, st, t)
    torch.cuda.synchronize()
    total = time.perf_counter() - T0
    k = args.steps
    ms = {a: 1e3 * b / k for a, b in t.items()}
    # message volume of one split-scoring level (counted by the library) beside the unfused protocol
    lvl_msgs = None
    if not args.no_roofline:           # left out of runs made for a kernel trace: it repeats the level once more
        g.train_import(h, st["M"], st["Tprev"], st["F"], st["C"], st["gamma"])
        g.stats_reset()
        g.train_level(h)
        lvl_rounds, lvl_wire, _ = g.stats()
        lvl_msgs = {"rounds": lvl_rounds, "bytes_sent_per_party": int(lvl_wire[0].sum()),
                    "payload_bits_counted_by_the_kernels_per_party": int(g.wire_bits_dev()[0].sum()),
                    "paper_literal_learning_bytes_per_party": paper_literal_ol_bytes(N, d, K, h, H),
                    "note": "the library fuses select-and-accumulate into inner products with one reshare per "
                            "output; the second figure prices the learning protocol as printed (analytic)"}
    ncand = (1 << h) * d
    value = ncand / (ms["level"] / 1e3)
    # sanity: predictions equal plaintext traversal on a sample of instances
    pred = g.rec(R)[:2000].astype(np.int64)
    Tt = np.concatenate([wi["feat"], wi["leaf"]]).astype(np.int64)
    idx = np.zeros(2000, dtype=np.int64)
    for _ in range(Hinf):
        idx = 2 * idx + 1 + wi["I"][np.arange(2000), Tt[idx]].astype(np.int64)
    assert np.array_equal(pred, Tt[idx]), "inference result differs from plaintext traversal"
    rounds, wire, _ = g.stats()
    g.close(); del g, st
    torch.cuda.empty_cache()

    out = {
        "metric": "secure split candidates scored/s per level", "value": value, "unit": "candidates/s",
        "n_gpus": 1, "steps": k, "warmup": args.warmup, "ms_per_step": 1e3 * total / k,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "C5 scale: %d samples x %d binary columns, %d classes, one split-scoring level over %d "
                               "nodes (%d candidates) + depth-%d inference on %d instances; 3 parties on 1 GPU, Z_2^64, tau=16"
                               % (N, d, K, 1 << h, ncand, Hinf, NI),
                   "value_from": "candidates / time of gt_train_level(h=%d)" % h},
        "breakdown_ms": {"a0_products": ms["a0"], "state_import_copies": ms["import"], "a1_a7_level": ms["level"],
                         "a1_a2_a8_label_level": ms["finish"], "b1_b5_inference": ms["infer"]},
        "inference_instances_per_s": NI / (ms["infer"] / 1e3), "inference_depth": Hinf,
        "level_messages": lvl_msgs,
    }

    if not args.no_roofline:
        # second timed region with a pair of HIP events around every kernel launch
        g, st = setup(True)
        step(g, st, None)
        g.stats_reset()
        pc = {}
        for _ in range(k):
            step(g, st, None, pc)
        prof = g.prof()
        g.close(); del g, st
        torch.cuda.empty_cache()
        # equality tests per step and kernel: array access over a shared array (partition over the tree
        # level), over the sample's own row (feature fetch), leaf one-hot (level and label level), and
        # the one-launch inference (node lookups, feature fetches, labels of all levels)
        n_var = {
            "eqgrid": N * (1 << (h - 1)) + N * (1 << h),
            "eqgrid_rows": N * d + N * d,
            "eqgrid_store": N * (1 << h) + N * (1 << (h + 1)),
            "infer": NI * ((1 << Hinf) - 1 + Hinf * d + (1 << Hinf)),
        }
        n_eq = sum(n_var.values())
        eq_ms = sum(prof[c][0] for c in n_var)
        eq_l = sum(prof[c][1] for c in n_var)
        cnt_ms, cnt_l = prof["count"]
        macs_level, macs_label = 6 * N * (1 << h) * CW, 6 * N * (1 << (h + 1)) * K   # ring MACs, all parties
        lvl_cnt_ms = pc["level_count_ms"] / k
        lbl_cnt_ms = max(cnt_ms / k - lvl_cnt_ms, 1e-9)
        lbl_bytes = 8.0 * N * (3 * (1 << (h + 1)) + 6 * K)            # L once per component, the K columns (own+next, own) per party
        eq_bytes_step = sum(EQ_HBM_BYTES[c] * n_var[c] for c in n_var)
        per_variant = {c: {"tests_per_step": n_var[c], "ms_per_step": prof[c][0] / k, "launches_per_step": prof[c][1] // k,
                           "tests_per_s": n_var[c] * k / (prof[c][0] / 1e3) if prof[c][0] else None,
                           "hbm_bytes_per_test": EQ_HBM_BYTES[c],
                           "hbm_GBps": EQ_HBM_BYTES[c] * n_var[c] * k / (prof[c][0] / 1e3) / 1e9 if prof[c][0] else None}
                       for c in n_var}
        kern = {
            "eqgrid": {"bound": "alu", "achieved": EQ_ALU_OPS * n_eq * k / (eq_ms / 1e3) / 1e12, "peak": LANE_OPS_PEAK,
                       "unit": "Tops/s", "traffic": eq_bytes_step * k / max(eq_l, 1),
                       "note": "the equality-test kernels together (three grid variants of training and the one-launch inference: most of the step); %d 32-bit ALU ops per "
                               "test for the three parties, of which %d are the dealer's PRF blocks (the daBits, offline material of the test: "
                               "the paper's timings exclude its generation, this simulation derives it in the kernel) and %d are "
                               "online work (mask words 150, protocol 150): counting online ops only the figure is %.2f of the "
                               "peak; peak = 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz nominal (the shader clock under this load "
                               "reads %.1f GHz); traffic = HBM bytes per launch = per-variant counter bytes per test "
                               "(profiles/pmc_traffic_micro.md) x this run's tests per variant; the >=50%% HBM target of the "
                               "workload description is not met and cannot be by this kernel: its messages stay in LDS and it "
                               "is bound by the PRF (VALU issue share 0.77-0.83, profiles/pmc_sq_micro.md), see eqgrid_hbm_view"
                               % (EQ_ALU_OPS, EQ_ALU_OPS_DEALER, EQ_ALU_OPS_ONLINE,
                                  EQ_ALU_OPS_ONLINE * n_eq * k / (eq_ms / 1e3) / 1e12 / LANE_OPS_PEAK, SHADER_CLOCK_MEASURED_GHZ),
                       "avg_launch_ms": eq_ms / max(eq_l, 1), "launches_per_step": eq_l // k,
                       "eq_tests_per_s": n_eq * k / (eq_ms / 1e3), "variants": per_variant},
            "eqgrid_hbm_view": {"bound": "hbm", "achieved": eq_bytes_step * k / (eq_ms / 1e3) / 1e9,
                                "peak": HBM_PEAK_GBS, "unit": "GB/s", "traffic": eq_bytes_step * k / max(eq_l, 1),
                                "note": "per-variant HBM bytes per test x tests/s: the protocol messages (24 B per test: 63 + 1 bits from each party) pass "
                                        "through LDS, HBM sees the operands and results only, so this is not the binding limit"},
            # the two launches of the contraction have different bounds: the level's (128 nodes x 260 columns)
            # is matrix-core work, the label level's (256 nodes x 4 class columns) streams L once
            "count": {"bound": "mfma", "achieved": 72.0 * macs_level / (lvl_cnt_ms / 1e3) / 1e12, "peak": 5000.0,
                      "unit": "TOP/s", "traffic": 19.0e9,
                      "note": "the contraction of the split-scoring level: ring MAC = 36 int8 limb products on the matrix "
                              "cores = 72 int8 ops; int8 dense peak 5.0 POP/s; %d ring MACs (every party's two products "
                              "are computed; the leaf one-hot is stored once per component, the copy that both of its "
                              "holders read); traffic: FETCH_SIZE + WRITE_SIZE of this launch in profiles/pmc_traffic_micro.md "
                              "(compulsory 15.6 GB)" % macs_level,
                      "avg_launch_ms": lvl_cnt_ms, "launches_per_step": 1},
            "count_label_level": {"bound": "hbm", "achieved": lbl_bytes / (lbl_cnt_ms / 1e3) / 1e9, "peak": HBM_PEAK_GBS,
                                  "unit": "GB/s", "traffic": lbl_bytes,
                                  "note": "class totals of the label level (%d nodes x %d class columns on 16-wide tiles): "
                                          "the three components of L and the class columns are read once "
                                          "(algorithmic bytes); %d ring MACs = %.2f of the int8 peak"
                                          % (1 << (h + 1), K, macs_label, 72.0 * macs_label / (lbl_cnt_ms / 1e3) / 1e12 / 5000.0),
                                  "avg_launch_ms": lbl_cnt_ms, "launches_per_step": 1},
        }
        for v in kern.values():
            v["frac"] = v["achieved"] / v["peak"]
        cls_ms = {c: prof[c][0] / k for c in prof}
        dom = "eqgrid" if eq_ms >= max(prof[c][0] for c in prof if c not in n_var) else max(
            (c for c in prof if c not in n_var), key=lambda c: prof[c][0])
        dom = dom if dom in kern else "eqgrid"
        # what a plain streaming kernel of the library reaches on this machine, beside the published 8 TB/s:
        # gt_reconstruct_a reads three words and writes one per element
        gs = gtree.GTree(wl.PROTOCOL_SEED, tau=16, K=K)
        sv = gs.new(1 << 26)
        pv = torch.zeros(1 << 26, dtype=torch.int64, device="cuda:0")
        gs.L.gt_reconstruct_a(gs.ctx, gtree._ref(sv), pv.data_ptr(), sv.n)
        torch.cuda.synchronize(); c0 = time.perf_counter()
        for _ in range(10):
            gs.L.gt_reconstruct_a(gs.ctx, gtree._ref(sv), pv.data_ptr(), sv.n)
        torch.cuda.synchronize()
        stream_gbs = 10 * 4 * 8 * (1 << 26) / (time.perf_counter() - c0) / 1e9
        gs.close(); del sv, pv
        torch.cuda.empty_cache()
        out["measured_stream_GBps"] = {"value": stream_gbs, "frac_of_hbm_peak": stream_gbs / HBM_PEAK_GBS,
                                       "kernel": "gt_reconstruct_a on 2^26 words (3 reads + 1 write per word), 10 launches"}
        out["roofline"] = dict(kern[dom], kernel=dom)
        out["kernel_classes_ms_per_step"] = cls_ms
        out["roofline_other"] = {c: v for c, v in kern.items() if c != dom}

    if not args.no_paper_shapes:
        out["paper_shape_workloads"] = paper_shapes(np, torch, gtree, wl)
        # the second half of the metric's name: 10^4 instances through a depth-7 tree with thresholds
        out["depth7_inference_instances_per_s"] = out["paper_shape_workloads"]["c4_infer_depth7"]["instances_per_s"]

    if args.cpu_samples > 0:
        from oracle import Oracle, orc

        def oracle_level(Ns, threads):
            ws = wl.c5_level(N=Ns, d=d, K=K, h=h)
            if threads:
                orc.set_threads(threads)
            o = Oracle(wl.PROTOCOL_SEED, tau=16, K=K)
            xs, ys = o.share(ws["X"].reshape(-1)), o.share(ws["Y"].reshape(-1))
            sto = [o.share(a) for a in (ws["M"], ws["Tprev"], ws["F"], np.zeros((1 << h) * CW, dtype=np.uint64), ws["gamma"].reshape(-1))]
            o.train_create(xs, ys, Ns, d, H)
            o.train_import(h, *sto)
            c0 = time.perf_counter()
            o.train_level(h)
            dt = time.perf_counter() - c0
            o.close()
            return dt

        all_threads = orc.get_threads()
        Ns = min(args.cpu_samples, N)
        cpu_s = oracle_level(Ns, 0)
        full = Ns == N
        out["cpu_baseline"] = {
            "value": ncand / (cpu_s * N / Ns), "unit": "candidates/s", "cores": all_threads, "kind": "oracle",
            "sample": ("full size: the same level on all %d samples took %.2f s on the host" % (N, cpu_s)) if full else
                      ("the same level on %d of the %d samples took %.2f s on the host; scaled linearly in the sample count" % (Ns, N, cpu_s))}
        if args.cpu_single_samples > 0:
            N1 = min(args.cpu_single_samples, N)
            s1 = oracle_level(N1, 1)
            orc.set_threads(all_threads)
            out["cpu_baseline"]["single_thread"] = {
                "value": ncand / (s1 * N / N1), "unit": "candidates/s", "cores": 1,
                "sample": "the same level on %d of the %d samples took %.2f s on one thread; scaled linearly in the sample "
                          "count (the level's work is linear in the samples: per-sample equality tests and inner products)" % (N1, N, s1)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
