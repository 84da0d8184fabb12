"""GPU parity at the full benchmark sizes, in the launch configuration the
benchmark times (device-built CSR, row plan, rows on 128-byte lines, every chunk
width of the sweeps): the CSR is compared bit for bit with the CPU checker's and
the aggregation on EVERY destination row (attention: on 20,000 sampled rows)."""
import sys

import numpy as np
import pytest
import torch

import oracle
import workloads as W
from test_gpu_parity import assert_bits, assert_close, dev, host, say

pytestmark = pytest.mark.gpu


def sample_rows(rp, n=96, seed=0):
    deg = np.diff(rp)
    order = np.argsort(-deg, kind="stable")
    rng = np.random.default_rng(seed)
    pick = list(order[:8]) + list(order[-4:]) + list(order[len(order) // 2 - 4:len(order) // 2 + 4])
    pick += list(rng.choice(len(deg), size=n - len(pick), replace=False))
    return np.unique(np.array(pick, np.int64))


def close_all(got, ref, bf16=False, what=""):
    """The parity bar on every element of a large matrix, in row blocks (keeps the fp64 temporaries small)."""
    rtol = 1e-2 if bf16 else 1e-5
    for r0 in range(0, got.shape[0], 1 << 16):
        a = got[r0:r0 + (1 << 16)].astype(np.float64)
        b = ref[r0:r0 + (1 << 16)].astype(np.float64)
        ok = np.abs(a - b) <= 1e-6 + rtol * np.abs(b)
        if not ok.all():
            i = tuple(np.argwhere(~ok)[0])
            raise AssertionError("%s: %d elements off in rows %d.., first at row %d col %d: got %r want %r" %
                                 (what, int((~ok).sum()), r0, r0 + i[0], i[1], a[i], b[i]))


def test_config4_full_size_gcn_and_mean():
    """Every row of the dense benchmark graph against the checker, at every chunk width of the configuration's
    sweep (8, 16, 32, 64, all, and the library's own choice), in the benchmark's layout (rows on lines)."""
    import paper_2104_03058_amd as g
    N, src, dst = W.graph("c4")
    say("c4 full: N", N, "E", len(src))
    flags = oracle.SELF_LOOPS | oracle.NORM_SYM
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags, want_w=True, threads=16)
    say("c4 full: checker CSR done, nnz", len(ci), "max deg", int(np.diff(rp).max()))
    d_rp, d_ci, d_w, _ = g.gnnagg_build_csr(N, dev(src), dev(dst), flags, want_w=True)
    assert np.array_equal(host(d_rp), rp) and np.array_equal(host(d_ci), ci)
    assert_bits(host(d_w), w, "edge_w")
    say("c4 full: device CSR matches bit for bit")
    X = W.normal_f32((N, 602), seed=13)
    d_X = dev(X)
    plan = g.gnnagg_plan_rows(d_rp)
    Xp = g.pitched_empty(N, 602, torch.float32)
    Xp.copy_(d_X)
    assert g.gnnagg_auto_f_chunk(N, 602, g.F32, int(Xp.stride(0)), plan) == 32
    assert g.gnnagg_auto_f_chunk(N, 602, g.F32, 602, plan) == 602
    outp = g.pitched_empty(N, 602, torch.float32)
    # the blocked call as the benchmark's headline runs it: as many source blocks as the library recommends
    B = g.gnnagg_auto_source_blocks(g.WSUM, N, 602, g.F32, int(Xp.stride(0)), plan)
    assert B == 2 and g.gnnagg_auto_source_blocks(g.WSUM, N, 602, g.F32, 602, plan) == 1
    assert g.gnnagg_auto_source_blocks(g.MEAN, N, 602, g.F32, int(Xp.stride(0)), plan) == 4
    blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, B)
    ws = torch.empty(g.gnnagg_aggregate_blocked_workspace_bytes(N, 602, blocks), dtype=torch.uint8, device="cuda")
    ref = oracle.aggregate(oracle.WSUM, rp, ci, w, X, threads=16)
    say("c4 full: checker weighted sum done (all rows)")
    for fc in (g.F_CHUNK_AUTO, 32, 0):
        say("c4 full: wsum over", B, "source blocks, f_chunk", fc)
        outp.fill_(float("nan"))
        g.gnnagg_aggregate_blocked(g.WSUM, d_rp, d_ci, d_w, Xp, blocks, outp, fc, workspace=ws)
        close_all(host(outp), ref, what="c4 wsum blocked fc=%d" % fc)
    for fc in (8, 16, 32, 64, 0, g.F_CHUNK_AUTO):
        say("c4 full: wsum, rows on lines, f_chunk", fc)
        outp.fill_(float("nan"))
        g.gnnagg_aggregate(g.WSUM, d_rp, d_ci, d_w, Xp, outp, fc, plan)
        close_all(host(outp), ref, what="c4 wsum pitched fc=%d" % fc)
    for fc in (0, 64):
        say("c4 full: wsum, contiguous rows, f_chunk", fc)
        out = g.gnnagg_aggregate(g.WSUM, d_rp, d_ci, d_w, d_X, None, fc, plan)
        close_all(host(out), ref, what="c4 wsum fc=%d" % fc)
        del out
    # the same aggregation with the weights in factored form (s_j into the rows, a plain sum, s_i at the store),
    # over as many source blocks as the library recommends for it: every row against the per-edge weighted sum
    s = g.gnnagg_gcn_factors(d_rp)
    assert_bits(host(s), oracle.gcn_factors(rp), "gcn factors")
    Xs = g.gnnagg_scale_rows(Xp, s)
    sample = sample_rows(rp)
    assert_bits(host(Xs[torch.from_numpy(sample).cuda()]), oracle.scale_rows(X[sample], host(s)[sample]), "scaled rows")
    Bf = g.gnnagg_auto_source_blocks(g.SUM_SCALED, N, 602, g.F32, int(Xs.stride(0)), plan)
    assert Bf == 4
    blocks_f = g.gnnagg_plan_source_blocks(d_rp, d_ci, Bf)
    say("c4 full: factored weights over", Bf, "source blocks")
    outp.fill_(float("nan"))
    g.gnnagg_aggregate_blocked(g.SUM_SCALED, d_rp, d_ci, s, Xs, blocks_f, outp, g.F_CHUNK_AUTO)
    close_all(host(outp), ref, what="c4 factored gcn blocked")
    outp.fill_(float("nan"))
    g.gnnagg_aggregate(g.SUM_SCALED, d_rp, d_ci, s, Xs, outp, g.F_CHUNK_AUTO, plan)
    close_all(host(outp), ref, what="c4 factored gcn")
    del Xs, blocks_f, s
    ref = oracle.aggregate(oracle.MEAN, rp, ci, None, X, threads=16)
    for fc in (8, 16, 32, 64, 0, g.F_CHUNK_AUTO):
        say("c4 full: mean, rows on lines, f_chunk", fc)
        outp.fill_(float("nan"))
        g.gnnagg_aggregate(g.MEAN, d_rp, d_ci, None, Xp, outp, fc, plan)
        close_all(host(outp), ref, what="c4 mean pitched fc=%d" % fc)
    # sum, mean and max get 4 blocks on this graph (no stream of edge weights that blocks do nothing for)
    del blocks, ws
    B = g.gnnagg_auto_source_blocks(g.MEAN, N, 602, g.F32, int(Xp.stride(0)), plan)
    blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, B)
    ws = torch.empty(g.gnnagg_aggregate_blocked_workspace_bytes(N, 602, blocks), dtype=torch.uint8, device="cuda")
    say("c4 full: mean over", B, "source blocks")
    outp.fill_(float("nan"))
    g.gnnagg_aggregate_blocked(g.MEAN, d_rp, d_ci, None, Xp, blocks, outp, g.F_CHUNK_AUTO, workspace=ws)
    close_all(host(outp), ref, what="c4 mean blocked")
    ref = oracle.aggregate(oracle.MAX, rp, ci, None, X, threads=16)
    for fc in (32, 0, g.F_CHUNK_AUTO):
        say("c4 full: max, rows on lines, f_chunk", fc)
        outp.fill_(float("nan"))
        g.gnnagg_aggregate(g.MAX, d_rp, d_ci, None, Xp, outp, fc, plan)
        assert_bits(host(outp), ref, "c4 max pitched fc=%d" % fc)
    say("c4 full: max over", B, "source blocks")
    outp.fill_(float("nan"))
    g.gnnagg_aggregate_blocked(g.MAX, d_rp, d_ci, None, Xp, blocks, outp, g.F_CHUNK_AUTO, workspace=ws)
    assert_bits(host(outp), ref, "c4 max blocked")
    del Xp, outp, ref, blocks, ws
    # property that holds at any size: the all-ones matrix aggregates to the row degree, exactly
    ones = torch.ones((N, 8), dtype=torch.float32, device="cuda")
    deg = host(g.gnnagg_aggregate(g.SUM, d_rp, d_ci, None, ones, None, 0, plan))
    assert np.array_equal(deg[:, 0], np.diff(rp).astype(np.float32)) and np.array_equal(deg[:, 7], deg[:, 0])


@pytest.mark.parametrize("F", [100, 32, 16])
def test_config5_full_size_bf16_sum_and_max(F):
    """Every row of the sparse benchmark graph, in the benchmark's layout and with contiguous rows."""
    import paper_2104_03058_amd as g
    N, src, dst = W.graph("c5")
    say("c5 full: N", N, "E", len(src), "F", F)
    rp, ci, _, _ = oracle.build_csr(N, src, dst, 0, threads=16)
    d_rp, d_ci, _, _ = g.gnnagg_build_csr(N, dev(src), dev(dst), 0)
    assert np.array_equal(host(d_rp), rp) and np.array_equal(host(d_ci), ci)
    X = W.normal_bf16((N, F), seed=14 + F)
    d_X = dev(X)
    Xp = g.pitched_empty(N, F, torch.bfloat16)
    Xp.copy_(d_X)
    plan = g.gnnagg_plan_rows(d_rp)
    for name, gop, rop in (("sum", g.SUM, oracle.SUM), ("max", g.MAX, oracle.MAX)):
        ref = oracle.aggregate(rop, rp, ci, None, X, threads=16)
        for xin, layout in ((Xp, "rows on lines"), (d_X, "contiguous")):
            say("c5 full:", name, layout)
            out = g.gnnagg_aggregate(gop, d_rp, d_ci, None, xin, None, g.F_CHUNK_AUTO, plan)
            if name == "max":
                assert_bits(host(out), ref, "c5 max F=%d %s" % (F, layout))
            else:
                close_all(host(out), ref, bf16=True, what="c5 sum F=%d %s" % (F, layout))
            del out
    if F < 100:
        # the rows in popularity order (what the benchmark's "-ranked" workloads run): the same bits
        rank, ranked = g.gnnagg_rank_sources(N, d_ci)
        Xr = torch.empty_like(d_X)
        Xr[rank.long()] = d_X
        a = g.gnnagg_aggregate(g.SUM, d_rp, ranked, None, Xr, None, 0, plan)
        b = g.gnnagg_aggregate(g.SUM, d_rp, d_ci, None, d_X, None, 0, plan)
        assert_bits(host(a), host(b), "c5 ranked sum F=%d" % F)


@pytest.mark.parametrize("F", [8, 16, 32])
def test_dense_small_graph_hidden_widths(F):
    """The paper's regime (Section III): Combination first, Aggregation at hidden width 8/16/32, on the graph
    shaped like its third dataset (132,534 vertices, average degree 597); every row."""
    import paper_2104_03058_amd as g
    N, src, dst = W.graph("c6")
    say("c6 full: N", N, "E", len(src), "F", F)
    flags = oracle.SELF_LOOPS | oracle.NORM_SYM
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags, want_w=True, threads=16)
    d_rp, d_ci, d_w, _ = g.gnnagg_build_csr(N, dev(src), dev(dst), flags, want_w=True)
    assert np.array_equal(host(d_rp), rp) and np.array_equal(host(d_ci), ci)
    assert_bits(host(d_w), w, "edge_w")
    X = W.normal_f32((N, F), seed=40 + F)
    d_X = dev(X)
    plan = g.gnnagg_plan_rows(d_rp)
    for name, gop, rop, fc in (("wsum", g.WSUM, oracle.WSUM, 0), ("wsum", g.WSUM, oracle.WSUM, 4),
                               ("mean", g.MEAN, oracle.MEAN, 0), ("max", g.MAX, oracle.MAX, 0)):
        out = g.gnnagg_aggregate(gop, d_rp, d_ci, d_w, d_X, None, fc, plan)
        ref = oracle.aggregate(rop, rp, ci, w, X, threads=16)
        if name == "max":
            assert_bits(host(out), ref, "c6 max F=%d" % F)
        else:
            close_all(host(out), ref, what="c6 %s F=%d fc=%d" % (name, F, fc))


def test_dense_small_graph_at_input_width_over_source_blocks():
    """The third graph shape at the dense graph's input width (602 fp32 columns), plain and over the source blocks
    the library recommends - the shape blocks gain most on; every row of both against the checker."""
    import paper_2104_03058_amd as g
    N, src, dst = W.graph("c6")
    flags = oracle.SELF_LOOPS | oracle.NORM_SYM
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags, want_w=True, threads=16)
    d_rp, d_ci, d_w, _ = g.gnnagg_build_csr(N, dev(src), dev(dst), flags, want_w=True)
    X = W.normal_f32((N, 602), seed=46)
    Xp = g.pitched_empty(N, 602, torch.float32)
    Xp.copy_(dev(X))
    plan = g.gnnagg_plan_rows(d_rp)
    B = g.gnnagg_auto_source_blocks(g.WSUM, N, 602, g.F32, int(Xp.stride(0)), plan)
    assert B == 4
    blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, B)
    ref = oracle.aggregate(oracle.WSUM, rp, ci, w, X, threads=16)
    say("c6 F=602: plain")
    out = g.gnnagg_aggregate(g.WSUM, d_rp, d_ci, d_w, Xp, g.pitched_empty(N, 602, torch.float32), g.F_CHUNK_AUTO, plan)
    close_all(host(out), ref, what="c6 wsum F=602 plain")
    say("c6 F=602: over", B, "source blocks")
    out.fill_(float("nan"))
    g.gnnagg_aggregate_blocked(g.WSUM, d_rp, d_ci, d_w, Xp, blocks, out, g.F_CHUNK_AUTO)
    close_all(host(out), ref, what="c6 wsum F=602 blocked")
    say("c6 F=602: weights in factored form, in place, over the same blocks")
    fac = g.gnnagg_gcn_factors(d_rp)
    g.gnnagg_scale_rows(Xp, fac, Xp)
    out.fill_(float("nan"))
    g.gnnagg_aggregate_blocked(g.SUM_SCALED, d_rp, d_ci, fac, Xp, blocks, out, g.F_CHUNK_AUTO)
    close_all(host(out), ref, what="c6 factored gcn F=602 blocked")


def test_config4_graph_attention_full_size():
    """Attention at the size of the paper's largest graph (its GAT sweep, Section III), 8 heads x 8 channels:
    20,000 destination rows (the checker forms every exponential of a row once per column)."""
    import paper_2104_03058_amd as g
    N, src, dst = W.graph("c4")
    rp, ci, _, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS, threads=16)
    d_rp, d_ci, _, _ = g.gnnagg_build_csr(N, dev(src), dev(dst), oracle.SELF_LOOPS)
    assert np.array_equal(host(d_rp), rp) and np.array_equal(host(d_ci), ci)
    H = W.normal_f32((N, 8, 8), seed=50)
    a_s = W.normal_f32((8, 8), seed=51, std=0.1)
    a_d = W.normal_f32((8, 8), seed=52, std=0.1)
    plan = g.gnnagg_plan_rows(d_rp)
    rows = sample_rows(rp, n=20000)
    idx = torch.from_numpy(rows).cuda()
    ref = oracle.gat_attention_rows(rows, rp, ci, H, a_s, a_d, 0.2, threads=16)
    outs = {}
    for fc in (0, 8):
        say("c4 gat full: f_chunk", fc)
        _, outs[fc] = g.gnnagg_gat_attention(d_rp, d_ci, dev(H), dev(a_s), dev(a_d), 0.2, False, True, fc, plan)
        assert_close(host(outs[fc][idx]), ref, what="c4 gat fc=%d" % fc)
    # with alpha the score arrays are used instead of the in-register scores: the same output bits
    alpha, out2 = g.gnnagg_gat_attention(d_rp, d_ci, dev(H), dev(a_s), dev(a_d), 0.2, True, True, 0, plan)
    assert_bits(host(out2), host(outs[0]), "c4 gat with and without alpha")
    sums = host(torch.zeros(N, 8, device="cuda").index_add_(
        0, torch.repeat_interleave(torch.arange(N, device="cuda"), d_rp[1:] - d_rp[:-1]), alpha))
    assert np.all(np.abs(sums - 1.0) < 1e-4)  # the weights of every destination add up to 1, per head


def test_automatic_chunk_width_on_a_feature_matrix_beyond_the_cache():
    """X = 2.4 M x 128 fp32 (1.25 GB) is past the point where one chunk is fastest: GNNAGG_F_CHUNK_AUTO
    picks 32-column chunks; the result must equal the unchunked one (sums here are fp64-accumulated, and
    each element sees the same operands in the same order whatever the chunk width)."""
    import paper_2104_03058_amd as g
    N, src, dst = W.graph("c5")
    F = 128
    assert g.gnnagg_auto_f_chunk(N, F, g.F32) == 32  # 1.25 GB of X: the capacity rule
    rp, ci, _, _ = oracle.build_csr(N, src, dst, 0, threads=16)
    d_rp, d_ci = dev(rp), dev(ci)
    X = W.normal_f32((N, F), seed=60)
    d_X = dev(X)
    plan = g.gnnagg_plan_rows(d_rp)
    rows = sample_rows(rp, n=256)
    idx = torch.from_numpy(rows).cuda()
    ref = oracle.aggregate_rows(oracle.MEAN, rows, rp, ci, None, X, threads=16)
    out_auto = g.gnnagg_aggregate(g.MEAN, d_rp, d_ci, None, d_X, None, g.F_CHUNK_AUTO, plan)
    assert_close(host(out_auto[idx]), ref, what="auto chunk mean")
    out_one = g.gnnagg_aggregate(g.MEAN, d_rp, d_ci, None, d_X, None, 0, plan)
    assert_close(host(out_one[idx]), ref, what="one chunk mean")
    mx_auto = g.gnnagg_aggregate(g.MAX, d_rp, d_ci, None, d_X, None, g.F_CHUNK_AUTO, plan)
    mx_one = g.gnnagg_aggregate(g.MAX, d_rp, d_ci, None, d_X, None, 0, plan)
    assert torch.equal(mx_auto, mx_one)


def test_combination_at_the_dense_graph_size_and_the_layer_built_from_it():
    """Combination at the benchmark's size (602 -> 32 on 232,965 vertices) on sampled rows, then the
    GCN layer in the order the benchmark times (Combination first, aggregation at width 32): sampled
    rows against the checker run in the other order (aggregate at width 602, then project)."""
    import paper_2104_03058_amd as g
    N, src, dst = W.graph("c4")
    X = W.normal_f32((N, 602), seed=13)
    Wt = W.normal_f32((602, 32), seed=16, std=0.05)
    b = W.normal_f32((32,), seed=17, std=0.1)
    d_X = dev(X)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, 1, 127, 128, N - 129, N - 128, N - 1],
                                     rng.choice(N, size=500, replace=False)])).astype(np.int64)
    say("c4 full: combination")
    hid = g.gnnagg_combine(d_X, dev(Wt), dev(b), True)
    assert_close(host(hid[torch.from_numpy(rows).cuda()]), oracle.combine(X[rows], Wt, b, True), what="combine relu")
    hid = g.gnnagg_combine(d_X, dev(Wt))
    assert_close(host(hid[torch.from_numpy(rows).cuda()]), oracle.combine(X[rows], Wt), what="combine")
    say("c4 full: layer, combination first")
    flags = oracle.SELF_LOOPS | oracle.NORM_SYM
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags, want_w=True, threads=16)
    d_rp, d_ci, d_w, _ = g.gnnagg_build_csr(N, dev(src), dev(dst), flags, want_w=True)
    out = g.gnnagg_aggregate(g.WSUM, d_rp, d_ci, d_w, hid, None, 0, g.gnnagg_plan_rows(d_rp))
    some = sample_rows(rp, n=48)
    agg = oracle.aggregate_rows(oracle.WSUM, some, rp, ci, w, X, threads=16)  # [rows, 602], fp32
    ref = agg.astype(np.float64) @ Wt.astype(np.float64)
    got = host(out[torch.from_numpy(some).cuda()]).astype(np.float64)
    # each side rounds an intermediate to fp32 once (hidden features / aggregated features): a few ulp of
    # the magnitude sum  sum_j w_ij sum_k |x_jk| |W_kh|
    mag = oracle.aggregate_rows(oracle.WSUM, some, rp, ci, w, np.abs(X), threads=16)
    scale = mag.astype(np.float64) @ np.abs(Wt).astype(np.float64)
    assert np.all(np.abs(got - ref) <= 1e-6 + 1e-6 * scale), float(np.max(np.abs(got - ref) / (1e-6 + 1e-6 * scale)))


def test_more_than_two_to_the_31_edges():
    """2.3e9 edges (beyond 2^31 edge positions, below the 2^32 limit of the CSR build) on 50,000 vertices.
    No checker can run at this size; everything asserted is a property that holds exactly at any size:
    row lengths equal the in-degree counts, rows are sorted and hold the right multiset of sources, the
    all-ones matrix aggregates to the degree, a small-integer matrix to the exact integer sums, and max of
    X[j] = j to the largest source of the row.  Every row is long enough to be split over workgroups."""
    import paper_2104_03058_amd as g
    free, _ = torch.cuda.mem_get_info()
    if free < 160 * (1 << 30):
        pytest.skip("needs about 150 GB of free device memory")
    N, E = 50_000, 2_300_000_000
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2104)
    src = torch.randint(0, N, (E,), dtype=torch.int32, device="cuda", generator=gen)
    dst = torch.randint(0, N, (E,), dtype=torch.int32, device="cuda", generator=gen)
    say("big: edges drawn")
    rp, ci, _, _ = g.gnnagg_build_csr(N, src, dst, 0)
    torch.cuda.synchronize()
    say("big: CSR built")
    deg = torch.bincount(dst.long(), minlength=N)
    assert int(rp[0]) == 0 and int(rp[N]) == E
    assert torch.equal(rp[1:] - rp[:-1], deg)
    # inside a row the sources ascend: a descent may only sit where a row starts
    starts = torch.zeros(E + 1, dtype=torch.bool, device="cuda")
    starts[rp] = True
    descent = ci[1:] < ci[:-1]
    assert bool((~descent | starts[1:E]).all())
    del descent, starts
    # the same multiset of sources per row, seen through two exact integer sums
    rows_of = torch.repeat_interleave(torch.arange(N, device="cuda"), deg)
    for power in (1, 2):
        want = torch.zeros(N, dtype=torch.int64, device="cuda").index_add_(0, dst.long(), src.long() ** power)
        got = torch.zeros(N, dtype=torch.int64, device="cuda").index_add_(0, rows_of, ci.long() ** power)
        assert torch.equal(got, want)
    want_max = torch.full((N,), -1, dtype=torch.int64, device="cuda").scatter_reduce_(0, dst.long(), src.long(), "amax")
    del src, dst, rows_of
    say("big: CSR properties hold")
    plan = g.gnnagg_plan_rows(rp)
    assert g.gnnagg_aggregate_workspace_bytes(N, 8, plan) > 0  # mean degree 46,000: rows are split
    ones = torch.ones((N, 8), dtype=torch.float32, device="cuda")
    out = g.gnnagg_aggregate(g.SUM, rp, ci, None, ones, None, 0, plan)
    assert torch.equal(out[:, 0].long(), deg) and torch.equal(out[:, 7], out[:, 0])
    ids = torch.arange(N, device="cuda")
    X = torch.stack([(ids % 7).float(), ids.float(), (ids % 3).float(), torch.ones_like(ids).float()], dim=1).contiguous()
    s = g.gnnagg_aggregate(g.SUM, rp, ci, None, X, None, 0, plan)  # sums stay below 2^24: exact in fp32
    want7 = torch.zeros(N, dtype=torch.int64, device="cuda").index_add_(
        0, torch.repeat_interleave(torch.arange(N, device="cuda"), deg), ci.long() % 7)
    assert torch.equal(s[:, 0].long(), want7) and torch.equal(s[:, 3].long(), deg)
    m = g.gnnagg_aggregate(g.MAX, rp, ci, None, X, None, 0, plan)
    assert torch.equal(m[:, 1].long(), want_max)
    m2 = g.gnnagg_aggregate(g.MAX, rp, ci, None, X, None, 0, plan, split_long_rows=False)
    assert torch.equal(m, m2)
    say("big: aggregation properties hold")
