"""GPU parity of GCN's aggregation in factored form (the GCN operator of Section III): the weights
1/sqrt(d_i d_j) are a product s_i s_j, so the sources' factors go into the feature rows once
(gnnagg_scale_rows), the aggregation is a plain sum, and the destination's factor joins at the store
(GNNAGG_SUM_SCALED).  Bars: factors and scaled rows bit for bit (one correctly rounded operation each); the
scaled sum within 1e-6 + 1e-5 |r| of the CPU checker's scaled sum; and the whole factored path within the
same bar of the checker's weighted sum over per-edge weights, which is what it replaces."""
import sys

import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

g = None


def setup_module(module):
    global g
    import paper_2104_03058_amd as lib
    lib.load_library()  # raises if the HIP library has not been built: no fallback
    g = lib


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:  # bf16 bit patterns
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def assert_close(got, ref, what, rel=1e-5):
    ok = np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= 1e-6 + rel * np.abs(ref.astype(np.float64))
    if not ok.all():
        bad = np.argwhere(~ok)
        i = tuple(bad[0])
        raise AssertionError("%s: %d of %d elements off, first at %s: got %r want %r" %
                             (what, len(bad), ok.size, i, got[i], ref[i]))


def assert_bits(got, ref, what):
    a, b = np.ascontiguousarray(got).view(np.uint32), np.ascontiguousarray(ref).view(np.uint32)
    if not np.array_equal(a, b):
        bad = np.argwhere(a != b)
        i = tuple(bad[0])
        raise AssertionError("%s: %d elements differ bitwise, first at %s: got %r want %r" %
                             (what, len(bad), i, got[i], ref[i]))


def long_rows_graph(N, lengths, seed):
    """Rows 3, 4, ... receive lengths[k] in-edges from pseudo-random sources; plus a sparse background."""
    rng = np.random.default_rng(seed)
    parts_s, parts_d = [], []
    for k, n in enumerate(lengths):
        parts_s.append(rng.integers(0, N, size=n).astype(np.int32))
        parts_d.append(np.full(n, 3 + k, np.int32))
    s2, d2 = W.random_digraph(N, 4 * N, seed + 1)
    keep = (d2 < 3) | (d2 >= 3 + len(lengths))
    return np.concatenate(parts_s + [s2[keep]]), np.concatenate(parts_d + [d2[keep]])


def test_gcn_factors_bit_exact():
    for key, flags in (("c1", oracle.SELF_LOOPS), ("c2", 0)):  # without self-loops: rows of degree 0 as well
        N, src, dst = W.graph(key)
        rp, _, _, _ = oracle.build_csr(N, src, dst, flags)
        say("  factors", key, "N", N, "empty rows", int((np.diff(rp) == 0).sum()))
        assert_bits(host(g.gnnagg_gcn_factors(dev(rp))), oracle.gcn_factors(rp), "factors " + key)
    rp = np.array([0, 0, 1, 5, 21, 24], np.int64)
    assert host(g.gnnagg_gcn_factors(dev(rp))).tolist()[:4] == [0.0, 1.0, 0.5, 0.25]
    assert g.gnnagg_gcn_factors(dev(np.zeros(1, np.int64))).numel() == 0


@pytest.mark.parametrize("F", [1, 3, 4, 7, 32, 61, 64, 300, 602])
def test_scale_rows_bit_exact(F):
    N = 1237
    X = W.normal_f32((N, F), seed=F)
    s = W.normal_f32((N,), seed=1000 + F)
    ref = oracle.scale_rows(X, s)
    d_X, d_s = dev(X), dev(s)
    say("  scale rows F", F)
    assert_bits(host(g.gnnagg_scale_rows(d_X, d_s)), ref, "fresh pitched out")
    out = torch.full((N, F), float("nan"), dtype=torch.float32, device="cuda")
    g.gnnagg_scale_rows(d_X, d_s, out)
    assert_bits(host(out), ref, "contiguous out")
    # pitched input, columns beyond F poisoned on both sides: never read, never written
    Xp = torch.full((N, F + 5), float("nan"), dtype=torch.float32, device="cuda")
    Xp[:, :F] = d_X
    op = torch.full((N, F + 3), -7.0, dtype=torch.float32, device="cuda")
    g.gnnagg_scale_rows(Xp[:, :F], d_s, op[:, :F])
    assert_bits(host(op[:, :F]), ref, "pitched both")
    assert (host(op[:, F:]) == -7.0).all()
    # in place
    g.gnnagg_scale_rows(Xp[:, :F], d_s, Xp[:, :F])
    assert_bits(host(Xp[:, :F]), ref, "in place")
    assert np.isnan(host(Xp[:, F:])).all()
    # bf16 rows are widened, then scaled in fp32
    B = W.normal_bf16((N, F), seed=2000 + F)
    assert_bits(host(g.gnnagg_scale_rows(dev(B), d_s)), oracle.scale_rows(B, s), "bf16 in")


def test_scale_rows_single_row_and_empty():
    X = W.normal_f32((1, 10), seed=1)
    s = np.array([3.0], np.float32)
    assert_bits(host(g.gnnagg_scale_rows(dev(X), dev(s))), oracle.scale_rows(X, s), "one row")
    assert g.gnnagg_scale_rows(torch.empty((0, 4), device="cuda"), torch.empty(0, device="cuda")).shape == (0, 4)


@pytest.mark.parametrize("F,bf16", [(1, False), (7, False), (32, False), (100, True), (300, False), (602, False)])
def test_scaled_sum_matches_the_checker_through_every_entry_point(F, bf16):
    """Short rows sharing a wavefront, a hub row, rows split over workgroups; contiguous and pitched rows;
    chunked; with and without a plan; the Update step; source blocks; the call that allocates nothing."""
    N = 600
    src, dst = long_rows_graph(N, [40000, 33000, 9000, 300], seed=F)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    X = W.normal_bf16((N, F), seed=10 + F) if bf16 else W.normal_f32((N, F), seed=10 + F)
    s = W.normal_f32((N,), seed=20 + F)
    ref = oracle.aggregate(oracle.SUM_SCALED, rp, ci, s, X, threads=8)
    rel = 1e-2 if bf16 else 1e-5
    d_rp, d_ci, d_X, d_s = dev(rp), dev(ci), dev(X), dev(s)
    plan = g.gnnagg_plan_rows(d_rp)
    for use_plan in (True, False):
        for fc in (0, 5, g.F_CHUNK_AUTO):
            say("  scaled sum F", F, "plan", use_plan, "f_chunk", fc)
            out = torch.full((N, F), float("nan"), dtype=torch.float32, device="cuda")
            g.gnnagg_aggregate(g.SUM_SCALED, d_rp, d_ci, d_s, d_X, out, fc, plan if use_plan else None)
            assert_close(host(out), ref, "plain plan=%s fc=%d" % (use_plan, fc), rel)
    whole = g.gnnagg_aggregate(g.SUM_SCALED, d_rp, d_ci, d_s, d_X, None, 0, plan, split_long_rows=False)
    assert_close(host(whole), ref, "one workgroup per row", rel)
    # rows on 128-byte lines
    Xp = g.pitched_empty(N, F, d_X.dtype)
    Xp.copy_(d_X)
    outp = g.pitched_empty(N, F, torch.float32)
    for fc in (0, g.F_CHUNK_AUTO):
        outp.fill_(float("nan"))
        g.gnnagg_aggregate(g.SUM_SCALED, d_rp, d_ci, d_s, Xp, outp, fc, plan)
        assert_close(host(outp), ref, "pitched fc=%d" % fc, rel)
    # the call that allocates nothing
    outp.fill_(float("nan"))
    g.gnnagg_aggregate_noalloc(g.SUM_SCALED, d_rp, d_ci, d_s, Xp, outp, 0, plan)
    assert_close(host(outp), ref, "noalloc", rel)
    # source blocks: the factor joins when the last block finishes the row
    for B in (1, 3):
        blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, B)
        outp.fill_(float("nan"))
        g.gnnagg_aggregate_blocked(g.SUM_SCALED, d_rp, d_ci, d_s, Xp, blocks, outp, 0)
        assert_close(host(outp), ref, "blocked B=%d" % B, rel)
    # the Update step follows the scaling: act(s_i * sum + bias)
    bias = W.normal_f32((F,), seed=30 + F)
    got = g.gnnagg_aggregate_update(g.SUM_SCALED, d_rp, d_ci, d_s, d_X, None, dev(bias), True, None, 0, plan)
    assert_close(host(got), oracle.update(ref, bias, True), "bias + relu", rel)
    if F <= 64:
        W2 = W.normal_f32((F, 24), seed=40 + F)
        b2 = W.normal_f32((24,), seed=50 + F)
        got = g.gnnagg_aggregate_update(g.SUM_SCALED, d_rp, d_ci, d_s, d_X, dev(W2), dev(b2), True, None, 0, plan)
        assert_close(host(got), oracle.combine(ref, W2, b2, True), "fused dense layer", max(rel, 2e-5))
    # bf16 output: the scaled fp32 result rounded to nearest even
    ob = torch.empty((N, F), dtype=torch.bfloat16, device="cuda")
    g.gnnagg_aggregate(g.SUM_SCALED, d_rp, d_ci, d_s, d_X, ob, 0, plan)
    assert_close(W.bf16_to_f32(host(ob.view(torch.int16)).view(np.uint16)), W.bf16_to_f32(W.f32_to_bf16(ref)), "bf16 out",
                 1e-2)


def test_scaled_sum_with_unit_factors_is_the_sum_bit_for_bit():
    N, src, dst = W.graph("c1")
    rp, ci, _, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS)
    d_rp, d_ci = dev(rp), dev(ci)
    X = dev(W.normal_f32((N, 96), seed=5))
    plan = g.gnnagg_plan_rows(d_rp)
    ones = torch.ones(N, dtype=torch.float32, device="cuda")
    a = g.gnnagg_aggregate(g.SUM_SCALED, d_rp, d_ci, ones, X, None, 32, plan)
    b = g.gnnagg_aggregate(g.SUM, d_rp, d_ci, None, X, None, 32, plan)
    assert_bits(host(a), host(b), "unit factors")


@pytest.mark.parametrize("key,scale,F", [("c1", 1.0, 602), ("c2", 1.0, 100), ("c4", 0.02, 64)])
def test_factored_gcn_meets_the_bar_of_the_weighted_sum_it_replaces(key, scale, F):
    """gcn_factors -> scale_rows -> SUM_SCALED on the device against the checker's weighted sum over the
    per-edge weights 1/sqrt(d_i d_j): the two differ by how the weights are rounded, far inside the bar."""
    N, src, dst = W.graph(key, scale)
    flags = oracle.SELF_LOOPS | oracle.NORM_SYM
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags, want_w=True, threads=8)
    X = W.normal_f32((N, F), seed=77)
    ref = oracle.aggregate(oracle.WSUM, rp, ci, w, X, threads=8)
    d_rp, d_ci, _, _ = g.gnnagg_build_csr(N, dev(src), dev(dst), flags)
    plan = g.gnnagg_plan_rows(d_rp)
    s = g.gnnagg_gcn_factors(d_rp)
    Xs = g.gnnagg_scale_rows(dev(X), s)
    say("  factored gcn", key, "F", F)
    out = g.gnnagg_aggregate(g.SUM_SCALED, d_rp, d_ci, s, Xs, g.pitched_empty(N, F), g.F_CHUNK_AUTO, plan)
    assert_close(host(out), ref, "factored vs per-edge weights")
    # and the definition itself: the checker's scaled sum of the checker's scaled rows
    s_ref = oracle.gcn_factors(rp)
    ref2 = oracle.aggregate(oracle.SUM_SCALED, rp, ci, s_ref, oracle.scale_rows(X, s_ref), threads=8)
    assert_close(host(out), ref2, "factored vs the checker's factored form")
    blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, 4)
    outb = g.gnnagg_aggregate_blocked(g.SUM_SCALED, d_rp, d_ci, s, Xs, blocks, None, g.F_CHUNK_AUTO)
    assert_close(host(outb), ref, "factored, 4 source blocks")


@pytest.mark.parametrize("F,H,bf16", [(96, 16, False), (602, 32, False), (100, 41, True), (7, 130, False)])
def test_combination_with_scaled_rows_equals_combination_then_scaling(F, H, bf16):
    N = 1500
    X = W.normal_bf16((N, F), seed=F) if bf16 else W.normal_f32((N, F), seed=F)
    Wt = W.normal_f32((F, H), seed=F + 1, std=0.1)
    b = W.normal_f32((H,), seed=F + 2)
    s = W.normal_f32((N,), seed=F + 3)
    d_X, d_W, d_b, d_s = dev(X), dev(Wt), dev(b), dev(s)
    say("  combine_scaled F", F, "H", H)
    for bias, relu in ((None, False), (d_b, True)):
        fused = g.gnnagg_combine(d_X, d_W, bias, relu, row_scale=d_s)
        plain = g.gnnagg_combine(d_X, d_W, bias, relu)
        assert_bits(host(fused), host(g.gnnagg_scale_rows(plain, d_s, torch.empty_like(plain))), "fused vs two calls")
        ref = oracle.scale_rows(oracle.combine(X, Wt, b if bias is not None else None, relu, threads=8), s)
        assert_close(host(fused), ref, "vs checker")
    # with the rows also stored in another order
    perm = torch.randperm(N, device="cuda", generator=torch.Generator(device="cuda").manual_seed(1)).to(torch.int32)
    moved = g.gnnagg_combine(d_X, d_W, d_b, True, out_rows=perm, row_scale=d_s)
    straight = g.gnnagg_combine(d_X, d_W, d_b, True, row_scale=d_s)
    assert_bits(host(moved[perm.long()]), host(straight), "out_rows + row_scale")


def test_gcn_layer_in_factored_form_against_the_checkers_layer_with_per_edge_weights():
    """relu(A_hat (X W) + b): Combination writes s_j (X W)_j, the aggregation sums, scales by s_i and applies
    the Update step at its store - against the checker's combine, per-edge weighted sum and update."""
    N, src, dst = W.graph("c2")
    F, H = 500, 16
    flags = oracle.SELF_LOOPS | oracle.NORM_SYM
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags, want_w=True, threads=8)
    X = W.normal_f32((N, F), seed=3)
    Wt = W.normal_f32((F, H), seed=4, std=0.05)
    b = W.normal_f32((H,), seed=5, std=0.1)
    ref = oracle.update(oracle.aggregate(oracle.WSUM, rp, ci, w, oracle.combine(X, Wt, threads=8), threads=8), b, True)
    d_rp, d_ci, _, _ = g.gnnagg_build_csr(N, dev(src), dev(dst), flags)
    plan = g.gnnagg_plan_rows(d_rp)
    s = g.gnnagg_gcn_factors(d_rp)
    hid = g.gnnagg_combine(dev(X), dev(Wt), None, False, row_scale=s)
    out = g.gnnagg_aggregate_update(g.SUM_SCALED, d_rp, d_ci, s, hid, None, dev(b), True, None, 0, plan)
    assert_close(host(out), ref, "factored layer")


def test_factored_path_can_be_captured_in_a_graph_and_replayed():
    """Factors, row scaling and the scaled sum over source blocks only enqueue kernels: captured once, every
    replay - fresh inputs copied in place, eager work in between - gives the bits of the eager calls."""
    N, src, dst = W.graph("c4", 0.01)
    flags = oracle.SELF_LOOPS | oracle.NORM_SYM
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags, want_w=True)
    d_rp, d_ci = dev(rp), dev(ci)
    blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, 3)
    F = 160
    X = torch.zeros((N, F), dtype=torch.float32, device="cuda")
    Xs = torch.empty((N, F), dtype=torch.float32, device="cuda")
    s = torch.empty(N, dtype=torch.float32, device="cuda")
    out = torch.empty((N, F), dtype=torch.float32, device="cuda")
    ws = torch.empty(g.gnnagg_aggregate_blocked_workspace_bytes(N, F, blocks), dtype=torch.uint8, device="cuda")

    def call():
        g.gnnagg_gcn_factors(d_rp, s)
        g.gnnagg_scale_rows(X, s, Xs)
        g.gnnagg_aggregate_blocked(g.SUM_SCALED, d_rp, d_ci, s, Xs, blocks, out, 32, workspace=ws)

    call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for k in range(3):
        Xh = W.normal_f32((N, F), seed=880 + k)
        X.copy_(dev(Xh))
        s.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        out.zero_()
        Xs.zero_()
        s.zero_()
        ws.fill_(0x7F)
        call()
        torch.cuda.synchronize()
        assert torch.equal(got, out), "replay %d differs from the eager calls" % k
        assert_close(host(out), oracle.aggregate(oracle.WSUM, rp, ci, w, Xh, threads=8), "captured factored path %d" % k)


def test_seeded_sweep_of_small_random_cases_for_the_scaled_sum():
    """Thirty small cases with shapes drawn from a seeded generator: graph size (one vertex and edgeless graphs
    among them), a planted hub, feature width, chunk width, input type, with and without a row plan."""
    rng = np.random.default_rng(31337)
    for case in range(30):
        N = int(rng.integers(1, 400))
        E = int(rng.integers(0, 12 * N + 1))
        src, dst = (W.random_digraph(N, E, 6000 + case) if E else (np.zeros(0, np.int32), np.zeros(0, np.int32)))
        if N > 8 and case % 3 == 0:
            hub_src = rng.integers(0, N, size=int(rng.integers(300, 3000))).astype(np.int32)
            src = np.concatenate([src, hub_src])
            dst = np.concatenate([dst, np.full(len(hub_src), int(rng.integers(0, N)), np.int32)])
        F = int(rng.choice([1, 2, 3, 5, 8, 12, 17, 31, 32, 33, 64, 100, 129, 260, 513]))
        fc = int(rng.choice([0, 0, 1, 3, 4, 8, 16, 50, g.F_CHUNK_AUTO]))
        bf16 = bool(rng.integers(0, 2))
        rp, ci, _, _ = oracle.build_csr(N, src, dst, int(rng.choice([0, oracle.SELF_LOOPS])))
        X = W.normal_bf16((N, F), seed=6100 + case) if bf16 else W.normal_f32((N, F), seed=6100 + case)
        s = W.normal_f32((N,), seed=6200 + case)
        say("  scaled-sum sweep case", case, "N", N, "nnz", len(ci), "F", F, "fc", fc, "bf16", bf16)
        ref = oracle.aggregate(oracle.SUM_SCALED, rp, ci, s, X)
        d_rp = dev(rp)
        plan = g.gnnagg_plan_rows(d_rp) if case & 1 else None
        d_ci = dev(ci) if len(ci) else torch.zeros(1, dtype=torch.int32, device="cuda")
        out = torch.full((N, F), float("nan"), dtype=torch.float32, device="cuda")
        g.gnnagg_aggregate(g.SUM_SCALED, d_rp, d_ci, dev(s), dev(X), out, fc, plan)
        assert_close(host(out), ref, "sweep %d" % case, 1e-2 if bf16 else 1e-5)
