"""GPU parity: every call goes through the C ABI (ctypes binding) and is compared
element by element with the CPU checker on the same seeded inputs.

Bars (stated where they are used):
  * CSR structure, row plan, max aggregation: bit-exact.
  * fp32 sum / weighted sum / mean / attention: |g - r| <= 1e-6 + 1e-5 |r|.
  * bf16-stored inputs (fp32 accumulate): |g - r| <= 1e-6 + 1e-2 |r|.
"""
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


def close_f32(got, ref):
    return np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= 1e-6 + 1e-5 * np.abs(ref.astype(np.float64))


def close_bf16(got, ref):
    return np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= 1e-6 + 1e-2 * np.abs(ref.astype(np.float64))


def assert_close(got, ref, bf16=False, what=""):
    ok = close_bf16(got, ref) if bf16 else close_f32(got, ref)
    if not ok.all():
        bad = np.argwhere(~ok)
        i = tuple(bad[0])
        raise AssertionError("%s: %d of %d elements off, first at %s: got %r want %r" %
                             (what, len(bad), ok.size, i, got[i], ref[i]))


def assert_bits(got, ref, what=""):
    a, b = got.view(np.uint32), ref.view(np.uint32)
    if not np.array_equal(a, b):
        bad = np.argwhere(a != b)
        i = tuple(bad[0])
        raise AssertionError("%s: %d elements differ bitwise, first at %s: got %r want %r" %
                             (what, len(bad), i, got[i], ref[i]))


def gpu_csr(N, src, dst, flags=0, want_w=False, want_perm=False):
    rp, ci, w, perm = g.gnnagg_build_csr(N, dev(src), dev(dst), flags, want_w, want_perm)
    return rp, ci, w, perm


OPS = {"sum": (0, oracle.SUM), "wsum": (1, oracle.WSUM), "mean": (2, oracle.MEAN), "max": (3, oracle.MAX)}


def check_aggregate(N, rp, ci, w, X, ops, f_chunks=(0,), plans=(True, False), bf16=False, what=""):
    d_rp, d_ci = dev(rp), dev(ci)
    d_w = dev(w) if w is not None else None
    d_X = dev(X)
    plan = g.gnnagg_plan_rows(d_rp)
    for name in ops:
        gop, rop = OPS[name]
        ref = oracle.aggregate(rop, rp, ci, w, X, threads=8)
        for use_plan in plans:
            for fc in f_chunks:
                say("  aggregate", what, name, "f_chunk", fc, "plan", use_plan)
                out = torch.full((N, X.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
                g.gnnagg_aggregate(gop, d_rp, d_ci, d_w if name == "wsum" else None, d_X, out, fc,
                                   plan if use_plan else None)
                got = host(out)
                tag = "%s %s fc=%d plan=%s" % (what, name, fc, use_plan)
                if name == "max":
                    assert_bits(got, ref, tag)
                else:
                    assert_close(got, ref, bf16, tag)


# ------------------------------------------------------------------ CSR build
def tiny_digraphs():
    cases = []
    for k, (N, E) in enumerate([(5, 9), (17, 60), (33, 300), (64, 257), (8, 0), (1, 0), (1, 3), (300, 5000)]):
        if E:
            src, dst = W.random_digraph(N, E, 200 + k)
        else:
            src, dst = np.zeros(0, np.int32), np.zeros(0, np.int32)
        cases.append((N, src, dst))
    return cases


@pytest.mark.parametrize("flags", [0, 1, 3, 2])
def test_csr_tiny_digraphs_bit_exact(flags):
    for N, src, dst in tiny_digraphs():
        say("csr tiny N", N, "E", len(src), "flags", flags)
        rp, ci, w, perm = oracle.build_csr(N, src, dst, flags, want_w=True, want_perm=True)
        if len(src) == 0:
            d_src = torch.zeros(0, dtype=torch.int32, device="cuda")
            d_dst = torch.zeros(0, dtype=torch.int32, device="cuda")
            grp, gci, gw, gperm = g.gnnagg_build_csr(N, d_src, d_dst, flags, True, True)
        else:
            grp, gci, gw, gperm = gpu_csr(N, src, dst, flags, True, True)
        assert np.array_equal(host(grp), rp)
        assert np.array_equal(host(gci), ci)
        assert np.array_equal(host(gperm), perm)
        assert_bits(host(gw), w, "edge_w")


@pytest.mark.parametrize("key,scale", [("c1", 1.0), ("c2", 1.0), ("c4", 0.02), ("c5", 0.02)])
def test_csr_benchmark_graphs_bit_exact(key, scale):
    N, src, dst = W.graph(key, scale)
    say("csr", key, "N", N, "E", len(src))
    flags = oracle.SELF_LOOPS | oracle.NORM_SYM
    rp, ci, w, perm = oracle.build_csr(N, src, dst, flags, want_w=True, want_perm=True, threads=8)
    grp, gci, gw, gperm = gpu_csr(N, src, dst, flags, True, True)
    assert np.array_equal(host(grp), rp) and np.array_equal(host(gci), ci) and np.array_equal(host(gperm), perm)
    assert_bits(host(gw), w, "edge_w")
    # the structure does not depend on the order of the input edges
    sh = np.random.default_rng(1).permutation(len(src))
    grp2, gci2, _, _ = gpu_csr(N, src[sh], dst[sh], flags)
    assert np.array_equal(host(grp2), rp) and np.array_equal(host(gci2), ci)


def test_csr_reports_out_of_range_vertex():
    src = np.array([0, 1, 9, 2], np.int32)
    dst = np.array([1, 2, 0, -1], np.int32)
    with pytest.raises(g.GnnaggError) as e:
        gpu_csr(4, src, dst)
    assert e.value.status == -1


# ------------------------------------------------------------------ row plan
@pytest.mark.parametrize("key,scale", [("c2", 1.0), ("c4", 0.02), ("c5", 0.02)])
def test_plan_rows_sorted_by_degree(key, scale):
    N, src, dst = W.graph(key, scale)
    rp, _, _, _ = oracle.build_csr(N, src, dst, threads=8)
    plan = g.gnnagg_plan_rows(dev(rp))
    order = host(plan.row_order)
    deg = np.diff(rp)
    # unique answer: degree descending, ties by row id
    expect = np.lexsort((np.arange(N), -deg)).astype(np.int32)
    assert np.array_equal(order, expect)
    off = plan.class_offsets()
    assert off[0] == 0 and off[-1] == N and all(a <= b for a, b in zip(off, off[1:]))
    cls = np.where(deg > 0, 1 + np.floor(np.log2(np.maximum(deg, 1))).astype(np.int64), 0)
    for c in range(33):
        lo, hi = off[32 - c], off[33 - c]
        assert np.all(cls[order[lo:hi]] == c), c


# ------------------------------------------------------------------ aggregation on the benchmark shapes
def test_config1_gcn_tiny_chunk_sweep():
    N, src, dst = W.graph("c1")
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    X = W.bernoulli_f32((N, 1433), 0.013, seed=100)
    check_aggregate(N, rp, ci, w, X, ["wsum"], f_chunks=(16, 64, 0), what="c1")


def test_config2_sage_mean_mid():
    N, src, dst = W.graph("c2")
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    X = W.normal_f32((N, 500), seed=101)
    check_aggregate(N, rp, ci, None, X, ["mean", "sum", "max"], f_chunks=(0, 4), what="c2")


def test_config4_shape_scaled_dense_chunk_sweep():
    # the dense graph at 2 % of its vertices and edges: same mean degree (~492), hubs of several thousand
    N, src, dst = W.graph("c4", 0.02)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True, threads=8)
    say("c4 scaled N", N, "nnz", len(ci), "max deg", int(np.diff(rp).max()))
    X = W.normal_f32((N, 602), seed=102)
    check_aggregate(N, rp, ci, w, X, ["wsum"], f_chunks=(8, 16, 32, 64, 0), plans=(True,), what="c4s")
    check_aggregate(N, rp, ci, w, X, ["mean", "sum"], f_chunks=(0,), plans=(True, False), what="c4s")


@pytest.mark.parametrize("F", [100, 32, 16])
def test_config5_shape_scaled_sparse_bf16(F):
    N, src, dst = W.graph("c5", 0.02)
    rp, ci, _, _ = oracle.build_csr(N, src, dst, threads=8)
    say("c5 scaled N", N, "nnz", len(ci), "max deg", int(np.diff(rp).max()))
    X = W.normal_bf16((N, F), seed=103 + F)
    check_aggregate(N, rp, ci, None, X, ["sum", "max", "mean"], f_chunks=(0,), bf16=True, what="c5s F=%d" % F)


# ------------------------------------------------------------------ edge cases
def star(N, hub, n_in, seed):
    """n_in distinct sources (cycling) into one hub row, plus a few stray edges."""
    src = (np.arange(n_in, dtype=np.int32) * 7 + 1) % N
    dst = np.full(n_in, hub, np.int32)
    s2, d2 = W.random_digraph(N, 3 * N, seed)
    return np.concatenate([src, s2]), np.concatenate([dst, d2])


@pytest.mark.parametrize("F,fc", [(1, 0), (3, 0), (5, 2), (4, 0), (64, 0), (300, 0), (257, 0), (1030, 0), (9, 4)])
def test_hub_row_and_ragged_widths_fp32(F, fc):
    N = 700
    src, dst = star(N, hub=13, n_in=6000, seed=F)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    w = W.normal_f32((len(ci),), seed=7)
    X = W.normal_f32((N, F), seed=300 + F)
    check_aggregate(N, rp, ci, w, X, ["sum", "wsum", "mean", "max"], f_chunks=(fc,), what="hub F=%d" % F)


@pytest.mark.parametrize("F", [1, 2, 7, 8, 15, 100, 1000])
def test_hub_row_and_ragged_widths_bf16(F):
    N = 500
    src, dst = star(N, hub=2, n_in=5000, seed=50 + F)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    w = W.normal_f32((len(ci),), seed=8)
    X = W.normal_bf16((N, F), seed=400 + F)
    check_aggregate(N, rp, ci, w, X, ["sum", "wsum", "max"], f_chunks=(0,), bf16=True, what="hub bf16 F=%d" % F)


def test_empty_rows_single_vertex_and_directed():
    # no edges at all: sum/mean/max of an empty neighbourhood are +0
    for N in (1, 5, 300):
        rp = np.zeros(N + 1, np.int64)
        ci = np.zeros(1, np.int32)  # a valid non-empty buffer; never read
        X = W.normal_f32((N, 6), seed=N)
        for name in ("sum", "mean", "max"):
            out = g.gnnagg_aggregate(OPS[name][0], dev(rp), dev(ci), None, dev(X))
            assert_bits(host(out), np.zeros((N, 6), np.float32), "empty " + name)
    # one directed edge 2 -> 5: only row 5 receives
    src, dst = np.array([2], np.int32), np.array([5], np.int32)
    rp, ci, _, _ = gpu_csr(8, src, dst)
    X = W.normal_f32((8, 3), seed=1)
    out = host(g.gnnagg_aggregate(0, rp, ci, None, dev(X)))
    ref = np.zeros((8, 3), np.float32)
    ref[5] = X[2]
    assert_bits(out, ref, "directed")


def test_max_signed_zero_and_infinities_bit_exact():
    src = np.array([1, 2, 2, 1, 1, 3, 4], np.int32)
    dst = np.array([0, 0, 1, 1, 3, 4, 4], np.int32)
    X = np.array([[5.0, 1.0], [-0.0, -np.inf], [0.0, -3.0], [1.0, np.inf], [-2.0, 7.0]], np.float32)
    rp, ci, _, _ = oracle.build_csr(5, src, dst)
    for Xc in (X, W.f32_to_bf16(X)):
        ref = oracle.aggregate(oracle.MAX, rp, ci, None, Xc)
        out = host(g.gnnagg_aggregate(3, dev(rp), dev(ci), None, dev(Xc)))
        assert_bits(out, ref, "max special values")
    assert out.view(np.uint32)[3, 0] == 0x80000000  # the only neighbour holds -0


def test_same_bits_on_every_run_and_for_every_chunk_width_of_max():
    N, src, dst = W.graph("c4", 0.01)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, 3, want_w=True, threads=8)
    X = W.normal_f32((N, 130), seed=9)
    d = [dev(rp), dev(ci), dev(w), dev(X)]
    plan = g.gnnagg_plan_rows(d[0])
    a = host(g.gnnagg_aggregate(1, d[0], d[1], d[2], d[3], None, 0, plan))
    b = host(g.gnnagg_aggregate(1, d[0], d[1], d[2], d[3], None, 0, plan))
    assert_bits(a, b, "run-to-run")
    m0 = host(g.gnnagg_aggregate(3, d[0], d[1], None, d[3], None, 0, plan))
    for fc in (1, 8, 33, 64):
        assert_bits(host(g.gnnagg_aggregate(3, d[0], d[1], None, d[3], None, fc, plan)), m0, "max fc=%d" % fc)


def bf16_rne_bits(x):
    """fp32 array -> bf16 bit patterns, round to nearest even (numpy, independent of both implementations)."""
    b = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    return ((b + 0x7fff + ((b >> 16) & 1)) >> 16).astype(np.uint16)


@pytest.mark.parametrize("F", [1, 7, 32, 100, 300])
def test_bf16_output_is_the_rounded_fp32_result(F):
    N, src, dst = W.graph("c5", 0.01)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    Xb = W.normal_bf16((N, F), seed=70 + F)
    d_rp, d_ci, d_X = dev(rp), dev(ci), dev(Xb)
    plan = g.gnnagg_plan_rows(d_rp)
    for name in ("sum", "mean", "max"):
        gop, rop = OPS[name]
        ref32 = oracle.aggregate(rop, rp, ci, None, Xb)
        out = torch.zeros((N, F), dtype=torch.bfloat16, device="cuda")
        g.gnnagg_aggregate(gop, d_rp, d_ci, None, d_X, out, 0, plan)
        got = host(out.view(torch.int16)).view(np.uint16)
        want = bf16_rne_bits(ref32)
        if name == "max":  # the maximum of bf16 values is a bf16 value: exact
            assert np.array_equal(got, want)
        else:              # the fp32 results agree to ~1e-7, so the bf16 values differ by at most one step, rarely
            gf, wf = W.bf16_to_f32(got).astype(np.float64), W.bf16_to_f32(want).astype(np.float64)
            assert np.all(np.abs(gf - wf) <= 2.0 ** -7 * np.abs(wf) + 1e-30)
            assert np.mean(got != want) < 1e-3
    # fp32 features, bf16 output
    Xf = W.normal_f32((N, F), seed=71)
    ref32 = oracle.aggregate(oracle.SUM, rp, ci, None, Xf)
    out = torch.zeros((N, F), dtype=torch.bfloat16, device="cuda")
    g.gnnagg_aggregate(0, d_rp, d_ci, None, dev(Xf), out, 0, plan)
    got, want = host(out.view(torch.int16)).view(np.uint16), bf16_rne_bits(ref32)
    assert np.mean(got != want) < 1e-3


def test_auto_chunk_width_is_accepted_and_matches_one_chunk_on_small_inputs():
    N, src, dst = W.graph("c2")
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    X = W.normal_f32((N, 70), seed=12)
    d = [dev(rp), dev(ci), dev(X)]
    a = host(g.gnnagg_aggregate(0, d[0], d[1], None, d[2], None, g.F_CHUNK_AUTO))
    b = host(g.gnnagg_aggregate(0, d[0], d[1], None, d[2], None, 0))
    assert_bits(a, b, "auto vs one chunk")
    with pytest.raises(g.GnnaggError):
        g.gnnagg_aggregate(0, d[0], d[1], None, d[2], None, -2)


def test_measured_chunk_width_tuner_returns_a_valid_width_and_leaves_a_valid_result():
    N, src, dst = W.graph("c4", 0.02)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True, threads=8)
    X = W.normal_f32((N, 300), seed=77)
    d_rp, d_ci, d_w = dev(rp), dev(ci), dev(w)
    plan = g.gnnagg_plan_rows(d_rp)
    Xp = g.pitched_empty(N, 300, torch.float32)
    Xp.copy_(dev(X))
    out = g.pitched_empty(N, 300, torch.float32)
    out.fill_(float("nan"))
    best, ms = g.gnnagg_tune_f_chunk(g.WSUM, d_rp, d_ci, d_w, Xp, out, plan)
    assert best in (300, 32, 64, 128, 256, g.gnnagg_auto_f_chunk(N, 300, g.F32, int(Xp.stride(0)), plan)) and ms > 0
    assert_close(host(out), oracle.aggregate(oracle.WSUM, rp, ci, w, X, threads=8), what="result left by the tuner")
    # the width it returns is an ordinary f_chunk
    again = g.gnnagg_aggregate(g.WSUM, d_rp, d_ci, d_w, Xp, None, best, plan)
    assert_close(host(again), host(out), what="tuned width")
    g.gnnagg_set_workgroup_cap(2)   # the measurement override changes timing only
    capped = g.gnnagg_aggregate(g.WSUM, d_rp, d_ci, d_w, Xp, None, best, plan)
    g.gnnagg_set_workgroup_cap(-1)
    assert_bits(host(capped), host(again), "workgroup cap override")


def test_compensated_sum_survives_cancellation():
    # 20000 values of size ~1e3 that cancel to O(1): a plain fp32 running sum would be off by ~1e-2
    N, n_in = 64, 20000
    src = (np.arange(n_in, dtype=np.int32) % (N - 1)) + 1
    dst = np.zeros(n_in, np.int32)
    X = (1000.0 * W.normal_f32((N, 8), seed=5)).astype(np.float32)
    X[1:] -= X[1:].mean(axis=0, keepdims=True).astype(np.float32)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    ref = oracle.aggregate(oracle.SUM, rp, ci, None, X)
    d_rp = dev(rp)
    out = host(g.gnnagg_aggregate(0, d_rp, dev(ci), None, dev(X), None, 0, g.gnnagg_plan_rows(d_rp)))
    assert_close(out, ref, what="cancellation")


# ------------------------------------------------------------------ attention
def check_gat(N, rp, ci, H, a_s, a_d, f_chunks=(0,), plans=(True, False), what=""):
    ralpha, rout = oracle.gat_attention(rp, ci, H, a_s, a_d, 0.2, threads=8)
    d_rp, d_ci, d_H, d_as, d_ad = dev(rp), dev(ci), dev(H), dev(a_s), dev(a_d)
    plan = g.gnnagg_plan_rows(d_rp)
    for use_plan in plans:
        for fc in f_chunks:
            say("  gat", what, "f_chunk", fc, "plan", use_plan)
            alpha, out = g.gnnagg_gat_attention(d_rp, d_ci, d_H, d_as, d_ad, 0.2, True, True, fc,
                                                plan if use_plan else None)
            assert_close(host(out), rout, what="%s out fc=%d plan=%s" % (what, fc, use_plan))
            assert_close(host(alpha), ralpha, what="%s alpha fc=%d plan=%s" % (what, fc, use_plan))
            # without alpha, heads of 4 / 8 / 16 channels run as one launch that recomputes both scores in
            # registers, in the summation order of the score kernel: the same bits
            _, out2 = g.gnnagg_gat_attention(d_rp, d_ci, d_H, d_as, d_ad, 0.2, False, True, fc,
                                             plan if use_plan else None)
            assert_close(host(out2), rout, what="%s out (no alpha) fc=%d plan=%s" % (what, fc, use_plan))
            assert_bits(host(out2), host(out), "%s out with and without alpha fc=%d plan=%s" % (what, fc, use_plan))


def test_config3_gat_mid_graph():
    N, src, dst = W.graph("c2")
    rp, ci, _, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS)
    H = W.normal_f32((N, 8, 8), seed=110)
    a_s = W.normal_f32((8, 8), seed=111, std=0.1)
    a_d = W.normal_f32((8, 8), seed=112, std=0.1)
    check_gat(N, rp, ci, H, a_s, a_d, f_chunks=(0, 8, 16, 24), what="c3")


# (2,4) (1,8) (4,16) (64,8): a head on 1 / 2 / 4 lanes, narrow to wave-wide slices (scores recomputed from the
# gathered rows); (33,8): slices that cut heads; (2,32) (3,5) (4,6) (1,1): scores gathered
@pytest.mark.parametrize("heads,C", [(8, 8), (3, 5), (1, 1), (4, 6), (40, 8), (2, 4), (1, 8), (4, 16), (64, 8),
                                     (33, 8), (2, 32)])
def test_gat_hub_rows_and_odd_head_shapes(heads, C):
    N = 400
    src, dst = star(N, hub=7, n_in=5000, seed=heads * 10 + C)
    rp, ci, _, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS)
    H = W.normal_f32((N, heads, C), seed=120)
    a_s = W.normal_f32((heads, C), seed=121, std=0.5)
    a_d = W.normal_f32((heads, C), seed=122, std=0.5)
    check_gat(N, rp, ci, H, a_s, a_d, f_chunks=(0, C), what="gat hub %dx%d" % (heads, C))


def test_gat_dense_scaled_graph():
    N, src, dst = W.graph("c4", 0.01)
    rp, ci, _, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS, threads=8)
    H = W.normal_f32((N, 8, 8), seed=130)
    a_s = W.normal_f32((8, 8), seed=131, std=0.1)
    a_d = W.normal_f32((8, 8), seed=132, std=0.1)
    check_gat(N, rp, ci, H, a_s, a_d, f_chunks=(0, 8), plans=(True,), what="gat c4s")


def test_gat_special_cases():
    # a row with one in-edge copies its neighbour bit for bit and has weight exactly 1; empty rows give 0
    src = np.array([3, 1, 2], np.int32)
    dst = np.array([0, 0, 4], np.int32)
    H = W.normal_f32((5, 2, 4), seed=140)
    a_s = W.normal_f32((2, 4), seed=141)
    a_d = W.normal_f32((2, 4), seed=142)
    rp, ci, _, _ = oracle.build_csr(5, src, dst)
    alpha, out = g.gnnagg_gat_attention(dev(rp), dev(ci), dev(H), dev(a_s), dev(a_d), 0.2, True, True)
    alpha, out = host(alpha), host(out)
    assert_bits(out[4], H[2], "single edge")
    assert np.array_equal(alpha[rp[4]], np.ones(2, np.float32))
    assert_bits(out[1], np.zeros((2, 4), np.float32), "empty row")
    # scores scaled by 100: no overflow, weights collapse on the arg-max
    big = (100.0 * a_s).astype(np.float32)
    ralpha, rout = oracle.gat_attention(rp, ci, H, big, a_d, 0.2)
    alpha2, out2 = g.gnnagg_gat_attention(dev(rp), dev(ci), dev(H), dev(big), dev(a_d), 0.2, True, True)
    assert np.all(np.isfinite(host(out2)))
    # logits of size ~100 carry an fp32 rounding error of ~1e-5, which the exponential turns into a relative
    # error of the weights: this case checks robustness, not the parity bar
    assert np.allclose(host(out2), rout, rtol=2e-3, atol=1e-5)
    assert np.allclose(host(alpha2), ralpha, rtol=2e-3, atol=1e-6)


# ------------------------------------------------------------------ Update step inside the aggregation kernels
def check_update(N, rp, ci, w, X, ops, f_chunks=(0,), bf16=False, what="", seed=0):
    """act(aggregate(X) + bias) against the checker's aggregate followed by its Update step."""
    F = X.shape[1]
    d_rp, d_ci, d_X = dev(rp), dev(ci), dev(X)
    d_w = dev(w) if w is not None else None
    plan = g.gnnagg_plan_rows(d_rp)
    bias = W.normal_f32((F,), seed=900 + seed)
    d_b = dev(bias)
    for name in ops:
        gop, rop = OPS[name]
        agg = oracle.aggregate(rop, rp, ci, w, X, threads=8)
        for relu in (False, True):
            for use_bias in (True, False):
                ref = oracle.update(agg, bias if use_bias else None, relu)
                for fc in f_chunks:
                    for use_plan in (True, False):
                        say("  update", what, name, "relu", relu, "bias", use_bias, "fc", fc, "plan", use_plan)
                        out = torch.full((N, F), float("nan"), dtype=torch.float32, device="cuda")
                        g.gnnagg_aggregate_update(gop, d_rp, d_ci, d_w if name == "wsum" else None, d_X, None,
                                                  d_b if use_bias else None, relu, out, fc,
                                                  plan if use_plan else None)
                        tag = "%s %s relu=%s bias=%s fc=%d plan=%s" % (what, name, relu, use_bias, fc, use_plan)
                        if name == "max" and not use_bias:
                            assert_bits(host(out), ref, tag)
                        else:
                            assert_close(host(out), ref, bf16, tag)


def test_update_bias_and_activation_at_the_store():
    N, src, dst = W.graph("c1")
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    check_update(N, rp, ci, w, W.normal_f32((N, 96), seed=901), ("wsum", "mean", "max"), f_chunks=(0, 32, 40),
                 what="c1 F=96", seed=1)
    check_update(N, rp, ci, w, W.normal_f32((N, 602), seed=902), ("sum",), f_chunks=(0, 64), what="c1 F=602", seed=2)
    check_update(N, rp, ci, w, W.normal_bf16((N, 100), seed=903), ("sum", "max"), bf16=True, what="c1 bf16", seed=3)
    # a hub row (whole workgroup) and rows split over workgroups keep the epilogue
    N2 = 300
    src2, dst2 = long_rows_graph(N2, [40000, 9000, 300], seed=5)
    rp2, ci2, _, _ = oracle.build_csr(N2, src2, dst2)
    w2 = W.normal_f32((len(ci2),), seed=12)
    check_update(N2, rp2, ci2, w2, W.normal_f32((N2, 33), seed=904), ("wsum", "max"), f_chunks=(0, 8),
                 what="long rows", seed=4)
    # bf16 output: rounded after the activation
    X = W.normal_f32((N, 40), seed=905)
    bias = W.normal_f32((40,), seed=906)
    ref = oracle.update(oracle.aggregate(oracle.WSUM, rp, ci, w, X), bias, True)
    out = torch.empty((N, 40), dtype=torch.bfloat16, device="cuda")
    g.gnnagg_aggregate_update(g.WSUM, dev(rp), dev(ci), dev(w), dev(X), None, dev(bias), True, out, 0,
                              g.gnnagg_plan_rows(dev(rp)))
    got = W.bf16_to_f32(host(out.view(torch.int16)).view(np.uint16))
    assert_close(got, W.bf16_to_f32(W.f32_to_bf16(ref)), bf16=True, what="bf16 out after relu")


@pytest.mark.parametrize("F,H2,bf16", [(32, 32, False), (16, 41, False), (64, 7, False), (8, 1, False), (1, 3, False),
                                       (33, 64, False), (5, 300, False), (32, 16, True), (24, 40, True)])
def test_update_fused_dense_layer_on_the_aggregated_row(F, H2, bf16):
    """act(aggregate(X) W2 + b) in the aggregation kernel against the checker's aggregate then its dense layer:
    every operator, short rows sharing a wavefront, a hub row, rows split over workgroups, pitched rows."""
    N = 700
    src, dst = long_rows_graph(N, [33000, 9000, 700, 70], seed=F * 7 + H2)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    w = W.normal_f32((len(ci),), seed=13, std=0.05)
    X = W.normal_bf16((N, F), seed=910 + F) if bf16 else W.normal_f32((N, F), seed=910 + F)
    W2 = W.normal_f32((F, H2), seed=920 + H2, std=0.3)
    bias = W.normal_f32((H2,), seed=930 + H2)
    d_rp, d_ci, d_w, d_W2, d_b = dev(rp), dev(ci), dev(w), dev(W2), dev(bias)
    plan = g.gnnagg_plan_rows(d_rp)
    d_X = g.pitched_empty(N, F, torch.bfloat16 if bf16 else torch.float32)
    d_X.copy_(dev(X))
    for name in ("sum", "wsum", "mean", "max"):
        gop, rop = OPS[name]
        agg = oracle.aggregate(rop, rp, ci, w, X, threads=8)
        for relu, use_bias, use_plan in ((True, True, True), (False, False, True), (False, True, False)):
            say("  fused layer", name, "F", F, "H2", H2, "relu", relu, "bias", use_bias, "plan", use_plan)
            ref = oracle.combine(agg, W2, bias if use_bias else None, relu, threads=8)
            out = g.pitched_empty(N, H2, torch.float32)
            out.fill_(float("nan"))
            g.gnnagg_aggregate_update(gop, d_rp, d_ci, d_w if name == "wsum" else None, d_X, d_W2,
                                      d_b if use_bias else None, relu, out, 0, plan if use_plan else None)
            assert_close(host(out), ref, what="fused %s relu=%s bias=%s plan=%s" % (name, relu, use_bias, use_plan))
            # the same layer as two calls: identical up to the order of the fp64 additions
            two = g.gnnagg_combine(g.gnnagg_aggregate(gop, d_rp, d_ci, d_w if name == "wsum" else None, d_X, None, 0,
                                                      plan if use_plan else None).contiguous(),
                                   d_W2, d_b if use_bias else None, relu)
            assert_close(host(out), host(two), what="fused vs two calls " + name)


def test_update_layer_on_the_tiny_benchmark_graph_both_orders():
    """One GCN layer act(A X W + b) on the config 1 graph: Combination first then the aggregation with the
    epilogue, and aggregation at a hidden width with the fused dense layer; both against the checker."""
    N, src, dst = W.graph("c1")
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    d_rp, d_ci, d_w = dev(rp), dev(ci), dev(w)
    plan = g.gnnagg_plan_rows(d_rp)
    X = W.bernoulli_f32((N, 1433), 0.013, seed=940)
    W1 = W.normal_f32((1433, 16), seed=941, std=0.1)
    b1 = W.normal_f32((16,), seed=942, std=0.1)
    hid = g.gnnagg_combine(dev(X), dev(W1))
    out = g.gnnagg_aggregate_update(g.WSUM, d_rp, d_ci, d_w, hid, None, dev(b1), True, None, 0, plan)
    ref_hid = oracle.combine(X, W1)
    ref = oracle.update(oracle.aggregate(oracle.WSUM, rp, ci, w, ref_hid), b1, True)
    assert_close(host(out), ref, what="combination first, epilogue")
    W2 = W.normal_f32((16, 7), seed=943, std=0.3)
    b2 = W.normal_f32((7,), seed=944)
    out2 = g.gnnagg_aggregate_update(g.WSUM, d_rp, d_ci, d_w, out, dev(W2), dev(b2), False, None, 0, plan)
    ref2 = oracle.combine(oracle.aggregate(oracle.WSUM, rp, ci, w, ref), W2, b2, False)
    assert_close(host(out2), ref2, what="second layer, fused dense layer")


# ------------------------------------------------------------------ combination (dense layer on the matrix cores)
@pytest.mark.parametrize("N,F,H", [(1, 1, 1), (130, 33, 5), (1000, 602, 32), (257, 100, 200), (513, 64, 129),
                                   (4096, 31, 16), (127, 1433, 8)])
def test_combine_matches_checker(N, F, H):
    Wt = W.normal_f32((F, H), seed=500, std=0.3)
    b = W.normal_f32((H,), seed=501)
    for X in (W.normal_f32((N, F), seed=502), W.normal_bf16((N, F), seed=503)):
        for bias, relu in ((None, False), (b, False), (b, True)):
            ref = oracle.combine(X, Wt, bias, relu, threads=8)
            out = torch.full((N, H), float("nan"), dtype=torch.float32, device="cuda")
            g.gnnagg_combine(dev(X), dev(Wt), dev(bias) if bias is not None else None, relu, out)
            assert_close(host(out), ref, what="combine N=%d F=%d H=%d bias=%s relu=%s" % (N, F, H, bias is not None, relu))


def test_combination_first_equals_aggregation_first():
    # Section III runs Combination ahead of Aggregation; for the linear aggregators both orders agree
    N, src, dst = W.graph("c4", 0.01)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True, threads=8)
    X = W.normal_f32((N, 96), seed=510)
    Wt = W.normal_f32((96, 16), seed=511, std=0.2)
    d_rp, d_ci, d_w, d_X, d_W = dev(rp), dev(ci), dev(w), dev(X), dev(Wt)
    plan = g.gnnagg_plan_rows(d_rp)
    first = g.gnnagg_aggregate(1, d_rp, d_ci, d_w, g.gnnagg_combine(d_X, d_W), None, 0, plan)
    last = g.gnnagg_combine(g.gnnagg_aggregate(1, d_rp, d_ci, d_w, d_X, None, 0, plan), d_W)
    ref = oracle.aggregate(oracle.WSUM, rp, ci, w, oracle.combine(X, Wt, threads=8), threads=8)
    assert_close(host(first), ref, what="combine then aggregate")
    assert np.allclose(host(last), ref, rtol=1e-4, atol=1e-5)  # two fp32 roundings in a different place


# ------------------------------------------------------------------ seeded sweep of small random cases, streams
def test_seeded_sweep_of_small_random_cases():
    """Forty small cases with shapes drawn from a seeded generator: graph size, density, a planted hub,
    feature width, chunk width, input type, operator, with and without a row plan."""
    rng = np.random.default_rng(20240)
    for case in range(40):
        N = int(rng.integers(1, 400))
        E = int(rng.integers(0, 12 * N + 1))
        src, dst = (W.random_digraph(N, E, 7000 + case) if E else (np.zeros(0, np.int32), np.zeros(0, np.int32)))
        if N > 8 and case % 3 == 0:  # a hub row that needs a whole workgroup
            hub_src = rng.integers(0, N, size=int(rng.integers(300, 3000))).astype(np.int32)
            src = np.concatenate([src, hub_src])
            dst = np.concatenate([dst, np.full(len(hub_src), int(rng.integers(0, N)), np.int32)])
        F = int(rng.choice([1, 2, 3, 5, 8, 12, 17, 31, 32, 33, 64, 100, 129, 260, 513]))
        fc = int(rng.choice([0, 0, 1, 3, 4, 8, 16, 50, g.F_CHUNK_AUTO]))
        bf16 = bool(rng.integers(0, 2))
        flags = int(rng.choice([0, oracle.SELF_LOOPS, oracle.SELF_LOOPS | oracle.NORM_SYM]))
        rp, ci, w, _ = oracle.build_csr(N, src, dst, flags, want_w=True)
        X = W.normal_bf16((N, F), seed=8000 + case) if bf16 else W.normal_f32((N, F), seed=8000 + case)
        name = ["sum", "wsum", "mean", "max"][case % 4]
        say("  sweep case", case, "N", N, "nnz", len(ci), "F", F, "fc", fc, "bf16", bf16, name)
        check_aggregate(N, rp, ci, w, X, [name], f_chunks=(fc,), plans=(bool(case & 1),), bf16=bf16,
                        what="sweep %d" % case)


def test_calls_are_ordered_on_the_callers_stream():
    """Work is enqueued on the stream that is current for the caller: a side stream's result is complete
    once that stream is, and back-to-back dependent calls need no synchronisation in between."""
    N, src, dst = W.graph("c2")
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    X = W.normal_f32((N, 48), seed=901)
    Wt = W.normal_f32((48, 16), seed=902, std=0.2)
    d_rp, d_ci, d_w, d_X, d_W = dev(rp), dev(ci), dev(w), dev(X), dev(Wt)
    plan = g.gnnagg_plan_rows(d_rp)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        hid = g.gnnagg_combine(d_X, d_W)
        one = g.gnnagg_aggregate(1, d_rp, d_ci, d_w, hid, None, 0, plan)
        two = g.gnnagg_aggregate(1, d_rp, d_ci, d_w, one, None, 0, plan)  # consumes the previous output
    side.synchronize()
    h = oracle.combine(X, Wt)
    r1 = oracle.aggregate(oracle.WSUM, rp, ci, w, h)
    assert_close(one.cpu().numpy(), r1, what="first hop on a side stream")
    assert_close(two.cpu().numpy(), oracle.aggregate(oracle.WSUM, rp, ci, w, one.cpu().numpy()), what="second hop")


def test_seeded_sweep_of_attention_and_csr_cases():
    rng = np.random.default_rng(4711)
    for case in range(24):
        N = int(rng.integers(1, 300))
        E = int(rng.integers(0, 10 * N + 1))
        src, dst = (W.random_digraph(N, E, 9000 + case) if E else (np.zeros(0, np.int32), np.zeros(0, np.int32)))
        if N > 8 and case % 4 == 0:
            hub_src = rng.integers(0, N, size=int(rng.integers(300, 2500))).astype(np.int32)
            src = np.concatenate([src, hub_src])
            dst = np.concatenate([dst, np.full(len(hub_src), int(rng.integers(0, N)), np.int32)])
        flags = int(rng.choice([0, oracle.SELF_LOOPS, oracle.SELF_LOOPS | oracle.NORM_SYM, oracle.NORM_SYM]))
        rp, ci, w, perm = oracle.build_csr(N, src, dst, flags, want_w=True, want_perm=True)
        d_rp, d_ci, d_w, d_perm = gpu_csr(N, src, dst, flags, want_w=True, want_perm=True)
        what = "sweep %d N=%d E=%d flags=%d" % (case, N, len(src), flags)
        assert np.array_equal(host(d_rp), rp) and np.array_equal(host(d_ci), ci), what
        assert np.array_equal(host(d_perm), perm), what
        assert_bits(host(d_w), w, what)
        heads, C = [(1, 4), (2, 8), (3, 16), (5, 3), (2, 12), (16, 8), (1, 32), (7, 1)][case % 8]
        fc = int(rng.choice([0, C, 2 * C]))
        H = W.normal_f32((N, heads, C), seed=9500 + case)
        a_s = W.normal_f32((heads, C), seed=9600 + case, std=0.7)
        a_d = W.normal_f32((heads, C), seed=9700 + case, std=0.7)
        check_gat(N, rp, ci, H, a_s, a_d, f_chunks=(fc,), plans=(bool(case & 1),), what=what + " %dx%d" % (heads, C))


# ------------------------------------------------------------------ very long rows, split over workgroups
def long_rows_graph(N, lengths, seed):
    """Rows 3, 4, ... receive lengths[k] in-edges from pseudo-random sources; plus a sparse background."""
    rng = np.random.default_rng(seed)
    parts_s, parts_d = [], []
    for k, n in enumerate(lengths):
        parts_s.append(rng.integers(0, N, size=n).astype(np.int32))
        parts_d.append(np.full(n, 3 + k, np.int32))
    s2, d2 = W.random_digraph(N, 4 * N, seed + 1)
    keep = (d2 < 3) | (d2 >= 3 + len(lengths))  # the long rows keep exactly the lengths asked for
    return np.concatenate(parts_s + [s2[keep]]), np.concatenate(parts_d + [d2[keep]])


@pytest.mark.parametrize("F,fc,bf16", [(100, 0, True), (602, 0, False), (33, 8, False), (8, 0, True), (1, 0, False)])
def test_rows_split_over_workgroups_match_the_checker(F, fc, bf16):
    """Rows of 2^15 edges or more are cut into pieces of 2^13 edges when the call has a workspace: piece
    boundaries (32768 = exactly four pieces, 32769, a row one short of a power of two), several degree
    classes, and rows just below the threshold that stay with one workgroup."""
    N = 500
    src, dst = long_rows_graph(N, [32768, 32769, 65535, 40000, 70001, 32767, 9000], seed=F)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    w = W.normal_f32((len(ci),), seed=11)
    X = W.normal_bf16((N, F), seed=600 + F) if bf16 else W.normal_f32((N, F), seed=600 + F)
    d_rp, d_ci, d_w, d_X = dev(rp), dev(ci), dev(w), dev(X)
    plan = g.gnnagg_plan_rows(d_rp)
    need = g.gnnagg_aggregate_workspace_bytes(N, F, plan)
    assert need == (4 * 8 + 16) * F * 8  # class 16 (32768, 32769, 65535, 40000): 8 pieces each; 17 (70001): 16
    for name in ("sum", "wsum", "mean", "max"):
        gop, rop = OPS[name]
        say("  split rows", name, "F", F, "fc", fc)
        ref = oracle.aggregate(rop, rp, ci, w, X, threads=8)
        out = torch.full((N, F), float("nan"), dtype=torch.float32, device="cuda")
        g.gnnagg_aggregate(gop, d_rp, d_ci, d_w if name == "wsum" else None, d_X, out, fc, plan)
        whole = g.gnnagg_aggregate(gop, d_rp, d_ci, d_w if name == "wsum" else None, d_X, None, fc, plan,
                                   split_long_rows=False)
        if name == "max":
            assert_bits(host(out), ref, "split max")
        else:
            assert_close(host(out), ref, bf16, "split " + name)
        assert_close(host(out), host(whole), bf16, "split vs one workgroup per row " + name)
    # bf16 output and a caller-provided workspace that is reused
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    a = g.gnnagg_aggregate(0, d_rp, d_ci, None, d_X, torch.empty((N, F), dtype=torch.bfloat16, device="cuda"), fc,
                           plan, workspace=ws)
    b = g.gnnagg_aggregate(0, d_rp, d_ci, None, d_X, torch.empty((N, F), dtype=torch.bfloat16, device="cuda"), fc,
                           plan, workspace=ws)
    ref = oracle.aggregate(oracle.SUM, rp, ci, None, X, threads=8)
    assert np.array_equal(host(a.view(torch.int16)), host(b.view(torch.int16)))
    assert np.array_equal(host(a.view(torch.int16)).view(np.uint16), W.f32_to_bf16(ref))


@pytest.mark.parametrize("heads,C,fc", [(8, 8, 0), (2, 5, 5), (1, 64, 0), (16, 8, 64)])
def test_attention_rows_split_over_workgroups_match_the_checker(heads, C, fc):
    """Attention on rows of 2^15 edges or more: pieces leave softmax states (reference, denominator,
    weighted sums) in the workspace, the merge kernel folds them, a third kernel writes the weights."""
    N = 400
    src, dst = long_rows_graph(N, [32768, 32769, 50000, 70001, 32767], seed=heads * C)
    rp, ci, _, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS)
    H = W.normal_f32((N, heads, C), seed=700 + C)
    a_s = W.normal_f32((heads, C), seed=701, std=0.6)
    a_d = W.normal_f32((heads, C), seed=702, std=0.6)
    d_rp = dev(rp)
    plan = g.gnnagg_plan_rows(d_rp)
    assert g.gnnagg_gat_workspace_bytes(N, heads, C, plan) > g.gnnagg_gat_workspace_bytes(N, heads, C)
    check_gat(N, rp, ci, H, a_s, a_d, f_chunks=(fc,), plans=(True, False), what="gat split %dx%d" % (heads, C))
    # weights only, and sums only
    ralpha, rout = oracle.gat_attention(rp, ci, H, a_s, a_d, 0.2, threads=8)
    alpha, none = g.gnnagg_gat_attention(d_rp, dev(ci), dev(H), dev(a_s), dev(a_d), 0.2, True, False, fc, plan)
    assert none is None
    assert_close(host(alpha), ralpha, what="weights only")
    sums = host(alpha).astype(np.float64)
    seg = np.add.reduceat(sums, rp[:-1][np.diff(rp) > 0], axis=0)
    assert np.allclose(seg, 1.0, atol=1e-5)


@pytest.mark.parametrize("F,bf16,fc", [(100, True, 0), (602, False, 0), (33, False, 8), (5, True, 0), (130, False, 64)])
def test_row_pitched_input_and_output(F, bf16, fc):
    """X and out as [N, F] views into allocations whose rows start on 128-byte lines: same results as the
    contiguous call; the padding columns are never read (they hold NaN) and never written."""
    N, src, dst = W.graph("c5", 0.004)
    long_s, long_d = long_rows_graph(N, [40000], seed=F)   # one row long enough to be split as well
    src, dst = np.concatenate([src, long_s]), np.concatenate([dst, long_d])
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    w = W.normal_f32((len(ci),), seed=12)
    X = W.normal_bf16((N, F), seed=800 + F) if bf16 else W.normal_f32((N, F), seed=800 + F)
    dt = torch.bfloat16 if bf16 else torch.float32
    pitch = g.gnnagg_row_pitch(F, dt)
    row_bytes = pitch * (2 if bf16 else 4)
    assert pitch >= F and (row_bytes % 128 == 0 or (row_bytes < 128 and row_bytes & (row_bytes - 1) == 0))
    Xp = g.pitched_empty(N, F, dt)
    assert Xp.stride(0) == pitch
    Xp.untyped_storage().fill_(0xFF)  # all-ones bit patterns: NaN in both types
    Xp.copy_(dev(X))
    d_rp, d_ci, d_w = dev(rp), dev(ci), dev(w)
    plan = g.gnnagg_plan_rows(d_rp)
    for name in ("sum", "wsum", "mean", "max"):
        gop, rop = OPS[name]
        ref = oracle.aggregate(rop, rp, ci, w, X, threads=8)
        out = g.pitched_empty(N, F, torch.float32)
        base = torch.full((N, out.stride(0)), -7.0, dtype=torch.float32, device="cuda")
        out = base[:, :F]
        g.gnnagg_aggregate(gop, d_rp, d_ci, d_w if name == "wsum" else None, Xp, out, fc, plan)
        got = host(out)
        if name == "max":
            assert_bits(got, ref, "pitched max")
        else:
            assert_close(got, ref, bf16, "pitched " + name)
        assert bool((base[:, F:] == -7.0).all()), "padding columns were written"
        # a pitched input with a contiguous output, and the other way round
        flat = g.gnnagg_aggregate(gop, d_rp, d_ci, d_w if name == "wsum" else None, Xp, None, fc, plan)
        assert np.array_equal(host(flat).view(np.uint32), got.view(np.uint32))
        out2 = torch.full((N, out.stride(0)), -7.0, dtype=torch.float32, device="cuda")[:, :F]
        g.gnnagg_aggregate(gop, d_rp, d_ci, d_w if name == "wsum" else None, dev(X), out2, fc, plan)
        assert np.array_equal(host(out2).view(np.uint32), got.view(np.uint32))


# ------------------------------------------------------------------ feature rows stored in popularity order
def test_rank_sources_and_gather_from_ranked_rows():
    """rank orders the vertices by how often they are gathered (ties by id); aggregating (colidx_ranked, X stored
    by rank) gives bit for bit what (colidx, X) gives; Combination can write its rows by rank."""
    N, src, dst = W.graph("c5", 0.01)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    d_rp, d_ci = dev(rp), dev(ci)
    rank, ranked = g.gnnagg_rank_sources(N, d_ci)
    rank_h, ranked_h = host(rank), host(ranked)
    count = np.bincount(ci, minlength=N)
    want_order = np.lexsort((np.arange(N), -count))          # most frequent first, ties by id
    want_rank = np.empty(N, np.int32)
    want_rank[want_order] = np.arange(N, dtype=np.int32)
    assert np.array_equal(rank_h, want_rank)
    assert np.array_equal(ranked_h, want_rank[ci])
    plan = g.gnnagg_plan_rows(d_rp)
    X = W.normal_f32((N, 24), seed=950)
    Wt = W.normal_f32((24, 16), seed=951, std=0.3)
    hid = g.gnnagg_combine(dev(X), dev(Wt))
    hid_r = g.gnnagg_combine(dev(X), dev(Wt), out_rows=rank)
    assert_close(host(hid), oracle.combine(X, Wt), what="combine")
    assert np.array_equal(host(hid_r)[rank_h].view(np.uint32), host(hid).view(np.uint32))
    for gop in (0, 2, 3):
        a = g.gnnagg_aggregate(gop, d_rp, d_ci, None, hid, None, 0, plan)
        b = g.gnnagg_aggregate(gop, d_rp, ranked, None, hid_r, None, 0, plan)
        assert np.array_equal(host(a).view(np.uint32), host(b).view(np.uint32)), gop
    ref = oracle.aggregate(oracle.SUM, rp, ci, None, host(hid))
    assert_close(host(g.gnnagg_aggregate(0, d_rp, ranked, None, hid_r, None, 0, plan)), ref, what="ranked sum")
    # a graph without edges and a single vertex
    r1, c1 = g.gnnagg_rank_sources(3, torch.empty(0, dtype=torch.int32, device="cuda"))
    assert host(r1).tolist() == [0, 1, 2] and c1.numel() == 0


# ------------------------------------------------------------------ HIP graph capture of the enqueue-only calls
def test_calls_can_be_captured_in_a_graph_and_replayed():
    """Combination, aggregation and attention only enqueue kernels (no allocation, no synchronisation, no
    memset), so a layer can be captured once and replayed: every replay, with fresh inputs copied in place
    and ordinary eager work in between, must give the bits of the eager call."""
    N, src, dst = W.graph("c2")
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    d_rp, d_ci, d_w = dev(rp), dev(ci), dev(w)
    plan = g.gnnagg_plan_rows(d_rp)
    Wt = dev(W.normal_f32((48, 64), seed=971, std=0.2))
    a_s, a_d = dev(W.normal_f32((8, 8), seed=972, std=0.1)), dev(W.normal_f32((8, 8), seed=973, std=0.1))
    X = torch.zeros((N, 48), dtype=torch.float32, device="cuda")
    hid = torch.empty((N, 64), dtype=torch.float32, device="cuda")
    agg = torch.empty((N, 64), dtype=torch.float32, device="cuda")
    att = torch.empty((N, 8, 8), dtype=torch.float32, device="cuda")
    ws = torch.empty(g.gnnagg_gat_workspace_bytes(N, 8, 8, plan), dtype=torch.uint8, device="cuda")

    def layer():
        g.gnnagg_combine(X, Wt, None, True, hid)
        g.gnnagg_aggregate(g.WSUM, d_rp, d_ci, d_w, hid, agg, 0, plan)
        g.gnnagg_gat_attention(d_rp, d_ci, hid.view(N, 8, 8), a_s, a_d, 0.2, False, True, 0, plan, out=att, workspace=ws)

    layer()  # eager once: code objects loaded, nothing left to allocate
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer()
    for k in range(4):
        X.copy_(dev(W.normal_f32((N, 48), seed=980 + k)))
        graph.replay()
        torch.cuda.synchronize()
        got_agg, got_att = agg.clone(), att.clone()
        agg.zero_()
        att.zero_()
        layer()  # eager, same inputs
        torch.cuda.synchronize()
        assert torch.equal(got_agg, agg) and torch.equal(got_att, att), "replay %d differs from the eager call" % k
        ref = oracle.aggregate(oracle.WSUM, rp, ci, w, oracle.combine(host(X), host(Wt), None, True))
        assert_close(host(agg), ref, what="captured layer, replay %d" % k)


def test_check_csr_accepts_built_graphs_and_rejects_broken_ones():
    N, src, dst = W.graph("c2")
    rp, ci, _, _ = gpu_csr(N, src, dst, oracle.SELF_LOOPS)
    assert g.gnnagg_check_csr(rp, ci)
    bad = ci.clone()
    bad[1234] = N            # a source that does not exist
    assert not g.gnnagg_check_csr(rp, bad)
    bad[1234] = -1
    assert not g.gnnagg_check_csr(rp, bad)
    rp2 = rp.clone()
    rp2[100], rp2[101] = rp[101].item() + 1, rp[100].item()   # a row that ends before it starts
    assert not g.gnnagg_check_csr(rp2, ci)
    rp3 = rp.clone()
    rp3[N] = rp[N] + 5       # claims more entries than colidx holds
    assert not g.gnnagg_check_csr(rp3, ci)
    empty = torch.zeros(4, dtype=torch.int64, device="cuda")
    assert g.gnnagg_check_csr(empty, torch.empty(0, dtype=torch.int32, device="cuda"))
