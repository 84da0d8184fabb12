"""GPU parity of the blocked aggregation (gnnagg_plan_source_blocks + gnnagg_aggregate_blocked): the sources
are cut into B blocks of consecutive ids, every block is one pass of the aggregation kernels, and a
destination's state travels from block to block as doubles.  The result has to meet the same bars as the
plain call against the CPU checker: max bit for bit, sums within 1e-6 + 1e-5 |r|."""
import sys

import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

g = None
OPS = {"sum": (0, oracle.SUM), "wsum": (1, oracle.WSUM), "mean": (2, oracle.MEAN), "max": (3, oracle.MAX)}


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


def assert_close(got, ref, what):
    ok = np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= 1e-6 + 1e-5 * np.abs(ref.astype(np.float64))
    if not ok.all():
        bad = np.argwhere(~ok)
        i = tuple(bad[0])
        raise AssertionError("%s: %d of %d elements off, first at %s: got %r want %r" %
                             (what, len(bad), ok.size, i, got[i], ref[i]))


def assert_bits(got, ref, what):
    a, b = got.view(np.uint32), ref.view(np.uint32)
    if not np.array_equal(a, b):
        bad = np.argwhere(a != b)
        i = tuple(bad[0])
        raise AssertionError("%s: %d elements differ bitwise, first at %s: got %r want %r" %
                             (what, len(bad), i, got[i], ref[i]))


def check_blocked(N, rp, ci, w, X, Bs, f_chunks, what, ops=("sum", "wsum", "mean", "max"), pitched=False):
    d_rp, d_ci, d_w = dev(rp), dev(ci), dev(w)
    F = X.shape[1]
    if pitched:
        d_X = g.pitched_empty(N, F, torch.bfloat16 if X.dtype == np.uint16 else torch.float32)
        d_X.untyped_storage().fill_(0xFF)  # NaN in the padding columns: they must never be read
        d_X.copy_(dev(X))
    else:
        d_X = dev(X)
    refs = {name: oracle.aggregate(OPS[name][1], rp, ci, w, X, threads=8) for name in ops}
    for B in Bs:
        blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, B)
        # the table itself: block b of row r is the run of its (ascending) sources inside block b's id range
        bp = host(blocks.block_ptr)[: (B + 1) * N].reshape(B + 1, N)
        per = -(-N // B)
        assert np.array_equal(bp[0], rp[:-1]) and np.array_equal(bp[B], rp[1:])
        assert (np.diff(bp, axis=0) >= 0).all()
        for r in np.random.default_rng(B).choice(N, size=min(N, 50), replace=False):
            srcs = ci[rp[r]:rp[r + 1]]
            want = rp[r] + np.searchsorted(srcs, np.arange(B + 1) * per, side="left")
            want[B] = rp[r + 1]
            assert np.array_equal(bp[:, r], want), (B, r)
        order = host(blocks.row_order)[: B * N].reshape(B, N)
        for b in range(B):  # every block's order is a permutation of the rows, by that block's degree
            assert np.array_equal(np.sort(order[b]), np.arange(N))
            deg = (bp[b + 1] - bp[b])[order[b]]
            assert (np.diff(deg) <= 0).all()
        for name in ops:
            gop, _ = OPS[name]
            for fc in f_chunks:
                say("  blocked", what, name, "B", B, "f_chunk", fc)
                if pitched:
                    base = torch.full((N, g.gnnagg_row_pitch(F)), -7.0, dtype=torch.float32, device="cuda")
                    out = base[:, :F]
                else:
                    out = torch.full((N, F), float("nan"), dtype=torch.float32, device="cuda")
                g.gnnagg_aggregate_blocked(gop, d_rp, d_ci, d_w if name == "wsum" else None, d_X, blocks, out, fc)
                got = host(out)
                tag = "%s %s B=%d fc=%d" % (what, name, B, fc)
                if name == "max":
                    assert_bits(got, refs[name], tag)
                else:
                    assert_close(got, refs[name], tag)
                if pitched:
                    assert bool((base[:, F:] == -7.0).all()), "padding columns were written"


@pytest.mark.parametrize("key,scale,F", [("c4", 0.02, 602), ("c4", 0.02, 32), ("c5", 0.01, 100), ("c2", 1.0, 500),
                                         ("c1", 1.0, 7)])
def test_blocked_matches_the_checker_on_benchmark_shapes(key, scale, F):
    N, src, dst = W.graph(key, scale)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    X = W.normal_f32((N, F), seed=40 + F)
    check_blocked(N, rp, ci, w, X, Bs=(1, 2, 3, 8), f_chunks=(0, 32, g.F_CHUNK_AUTO), what="%s F=%d" % (key, F),
                  pitched=(F % 32 != 0))


def test_blocked_bf16_input_and_bf16_output():
    N, src, dst = W.graph("c5", 0.01)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    w = W.normal_f32((len(ci),), seed=3)
    X = W.normal_bf16((N, 200), seed=77)
    check_blocked(N, rp, ci, w, X, Bs=(2, 5), f_chunks=(0, 128, g.F_CHUNK_AUTO), what="bf16", pitched=True)
    d_rp, d_ci, d_X = dev(rp), dev(ci), dev(X)
    blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, 4)
    out = torch.empty((N, 200), dtype=torch.bfloat16, device="cuda")
    g.gnnagg_aggregate_blocked(0, d_rp, d_ci, None, d_X, blocks, out, 0)
    ref = oracle.aggregate(oracle.SUM, rp, ci, None, X, threads=8)
    assert np.array_equal(host(out.view(torch.int16)).view(np.uint16), W.f32_to_bf16(ref))


@pytest.mark.parametrize("F,fc", [(100, 0), (33, 8), (602, 32)])
def test_blocked_with_rows_split_over_workgroups(F, fc):
    """Rows long enough to be cut into pieces inside a block (2^15 edges or more from one block's sources), rows
    that are long only as a whole, empty rows and rows with all sources in one block."""
    N = 600
    rng = np.random.default_rng(F)
    parts_s, parts_d = [], []
    for k, (n, lo, hi) in enumerate([(70000, 0, N), (40000, 0, 150), (33000, 450, 600), (90000, 0, N), (20000, 0, N)]):
        parts_s.append(rng.integers(lo, hi, size=n).astype(np.int32))
        parts_d.append(np.full(n, 3 + k, np.int32))
    s2, d2 = W.random_digraph(N, 4 * N, 5)
    keep = (d2 < 3) | (d2 >= 20)
    src, dst = np.concatenate(parts_s + [s2[keep]]), np.concatenate(parts_d + [d2[keep]])
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    assert (np.diff(rp) == 0).any()
    w = W.normal_f32((len(ci),), seed=11)
    X = W.normal_f32((N, F), seed=600 + F)
    check_blocked(N, rp, ci, w, X, Bs=(1, 2, 4), f_chunks=(fc,), what="split rows F=%d" % F)


def test_blocked_states_in_transit_are_exact_for_integer_data():
    """Integer-valued features: every partial sum is exact, so the blocked result equals the plain call bit for bit
    whatever B is (the states carried between blocks lose nothing)."""
    N, src, dst = W.graph("c4", 0.01)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    X = np.random.default_rng(2).integers(-50, 50, size=(N, 70)).astype(np.float32)
    d_rp, d_ci, d_X = dev(rp), dev(ci), dev(X)
    plain = host(g.gnnagg_aggregate(0, d_rp, d_ci, None, d_X, None, 0, g.gnnagg_plan_rows(d_rp)))
    ref = oracle.aggregate(oracle.SUM, rp, ci, None, X, threads=8)
    assert np.array_equal(plain, ref)
    for B in (2, 7, 64):
        blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, B)
        assert np.array_equal(host(g.gnnagg_aggregate_blocked(0, d_rp, d_ci, None, d_X, blocks, None, 0)), ref), B


def test_blocked_twice_in_a_row_with_one_workspace_gives_the_same_bits():
    N, src, dst = W.graph("c4", 0.01)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    X = W.normal_f32((N, 96), seed=8)
    d_rp, d_ci, d_X = dev(rp), dev(ci), dev(X)
    blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, 3)
    need = g.gnnagg_aggregate_blocked_workspace_bytes(N, 96, blocks)
    assert need >= 2 * N * 96 * 8
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    a = host(g.gnnagg_aggregate_blocked(2, d_rp, d_ci, None, d_X, blocks, None, 32, workspace=ws))
    ws.fill_(0xFF)  # whatever the workspace holds beforehand must not matter
    b = host(g.gnnagg_aggregate_blocked(2, d_rp, d_ci, None, d_X, blocks, None, 32, workspace=ws))
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    small = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(g.GnnaggError) as e:
        g.gnnagg_aggregate_blocked(2, d_rp, d_ci, None, d_X, blocks, None, 32, workspace=small)
    assert e.value.status == -4


def test_plan_source_blocks_rejects_rows_that_are_not_ascending_and_bad_block_counts():
    rp = np.array([0, 3, 5], np.int64)
    ci = np.array([0, 1, 1, 1, 0], np.int32)  # row 1 lists 1 before 0
    with pytest.raises(g.GnnaggError) as e:
        g.gnnagg_plan_source_blocks(dev(rp), dev(ci), 2)
    assert e.value.status == -1
    ci_ok = np.array([0, 1, 1, 0, 1], np.int32)
    blocks = g.gnnagg_plan_source_blocks(dev(rp), dev(ci_ok), 2)
    assert host(blocks.block_ptr)[:6].tolist() == [0, 3, 1, 4, 3, 5]
    for B in (0, -1, 65):
        with pytest.raises(g.GnnaggError) as e:
            g.gnnagg_plan_source_blocks(dev(rp), dev(ci_ok), B)
        assert e.value.status == -1


def test_measured_tuner_of_the_blocked_call_returns_a_valid_width_and_leaves_a_valid_result():
    N, src, dst = W.graph("c4", 0.02)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    F = 300
    X = W.normal_f32((N, F), seed=21)
    d_rp, d_ci, d_w = dev(rp), dev(ci), dev(w)
    Xp = g.pitched_empty(N, F, torch.float32)
    Xp.copy_(dev(X))
    out = g.pitched_empty(N, F, torch.float32)
    ref = oracle.aggregate(oracle.WSUM, rp, ci, w, X, threads=8)
    times = {}
    for B in (1, 2, 4):
        blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, B)
        out.fill_(float("nan"))
        width, ms = g.gnnagg_tune_blocked(g.WSUM, d_rp, d_ci, d_w, Xp, out, blocks)
        assert width in (32, 64, 128) and ms > 0.0, (B, width, ms)
        assert_close(host(out), ref, "after tuning with %d blocks" % B)   # the last timed call left a whole result
        times[B] = ms
    plain_width, plain_ms = g.gnnagg_tune_f_chunk(g.WSUM, d_rp, d_ci, d_w, Xp, out, g.gnnagg_plan_rows(d_rp))
    assert plain_ms > 0.0 and plain_width > 0
    say("  tuned: plain %.3f ms at %d; blocked %s" % (plain_ms, plain_width, times))


def test_blocked_call_can_be_captured_in_a_graph_and_replayed():
    """The blocked call only enqueues kernels, so it can be captured once and replayed: every replay, with fresh
    inputs copied in place and eager work in between, gives the bits of the eager call."""
    N, src, dst = W.graph("c4", 0.01)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    d_rp, d_ci, d_w = dev(rp), dev(ci), dev(w)
    blocks = g.gnnagg_plan_source_blocks(d_rp, d_ci, 3)
    F = 160
    X = torch.zeros((N, F), dtype=torch.float32, device="cuda")
    out = torch.empty((N, F), dtype=torch.float32, device="cuda")
    ws = torch.empty(g.gnnagg_aggregate_blocked_workspace_bytes(N, F, blocks), dtype=torch.uint8, device="cuda")

    def call():
        g.gnnagg_aggregate_blocked(g.WSUM, d_rp, d_ci, d_w, X, blocks, out, 32, workspace=ws)

    call()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for k in range(3):
        Xh = W.normal_f32((N, F), seed=990 + k)
        X.copy_(dev(Xh))
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        out.zero_()
        ws.fill_(0x7F)
        call()
        torch.cuda.synchronize()
        assert torch.equal(got, out), "replay %d differs from the eager call" % k
        assert_close(host(out), oracle.aggregate(oracle.WSUM, rp, ci, w, Xh, threads=8), "captured blocked call %d" % k)
