"""Pins for the CPU checker: every expected value here comes from something
other than the checker itself - a hand-verifiable worked example on the
paper's Fig. 2 topology, dense brute force written with numpy, scipy's
sparse routines, closed forms and invariants.  CPU only."""
import os

import numpy as np
import pytest
import scipy.sparse as sp
import scipy.special

import oracle
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "star_fig2.txt")


def read_golden(path):
    sections, cur = {}, None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line[0].isalpha():
            cur = line
            sections[cur] = []
        else:
            sections[cur].append([float(t) for t in line.split()])
    return {k: np.array(v) for k, v in sections.items()}


# ---------------------------------------------------------------- helpers
def dense_count(N, src, dst, self_loops=False):
    """C[i, j] = number of edges j -> i (numpy brute force)."""
    C = np.zeros((N, N), dtype=np.float64)
    for s, d in zip(src.tolist(), dst.tolist()):
        C[d, s] += 1.0
    if self_loops:
        C += np.eye(N)
    return C


def brute_csr(N, src, dst, self_loops=False):
    s = list(src.tolist())
    d = list(dst.tolist())
    if self_loops:
        s += list(range(N))
        d += list(range(N))
    rowptr, colidx, perm = [0], [], []
    for i in range(N):
        ent = sorted((s[k], k) for k in range(len(s)) if d[k] == i)
        colidx += [e[0] for e in ent]
        perm += [e[1] for e in ent]
        rowptr.append(len(colidx))
    return np.array(rowptr, np.int64), np.array(colidx, np.int32), np.array(perm, np.int64)


def tiny_graphs():
    out = []
    for seed, (N, E) in enumerate([(5, 9), (17, 60), (33, 300), (64, 257), (8, 0)]):
        src, dst = W.random_digraph(N, E, seed + 100) if E else (np.zeros(0, np.int32), np.zeros(0, np.int32))
        out.append((N, src, dst))
    return out


# ---------------------------------------------------------------- golden
def test_star_example_matches_hand_values():
    g = read_golden(GOLDEN)
    src = g["edges"][:, 0].astype(np.int32)
    dst = g["edges"][:, 1].astype(np.int32)
    X = g["features"].astype(np.float32)
    rowptr, colidx, _, perm = oracle.build_csr(4, src, dst, want_perm=True)
    assert rowptr.tolist() == g["rowptr"].ravel().astype(int).tolist()
    assert colidx.tolist() == g["colidx"].ravel().astype(int).tolist()
    assert perm.tolist() == g["perm"].ravel().astype(int).tolist()
    for name, op in [("sum", oracle.SUM), ("mean", oracle.MEAN), ("max", oracle.MAX)]:
        for fc in (0, 2, 1, 3):  # P = 1, 2 (the figure's case), 4, and a ragged split
            for form in (0, 1):
                got = oracle.aggregate(op, rowptr, colidx, None, X, f_chunk=fc, form=form)
                assert np.array_equal(got, g[name].astype(np.float32)), (name, fc, form)
    rp, ci, w, _ = oracle.build_csr(4, src, dst, flags=oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    assert ci[rp[0]:rp[1]].tolist() == [0, 1, 2, 3]
    assert np.array_equal(w[rp[0]:rp[1]], g["gcn_w_row0"].ravel().astype(np.float32))


# ---------------------------------------------------------------- CSR
@pytest.mark.parametrize("loops", [False, True])
def test_csr_matches_brute_force(loops):
    for N, src, dst in tiny_graphs():
        rp, ci, _, perm = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS if loops else 0, want_perm=True)
        brp, bci, bperm = brute_csr(N, src, dst, loops)
        assert np.array_equal(rp, brp) and np.array_equal(ci, bci) and np.array_equal(perm, bperm)


def test_csr_direction_rows_are_destinations():
    # one edge 2 -> 5: row 5 must list source 2, row 2 must be empty
    rp, ci, _, _ = oracle.build_csr(8, np.array([2], np.int32), np.array([5], np.int32))
    assert rp.tolist() == [0, 0, 0, 0, 0, 0, 1, 1, 1] and ci.tolist() == [2]


def test_csr_invariants_and_shuffle_invariance():
    N, src, dst = W.graph("c2")
    rp, ci, _, perm = oracle.build_csr(N, src, dst, want_perm=True)
    assert rp[0] == 0 and rp[-1] == len(src) and np.all(np.diff(rp) >= 0)
    assert np.array_equal(np.sort(perm), np.arange(len(src)))
    rows = np.repeat(np.arange(N), np.diff(rp))
    assert np.array_equal(dst[perm], rows) and np.array_equal(src[perm], ci)
    # sorted within each row: (row, col) pairs non-decreasing lexicographically
    key = rows.astype(np.int64) * N + ci
    assert np.all(np.diff(key) >= 0)
    sh = np.random.default_rng(0).permutation(len(src))
    rp2, ci2, _, _ = oracle.build_csr(N, src[sh], dst[sh])
    assert np.array_equal(rp, rp2) and np.array_equal(ci, ci2)


def test_csr_matches_scipy_on_simple_graph():
    N, src, dst = W.graph("c1")
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    A = sp.coo_matrix((np.ones(len(src)), (dst, src)), shape=(N, N)).tocsr()
    A.sort_indices()
    assert np.array_equal(rp, A.indptr.astype(np.int64)) and np.array_equal(ci, A.indices.astype(np.int32))


def test_csr_rejects_out_of_range():
    with pytest.raises(ValueError):
        oracle.build_csr(4, np.array([0, 4], np.int32), np.array([1, 1], np.int32))


def test_gcn_weights_closed_form():
    N, src, dst = W.graph("c1")
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    deg = np.bincount(dst, minlength=N).astype(np.float64) + 1.0
    rows = np.repeat(np.arange(N), np.diff(rp))
    expect = (1.0 / np.sqrt(deg[rows] * deg[ci])).astype(np.float32)
    assert np.array_equal(w, expect)


# ---------------------------------------------------------------- sum / wsum
def test_sum_wsum_match_dense_brute_force():
    for k, (N, src, dst) in enumerate(tiny_graphs()):
        X = W.normal_f32((N, 7), seed=k)
        C = dense_count(N, src, dst)
        rp, ci, _, _ = oracle.build_csr(N, src, dst)
        got = oracle.aggregate(oracle.SUM, rp, ci, None, X)
        assert np.array_equal(got, (C @ X.astype(np.float64)).astype(np.float32)) or \
            np.allclose(got, C @ X.astype(np.float64), rtol=1e-6, atol=1e-6)
        # weighted: arbitrary per-edge weights against a dense weight matrix
        w = W.normal_f32((len(ci),), seed=50 + k)
        Wd = np.zeros((N, N))
        rows = np.repeat(np.arange(N), np.diff(rp))
        np.add.at(Wd, (rows, ci), w.astype(np.float64))
        gotw = oracle.aggregate(oracle.WSUM, rp, ci, w, X)
        assert np.allclose(gotw, Wd @ X.astype(np.float64), rtol=1e-6, atol=1e-6)


def test_gcn_matches_dense_normalised_adjacency():
    for k, (N, src, dst) in enumerate(tiny_graphs()):
        X = W.normal_f32((N, 5), seed=k + 7)
        C = dense_count(N, src, dst, self_loops=True)
        d = C.sum(axis=1)
        Ahat = C / np.sqrt(np.outer(d, d))
        rp, ci, w, _ = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
        got = oracle.aggregate(oracle.WSUM, rp, ci, w, X)
        assert np.allclose(got, Ahat @ X.astype(np.float64), rtol=2e-6, atol=1e-6)


# ---------------------------------------------------------------- GCN in factored form
def test_gcn_factors_closed_form():
    # rows of 0, 1, 4, 16 and 3 in-edges: 0, 1, 1/2, 1/4 exactly, and 1/sqrt(3) rounded once
    deg = [0, 1, 4, 16, 3]
    rp = np.concatenate([[0], np.cumsum(deg)]).astype(np.int64)
    s = oracle.gcn_factors(rp)
    assert s.dtype == np.float32
    assert s[:4].tolist() == [0.0, 1.0, 0.5, 0.25]
    assert s[4] == np.float32(1.0 / np.sqrt(3.0))
    N, src, dst = W.graph("c1")
    rp, _, _, _ = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS)
    d = np.bincount(dst, minlength=N).astype(np.float64) + 1.0
    assert np.array_equal(oracle.gcn_factors(rp), (1.0 / np.sqrt(d)).astype(np.float32))


def test_scale_rows_is_the_rounded_fp32_product():
    X = W.normal_f32((23, 9), seed=3)
    s = W.normal_f32((23,), seed=4)
    assert np.array_equal(oracle.scale_rows(X, s), X * s[:, None])          # numpy's fp32 product rounds correctly
    assert np.array_equal(oracle.scale_rows(X, np.full(23, 0.25, np.float32)), X / 4)   # a power of two: exact
    B = W.normal_bf16((23, 9), seed=5)
    assert np.array_equal(oracle.scale_rows(B, s), W.bf16_to_f32(B) * s[:, None])
    # the factor belongs to the ROW (a transposed operand scales columns): row 1 only
    one = np.zeros(23, np.float32)
    one[1] = 2.0
    got = oracle.scale_rows(X, one)
    assert np.array_equal(got[1], 2 * X[1]) and not got[[0] + list(range(2, 23))].any()


def test_scaled_sum_matches_dense_brute_force_and_its_special_cases():
    for k, (N, src, dst) in enumerate(tiny_graphs()):
        X = W.normal_f32((N, 6), seed=20 + k)
        C = dense_count(N, src, dst)
        rp, ci, _, _ = oracle.build_csr(N, src, dst)
        s = W.normal_f32((N,), seed=30 + k)
        got = oracle.aggregate(oracle.SUM_SCALED, rp, ci, s, X)
        assert np.allclose(got, s.astype(np.float64)[:, None] * (C @ X.astype(np.float64)), rtol=1e-6, atol=1e-6)
        plain = oracle.aggregate(oracle.SUM, rp, ci, None, X)
        # factor 1: the plain sum, bit for bit; a power of two: the plain sum scaled exactly
        assert np.array_equal(oracle.aggregate(oracle.SUM_SCALED, rp, ci, np.ones(N, np.float32), X), plain)
        assert np.array_equal(oracle.aggregate(oracle.SUM_SCALED, rp, ci, np.full(N, -0.5, np.float32), X), -plain / 2)
        # the factor is the DESTINATION's: only row 0's factor moves row 0
        s2 = s.copy()
        s2[0] += 1.0
        got2 = oracle.aggregate(oracle.SUM_SCALED, rp, ci, s2, X)
        assert np.array_equal(got2[1:], got[1:])
        if rp[1] > rp[0] and np.abs(plain[0]).max() > 1e-3:
            assert not np.array_equal(got2[0], got[0])
        assert np.array_equal(oracle.aggregate_rows(oracle.SUM_SCALED, np.arange(N), rp, ci, s, X), got)


@pytest.mark.parametrize("key", ["c1", "c2"])
def test_factored_gcn_is_the_gcn_weighted_sum_up_to_the_rounding_of_the_weights(key):
    # s_i * sum_j (s_j x_j) against sum_j fl(1/sqrt(d_i d_j)) x_j, the latter pinned above against scipy and the
    # dense normalised adjacency.  Each term differs by at most three roundings to fp32 (s_i, s_j, s_j x_j) on one
    # side and one (the edge weight) on the other: 4 * 2^-24 of the sum of the terms' magnitudes, plus half an ulp
    # of each result.
    N, src, dst = W.graph(key)
    X = W.normal_f32((N, 19), seed=8)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    s = oracle.gcn_factors(rp)
    got = oracle.aggregate(oracle.SUM_SCALED, rp, ci, s, oracle.scale_rows(X, s))
    ref = oracle.aggregate(oracle.WSUM, rp, ci, w, X)
    mag = oracle.aggregate(oracle.WSUM, rp, ci, w, np.abs(X))
    assert np.all(np.abs(got.astype(np.float64) - ref) <= 4 * 2.0 ** -24 * mag + 2.0 ** -23 * np.abs(ref))
    assert np.abs(got - ref).max() > 0          # and they are two roundings of it, not one computation


@pytest.mark.parametrize("key", ["c1", "c2"])
def test_sum_matches_scipy_spmm(key):
    N, src, dst = W.graph(key)
    F = 37
    X = W.normal_f32((N, F), seed=11)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    A = sp.csr_matrix((w.astype(np.float64), ci, rp), shape=(N, N))
    ref = A @ X.astype(np.float64)
    got = oracle.aggregate(oracle.WSUM, rp, ci, w, X)
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-7)


def test_sum_of_ones_is_degree_exactly():
    N, src, dst = W.graph("c2")
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    got = oracle.aggregate(oracle.SUM, rp, ci, None, np.ones((N, 3), np.float32))
    assert np.array_equal(got, np.repeat(np.diff(rp)[:, None], 3, axis=1).astype(np.float32))


def test_gcn_sqrt_degree_is_fixed_point():
    # x_j = sqrt(d_j) is an eigenvector of D^-1/2 (A+I) D^-1/2 with eigenvalue 1
    N, src, dst = W.graph("c1")
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    d = np.diff(rp).astype(np.float64)
    X = np.sqrt(d)[:, None].astype(np.float32)
    got = oracle.aggregate(oracle.WSUM, rp, ci, w, X)
    assert np.allclose(got[:, 0], np.sqrt(d), rtol=1e-6)


def test_wsum_symmetry_of_normalised_operator():
    N, src, dst = W.graph("c1")
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    x = W.normal_f32((N, 1), seed=1)
    y = W.normal_f32((N, 1), seed=2)
    Ax = oracle.aggregate(oracle.WSUM, rp, ci, w, x).astype(np.float64)
    Ay = oracle.aggregate(oracle.WSUM, rp, ci, w, y).astype(np.float64)
    assert abs(float((y.T @ Ax)[0, 0]) - float((x.T @ Ay)[0, 0])) < 1e-4


# ---------------------------------------------------------------- mean
def test_mean_constant_and_isolated():
    N, src, dst = W.graph("c2")
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    deg = np.diff(rp)
    assert (deg == 0).any()  # config 2 allows isolated vertices
    got = oracle.aggregate(oracle.MEAN, rp, ci, None, np.full((N, 2), 2.5, np.float32))
    assert np.array_equal(got[deg > 0], np.full((int((deg > 0).sum()), 2), 2.5, np.float32))
    assert np.array_equal(got[deg == 0], np.zeros((int((deg == 0).sum()), 2), np.float32))


def test_mean_matches_dense_and_excludes_self():
    for k, (N, src, dst) in enumerate(tiny_graphs()):
        X = W.normal_f32((N, 4), seed=k + 20)
        C = dense_count(N, src, dst)
        d = C.sum(axis=1, keepdims=True)
        ref = np.where(d > 0, (C @ X.astype(np.float64)) / np.maximum(d, 1), 0.0)
        rp, ci, _, _ = oracle.build_csr(N, src, dst)
        got = oracle.aggregate(oracle.MEAN, rp, ci, None, X)
        assert np.allclose(got, ref, rtol=1e-6, atol=1e-7)


def test_mean_one_hot_gives_multiplicity_over_degree():
    src, dst = W.random_digraph(20, 120, 5)
    rp, ci, _, _ = oracle.build_csr(20, src, dst)
    C = dense_count(20, src, dst)
    j = 3
    X = np.zeros((20, 1), np.float32)
    X[j] = 1.0
    got = oracle.aggregate(oracle.MEAN, rp, ci, None, X)[:, 0]
    d = C.sum(axis=1)
    ref = np.where(d > 0, C[:, j] / np.maximum(d, 1), 0)
    assert np.allclose(got, ref, rtol=1e-7)


# ---------------------------------------------------------------- max
def test_max_of_vertex_id_is_last_neighbour():
    N, src, dst = W.graph("c2")
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    X = np.arange(N, dtype=np.float32)[:, None].repeat(2, axis=1)
    got = oracle.aggregate(oracle.MAX, rp, ci, None, X)
    deg = np.diff(rp)
    last = np.where(deg > 0, ci[np.maximum(rp[1:] - 1, 0)], 0).astype(np.float32)
    assert np.array_equal(got[:, 0], last) and np.array_equal(got[:, 1], last)


def test_max_matches_dense_masked_max_and_is_order_independent():
    for k, (N, src, dst) in enumerate(tiny_graphs()):
        X = W.normal_f32((N, 6), seed=k + 30)
        C = dense_count(N, src, dst)
        ref = np.zeros((N, 6), np.float32)
        for i in range(N):
            nb = np.nonzero(C[i])[0]
            if len(nb):
                ref[i] = X[nb].max(axis=0)
        rp, ci, _, _ = oracle.build_csr(N, src, dst)
        got = oracle.aggregate(oracle.MAX, rp, ci, None, X)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))
        # reversing each row's neighbour order changes nothing bitwise
        ci_rev = ci.copy()
        for i in range(N):
            ci_rev[rp[i]:rp[i + 1]] = ci[rp[i]:rp[i + 1]][::-1]
        got2 = oracle.aggregate(oracle.MAX, rp, ci_rev, None, X)
        assert np.array_equal(got.view(np.uint32), got2.view(np.uint32))


def test_max_signed_zero_and_empty_row():
    # row 0 <- {1: -0.0, 2: +0.0}; row 1 <- {2: +0.0, 1: -0.0} in the other order; row 3 <- {1: -0.0}
    src = np.array([1, 2, 2, 1, 1], np.int32)
    dst = np.array([0, 0, 1, 1, 3], np.int32)
    X = np.array([[5.0], [-0.0], [0.0], [1.0]], np.float32)
    rp, ci, _, _ = oracle.build_csr(4, src, dst)
    got = oracle.aggregate(oracle.MAX, rp, ci, None, X).view(np.uint32)[:, 0]
    assert got.tolist() == [0x00000000, 0x00000000, 0x00000000, 0x80000000]  # row 2 is empty -> +0


def test_max_with_infinities():
    src = np.array([1, 2, 1, 2], np.int32)
    dst = np.array([0, 0, 3, 3], np.int32)
    X = np.array([[0, 0], [-np.inf, np.inf], [-3.0, 2.0], [0, 0]], np.float32)
    rp, ci, _, _ = oracle.build_csr(4, src, dst)
    got = oracle.aggregate(oracle.MAX, rp, ci, None, X)
    assert got[0].tolist() == [-3.0, np.inf] and got[3].tolist() == [-3.0, np.inf]


# ---------------------------------------------------------------- bf16
def test_bf16_widening_is_exact():
    src, dst = W.random_digraph(40, 300, 9)
    rp, ci, _, _ = oracle.build_csr(40, src, dst)
    Xb = W.normal_bf16((40, 10), seed=3)
    Xf = W.bf16_to_f32(Xb)
    for op in (oracle.SUM, oracle.MEAN, oracle.MAX):
        a = oracle.aggregate(op, rp, ci, None, Xb)
        b = oracle.aggregate(op, rp, ci, None, Xf)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_bf16_generator_rounds_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1.0 + 2 ** -8 + 2 ** -20], np.float32)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1.0078125 -> even mantissa (1.0)
    # 1.01171875 = 1 + 3*2^-8 is a tie between 1.0078125 and 1.015625 -> even (1.015625)
    got = W.bf16_to_f32(W.f32_to_bf16(x))
    assert got.tolist()[:4] == [1.0, 1.0, 1.015625, -2.5]
    assert got[5] == np.float32(1.0078125)


# ---------------------------------------------------------------- decomposition (Alg. 1)
@pytest.mark.parametrize("op", [oracle.SUM, oracle.WSUM, oracle.MEAN, oracle.MAX])
def test_chunked_equals_unchunked_bitwise(op):
    N, src, dst = W.graph("c1")
    F = 45
    X = W.normal_f32((N, F), seed=4)
    rp, ci, w, _ = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    base = oracle.aggregate(op, rp, ci, w, X, form=0)
    for fc in (1, 4, 8, 16, 44, 45, 64, 0):
        got = oracle.aggregate(op, rp, ci, w, X, f_chunk=fc, form=1)
        assert np.array_equal(base.view(np.uint32), got.view(np.uint32)), fc


def test_rows_subset_and_threads_agree_with_full():
    N, src, dst = W.graph("c1")
    X = W.normal_f32((N, 9), seed=5)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    full = oracle.aggregate(oracle.SUM, rp, ci, None, X)
    rows = np.array([0, 5, 77, N - 1], np.int64)
    part = oracle.aggregate_rows(oracle.SUM, rows, rp, ci, None, X)
    assert np.array_equal(full[rows], part)
    assert np.array_equal(full, oracle.aggregate(oracle.SUM, rp, ci, None, X, threads=4))


# ---------------------------------------------------------------- GAT
def dense_gat(N, src, dst, H, a_src, a_dst, slope):
    C = dense_count(N, src, dst)
    Hd = H.astype(np.float64)
    ssrc = np.einsum("nhc,hc->nh", Hd, a_src.astype(np.float64))
    sdst = np.einsum("nhc,hc->nh", Hd, a_dst.astype(np.float64))
    out = np.zeros_like(Hd)
    for h in range(H.shape[1]):
        s = sdst[:, h][:, None] + ssrc[:, h][None, :]  # [i, j]
        e = np.where(s >= 0, s, slope * s)
        e = np.where(C > 0, e, -np.inf)
        with np.errstate(invalid="ignore"):
            p = C * np.exp(e - np.max(e, axis=1, keepdims=True, initial=-1e300))
        p = np.nan_to_num(p)
        z = p.sum(axis=1, keepdims=True)
        a = np.divide(p, z, out=np.zeros_like(p), where=z > 0)
        out[:, h, :] = a @ Hd[:, h, :]
    return out


def test_gat_matches_dense_masked_softmax():
    for k, (N, src, dst) in enumerate(tiny_graphs()):
        H = W.normal_f32((N, 3, 5), seed=k + 40)
        a_s = W.normal_f32((3, 5), seed=k + 41, std=0.7)
        a_d = W.normal_f32((3, 5), seed=k + 42, std=0.7)
        rp, ci, _, _ = oracle.build_csr(N, src, dst)
        alpha, out = oracle.gat_attention(rp, ci, H, a_s, a_d, 0.2)
        ref = dense_gat(N, src, dst, H, a_s, a_d, 0.2)
        assert np.allclose(out, ref, rtol=2e-6, atol=1e-7)
        # softmax weights of every non-empty row sum to one, per head
        rows = np.repeat(np.arange(N), np.diff(rp))
        tot = np.zeros((N, 3))
        np.add.at(tot, rows, alpha.astype(np.float64))
        assert np.allclose(tot[np.diff(rp) > 0], 1.0, atol=1e-6)


def test_gat_softmax_matches_scipy_on_one_row():
    # complete in-neighbourhood: row 0 receives from every vertex once
    N = 12
    src = np.arange(N, dtype=np.int32)
    dst = np.zeros(N, np.int32)
    H = W.normal_f32((N, 2, 4), seed=60)
    a_s = W.normal_f32((2, 4), seed=61)
    a_d = W.normal_f32((2, 4), seed=62)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    alpha, out = oracle.gat_attention(rp, ci, H, a_s, a_d, 0.2)
    Hd = H.astype(np.float64)
    s = np.einsum("nhc,hc->nh", Hd, a_s.astype(np.float64)) + np.einsum("hc,hc->h", Hd[0], a_d.astype(np.float64))
    e = np.where(s >= 0, s, 0.2 * s)
    sm = scipy.special.softmax(e, axis=0)  # [j, h]
    assert np.allclose(alpha, sm, rtol=1e-6, atol=1e-8)
    assert np.allclose(out[0], np.einsum("jh,jhc->hc", sm, Hd), rtol=1e-6, atol=1e-7)


def test_gat_zero_attention_is_mean_with_self_loops():
    N, src, dst = W.graph("c2")
    rp, ci, _, _ = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS)
    H = W.normal_f32((N, 8, 8), seed=70)
    z = np.zeros((8, 8), np.float32)
    _, out = oracle.gat_attention(rp, ci, H, z, z, 0.2, want_alpha=False)
    A = sp.csr_matrix((np.ones(len(ci)), ci, rp), shape=(N, N))
    ref = (A @ H.reshape(N, 64).astype(np.float64)) / np.diff(rp)[:, None]
    assert np.allclose(out.reshape(N, 64), ref, rtol=1e-6, atol=1e-7)


def test_gat_constant_head_and_single_edge_rows():
    N, src, dst = W.graph("c1")
    rp, ci, _, _ = oracle.build_csr(N, src, dst, flags=oracle.SELF_LOOPS)
    # H constant within a head across vertices -> weights sum to one -> out == H
    Hc = np.tile(W.normal_f32((1, 4, 3), seed=80), (N, 1, 1))
    a_s = W.normal_f32((4, 3), seed=81)
    a_d = W.normal_f32((4, 3), seed=82)
    _, out = oracle.gat_attention(rp, ci, Hc, a_s, a_d, 0.2)
    assert np.allclose(out, Hc, rtol=1e-6, atol=1e-7)
    # a row with exactly one in-edge copies that neighbour bit for bit
    src1 = np.array([3, 1, 2], np.int32)
    dst1 = np.array([0, 0, 4], np.int32)
    H = W.normal_f32((5, 2, 3), seed=83)
    rp1, ci1, _, _ = oracle.build_csr(5, src1, dst1)
    alpha, out1 = oracle.gat_attention(rp1, ci1, H, a_s[:2], a_d[:2], 0.2)
    assert np.array_equal(out1[4].view(np.uint32), H[2].view(np.uint32))
    assert np.array_equal(alpha[rp1[4]], np.ones(2, np.float32))
    assert np.array_equal(out1[1], np.zeros((2, 3), np.float32))  # empty row


def test_gat_large_scores_select_argmax_without_overflow():
    N = 6
    src = np.array([1, 2, 3, 4, 5], np.int32)
    dst = np.zeros(5, np.int32)
    H = W.normal_f32((N, 1, 4), seed=90)
    a_s = 100.0 * W.normal_f32((1, 4), seed=91)
    a_d = np.zeros((1, 4), np.float32)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    alpha, out = oracle.gat_attention(rp, ci, H, a_s, a_d, 0.2)
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(alpha))
    s = (H[1:, 0, :].astype(np.float64) @ a_s[0].astype(np.float64))
    jbest = 1 + int(np.argmax(np.where(s >= 0, s, 0.2 * s)))
    assert np.allclose(out[0, 0], H[jbest, 0], atol=1e-5)


def test_gat_leaky_slope_matters():
    # negative scores: slope 0.2 and slope 1.0 must give different weights
    N = 4
    src = np.array([1, 2, 3], np.int32)
    dst = np.zeros(3, np.int32)
    H = np.zeros((N, 1, 1), np.float32)
    H[1:, 0, 0] = [-1.0, -2.0, -3.0]
    a_s = np.ones((1, 1), np.float32)
    a_d = np.zeros((1, 1), np.float32)
    rp, ci, _, _ = oracle.build_csr(N, src, dst)
    alpha, _ = oracle.gat_attention(rp, ci, H, a_s, a_d, 0.2)
    e = np.array([-0.2, -0.4, -0.6])
    assert np.allclose(alpha[:, 0], np.exp(e) / np.exp(e).sum(), rtol=1e-6)


def test_gat_rows_subset_agrees_with_full_and_dense():
    # the row-subset form shares no score arrays with the full form; both must match the dense softmax
    for k, (N, src, dst) in enumerate(tiny_graphs()[:4]):
        H = W.normal_f32((N, 2, 3), seed=k + 200)
        a_s = W.normal_f32((2, 3), seed=k + 201, std=0.7)
        a_d = W.normal_f32((2, 3), seed=k + 202, std=0.7)
        rp, ci, _, _ = oracle.build_csr(N, src, dst)
        _, full = oracle.gat_attention(rp, ci, H, a_s, a_d, 0.2, want_alpha=False)
        rows = np.arange(N, dtype=np.int64)[::2]
        part = oracle.gat_attention_rows(rows, rp, ci, H, a_s, a_d, 0.2, threads=2)
        ref = dense_gat(N, src, dst, H, a_s, a_d, 0.2)
        assert np.allclose(part, ref[rows], rtol=2e-6, atol=1e-7)
        assert np.allclose(part, full[rows], rtol=1e-6, atol=1e-7)


# ---------------------------------------------------------------- combination (dense layer)
def test_combine_matches_library_matmul_and_special_cases():
    X = W.normal_f32((37, 19), seed=300)
    Wt = W.normal_f32((19, 5), seed=301)
    b = W.normal_f32((5,), seed=302)
    ref = X.astype(np.float64) @ Wt.astype(np.float64) + b.astype(np.float64)
    assert np.allclose(oracle.combine(X, Wt, b), ref, rtol=1e-6, atol=1e-7)
    assert np.allclose(oracle.combine(X, Wt, b, relu=True), np.maximum(ref, 0.0), rtol=1e-6, atol=1e-7)
    assert np.allclose(oracle.combine(X, Wt), ref - b, rtol=1e-6, atol=1e-6)
    # identity weights copy the input bit for bit; a one-hot column picks a column
    assert np.array_equal(oracle.combine(X, np.eye(19, dtype=np.float32)), X)
    e3 = np.zeros((19, 1), np.float32)
    e3[3] = 1.0
    assert np.array_equal(oracle.combine(X, e3)[:, 0], X[:, 3])
    # operand order: W is [F,H], not its transpose
    Wr = W.normal_f32((19, 19), seed=303)
    assert not np.allclose(oracle.combine(X, Wr), X.astype(np.float64) @ Wr.T.astype(np.float64), atol=1e-3)
    # bf16 features widen exactly
    Xb = W.normal_bf16((37, 19), seed=304)
    assert np.array_equal(oracle.combine(Xb, Wt, b), oracle.combine(W.bf16_to_f32(Xb), Wt, b))


def test_combination_commutes_with_linear_aggregation():
    # aggregate(X) W = aggregate(X W) for sum / weighted sum / mean (the reason Combination can run first)
    N, src, dst = W.graph("c1")
    rp, ci, w, _ = oracle.build_csr(N, src, dst, oracle.SELF_LOOPS | oracle.NORM_SYM, want_w=True)
    X = W.normal_f32((N, 24), seed=310)
    Wt = W.normal_f32((24, 6), seed=311)
    for op in (oracle.SUM, oracle.WSUM, oracle.MEAN):
        a = oracle.combine(oracle.aggregate(op, rp, ci, w, X), Wt).astype(np.float64)
        b = oracle.aggregate(op, rp, ci, w, oracle.combine(X, Wt)).astype(np.float64)
        assert np.allclose(a, b, rtol=1e-4, atol=1e-4)


def test_update_without_weights_is_a_rounded_addition_then_the_activation():
    # pinned by the closed form on exactly representable values and by numpy on random ones
    A = np.array([[1.0, -2.0, 0.5, -0.0], [3.0, 0.25, -8.0, 16.0]], np.float32)
    b = np.array([0.5, 1.0, -0.5, 0.0], np.float32)
    assert np.array_equal(oracle.update(A, b), np.array([[1.5, -1.0, 0.0, 0.0], [3.5, 1.25, -8.5, 16.0]], np.float32))
    got = oracle.update(A, b, relu=True)
    assert np.array_equal(got, np.array([[1.5, 0.0, 0.0, 0.0], [3.5, 1.25, 0.0, 16.0]], np.float32))
    assert not np.signbit(got).any()  # max(0, .) never returns -0
    assert np.array_equal(oracle.update(A), A) and np.array_equal(oracle.update(A, relu=True), np.maximum(A, 0))
    R = W.normal_f32((50, 7), seed=320)
    rb = W.normal_f32((7,), seed=321)
    want = (R.astype(np.float64) + rb.astype(np.float64)).astype(np.float32)
    assert np.array_equal(oracle.update(R, rb), want)  # a sum of two floats is exact in fp64: one rounding
    assert np.array_equal(oracle.update(R, rb, relu=True), np.maximum(want, np.float32(0)))
    # the bias belongs to the column, not the row
    assert not np.array_equal(oracle.update(R[:7], rb), (R[:7].T.astype(np.float64) + rb).T.astype(np.float32))
