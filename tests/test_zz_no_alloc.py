"""The entry point that allocates nothing (gnnagg_aggregate_noalloc) against gnnagg_aggregate_ws: same
kernels, the partial results of split rows in the library's fixed scratch array instead of a caller
workspace.  Two calls in a row on the same GPU, the second on a smaller input, so that whatever the first
call left in the array is there when the second runs."""
import ctypes
import sys

import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def long_rows(N, lengths, seed):
    rng = np.random.default_rng(seed)
    s, d = [], []
    for k, n in enumerate(lengths):
        s.append(rng.integers(0, N, size=n).astype(np.int32))
        d.append(np.full(n, 3 + k, np.int32))
    s2, d2 = W.random_digraph(N, 6 * N, seed + 1)
    return np.concatenate(s + [s2]), np.concatenate(d + [d2])


def run_case(g, N, lengths, F, seed, bf16):
    src, dst = long_rows(N, lengths, seed)
    d_src, d_dst = torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda()
    rp, ci, _, _ = g.gnnagg_build_csr(N, d_src, d_dst, 0)
    plan = g.gnnagg_plan_rows(rp)
    need = g.gnnagg_aggregate_workspace_bytes(N, F, plan)
    assert 0 < need <= 8 << 20, need  # the case must use the scratch array and fit it
    w = torch.from_numpy(W.normal_f32((int(ci.shape[0]),), seed=seed + 2)).cuda()
    if bf16:
        X = torch.from_numpy(W.normal_bf16((N, F), seed=seed + 3).view(np.int16)).cuda().view(torch.bfloat16)
    else:
        X = torch.from_numpy(W.normal_f32((N, F), seed=seed + 3)).cuda()
    Xp = g.pitched_empty(N, F, X.dtype)
    Xp.copy_(X)
    for op in (g.SUM, g.WSUM, g.MEAN, g.MAX):
        for fc in (0, 16):
            say("  no-alloc N", N, "F", F, "op", op, "f_chunk", fc, "scratch bytes", need)
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            want = g.pitched_empty(N, F, torch.float32)
            want.fill_(float("nan"))
            g.gnnagg_aggregate(op, rp, ci, w if op == g.WSUM else None, Xp, want, fc, plan, workspace=ws)
            got = g.pitched_empty(N, F, torch.float32)
            got.fill_(float("nan"))
            g.gnnagg_aggregate_noalloc(op, rp, ci, w if op == g.WSUM else None, Xp, got, fc, plan)
            torch.cuda.synchronize()
            a, b = got.cpu().numpy(), want.cpu().numpy()
            assert not np.isnan(a).any()
            # same kernels, same launch geometry, no atomics: the bar is the parity bar of the operator
            # (bit-exact for max, 1e-6 + 1e-5 |r| for sums, 1e-2 relative for bf16 inputs); the bits agree
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), (op, fc)


def test_no_alloc_entry_point_matches_the_workspace_entry_point_twice_in_a_row():
    import paper_2104_03058_amd as g
    g.load_library()
    run_case(g, 900, [70001, 32768, 40000, 500], F=100, seed=21, bf16=True)
    run_case(g, 300, [33000, 64], F=33, seed=22, bf16=False)  # smaller input, the array still holds the first call's data


def test_no_alloc_entry_point_rejects_a_plan_beyond_its_scratch_array():
    import paper_2104_03058_amd as g
    lib = g.load_library()
    # host-side decision: 600 rows of class 16 at F = 1024 need 600 * 8 * 1024 * 8 bytes = 39 MB > 8 MiB
    N, F = 1000, 1024
    off = (ctypes.c_int64 * 34)()
    for k in range(34):
        off[k] = 0 if k <= 16 else (600 if k < 33 else N)  # class 16 holds rows [0, 600), class 0 the rest
    order = torch.arange(N, dtype=torch.int32, device="cuda")
    rp = torch.zeros(N + 1, dtype=torch.int64, device="cuda")
    ci = torch.zeros(1, dtype=torch.int32, device="cuda")
    X = torch.zeros((N, F), dtype=torch.float32, device="cuda")
    out = torch.full((N, F), 7.0, dtype=torch.float32, device="cuda")
    need = ctypes.c_size_t(0)
    rc = lib.gnnagg_aggregate_ws(0, N, None, None, None, None, 0, 0, None, 0, 0, F, 0, ctypes.c_void_p(order.data_ptr()),
                                 ctypes.cast(off, ctypes.c_void_p), None, ctypes.byref(need), None)
    assert rc == 0 and need.value == 600 * 8 * F * 8
    rc = lib.gnnagg_aggregate_noalloc(0, N, ctypes.c_void_p(rp.data_ptr()), ctypes.c_void_p(ci.data_ptr()), None,
                                      ctypes.c_void_p(X.data_ptr()), 0, 0, ctypes.c_void_p(out.data_ptr()), 0, 0, F, 0,
                                      ctypes.c_void_p(order.data_ptr()), ctypes.cast(off, ctypes.c_void_p), None)
    assert rc == -4  # GNNAGG_EWORKSPACE, before anything is launched
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
