"""CPU-only checks of the GPU library's host side: the shared object loads and
exports every symbol the header declares, argument validation answers before
anything is launched, and the launch geometry (feature slices x degree-class
lane groups) covers every output element and every edge exactly as intended."""
import ctypes
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "gnnagg.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2104_03058_amd as g
    from paper_2104_03058_amd import build
    if not os.path.exists(g.library_path()):
        build.build()
    return g.load_library()


def declared_symbols():
    text = open(HEADER).read()
    return sorted(set(re.findall(r"GNNAGG_API\s+[\w\s\*]+?\b(gnnagg_\w+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_symbols()
    for must in ["gnnagg_build_csr", "gnnagg_aggregate", "gnnagg_gat_attention", "gnnagg_plan_rows",
                 "gnnagg_combine", "gnnagg_auto_f_chunk", "gnnagg_strerror", "gnnagg_version"]:
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_version_and_strerror(lib):
    import paper_2104_03058_amd as g
    assert g.gnnagg_version() >= 100
    assert g.gnnagg_strerror(0) == "ok"
    assert "invalid" in g.gnnagg_strerror(-1)
    assert g.gnnagg_strerror(-99) == "unknown status"


def other_ptr():
    return ctypes.c_void_p(8192)


def test_argument_validation_returns_before_any_launch(lib):
    """All of these are rejected on the host; no HIP call is reached, so they run without a GPU."""
    EINVAL, ENULL, EUNSUP, EWS = -1, -2, -3, -4
    one = ctypes.c_void_p(4096)  # a non-null, aligned stand-in pointer that is never dereferenced
    agg = lib.gnnagg_aggregate
    assert agg(7, 4, one, one, one, one, 0, one, 0, 8, 0, None, None, None) == EINVAL      # op
    assert agg(0, -1, one, one, one, one, 0, one, 0, 8, 0, None, None, None) == EINVAL     # N
    assert agg(0, 4, one, one, one, one, 0, one, 0, 0, 0, None, None, None) == EINVAL      # F
    assert agg(0, 4, one, one, one, one, 0, one, 0, 8, -2, None, None, None) == EINVAL     # f_chunk (-1 = auto)
    assert agg(0, 4, one, one, one, one, 5, one, 0, 8, 0, None, None, None) == EINVAL      # x_dtype
    assert agg(0, 4, one, one, one, one, 0, one, 2, 8, 0, None, None, None) == EINVAL      # out_dtype
    assert agg(0, 4, None, one, one, one, 0, one, 0, 8, 0, None, None, None) == ENULL      # rowptr
    assert agg(1, 4, one, one, None, one, 0, one, 0, 8, 0, None, None, None) == ENULL      # wsum needs edge_w
    assert agg(0, 4, one, one, one, one, 0, one, 0, 8, 0, one, None, None) == EINVAL       # half a plan
    assert agg(0, 4, one, one, one, one, 0, one, 0, 8, 0, None, None, None) == EINVAL      # X aliases out
    assert agg(0, 4, one, one, one, ctypes.c_void_p(4098), 0, one, 0, 8, 0, None, None, None) == EINVAL  # alignment
    assert agg(0, 0, None, None, None, None, 0, None, 0, 8, 0, None, None, None) == 0      # empty graph: nothing to do

    need = ctypes.c_size_t(0)
    csr = lib.gnnagg_build_csr
    assert csr(-1, 0, None, None, 0, None, None, None, None, None, ctypes.byref(need), None) == EINVAL
    assert csr(4, 2, None, None, 8, None, None, None, None, None, ctypes.byref(need), None) == EINVAL  # flags
    assert csr(4, 2, None, None, 0, None, None, None, None, None, None, None) == ENULL
    assert csr(4, 1 << 32, None, None, 0, None, None, None, None, None, ctypes.byref(need), None) == EUNSUP
    assert csr(4, 2, None, None, 0, None, None, None, None, None, ctypes.byref(need), None) == 0
    assert need.value > 0 and need.value % 256 == 0
    small = ctypes.c_size_t(16)
    assert csr(4, 2, one, one, 0, one, one, None, None, one, ctypes.byref(small), None) == EWS
    big = ctypes.c_size_t(need.value)
    assert csr(4, 2, one, one, 0, one, one, None, None, ctypes.c_void_p(4097), ctypes.byref(big), None) == EWS
    assert csr(4, 2, None, one, 0, one, one, None, None, one, ctypes.byref(big), None) == ENULL

    plan = lib.gnnagg_plan_rows
    assert plan(-3, None, None, None, None, ctypes.byref(need), None) == EINVAL
    assert plan(10, None, None, None, None, ctypes.byref(need), None) == 0 and need.value > 0

    gat = lib.gnnagg_gat_attention
    f = ctypes.c_float(0.2)
    assert gat(4, one, one, one, one, one, 0, 8, f, None, one, 0, None, None, None, ctypes.byref(need), None) == EINVAL
    assert gat(4, one, one, one, one, one, 8, 8, f, None, one, 12, None, None, None, ctypes.byref(need), None) == EINVAL
    assert gat(4, one, one, one, one, one, 8, 8, f, None, one, 16, None, None, None, ctypes.byref(need), None) == 0
    assert need.value >= 2 * 4 * 8 * 4
    assert gat(4, one, one, one, one, one, 8, 8, f, None, one, 0, None, None, one, ctypes.byref(small), None) == EWS

    aggws = lib.gnnagg_aggregate_ws
    off = (ctypes.c_int64 * 34)()
    rows = [0] * 33
    rows[32 - 16], rows[32 - 17], rows[32 - 3] = 2, 1, 97  # two rows of class 16 (8 pieces), one of class 17 (16)
    for k in range(33):
        off[k + 1] = off[k] + rows[k]
    offp = ctypes.cast(off, ctypes.c_void_p)
    need = ctypes.c_size_t(77)
    assert aggws(0, 100, one, one, one, one, 0, 0, other_ptr(), 0, 0, 8, 0, one, offp, None, None, None) == ENULL
    assert aggws(0, 100, None, None, None, None, 0, 0, None, 0, 0, 8, 0, one, offp, None, ctypes.byref(need), None) == 0
    assert need.value == (2 * 8 + 16) * 8 * 8          # slots x F x sizeof(double)
    assert aggws(0, 100, None, None, None, None, 0, 0, None, 0, 0, 8, 0, None, None, None, ctypes.byref(need), None) == 0
    assert need.value == 0                               # no plan: nothing is split
    small = ctypes.c_size_t(64)
    assert aggws(0, 100, one, one, one, one, 0, 0, other_ptr(), 0, 0, 8, 0, one, offp, one, ctypes.byref(small), None) == EWS
    big = ctypes.c_size_t(1 << 20)
    assert aggws(0, 100, one, one, one, one, 0, 0, other_ptr(), 0, 0, 8, 0, one, offp, ctypes.c_void_p(4100),
                 ctypes.byref(big), None) == EWS        # misaligned
    assert aggws(9, 100, one, one, one, one, 0, 0, other_ptr(), 0, 0, 8, 0, one, offp, one, ctypes.byref(big),
                 None) == EINVAL
    assert aggws(0, 100, one, one, one, one, 0, 7, other_ptr(), 0, 0, 8, 0, one, offp, one, ctypes.byref(big),
                 None) == EINVAL                        # a pitch below F
    assert aggws(0, 100, one, one, one, one, 0, 0, other_ptr(), 0, 5, 8, 0, one, offp, one, ctypes.byref(big),
                 None) == EINVAL
    pitch = lib.gnnagg_row_pitch
    assert [pitch(100, 1), pitch(602, 0), pitch(32, 0), pitch(16, 1), pitch(33, 0), pitch(3, 0), pitch(50, 1),
            pitch(64, 1), pitch(1, 1)] == [128, 608, 32, 16, 64, 4, 64, 64, 1]
    assert pitch(0, 0) == 0 and pitch(8, 7) == 0

    chk = lib.gnnagg_check_csr
    assert chk(-1, 0, one, one, one, ctypes.byref(need), None) == EINVAL
    assert chk(4, 3, one, one, None, None, None) == ENULL
    assert chk(4, 3, None, None, None, ctypes.byref(need), None) == 0 and need.value >= 256
    assert chk(4, 3, one, one, one, ctypes.byref(ctypes.c_size_t(8)), None) == EWS
    assert chk(4, 3, None, one, one, ctypes.byref(ctypes.c_size_t(4096)), None) == ENULL

    ranks = lib.gnnagg_rank_sources
    assert ranks(-1, 0, None, None, None, None, ctypes.byref(need), None) == EINVAL
    assert ranks(5, 1 << 32, None, None, None, None, ctypes.byref(need), None) == EUNSUP
    assert ranks(5, 9, None, None, None, None, None, None) == ENULL
    assert ranks(5, 9, None, None, None, None, ctypes.byref(need), None) == 0 and need.value > 0
    tiny = ctypes.c_size_t(8)
    assert ranks(5, 9, one, one, one, one, ctypes.byref(tiny), None) == EWS
    roomy = ctypes.c_size_t(need.value)
    assert ranks(5, 9, None, one, one, one, ctypes.byref(roomy), None) == ENULL

    comb = lib.gnnagg_combine
    other = ctypes.c_void_p(8192)
    assert comb(-1, one, 0, 8, one, None, 4, 0, other, None, None) == EINVAL   # N
    assert comb(4, one, 0, 0, one, None, 4, 0, other, None, None) == EINVAL    # F
    assert comb(4, one, 0, 8, one, None, 0, 0, other, None, None) == EINVAL    # H
    assert comb(4, one, 3, 8, one, None, 4, 0, other, None, None) == EINVAL    # x_dtype
    assert comb(4, one, 0, 8, one, None, 4, 2, other, None, None) == EINVAL    # relu flag
    assert comb(4, None, 0, 8, one, None, 4, 0, other, None, None) == ENULL    # X
    assert comb(4, one, 0, 8, None, None, 4, 0, other, None, None) == ENULL    # W
    assert comb(4, one, 0, 8, one, None, 4, 0, None, None, None) == ENULL      # out
    assert comb(4, one, 0, 8, one, None, 4, 0, one, None, None) == EINVAL      # out aliases X
    assert comb(4, ctypes.c_void_p(4098), 0, 8, one, None, 4, 0, other, None, None) == EINVAL  # fp32 X on a 2-byte boundary
    assert comb(0, None, 0, 8, None, None, 4, 0, None, None, None) == 0        # no rows: nothing to do


def test_update_and_no_alloc_entry_points_validate_on_the_host(lib):
    EINVAL, ENULL, EUNSUP, EWS = -1, -2, -3, -4
    one, other = ctypes.c_void_p(4096), ctypes.c_void_p(8192)
    need = ctypes.c_size_t(0)
    big = ctypes.c_size_t(1 << 20)
    upd = lib.gnnagg_aggregate_update

    def call(op=0, N=100, X=one, F=8, fc=0, W2=None, H2=0, bias=None, relu=0, out=other, x_pitch=0, out_pitch=0,
             ws=one, wsb=big):
        return upd(op, N, one, one, one, X, 0, x_pitch, F, fc, W2, H2, bias, relu, out, 0, out_pitch, None, None, ws,
                   ctypes.byref(wsb) if wsb is not None else None, None)

    assert call(wsb=None) == ENULL
    assert call(relu=2) == EINVAL
    assert call(H2=5) == EINVAL                       # a width without a matrix
    assert call(W2=one, H2=0) == EINVAL               # a matrix without a width
    assert call(W2=one, H2=4097) == EINVAL
    assert call(W2=one, H2=8, F=65) == EUNSUP         # the fused layer holds rows of at most 64 columns
    assert call(W2=one, H2=8, F=64, fc=16) == EINVAL  # ... and contracts them whole
    assert call(W2=one, H2=8, F=64, out_pitch=7) == EINVAL   # out has H2 columns
    assert call(W2=ctypes.c_void_p(4098), H2=8) == EINVAL    # alignment
    assert call(bias=ctypes.c_void_p(4098)) == EINVAL
    assert call(op=9) == EINVAL
    assert call(out=one) == EINVAL                    # out aliases X
    assert call(ws=None, wsb=need) == 0 and need.value == 0  # size query, no plan
    assert call(N=0, X=None, out=None) == 0

    na = lib.gnnagg_aggregate_noalloc
    assert na(0, -1, one, one, one, one, 0, 0, other, 0, 0, 8, 0, None, None, None) == EINVAL
    assert na(9, 10, one, one, one, one, 0, 0, other, 0, 0, 8, 0, None, None, None) == EINVAL
    assert na(0, 10, one, one, one, one, 0, 4, other, 0, 0, 8, 0, None, None, None) == EINVAL  # pitch below F
    assert na(0, 10, None, one, one, one, 0, 0, other, 0, 0, 8, 0, None, None, None) == ENULL
    assert na(0, 10, one, one, one, one, 0, 0, other, 0, 0, 8, 0, one, None, None) == EINVAL   # half a plan
    assert na(0, 0, None, None, None, None, 0, 0, None, 0, 0, 8, 0, None, None, None) == 0
    # a plan whose split rows need more than the fixed array: 600 rows of class 16, 1024 columns
    off = (ctypes.c_int64 * 34)()
    for k in range(34):
        off[k] = 0 if k <= 16 else (600 if k < 33 else 1000)
    assert na(0, 1000, one, one, one, one, 0, 0, other, 0, 0, 1024, 0, one, ctypes.cast(off, ctypes.c_void_p),
              None) == EWS
    text = open(HEADER).read()
    assert re.search(r"#define\s+GNNAGG_NOALLOC_SCRATCH_BYTES\s+\(8u << 20\)", text)


def test_source_block_entry_points_validate_on_the_host(lib):
    EINVAL, ENULL, EUNSUP, EWS = -1, -2, -3, -4
    one, other = ctypes.c_void_p(4096), ctypes.c_void_p(8192)
    need = ctypes.c_size_t(0)
    big = ctypes.c_size_t(1 << 30)
    off = (ctypes.c_int64 * (3 * 34))()
    for b in range(3):
        for k in range(34):
            off[b * 34 + k] = 0 if k <= 24 else 100  # 100 rows of 128..255 edges in every block
    offp = ctypes.cast(off, ctypes.c_void_p)
    plan = lib.gnnagg_plan_source_blocks
    assert plan(10, None, None, 2, None, None, None, None, None, None) == ENULL          # no size pointer
    for B in (0, -3, 65):
        assert plan(10, None, None, B, None, None, None, None, ctypes.byref(need), None) == EINVAL
    assert plan(-1, None, None, 2, None, None, None, None, ctypes.byref(need), None) == EINVAL
    assert plan(1 << 31, None, None, 2, None, None, None, None, ctypes.byref(need), None) == EUNSUP
    assert plan(1000, None, None, 2, None, None, None, None, ctypes.byref(need), None) == 0 and need.value > 0
    small = ctypes.c_size_t(need.value - 1)
    assert plan(1000, one, one, 2, one, one, offp, one, ctypes.byref(small), None) == EWS
    assert plan(1000, None, one, 2, one, one, offp, one, ctypes.byref(big), None) == ENULL
    assert plan(1000, one, one, 2, None, one, offp, one, ctypes.byref(big), None) == ENULL
    assert plan(1000, one, one, 2, one, one, None, one, ctypes.byref(big), None) == ENULL
    assert plan(1000, one, one, 2, ctypes.c_void_p(4100), one, offp, one, ctypes.byref(big), None) == EINVAL
    assert plan(0, one, one, 3, one, one, offp, one, ctypes.byref(big), None) == 0 and off[2 * 34 + 33] == 0
    for b in range(3):
        for k in range(34):
            off[b * 34 + k] = 0 if k <= 24 else 100

    blocked = lib.gnnagg_aggregate_blocked

    def call(op=0, N=100, X=one, F=8, fc=0, B=3, bp=one, order=one, co=offp, out=other, x_pitch=0, out_pitch=0,
             ws=one, wsb=big):
        return blocked(op, N, one, one, one, X, 0, x_pitch, out, 0, out_pitch, F, fc, B, bp, order, co, ws,
                       ctypes.byref(wsb) if wsb is not None else None, None)

    assert call(wsb=None) == ENULL
    assert call(B=0) == EINVAL and call(B=65) == EINVAL
    assert call(co=None) == ENULL and call(order=None) == ENULL and call(bp=None) == ENULL
    assert call(op=7) == EINVAL
    assert call(out=one) == EINVAL                     # out aliases X
    assert call(x_pitch=4) == EINVAL                   # a pitch below F
    assert call(bp=ctypes.c_void_p(4100)) == EINVAL
    # workspace: two arrays of N rows of 16 doubles (8 columns padded to a 128-byte line), no split rows
    assert call(ws=None, wsb=need) == 0 and need.value == 2 * 100 * 16 * 8
    assert call(ws=None, wsb=need, B=2) == 0 and need.value == 100 * 16 * 8
    assert call(ws=None, wsb=need, B=1) == 0 and need.value == 0
    assert call(ws=None, wsb=need, F=602) == 0 and need.value == 2 * 100 * 608 * 8
    assert call(wsb=ctypes.c_size_t(2 * 100 * 16 * 8 - 1)) == EWS
    assert call(ws=ctypes.c_void_p(4100)) == EWS
    empty = (ctypes.c_int64 * (3 * 34))()               # the plan of a graph without vertices
    assert call(N=0, X=None, out=None, bp=None, co=ctypes.cast(empty, ctypes.c_void_p)) == 0
    assert call(N=0, X=None, out=None, bp=None) == EINVAL  # a plan for 100 rows

    tune = lib.gnnagg_tune_blocked
    best, ms = ctypes.c_int32(-1), ctypes.c_float(-1.0)

    def tcall(op=0, N=100, X=one, F=8, B=3, bp=one, co=offp, out=other, ws=one, wsb=big, bestp=ctypes.byref(best)):
        return tune(op, N, one, one, one, X, 0, 0, out, 0, 0, F, B, bp, one, co, ws,
                    ctypes.byref(wsb) if wsb is not None else None, None, bestp, ctypes.byref(ms))

    assert tcall(wsb=None) == ENULL
    assert tcall(B=0) == EINVAL and tcall(co=None) == ENULL and tcall(op=7) == EINVAL
    assert tcall(ws=None, wsb=need, bestp=None) == 0 and need.value == 2 * 100 * 16 * 8   # size query needs no result slot
    assert tcall(bestp=None) == ENULL
    assert tcall(wsb=ctypes.c_size_t(16)) == EWS
    assert tcall(N=0, X=None, out=None, bp=None, co=ctypes.cast(empty, ctypes.c_void_p)) == 0 and best.value == 8


def test_factored_gcn_entry_points_validate_on_the_host(lib):
    EINVAL, ENULL = -1, -2
    one, other = ctypes.c_void_p(4096), other_ptr()
    agg = lib.gnnagg_aggregate
    assert agg(5, 4, one, one, one, one, 0, other, 0, 8, 0, None, None, None) == EINVAL    # one past the last operator
    assert agg(4, 4, one, one, None, one, 0, other, 0, 8, 0, None, None, None) == ENULL    # the factors are required
    assert lib.gnnagg_auto_source_blocks(5, 200000, 602, 0, 608, None) == 0
    fac = lib.gnnagg_gcn_factors
    assert fac(-1, one, other, None) == EINVAL
    assert fac(4, None, other, None) == ENULL
    assert fac(4, one, None, None) == ENULL
    assert fac(4, ctypes.c_void_p(4100), other, None) == EINVAL     # rowptr on a 4-byte boundary
    assert fac(0, None, None, None) == 0
    sc = lib.gnnagg_scale_rows
    assert sc(-1, 8, one, 0, 0, one, other, 0, None) == EINVAL      # N
    assert sc(4, 0, one, 0, 0, one, other, 0, None) == EINVAL       # F
    assert sc(4, 8, one, 2, 0, one, other, 0, None) == EINVAL       # x_dtype
    assert sc(4, 8, one, 0, 7, one, other, 0, None) == EINVAL       # pitch below F
    assert sc(4, 8, one, 0, 0, one, other, 4, None) == EINVAL
    assert sc(4, 8, None, 0, 0, one, other, 0, None) == ENULL
    assert sc(4, 8, one, 0, 0, None, other, 0, None) == ENULL
    assert sc(4, 8, one, 0, 0, one, None, 0, None) == ENULL
    assert sc(4, 8, ctypes.c_void_p(4098), 0, 0, one, other, 0, None) == EINVAL   # fp32 X on a 2-byte boundary
    assert sc(4, 8, one, 1, 0, one, one, 0, None) == EINVAL         # in place needs fp32 rows ...
    assert sc(4, 8, one, 0, 16, one, one, 8, None) == EINVAL        # ... at one pitch
    assert sc(0, 8, None, 0, 0, None, None, 0, None) == 0
    cs = lib.gnnagg_combine_scaled
    assert cs(4, one, 0, 8, one, None, 4, 0, None, other, None, None) == ENULL              # the factors are required
    assert cs(4, one, 0, 8, one, None, 4, 0, ctypes.c_void_p(4098), other, None, None) == EINVAL
    assert cs(4, one, 0, 0, one, None, 4, 0, one, other, None, None) == EINVAL              # F, as in gnnagg_combine
    assert cs(4, one, 0, 8, one, None, 4, 0, one, one, None, None) == EINVAL                # out aliases X
    assert cs(0, None, 0, 8, None, None, 4, 0, None, None, None, None) == 0


def test_line_gather_probe_validates_on_the_host(lib):
    EINVAL, ENULL = -1, -2
    one, other = ctypes.c_void_p(4096), ctypes.c_void_p(8192)
    f = lib.gnnagg_line_gather_probe
    assert f(None, 1 << 20, None, 1, 1, other, None) == ENULL and f(one, 1 << 20, None, 1, 1, None, None) == ENULL
    assert f(one, 100, None, 1, 1, other, None) == EINVAL          # not whole lines
    assert f(one, 0, None, 1, 1, other, None) == EINVAL
    assert f(ctypes.c_void_p(4100), 1 << 20, None, 1, 1, other, None) == EINVAL   # buffer not on a line
    assert f(one, 1 << 20, None, 0, 1, other, None) == EINVAL and f(one, 1 << 20, None, 1, 0, other, None) == EINVAL
    assert f(one, 1 << 40, None, 1, 1, other, None) == EINVAL      # more than 2^31 lines
    assert f(one, 1 << 20, ctypes.c_void_p(4098), 1, 1, other, None) == EINVAL    # index array not on 4 bytes


def test_source_block_rule(lib):
    """Blocks pay on dense fp32 graphs of at least 100,000 rows whose rows start on lines; nowhere else.  Four
    where the edges are spread over the rows, two where the longest tenth of the rows holds most of them."""
    import paper_2104_03058_amd as g
    N = 232965
    hubs = plan_of(N, {16: 30, 15: 300, 14: 2000, 13: 6000, 12: 10000, 10: 30000, 8: 60000,
                       6: 80000})                            # mean degree ~ 600, the top tenth holds ~ 3/4
    flat = plan_of(N, {11: 20000, 10: 80000, 9: 100000, 8: 32965})                      # ~ 600, top tenth ~ 1/5
    medium = plan_of(N, {11: 3000, 9: 20000, 8: 60000, 7: 80000, 6: 50000, 5: 19965})   # mean degree ~ 130
    assert g.gnnagg_auto_source_blocks(g.WSUM, N, 602, g.F32, 608, hubs) == 2
    assert g.gnnagg_auto_source_blocks(g.WSUM, N, 602, g.F32, 608, flat) == 4
    between = plan_of(N, {15: 300, 14: 2500, 13: 6500, 12: 10000, 11: 12000, 10: 25000, 9: 40000, 8: 50000,
                          7: 50000, 6: 36665})               # the top tenth holds about 65 % of the edges
    assert g.gnnagg_auto_source_blocks(g.WSUM, N, 602, g.F32, 608, between) == 2   # the weights' stream gains nothing
    for op in (g.SUM, g.MEAN, g.MAX):
        assert g.gnnagg_auto_source_blocks(op, N, 602, g.F32, 608, between) == 4
        assert g.gnnagg_auto_source_blocks(op, N, 602, g.F32, 608, hubs) == 2
    assert g.gnnagg_auto_source_blocks(9, N, 602, g.F32, 608, flat) == 0            # no such operator
    assert g.gnnagg_auto_source_blocks(g.WSUM, N, 128, g.F32, 128, flat) == 4
    assert g.gnnagg_auto_source_blocks(g.WSUM, N, 602, g.F32, 602, flat) == 1      # rows not on lines
    assert g.gnnagg_auto_source_blocks(g.WSUM, N, 64, g.F32, 64, flat) == 1        # narrow rows: one pass per block is short
    assert g.gnnagg_auto_source_blocks(g.WSUM, N, 512, g.BF16, 512, flat) == 1     # bf16
    assert g.gnnagg_auto_source_blocks(g.WSUM, N, 602, g.F32, 608, medium) == 1    # too few edges per row
    assert g.gnnagg_auto_source_blocks(g.WSUM, N, 602, g.F32, 608, None) == 1      # no plan
    small = plan_of(60000, {12: 2000, 10: 20000, 9: 38000})
    assert g.gnnagg_auto_source_blocks(g.WSUM, 60000, 602, g.F32, 608, small) == 1  # small graph
    assert g.gnnagg_auto_source_blocks(g.WSUM, 10, 0, g.F32) == 0 and g.gnnagg_auto_source_blocks(g.WSUM, 10, 8, 7) == 0
    assert g.gnnagg_auto_source_blocks(g.WSUM, 10, 8, g.F32, 4) == 0


# ------------------------------------------------------------------ launch geometry
@pytest.fixture(scope="module")
def checker(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("host") / "schedule_check")
    # AddressSanitizer and UBSan on the host side of the scheduling code (a CPU build: no GPU code runs)
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                           "-I" + os.path.join(ROOT, "include"),
                           "-I" + os.path.join(ROOT, "paper_2104_03058_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host", "schedule_check.cpp"), "-o", exe])
    return exe


def run_checker(exe, F, f_chunk, max_vec, vec_multiple, N, class_counts=None, split=False):
    args = [exe, str(F), str(f_chunk), str(max_vec), str(vec_multiple), str(N),
            ("2" if split else "1") if class_counts else "0"]
    if class_counts:
        args += [str(c) for c in class_counts]
    p = subprocess.run(args, capture_output=True, text=True)
    assert p.returncode == 0 and p.stdout.startswith("OK"), (args, p.stdout, p.stderr)
    return p.stdout


def counts(N, spread):
    """rows per class 32..0: `spread` maps class -> rows, the rest go to class 1."""
    c = [0] * 33
    used = 0
    for cls, n in spread.items():
        c[32 - cls] = n
        used += n
    c[32 - 1] += N - used
    assert c[32 - 1] >= 0
    return c


@pytest.mark.parametrize("F,f_chunk,max_vec", [
    (1433, 0, 4), (1433, 16, 4), (1433, 64, 4),          # config 1 sweep (ragged last chunk of width 9)
    (500, 0, 4), (602, 0, 4), (602, 8, 4), (602, 16, 4), (602, 32, 4), (602, 64, 4),
    (100, 0, 8), (16, 0, 8), (32, 0, 8), (100, 7, 8),    # bf16 widths; a chunk narrower than the vector
    (1, 0, 4), (3, 0, 4), (5, 2, 4), (257, 0, 4), (2051, 0, 8), (513, 512, 8),
])
def test_geometry_without_plan(checker, F, f_chunk, max_vec):
    run_checker(checker, F, f_chunk, max_vec, 0, 37)


@pytest.mark.parametrize("F,f_chunk,max_vec", [(602, 0, 4), (602, 64, 4), (100, 0, 8), (16, 0, 8), (9, 4, 4), (64, 8, 4)])
def test_geometry_with_degree_classes(checker, F, f_chunk, max_vec):
    N = 300
    cc = counts(N, {0: 7, 2: 40, 3: 33, 4: 29, 5: 21, 6: 17, 7: 13, 8: 9, 9: 6, 11: 5, 15: 3, 32: 1})
    run_checker(checker, F, f_chunk, max_vec, 0, N, cc)


@pytest.mark.parametrize("F,f_chunk,max_vec,line_cols", [(602, 0, 4, 32), (1433, 0, 4, 32), (1000, 0, 8, 64), (2051, 0, 8, 64),
                                                         (602, 256, 4, 32), (100, 0, 8, 64), (257, 0, 4, 32)])
def test_geometry_with_line_aligned_slices(checker, F, f_chunk, max_vec, line_cols):
    """When rows start on 128-byte lines the slices of a wide chunk end on line boundaries; coverage as before."""
    N = 150
    cc = counts(N, {0: 4, 2: 30, 4: 20, 6: 10, 9: 4, 13: 2})
    run_checker(checker, F, f_chunk, max_vec, "0:%d" % line_cols, N, cc)


@pytest.mark.parametrize("F,f_chunk,max_vec", [(602, 0, 4), (100, 0, 8), (16, 0, 8), (9, 4, 4), (1030, 64, 4)])
def test_geometry_with_split_rows(checker, F, f_chunk, max_vec):
    """Rows of 2^15 edges or more are cut into pieces when a workspace is available: every piece covers all
    columns in a slot of its own, nothing else changes.  Eight long classes exceed the table's seven split
    runs, so the shortest ones share a run."""
    N = 200
    spread = {0: 5, 3: 30, 6: 17, 9: 6, 12: 4, 14: 3, 15: 3, 16: 2, 17: 1, 18: 1, 19: 1, 20: 1, 21: 1, 22: 1, 23: 1}
    out = run_checker(checker, F, f_chunk, max_vec, 0, N, counts(N, spread), split=True)
    assert "split_rows=9 " in out, out
    # without permission to split the same plan is laid out as before
    assert "split_rows=0 slots=0" in run_checker(checker, F, f_chunk, max_vec, 0, N, counts(N, spread))


@pytest.mark.parametrize("heads,C,f_chunk", [(8, 8, 0), (8, 8, 8), (8, 8, 16), (3, 5, 0), (4, 6, 12), (40, 8, 0)])
def test_geometry_attention_lanes_stay_inside_heads(checker, heads, C, f_chunk):
    N = 120
    cc = counts(N, {0: 3, 2: 30, 4: 20, 6: 10, 9: 4, 13: 2})
    run_checker(checker, heads * C, f_chunk, 4, C, N, cc)


# ------------------------------------------------------------------ resident-workgroup cap
@pytest.fixture(scope="module")
def cap_checker(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("host") / "cap_check")
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                           "-I" + os.path.join(ROOT, "include"),
                           "-I" + os.path.join(ROOT, "paper_2104_03058_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host", "cap_check.cpp"), "-o", exe])
    return exe


def run_cap(exe, g, lanes, weighted, N, spread):
    out = subprocess.run([exe, str(g), str(lanes), str(int(weighted)), str(N)] + [str(c) for c in counts(N, spread)],
                         capture_output=True, text=True)
    assert out.returncode == 0, out.stderr
    return [int(t) for t in out.stdout.split()]


def test_workgroup_cap_follows_degree_and_bytes_in_flight(cap_checker):
    N = 1000
    dense = {10: 600, 9: 300, 8: 100}        # degrees 128..1023: mean ~ 580
    medium = {8: 700, 7: 300}                # degrees 64..255: mean ~ 160
    sparse = {3: 500, 2: 300, 5: 100}        # single digits
    cap, claim, noplan = run_cap(cap_checker, 6, 64, True, N, dense)
    assert cap == 2 and noplan == 0
    # exactly `cap` workgroups fit into 160 KB of LDS
    assert cap * claim <= 160 * 1024 < (cap + 1) * claim
    # the measured optima: (active lanes, weighted) -> cap
    for lanes, weighted, want in [(64, False, 2), (56, True, 2), (56, False, 3), (48, True, 2), (48, False, 3),
                                  (39, True, 3), (39, False, 4), (50, True, 2), (50, False, 3)]:
        cap, claim, _ = run_cap(cap_checker, 6, lanes, weighted, N, dense)
        assert cap == want, (lanes, weighted, cap)
        assert cap * claim <= 160 * 1024 < (cap + 1) * claim
    assert run_cap(cap_checker, 6, 64, True, N, medium)[0] == 2
    assert run_cap(cap_checker, 6, 64, True, N, sparse)[:2] == [0, 0]
    assert run_cap(cap_checker, 5, 64, True, N, dense)[0] == 2 and run_cap(cap_checker, 5, 50, True, N, dense)[0] == 3
    assert run_cap(cap_checker, 5, 64, True, N, medium)[0] == 0
    assert run_cap(cap_checker, 4, 64, True, N, dense)[0] == 0   # slices of 16 lanes or fewer are never capped
    assert run_cap(cap_checker, 2, 64, False, N, dense)[0] == 0


def test_auto_chunk_width(lib):
    import paper_2104_03058_amd as g
    assert g.gnnagg_auto_f_chunk(232965, 602, g.F32) == 602          # 561 MB, no plan: one chunk
    assert g.gnnagg_auto_f_chunk(2449029, 100, g.BF16) == 100        # 490 MB: one chunk
    assert g.gnnagg_auto_f_chunk(2449029, 512, g.F32) == 32          # 5 GB: ~300 MB column slices
    assert g.gnnagg_auto_f_chunk(2449029, 1024, g.BF16) == 64        # same bytes per row piece in bf16
    assert g.gnnagg_auto_f_chunk(50_000_000, 64, g.F32) == 32        # never under 128 bytes per row piece
    assert g.gnnagg_auto_f_chunk(10, 0, g.F32) == 0 and g.gnnagg_auto_f_chunk(10, 8, 7) == 0
    assert g.gnnagg_auto_f_chunk(10, 8, g.F32, 4) == 0               # a pitch below F


def plan_of(N, spread):
    import paper_2104_03058_amd as g
    off = (ctypes.c_int64 * 34)()
    for k, rows in enumerate(counts(N, spread)):
        off[k + 1] = off[k] + rows
    return g.RowPlan(None, off)


def test_auto_chunk_width_one_line_on_dense_skewed_graphs(lib):
    """Line-aligned fp32 rows on a dense graph whose 32,768 longest rows hold much of the edges: chunks of one
    128-byte line.  Any of the conditions missing: one chunk."""
    import paper_2104_03058_amd as g
    N = 232965
    skewed = plan_of(N, {15: 60, 14: 700, 13: 4000, 12: 12000, 11: 25000, 10: 40000, 9: 50000, 8: 45000, 7: 30000,
                         6: 15000, 5: 8000})                 # power-law shaped: mean ~ 500, long tail of hubs
    flat = plan_of(N, {8: N})                                 # every row 128..255 edges
    sparse = plan_of(N, {12: 5, 8: 100, 3: 100000, 2: 100000})   # mean degree ~ 5
    assert g.gnnagg_auto_f_chunk(N, 602, g.F32, 608, skewed) == 32
    assert g.gnnagg_auto_f_chunk(N, 256, g.F32, 256, skewed) == 32
    assert g.gnnagg_auto_f_chunk(N, 602, g.F32, 602, skewed) == 602    # rows not on lines
    assert g.gnnagg_auto_f_chunk(N, 602, g.F32, 608, None) == 602      # no plan
    assert g.gnnagg_auto_f_chunk(N, 602, g.F32, 608, flat) == 602      # no hubs
    assert g.gnnagg_auto_f_chunk(N, 602, g.F32, 608, sparse) == 602    # low mean degree
    assert g.gnnagg_auto_f_chunk(N, 64, g.F32, 64, skewed) == 64       # narrower than four lines
    assert g.gnnagg_auto_f_chunk(N, 512, g.BF16, 512, skewed) == 128   # bf16: two lines per piece
    assert g.gnnagg_auto_f_chunk(N, 200, g.BF16, 256, skewed) == 200   # bf16 rows narrower than four lines
    assert g.gnnagg_auto_f_chunk(20000, 602, g.F32, 608, plan_of(20000, {12: 500, 9: 19500})) == 602  # fits one L2
    # one line per piece whatever the row count (long rows)
    def skewed_of(n):
        return plan_of(n, {13: n // 100, 11: n // 10, 9: n // 4, 8: n - n // 100 - n // 10 - n // 4})
    for n in (40000, 50000, 100000, 132534, 250000):
        assert g.gnnagg_auto_f_chunk(n, 1433, g.F32, 1440, skewed_of(n)) == 32
    assert g.gnnagg_auto_f_chunk(150000, 602, g.BF16, 640, skewed_of(150000)) == 128
    assert g.gnnagg_auto_f_chunk(45000, 512, g.BF16, 512, skewed_of(45000)) == 128
    # short rows do not amortise a pass: wider pieces at low mean degree, while the slice stays in the Infinity Cache
    def short_rows(n, c):  # hubs for the hot share, everything else in degree class c
        return plan_of(n, {14: n // 400, c: n - n // 400})
    assert g.gnnagg_auto_f_chunk(160000, 2048, g.F32, 2048, short_rows(160000, 4)) == 64    # mean degree ~42
    assert g.gnnagg_auto_f_chunk(160000, 2048, g.F32, 2048, short_rows(160000, 6)) == 32    # mean degree ~78
    assert g.gnnagg_auto_f_chunk(700000, 300, g.F32, 320, short_rows(700000, 4)) == 32      # two lines would be 180 MB


def test_bench_module_is_importable_and_its_workloads_name_known_graphs():
    """bench.py must import without a GPU (the GPU is touched only inside main)."""
    import importlib
    import workloads as W
    bench = importlib.import_module("bench")
    for name, (gkey, opname, F, xdt, gcn) in bench.WORKLOADS.items():
        assert gkey in W.GRAPHS, name
        assert opname in ("sum", "wsum", "mean", "max", "sum-ranked", "gat", "combine", "layer", "layer-ranked",
                          "layer-fused", "agg-dense", "mean-srcblock", "gcn-factored", "layer-factored"), name
        assert xdt in ("f32", "bf16"), name
    for name in bench.DEFAULT_ALSO + list(bench.CPU_BASELINE_ALSO) + list(bench.SINGLE_THREAD_ALSO):
        assert bench.split_name(name)[0] in bench.WORKLOADS, name
    # the sweeps the two benchmark configurations name are part of the default run
    for name in ["c1-gcn@16", "c1-gcn@64", "c1-gcn@all"] + ["c4-%s@%s" % (o, w) for o in ("gcn", "mean")
                                                            for w in ("8", "16", "32", "64", "all")]:
        assert name in bench.DEFAULT_ALSO, name
    assert bench.split_name("c4-gcn#4@64") == ("c4-gcn", 4, "64") and bench.split_name("c4-gcn#auto") == ("c4-gcn", -1, "")
    assert bench.split_name("c1-gcn@all") == ("c1-gcn", 0, "all")
    # line requests per edge: rows on lines, summed over the chunk passes
    assert bench.gather_lines_per_edge(602, 4, 608, 602) == 19
    assert bench.gather_lines_per_edge(602, 4, 608, 32) == 19
    assert bench.gather_lines_per_edge(602, 4, 608, 8) == 76
    assert bench.gather_lines_per_edge(100, 2, 128, 100) == 2
    assert bench.gather_lines_per_edge(16, 2, 16, 16) == 1
    assert bench.gather_lines_per_edge(100, 2, 100, 100) is None  # 200-byte pitch: rows straddle lines
    # traffic records in profiles/ carry what bench.py checks before it uses them
    for rec in bench.measured_traffic().values():
        assert {"workload", "kernel_sources", "kernel_source_hash", "fetch_bytes", "write_bytes", "source"} <= set(rec)
    assert len(bench.kernel_source_hash(bench.AGGREGATE_SOURCES)) == 16
    assert bench.kernel_source_hash(bench.AGGREGATE_SOURCES) != bench.kernel_source_hash(bench.GAT_SOURCES)


def test_traffic_records_under_profiles_were_taken_with_the_kernels_in_the_tree():
    """bench.py reports the counted traffic of a workload only from a profile whose recorded fingerprint of the
    kernel sources equals the tree's; a record that has gone stale would silently turn `roofline.traffic` into
    null, so the records kept under profiles/ are checked against the sources here."""
    import importlib
    bench = importlib.import_module("bench")
    recs = bench.measured_traffic()
    assert "c4-gcn#auto" in recs and "c4-gcn" in recs and "c5-sum" in recs and "c4-gat" in recs
    for name, rec in recs.items():
        assert rec["kernel_source_hash"] == bench.kernel_source_hash(rec["kernel_sources"]), \
            "%s: %s was taken with other kernel sources" % (name, rec["source"])
        assert rec["fetch_bytes"] > 0 and rec["write_bytes"] >= 0
