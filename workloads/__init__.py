"""Seeded synthetic workloads: graphs and feature matrices shaped like the
paper's evaluation inputs (Section III, Table II), produced by ``synth.c``.

This package generates *inputs* only.  It contains none of the aggregation
arithmetic, and is the one module both the CPU checker's tests and the GPU
harness import, so that both sides consume identical bytes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "synth.c")
_LIB = os.path.join(_HERE, "libgnnagg_synth.so")


def build(force: bool = False) -> str:
    """Compile synth.c with gcc (a second or two)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, u64, dbl, f32, i32 = ctypes.c_int64, ctypes.c_uint64, ctypes.c_double, ctypes.c_float, ctypes.c_int32
        vp = ctypes.c_void_p
        lib.synth_powerlaw_graph.restype = i64
        lib.synth_powerlaw_graph.argtypes = [i64, i64, dbl, dbl, u64, ctypes.c_int, vp, vp]
        lib.synth_normal_f32.restype = None
        lib.synth_normal_f32.argtypes = [i64, u64, f32, f32, vp]
        lib.synth_normal_bf16.restype = None
        lib.synth_normal_bf16.argtypes = [i64, u64, f32, f32, vp]
        lib.synth_f32_to_bf16.restype = None
        lib.synth_f32_to_bf16.argtypes = [i64, vp, vp]
        lib.synth_bernoulli_f32.restype = None
        lib.synth_bernoulli_f32.argtypes = [i64, dbl, u64, vp]
        lib.synth_randint_i32.restype = None
        lib.synth_randint_i32.argtypes = [i64, i32, u64, u64, vp]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def powerlaw_graph(N: int, M: int, alpha: float, R: float, seed: int, cover_all: bool = False):
    """Symmetric simple graph: returns (src, dst) int32 arrays of 2*M directed edges."""
    src = np.empty(2 * M, dtype=np.int32)
    dst = np.empty(2 * M, dtype=np.int32)
    r = _load().synth_powerlaw_graph(N, M, alpha, R, seed, int(cover_all), _ptr(src), _ptr(dst))
    if r < 0:
        raise RuntimeError("graph generation failed (N=%d M=%d alpha=%g R=%g)" % (N, M, alpha, R))
    return src, dst


def normal_f32(shape, seed: int, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().synth_normal_f32(out.size, seed, mean, std, _ptr(out))
    return out


def normal_bf16(shape, seed: int, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """bf16 bit patterns (uint16), N(mean, std) rounded to nearest even."""
    out = np.empty(shape, dtype=np.uint16)
    _load().synth_normal_bf16(out.size, seed, mean, std, _ptr(out))
    return out


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    _load().synth_f32_to_bf16(x.size, _ptr(x), _ptr(out))
    return out


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns."""
    return (b.astype(np.uint32) << 16).view(np.float32)


def bernoulli_f32(shape, p: float, seed: int) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().synth_bernoulli_f32(out.size, p, seed, _ptr(out))
    return out


def randint_i32(n: int, hi: int, seed: int, stream: int = 0) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    _load().synth_randint_i32(n, hi, seed, stream, _ptr(out))
    return out


def random_digraph(N: int, E: int, seed: int):
    """Directed multigraph with E uniformly drawn edges (duplicates and self
    pairs allowed): the case that exposes a transposed CSR."""
    return randint_i32(E, N, seed, 0), randint_i32(E, N, seed, 1)


# --------------------------------------------------------------------------
# The five benchmark workloads.  (N, undirected M, Pareto exponent, cap R,
# seed, cover_all).  R bounds the propensity law.  It is calibrated so that the
# realised maximum degree is about 21k on the dense graph, about 20k on the
# very large sparse graph (an uncapped exponent-2 law would put several percent
# of all edges on one vertex) and 130-200 on the two small graphs.
# --------------------------------------------------------------------------
@dataclass
class GraphSpec:
    name: str
    N: int
    M: int
    alpha: float
    R: float
    seed: int
    cover_all: bool = False
    kind: str = "powerlaw"  # "uniform": M directed edges with independent uniform endpoints (alpha, R unused)


GRAPHS = {
    "c1": GraphSpec("c1-tiny", 2708, 5278, 2.1, 200.0, 0, True),
    "c2": GraphSpec("c2-mid", 19717, 44324, 2.1, 200.0, 1, False),
    "c4": GraphSpec("c4-dense", 232965, 57307946, 1.8, 680.0, 3, False),
    "c5": GraphSpec("c5-sparse", 2449029, 30950000, 2.0, 9000.0, 4, False),
    # the paper's third evaluation graph (Table II: 132,534 vertices, average degree 597): realised max degree ~6.6k
    "c6": GraphSpec("c6-dense-small", 132534, 39561252, 1.8, 60.0, 6, False),
    # Measurement aids, not benchmark shapes: uniform random directed graphs that pin the source rows of a
    # gather to one level of the memory system.  u-l2: the dense graph's edge count on so few vertices that
    # one 128-byte line per vertex (3.7 MB) stays in a 4 MB L2; u-hbm: 16.8 M vertices, so that even one
    # line per vertex (2.1 GB) is many times the 256 MB Infinity Cache and nearly every gather comes from HBM;
    "u-l2": GraphSpec("uniform-l2-resident", 29120, 114615892, 0.0, 0.0, 7, False, "uniform"),
    "u-hbm": GraphSpec("uniform-hbm-resident", 16777216, 67108864, 0.0, 0.0, 8, False, "uniform"),
    # u-mall: one line per vertex is 134 MB, 32 times one L2 and half the Infinity Cache; u-hbmw: 2.1 M
    # vertices for rows of 2.4 KB (5.1 GB), the dense benchmark's row width without any reuse.
    "u-mall": GraphSpec("uniform-infinity-cache-resident", 1048576, 67108864, 0.0, 0.0, 9, False, "uniform"),
    "u-hbmw": GraphSpec("uniform-hbm-resident-wide-rows", 2097152, 33554432, 0.0, 0.0, 10, False, "uniform"),
}


def graph(key: str, scale: float = 1.0):
    """COO edges of a benchmark graph.  scale < 1 shrinks N and M together
    (same mean degree and law) for parity cases the CPU checker finishes fast."""
    g = GRAPHS[key]
    N = max(16, int(round(g.N * scale)))
    M = max(8, int(round(g.M * scale)))
    if g.kind == "uniform":
        src, dst = random_digraph(N, M, g.seed)
        return N, src, dst
    src, dst = powerlaw_graph(N, M, g.alpha, g.R, g.seed, g.cover_all)
    return N, src, dst
