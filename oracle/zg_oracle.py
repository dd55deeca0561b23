"""ctypes access to the CPU checker (oracle/zg_oracle.c).  Test infrastructure only: tests,
the smoke check and the benchmark's CPU-baseline leg may import this; the product path never does.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libzg_oracle.so")
MAX_HOPS = 8


def build(force: bool = False) -> str:
    """Compile the checker with gcc (no fast-math, no FMA contraction)."""
    src = os.path.join(_HERE, "zg_oracle.c")
    hdr = os.path.join(_HERE, "zg_oracle.h")
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
        return _LIB_PATH
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-Wall", "-Wextra",
           "-o", _LIB_PATH, src]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


class _Graph(C.Structure):
    _fields_ = [("num_nodes", C.c_int64), ("num_edges", C.c_int64), ("offsets", C.c_void_p),
                ("offsets_is_i64", C.c_int32), ("indices", C.c_void_p)]


class _Blocks(C.Structure):
    _fields_ = [("num_hops", C.c_int32), ("n", C.c_int64 * (MAX_HOPS + 1)), ("E", C.c_int64 * MAX_HOPS),
                ("S", C.POINTER(C.c_int32)), ("row_ptr", C.POINTER(C.c_int32) * MAX_HOPS),
                ("nbr_gid", C.POINTER(C.c_int32) * MAX_HOPS), ("col", C.POINTER(C.c_int32) * MAX_HOPS)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB_PATH)
        L.zgo_philox4x32_10.argtypes = [C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        L.zgo_philox4x32_10.restype = None
        L.zgo_mulhi64.argtypes = [C.c_uint64, C.c_uint64]
        L.zgo_mulhi64.restype = C.c_uint64
        L.zgo_draw.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32]
        L.zgo_draw.restype = C.c_uint64
        L.zgo_floyd_resolve.argtypes = [C.c_int64, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.zgo_floyd_resolve.restype = None
        L.zgo_sample_positions.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int64, C.c_int32, C.c_int32,
                                           C.POINTER(C.c_int64)]
        L.zgo_sample_positions.restype = C.c_int32
        L.zgo_sample_blocks.argtypes = [C.POINTER(_Graph), C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32,
                                        C.c_uint64, C.c_int32, C.POINTER(_Blocks)]
        L.zgo_sample_blocks.restype = C.c_int
        L.zgo_blocks_free.argtypes = [C.POINTER(_Blocks)]
        L.zgo_blocks_free.restype = None
        L.zgo_gather.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64]
        L.zgo_gather.restype = None
        L.zgo_aggregate_mean.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32,
                                         C.c_void_p, C.c_int64]
        L.zgo_aggregate_mean.restype = None
        _lib = L
    return _lib


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> List[int]:
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().zgo_philox4x32_10(c, k, o)
    return list(o)


def mulhi64(a: int, b: int) -> int:
    return int(lib().zgo_mulhi64(a, b))


def draw(rng_key: int, hop: int, node: int, slot: int) -> int:
    return int(lib().zgo_draw(rng_key, hop, node, slot))


def floyd_resolve(deg: int, F: int, t: Sequence[int]) -> List[int]:
    tt = (C.c_int64 * F)(*t)
    pos = (C.c_int64 * F)()
    lib().zgo_floyd_resolve(deg, F, tt, pos)
    return list(pos)


def sample_positions(rng_key: int, hop: int, node: int, deg: int, F: int, with_replacement: bool = False) -> List[int]:
    pos = (C.c_int64 * max(F, 1))()
    k = lib().zgo_sample_positions(rng_key, hop, node, deg, F, int(with_replacement), pos)
    assert k >= 0
    return list(pos[:k])


@dataclass
class Blocks:
    n: List[int]            # n[0..H]
    E: List[int]            # E[0..H-1]
    S: np.ndarray           # int32 [n[H]]
    row_ptr: List[np.ndarray]
    nbr_gid: List[np.ndarray]
    col: List[np.ndarray]


class Graph:
    """Host CSR (numpy int32/int64 offsets, int32 indices) for the checker."""

    def __init__(self, offsets: np.ndarray, indices: np.ndarray):
        assert offsets.dtype in (np.int32, np.int64) and indices.dtype == np.int32
        self.offsets = np.ascontiguousarray(offsets)
        self.indices = np.ascontiguousarray(indices)
        self.num_nodes = self.offsets.shape[0] - 1
        self._c = _Graph(self.num_nodes, self.indices.shape[0], self.offsets.ctypes.data,
                         1 if offsets.dtype == np.int64 else 0, self.indices.ctypes.data)

    def sample_blocks(self, seeds: np.ndarray, fanouts: Sequence[int], rng_key: int,
                      with_replacement: bool = False) -> Blocks:
        seeds = np.ascontiguousarray(seeds, dtype=np.int32)
        H = len(fanouts)
        f = (C.c_int32 * H)(*fanouts)
        b = _Blocks()
        rc = lib().zgo_sample_blocks(C.byref(self._c), seeds.ctypes.data, seeds.shape[0], f, H,
                                     C.c_uint64(rng_key & 0xFFFFFFFFFFFFFFFF), int(with_replacement), C.byref(b))
        if rc != 0:
            raise ValueError(f"zgo_sample_blocks failed with {rc}")
        try:
            n = [int(b.n[h]) for h in range(H + 1)]
            E = [int(b.E[h]) for h in range(H)]
            S = np.ctypeslib.as_array(b.S, shape=(n[H],)).copy()
            rp = [np.ctypeslib.as_array(b.row_ptr[h], shape=(n[h] + 1,)).copy() for h in range(H)]
            nb = [np.ctypeslib.as_array(b.nbr_gid[h], shape=(max(E[h], 1),))[:E[h]].copy() for h in range(H)]
            col = [np.ctypeslib.as_array(b.col[h], shape=(max(E[h], 1),))[:E[h]].copy() for h in range(H)]
        finally:
            lib().zgo_blocks_free(C.byref(b))
        return Blocks(n, E, S, rp, nb, col)


def gather(feat: np.ndarray, ids: np.ndarray, dim: Optional[int] = None) -> np.ndarray:
    assert feat.dtype == np.float32 and feat.ndim == 2 and feat.strides[1] == 4
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    dim = feat.shape[1] if dim is None else dim
    X = np.empty((ids.shape[0], dim), dtype=np.float32)
    lib().zgo_gather(feat.ctypes.data, feat.strides[0] // 4, dim, ids.ctypes.data, ids.shape[0], X.ctypes.data, dim)
    return X


def aggregate_mean(row_ptr: np.ndarray, col: np.ndarray, X: np.ndarray) -> np.ndarray:
    assert X.dtype == np.float32 and X.ndim == 2 and X.strides[1] == 4
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    n_rows = row_ptr.shape[0] - 1
    dim = X.shape[1]
    out = np.empty((n_rows, dim), dtype=np.float32)
    lib().zgo_aggregate_mean(row_ptr.ctypes.data, col.ctypes.data, n_rows, X.ctypes.data, X.strides[0] // 4, dim,
                             out.ctypes.data, dim)
    return out


def step(graph: Graph, seeds: np.ndarray, fanouts: Sequence[int], rng_key: int, feat: Optional[np.ndarray] = None,
         with_replacement: bool = False):
    """One whole pass: blocks, gathered rows X for S_{H-1}, mean aggregation on the innermost block."""
    blocks = graph.sample_blocks(seeds, fanouts, rng_key, with_replacement)
    if feat is None:
        return blocks, None, None
    X = gather(feat, blocks.S)
    agg = aggregate_mean(blocks.row_ptr[-1], blocks.col[-1], X)
    return blocks, X, agg
