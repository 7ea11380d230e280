"""ctypes front end of the fp64 CPU oracle (oracle/psa_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests, the smoke check and the benchmark's
cpu_baseline leg may import this module.  It does not import the HIP binding and the HIP
binding does not import it.

Every array is numpy; 16-bit floating inputs travel as raw ``uint16`` bit patterns together with
``dtype`` (0 = IEEE binary16, 1 = bfloat16).  Shapes follow the C file's header.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "psa_oracle.c")
_LIB = os.path.join(_HERE, "libpsa_oracle.so")

F16, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over (request, query head) only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("batch", "num_q_heads", "num_kv_heads", "head_dim", "page_size", "num_pages",
                 "max_blocks", "dtype")]


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _p(a, ctype):
    return None if a is None else a.ctypes.data_as(C.POINTER(ctype))


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


@dataclass
class Problem:
    """One layer's paged KV, queries and tables, as the oracle consumes them."""
    q: np.ndarray            # uint16 [B][Hq][d]
    k_pool: np.ndarray       # uint16 [P][Hkv][T][d]
    v_pool: np.ndarray       # uint16 [P][Hkv][T][d]
    block_table: np.ndarray  # int32  [B][max_blocks]
    ctx_lens: np.ndarray     # int32  [B]
    dtype: int               # F16 or BF16

    def __post_init__(self):
        self.q, self.k_pool, self.v_pool = _u16(self.q), _u16(self.k_pool), _u16(self.v_pool)
        self.block_table, self.ctx_lens = _i32(self.block_table), _i32(self.ctx_lens)
        assert self.k_pool.shape == self.v_pool.shape and self.k_pool.ndim == 4
        assert self.q.ndim == 3 and self.q.shape[2] == self.k_pool.shape[3]
        assert self.q.shape[1] % self.k_pool.shape[1] == 0
        assert self.block_table.shape[0] == self.q.shape[0] == self.ctx_lens.shape[0]

    @property
    def shape(self) -> _Shape:
        P, H, T, D = self.k_pool.shape
        return _Shape(self.q.shape[0], self.q.shape[1], H, D, T, P, self.block_table.shape[1],
                      self.dtype)

    @property
    def dims(self):
        P, H, T, D = self.k_pool.shape
        return self.q.shape[0], self.q.shape[1], H, D, T, P, self.block_table.shape[1]

    def num_blocks(self) -> np.ndarray:
        T = self.k_pool.shape[2]
        return (self.ctx_lens + T - 1) // T

    def page_fill(self) -> np.ndarray:
        """Valid tokens per physical page implied by block_table and ctx_lens (0 = unused)."""
        P, _, T, _ = self.k_pool.shape
        fill = np.zeros(P, dtype=np.int32)
        for r, ctx in enumerate(self.ctx_lens):
            n = (int(ctx) + T - 1) // T
            if n == 0:
                continue
            pages = self.block_table[r, :n]
            fill[pages] = T
            fill[pages[-1]] = int(ctx) - (n - 1) * T
        return fill


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(C.c_int(n))


def decode(bits: np.ndarray, dtype: int) -> np.ndarray:
    """Exact decode of raw 16-bit patterns to float64 (numpy's own converters, for tests)."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def block_metadata(pb: Problem, page_fill=None) -> np.ndarray:
    P, H, T, D = pb.k_pool.shape
    meta = np.zeros((P, H, 2, D), dtype=np.uint16)
    fill = None if page_fill is None else _i32(page_fill)
    sh = pb.shape
    _load().oracle_block_metadata(C.byref(sh), _p(pb.k_pool, C.c_uint16), _p(fill, C.c_int32),
                                  _p(meta, C.c_uint16))
    return meta


def block_means(pb: Problem, page_fill=None) -> np.ndarray:
    """Mean-key metadata [P][H][D] (raw 16-bit patterns of the cache's type): see oracle_block_means."""
    P, H, T, D = pb.k_pool.shape
    means = np.zeros((P, H, D), dtype=np.uint16)
    fill = None if page_fill is None else _i32(page_fill)
    sh = pb.shape
    _load().oracle_block_means(C.byref(sh), _p(pb.k_pool, C.c_uint16), _p(fill, C.c_int32), _p(means, C.c_uint16))
    return means


UPPER_BOUND, CUBOID_CENTER, MEAN_KEY = 0, 1, 2      # scorers (Algorithm 1, line 5; see psa_oracle.c)


def block_scores(pb: Problem, meta: np.ndarray, scorer: int = UPPER_BOUND):
    """Returns (per-head scores [B][Hq][max_blocks], CS [B][Hkv][max_blocks]); -inf beyond each
    request's N."""
    B, Hq, H, D, T, P, MB = pb.dims
    ub = np.full((B, Hq, MB), -np.inf)
    cs = np.full((B, H, MB), -np.inf)
    sh = pb.shape
    _load().oracle_block_scores(C.byref(sh), _p(pb.q, C.c_uint16), _p(_u16(meta), C.c_uint16),
                                _p(pb.block_table, C.c_int32), _p(pb.ctx_lens, C.c_int32),
                                C.c_int32(scorer), _p(ub, C.c_double), _p(cs, C.c_double))
    return ub, cs


def block_order(pb: Problem, keys: np.ndarray) -> np.ndarray:
    B, Hq, H, D, T, P, MB = pb.dims
    keys = np.ascontiguousarray(keys, dtype=np.float64)
    assert keys.shape == (B, H, MB)
    order = np.full((B, H, MB), -1, dtype=np.int32)
    sh = pb.shape
    _load().oracle_block_order(C.byref(sh), _p(keys, C.c_double), _p(pb.ctx_lens, C.c_int32),
                               _p(order, C.c_int32))
    return order


def dense_attention(pb: Problem):
    B, Hq, H, D, T, P, MB = pb.dims
    out = np.zeros((B, Hq, D))
    lse = np.zeros((B, Hq))
    sh = pb.shape
    _load().oracle_dense_attention(C.byref(sh), _p(pb.q, C.c_uint16), _p(pb.k_pool, C.c_uint16),
                                   _p(pb.v_pool, C.c_uint16), _p(pb.block_table, C.c_int32),
                                   _p(pb.ctx_lens, C.c_int32), _p(out, C.c_double), _p(lse, C.c_double))
    return out, lse


def attend_prefix(pb: Problem, order: np.ndarray, n_take: np.ndarray, want_lse: bool = False):
    """Softmax attention over the first n_take ranked blocks, by the definition; with want_lse also
    the natural log of its denominator, sum over those tokens of exp(scaled logit)."""
    B, Hq, H, D, T, P, MB = pb.dims
    order, n_take = _i32(order), _i32(n_take)
    assert order.shape == (B, H, MB) and n_take.shape == (B, Hq)
    out = np.zeros((B, Hq, D))
    lse = np.zeros((B, Hq)) if want_lse else None
    sh = pb.shape
    _load().oracle_attend_prefix(C.byref(sh), _p(pb.q, C.c_uint16), _p(pb.k_pool, C.c_uint16),
                                 _p(pb.v_pool, C.c_uint16), _p(pb.block_table, C.c_int32),
                                 _p(pb.ctx_lens, C.c_int32), _p(order, C.c_int32),
                                 _p(n_take, C.c_int32), _p(out, C.c_double), _p(lse, C.c_double))
    return (out, lse) if want_lse else out


@dataclass
class DecodeResult:
    out: np.ndarray          # float64 [B][Hq][d]
    n_selected: np.ndarray   # int32 [B][Hq]
    mass_est: np.ndarray     # float64 [B][Hq]
    blocks_read: np.ndarray  # int32 [B][Hkv]
    order: np.ndarray        # int32 [B][Hkv][max_blocks]
    cs: np.ndarray | None = None           # float64 [B][Hkv][max_blocks]
    p_acc: np.ndarray | None = None        # float64 [B][Hq][max_blocks]
    true_mass: np.ndarray | None = None    # float64 [B][Hq][max_blocks]
    block_lse: np.ndarray | None = None    # float64 [B][Hq][max_blocks], in ranked order


def psa_decode_ordered(pb: Problem, order: np.ndarray, eps: float, m: int = 1,
                       curves: bool = False) -> DecodeResult:
    """Algorithm 1 over a GIVEN ranking (lines 7-19)."""
    B, Hq, H, D, T, P, MB = pb.dims
    order = _i32(order)
    assert order.shape == (B, H, MB)
    out = np.zeros((B, Hq, D))
    n_sel = np.zeros((B, Hq), dtype=np.int32)
    mass = np.zeros((B, Hq))
    bread = np.zeros((B, H), dtype=np.int32)
    pc = np.full((B, Hq, MB), np.nan) if curves else None
    tm = np.full((B, Hq, MB), np.nan) if curves else None
    ac = np.full((B, Hq, MB), np.nan) if curves else None
    sh = pb.shape
    _load().oracle_psa_decode(C.byref(sh), _p(pb.q, C.c_uint16), _p(pb.k_pool, C.c_uint16),
                              _p(pb.v_pool, C.c_uint16), _p(pb.block_table, C.c_int32),
                              _p(pb.ctx_lens, C.c_int32), _p(order, C.c_int32),
                              C.c_double(eps), C.c_int32(m), _p(out, C.c_double),
                              _p(n_sel, C.c_int32), _p(mass, C.c_double), _p(bread, C.c_int32),
                              _p(pc, C.c_double), _p(tm, C.c_double), _p(ac, C.c_double))
    return DecodeResult(out, n_sel, mass, bread, order, None, pc, tm, ac)


def psa_decode(pb: Problem, eps: float, m: int = 1, curves: bool = False,
               meta: np.ndarray | None = None, scorer: int = UPPER_BOUND) -> DecodeResult:
    """The whole path: metadata -> scores -> ranking -> progressive loop (Algorithm 1)."""
    if meta is None:
        meta = block_means(pb, pb.page_fill()) if scorer == MEAN_KEY else block_metadata(pb, pb.page_fill())
    _, cs = block_scores(pb, meta, scorer)
    order = block_order(pb, cs)
    res = psa_decode_ordered(pb, order, eps, m, curves)
    res.cs = cs
    return res


def topk_attention(pb: Problem, k: int, meta: np.ndarray | None = None,
                   scorer: int = UPPER_BOUND) -> DecodeResult:
    """Fixed-budget control (Sec. 1 and 2.2: what dynamic sparse attention does before PSA -- attend
    exactly the k blocks with the best criticality scores): metadata -> scores -> ranking, then the
    definition of attention over the first min(k, N) ranked blocks.  mass_est is Algorithm 1's P_acc
    evaluated there (lines 15-16), read off the full curve of a run that never stops."""
    if meta is None:
        meta = block_means(pb, pb.page_fill()) if scorer == MEAN_KEY else block_metadata(pb, pb.page_fill())
    _, cs = block_scores(pb, meta, scorer)
    order = block_order(pb, cs)
    B, Hq, H, D, T, P, MB = pb.dims
    G = Hq // H
    nb = pb.num_blocks()
    n_take = np.repeat(np.minimum(k, nb)[:, None], Hq, 1).astype(np.int32)
    out = attend_prefix(pb, order, n_take)
    curves = psa_decode_ordered(pb, order, 1.0, 1, curves=True)
    mass = np.zeros((B, Hq))
    for r in range(B):
        if nb[r]:
            mass[r] = curves.p_acc[r, :, n_take[r, 0] - 1]
    bread = n_take.reshape(B, H, G).max(-1).astype(np.int32)
    return DecodeResult(out, n_take, mass, bread, order, cs)


def append_kv(pb: Problem, k_new: np.ndarray, v_new: np.ndarray):
    """Incremental decode (Sec. 3.1: each step adds the new token's K/V to the cache; block metadata
    lives with the block): the cache after one more token per request.  k_new, v_new: uint16 bit
    patterns [B][Hkv][d].  Returns (the new Problem, status [B]) where status is 0, or 2 when the
    request's table row is full or its length is negative, or 1 when the table entry is outside the
    pool -- such a request is left as it was.  Metadata of the new cache is obtained the plain way,
    block_metadata(new, new.page_fill()): nothing incremental here."""
    B, Hq, H, D, T, P, MB = pb.dims
    k_pool, v_pool = pb.k_pool.copy(), pb.v_pool.copy()
    ctx = pb.ctx_lens.copy()
    status = np.zeros(B, dtype=np.int32)
    for r in range(B):
        c = int(ctx[r])
        if c < 0 or c >= MB * T:
            status[r] = 2
            continue
        page = int(pb.block_table[r, c // T])
        if page < 0 or page >= P:
            status[r] = 1
            continue
        k_pool[page, :, c % T, :] = k_new[r]
        v_pool[page, :, c % T, :] = v_new[r]
        ctx[r] = c + 1
    return Problem(pb.q, k_pool, v_pool, pb.block_table, ctx, pb.dtype), status
