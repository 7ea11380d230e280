"""Brute-force numpy/scipy helpers the oracle is pinned against.

They use library routines only (numpy matmul, scipy softmax / logsumexp, numpy's own fp16
converter) and never call the oracle's C code, so agreement between the two is evidence about
both.  Small inputs only.
"""
from __future__ import annotations

import numpy as np
from scipy.special import logsumexp, softmax

from oracle import psa_oracle as po


def random_problem(rng, B=2, Hq=4, Hkv=2, d=16, T=4, ctx=(9, 16), dtype=po.F16, shuffle=True,
                   spare_pages=2, scale=1.0):
    """A small paged problem with arbitrary sizes (the oracle is not tied to d=128, T=16)."""
    ctx = np.asarray(ctx, dtype=np.int32)
    assert len(ctx) == B
    nblk = (ctx + T - 1) // T
    P = int(nblk.sum()) + spare_pages
    pages = rng.permutation(P) if shuffle else np.arange(P)
    MB = max(1, int(nblk.max()))
    table = np.zeros((B, MB), dtype=np.int32)
    off = 0
    for r in range(B):
        table[r, :nblk[r]] = pages[off:off + nblk[r]]
        off += nblk[r]

    def draw(shape):
        x = (rng.standard_normal(shape) * scale).astype(np.float32)
        if dtype == po.F16:
            return x.astype(np.float16).view(np.uint16)
        bits = x.view(np.uint32)
        bits = (bits + 0x7FFF + ((bits >> 16) & 1)) >> 16  # round to nearest even
        return bits.astype(np.uint16)

    return po.Problem(draw((B, Hq, d)), draw((P, Hkv, T, d)), draw((P, Hkv, T, d)), table, ctx, dtype)


def stream_kv(pb, r, h):
    """Decoded keys and values of stream (r, h): [ctx][d] each, in logical token order."""
    T = pb.k_pool.shape[2]
    ctx = int(pb.ctx_lens[r])
    n = (ctx + T - 1) // T
    pages = pb.block_table[r, :n]
    k = po.decode(pb.k_pool[pages, h], pb.dtype).reshape(n * T, -1)[:ctx]
    v = po.decode(pb.v_pool[pages, h], pb.dtype).reshape(n * T, -1)[:ctx]
    return k, v


def logits(pb, r, hq):
    G = pb.q.shape[1] // pb.k_pool.shape[1]
    k, _ = stream_kv(pb, r, hq // G)
    q = po.decode(pb.q[r, hq], pb.dtype)
    return k @ q / np.sqrt(pb.q.shape[2])


def dense(pb):
    B, Hq, d = pb.q.shape
    G = Hq // pb.k_pool.shape[1]
    out = np.zeros((B, Hq, d))
    lse = np.full((B, Hq), -np.inf)
    for r in range(B):
        if pb.ctx_lens[r] == 0:
            continue
        for hq in range(Hq):
            s = logits(pb, r, hq)
            _, v = stream_kv(pb, r, hq // G)
            out[r, hq] = softmax(s) @ v
            lse[r, hq] = logsumexp(s)
    return out, lse


def attend_blocks(pb, r, hq, blocks):
    """Softmax attention of head (r, hq) over the tokens of the listed logical blocks."""
    T = pb.k_pool.shape[2]
    G = pb.q.shape[1] // pb.k_pool.shape[1]
    ctx = int(pb.ctx_lens[r])
    tok = np.concatenate([np.arange(b * T, min((b + 1) * T, ctx)) for b in blocks]) if len(blocks) \
        else np.zeros(0, dtype=int)
    if tok.size == 0:
        return np.zeros(pb.q.shape[2])
    s = logits(pb, r, hq)[tok]
    _, v = stream_kv(pb, r, hq // G)
    return softmax(s) @ v[tok]


def block_lse(pb, r, hq):
    """log of each logical block's sum of exponentiated logits (log AS_b)."""
    T = pb.k_pool.shape[2]
    s = logits(pb, r, hq)
    n = (len(s) + T - 1) // T
    return np.array([logsumexp(s[b * T:(b + 1) * T]) for b in range(n)])


def p_acc_curve(lse_ranked):
    """P_acc(n) of Algorithm 1 lines 12-16 from the ranked blocks' log AS, n = 1..N."""
    N = len(lse_ranked)
    ref = np.max(lse_ranked)
    a = np.exp(lse_ranked - ref)
    acc = np.cumsum(a)
    amin = np.minimum.accumulate(a)
    left = N - np.arange(1, N + 1)
    return acc / (acc + amin * left)


def first_stop(p, eps, m):
    """First n (1-based) that is a multiple of m, or N, with float32(P_acc) > float32(eps)."""
    N = len(p)
    for n in range(1, N + 1):
        if (n % m == 0 or n == N) and (np.float32(p[n - 1]) > np.float32(eps) or n == N):
            return n
    return N
