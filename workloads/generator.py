"""Seeded synthetic long-context decode inputs: planted-critical-token KV caches.

This module serves BOTH the CPU oracle's tests and the HIP path's tests / benchmark, and holds none
of the method's arithmetic: it only draws random numbers, plants structure, rounds to the storage
type and lays pages out.  The rounded 16-bit patterns it returns are *the* input; both sides
consume the same bytes.

They stand in for the long-context workloads the paper measures on (LongBench subsets run through
LWM-Text-7B and Llama-3.1-8B, Sec. 5.1), which need model weights and datasets that are not
available here.  The recipe keeps what matters to the method: a few tokens carry most of the
attention mass, how few differs strongly between KV heads, requests and layers (Sec. 2.3), contexts
reach 128K tokens, pages are 16 tokens and scattered through a pool.

Recipe, per (layer, request, KV head), from a sub-seed of (seed, layer, request, kv_head):
  * v: a random unit direction in R^d.
  * queries of the group: q_g = sqrt(d) * v + N(0, I), one draw per query head.
  * background keys N(0, I): scaled logits q.k/sqrt(d) are about N(0, 2).
  * critical keys N(0, I) + 6 v: about +6 on the logit.
  * critical tokens: the first 16 tokens, the last 64 tokens, and a fraction f of the positions in
    between, placed as runs of uniform length 1..16 whose starts are uniform (runs may overlap, so
    the realised fraction is a little below f).
  * values N(0, I).
  * "uniform" configs (no planted tokens): keys N(0, 0.1^2), queries N(0, I).
Everything is drawn in float32 and rounded to nearest-even to fp16 / bf16.
Choices the configs leave open, fixed here: v is drawn per (request, KV head); the fraction f is
drawn per KV head, per layer or fixed as the config says; context lengths of the ragged config are
log-uniform integers; a random block table is ONE random permutation of all physical pages.
Tokens of a last page beyond the context length are filled with NaN when ``poison_tail`` is set
(a real paged cache holds garbage there), else with zeros.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace

import numpy as np
import torch

PAGE = 16
HEAD_DIM = 128


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    index: int                 # 1..5, as the configs are numbered
    layers: int
    batch: int
    num_q_heads: int
    num_kv_heads: int
    ctx: int                   # fixed context length, or the upper bound when ragged
    dtype: str                 # "f16" | "bf16"
    threshold: float
    ctx_min: int = 0           # > 0: context lengths log-uniform in [ctx_min, ctx]
    frac: float = 0.01         # fixed critical fraction
    frac_range: tuple = ()     # (lo, hi): log-uniform draw
    frac_per: str = "fixed"    # "fixed" | "kv_head" | "layer"
    dense_layers: int = 0      # the first such layers use fraction 0.5
    random_table: bool = False
    planted: bool = True
    extra_thresholds: tuple = ()

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    def scaled(self, **kw) -> "WorkloadConfig":
        """A smaller copy of the same recipe (tests)."""
        return replace(self, **kw)


CONFIGS = {
    1: WorkloadConfig("c1_4k_b1", 1, 1, 1, 32, 8, 4096, "f16", 0.90, frac=0.01),
    2: WorkloadConfig("c2_32k_b8", 2, 1, 8, 32, 8, 32768, "f16", 0.95,
                      frac_range=(0.005, 0.10), frac_per="kv_head"),
    3: WorkloadConfig("c3_128k_b4_l32", 3, 32, 4, 32, 8, 131072, "bf16", 0.95,
                      frac_range=(0.002, 0.20), frac_per="layer", dense_layers=2,
                      random_table=True),
    4: WorkloadConfig("c4_ragged_b64_g8", 4, 1, 64, 64, 8, 131072, "f16", 0.98, ctx_min=4096,
                      frac=0.02, random_table=True),
    5: WorkloadConfig("c5_uniform_64k_b16", 5, 1, 16, 32, 8, 65536, "bf16", 0.95, planted=False,
                      extra_thresholds=(0.99,)),
}


def get_config(index: int) -> WorkloadConfig:
    return CONFIGS[index]


def base_seed(index: int) -> int:
    return 250300392 * 10 + index


def _torch_dtype(name: str):
    return {"f16": torch.float16, "bf16": torch.bfloat16}[name]


def _sub_seed(seed: int, *keys: int) -> int:
    """A 63-bit mix of the seed and integer keys (splitmix-style), independent of any device."""
    x = seed & 0xFFFFFFFFFFFFFFFF
    for k in keys:
        x = (x + 0x9E3779B97F4A7C15 + (k & 0xFFFFFFFF) * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 30
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 27
        x = (x * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
    return x & 0x7FFFFFFFFFFFFFFF


def _host_rng(seed: int, *keys: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(_sub_seed(seed, *keys)))


@dataclass
class LayerInputs:
    """One layer's inputs.  Tensors live on ``device``; 16-bit floats in the config's dtype."""
    cfg: WorkloadConfig
    layer: int
    q: torch.Tensor            # [B][Hq][d]
    k_pool: torch.Tensor       # [P][Hkv][16][d]
    v_pool: torch.Tensor       # [P][Hkv][16][d]
    block_table: torch.Tensor  # int32 [B][max_blocks]
    ctx_lens: torch.Tensor     # int32 [B]
    page_fill: torch.Tensor    # int32 [P]  valid tokens per physical page
    frac: np.ndarray = field(default=None)  # [B][Hkv] critical fraction used (0 when not planted)

    @property
    def dtype_code(self) -> int:
        return 0 if self.cfg.dtype == "f16" else 1

    @property
    def max_blocks(self) -> int:
        return self.block_table.shape[1]


def as_bits(t: torch.Tensor) -> np.ndarray:
    """Raw 16-bit patterns of an fp16 / bf16 tensor as a host uint16 array (a copy)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16).copy()


def context_lengths(cfg: WorkloadConfig, seed: int) -> np.ndarray:
    if cfg.ctx_min <= 0:
        return np.full(cfg.batch, cfg.ctx, dtype=np.int64)
    rng = _host_rng(seed, 101)
    u = rng.random(cfg.batch)
    lens = np.exp(np.log(cfg.ctx_min) + u * (np.log(cfg.ctx) - np.log(cfg.ctx_min)))
    return np.clip(np.rint(lens).astype(np.int64), cfg.ctx_min, cfg.ctx)


def critical_fractions(cfg: WorkloadConfig, seed: int, layer: int) -> np.ndarray:
    """[B][Hkv] fraction of planted critical positions."""
    B, H = cfg.batch, cfg.num_kv_heads
    if not cfg.planted:
        return np.zeros((B, H))
    if layer < cfg.dense_layers:
        return np.full((B, H), 0.5)
    if cfg.frac_per == "fixed":
        return np.full((B, H), cfg.frac)
    lo, hi = cfg.frac_range
    if cfg.frac_per == "layer":
        u = _host_rng(seed, 202, layer).random()
        return np.full((B, H), float(np.exp(np.log(lo) + u * (np.log(hi) - np.log(lo)))))
    u = _host_rng(seed, 203, layer).random((B, H))
    return np.exp(np.log(lo) + u * (np.log(hi) - np.log(lo)))


def _critical_mask(n_tok: int, frac: float, gen: torch.Generator, device) -> torch.Tensor:
    mask = torch.zeros(n_tok, dtype=torch.bool, device=device)
    mask[: min(16, n_tok)] = True
    mask[max(0, n_tok - 64):] = True
    lo, hi = 16, n_tok - 64
    if hi > lo and frac > 0:
        n_mid = hi - lo
        n_runs = max(1, int(round(frac * n_mid / 8.5)))
        starts = torch.randint(0, n_mid, (n_runs,), generator=gen, device=device)
        lens = torch.randint(1, 17, (n_runs,), generator=gen, device=device)
        ends = torch.clamp(starts + lens, max=n_mid)
        delta = torch.zeros(n_mid + 1, dtype=torch.int32, device=device)
        one = torch.ones(n_runs, dtype=torch.int32, device=device)
        delta.scatter_add_(0, starts, one)
        delta.scatter_add_(0, ends, -one)
        mask[lo:hi] |= torch.cumsum(delta[:-1], 0) > 0
    return mask


def generate_layer(cfg: WorkloadConfig, layer: int = 0, seed: int | None = None,
                   device: str | torch.device = "cpu", poison_tail: bool = False) -> LayerInputs:
    """Build one layer of ``cfg`` on ``device``.  Deterministic for a given (cfg, layer, seed,
    device type); the same call hands the same bytes to the oracle and to the HIP path."""
    if seed is None:
        seed = base_seed(cfg.index)
    device = torch.device(device)
    dt = _torch_dtype(cfg.dtype)
    B, Hq, H, G, d = cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.group, HEAD_DIM
    ctx = context_lengths(cfg, seed)
    nblk = (ctx + PAGE - 1) // PAGE
    max_blocks = int(nblk.max()) if B else 0
    total = int(nblk.sum())

    # block table: identity packing, or one random permutation of all physical pages
    if cfg.random_table:
        perm = _host_rng(seed, 303, layer).permutation(total).astype(np.int32)
    else:
        perm = np.arange(total, dtype=np.int32)
    table = np.zeros((B, max(max_blocks, 1)), dtype=np.int32)
    fill = np.zeros(max(total, 1), dtype=np.int32)
    off = 0
    for r in range(B):
        n = int(nblk[r])
        table[r, :n] = perm[off:off + n]
        if n:
            fill[perm[off:off + n]] = PAGE
            fill[perm[off + n - 1]] = int(ctx[r]) - (n - 1) * PAGE
        off += n

    fracs = critical_fractions(cfg, seed, layer)
    k_pool = torch.zeros((max(total, 1), H, PAGE, d), dtype=dt, device=device)
    v_pool = torch.zeros_like(k_pool)
    q = torch.zeros((B, Hq, d), dtype=dt, device=device)
    tail_fill = float("nan") if poison_tail else 0.0

    for r in range(B):
        n_tok, n = int(ctx[r]), int(nblk[r])
        pages = torch.from_numpy(table[r, :n].astype(np.int64)).to(device)
        for h in range(H):
            gen = torch.Generator(device=device)
            gen.manual_seed(_sub_seed(seed, 404, layer, r, h))
            if cfg.planted:
                v = torch.randn(d, generator=gen, device=device)
                v = v / v.norm()
                qg = math.sqrt(d) * v + torch.randn((G, d), generator=gen, device=device)
            else:
                qg = torch.randn((G, d), generator=gen, device=device)
            q[r, h * G:(h + 1) * G] = qg.to(dt)
            if n == 0:
                continue
            keys = torch.randn((n * PAGE, d), generator=gen, device=device)
            if cfg.planted:
                mask = _critical_mask(n_tok, float(fracs[r, h]), gen, device)
                keys[:n_tok][mask] += 6.0 * v
            else:
                keys *= 0.1
            vals = torch.randn((n * PAGE, d), generator=gen, device=device)
            if n_tok < n * PAGE:
                keys[n_tok:] = tail_fill
                vals[n_tok:] = tail_fill
            k_pool[pages, h] = keys.to(dt).view(n, PAGE, d)
            v_pool[pages, h] = vals.to(dt).view(n, PAGE, d)
            del keys, vals

    return LayerInputs(cfg, layer, q, k_pool, v_pool,
                       torch.from_numpy(table).to(device),
                       torch.from_numpy(ctx.astype(np.int32)).to(device),
                       torch.from_numpy(fill).to(device), fracs)


def add_headroom(li: LayerInputs, extra_tokens: int) -> LayerInputs:
    """The same cache with room to append `extra_tokens` tokens per request: every row of the block
    table is extended with fresh pages, which sit at the end of the pools (zero-filled, fill 0)."""
    B = li.ctx_lens.numel()
    ctx = li.ctx_lens.cpu().numpy().astype(np.int64)
    have = (ctx + PAGE - 1) // PAGE
    need = (ctx + extra_tokens + PAGE - 1) // PAGE
    extra = int((need - have).sum())
    P0 = li.k_pool.shape[0]
    pad = torch.zeros((extra,) + tuple(li.k_pool.shape[1:]), dtype=li.k_pool.dtype, device=li.k_pool.device)
    table = np.zeros((B, max(int(need.max()), 1)), dtype=np.int32)
    old = li.block_table.cpu().numpy()
    nxt = P0
    for r in range(B):
        table[r, :have[r]] = old[r, :have[r]]
        for b in range(int(have[r]), int(need[r])):
            table[r, b] = nxt
            nxt += 1
    dev = li.k_pool.device
    return LayerInputs(cfg=li.cfg, layer=li.layer, q=li.q.clone(),
                       k_pool=torch.cat([li.k_pool, pad]).contiguous(), v_pool=torch.cat([li.v_pool, pad]).contiguous(),
                       block_table=torch.from_numpy(table).to(dev), ctx_lens=li.ctx_lens.clone(),
                       page_fill=torch.cat([li.page_fill, torch.zeros(extra, dtype=torch.int32, device=dev)]).contiguous(),
                       frac=li.frac)


def step_inputs(li: LayerInputs, step: int, seed: int | None = None):
    """Inputs of decode step `step` = 1, 2, ... after the cache `li` was built: (q, k_new, v_new).
    Queries drift slowly (each step adds a small seeded perturbation to the previous step's query:
    consecutive decode queries are similar), the new token's keys and values are drawn like
    background tokens.  Rounded to the cache's 16-bit type; the rounded bits are the input."""
    if seed is None:
        seed = base_seed(li.cfg.index)
    dev = li.q.device
    dt = li.q.dtype
    B, Hq, d = li.q.shape
    H = li.k_pool.shape[1]
    q = li.q.float()
    for t in range(1, step + 1):
        g = torch.Generator(device="cpu")
        g.manual_seed(_sub_seed(seed, 707, li.layer, t))
        q = q + 0.15 * torch.randn((B, Hq, d), generator=g).to(dev)
    g = torch.Generator(device="cpu")
    g.manual_seed(_sub_seed(seed, 709, li.layer, step))
    k_new = torch.randn((B, H, d), generator=g).to(dev).to(dt)
    v_new = torch.randn((B, H, d), generator=g).to(dev).to(dt)
    return q.to(dt).contiguous(), k_new.contiguous(), v_new.contiguous()
