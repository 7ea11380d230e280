"""The seeded generator: determinism, layout and the planted structure the recipe promises."""
import numpy as np
import torch

import np_reference as ref
from oracle import psa_oracle as po
from workloads import CONFIGS, as_bits, generate_layer, get_config


def _problem(li):
    return po.Problem(as_bits(li.q), as_bits(li.k_pool), as_bits(li.v_pool),
                      li.block_table.numpy(), li.ctx_lens.numpy(), li.dtype_code)


def test_configs_match_the_five_named_workloads():
    c = CONFIGS
    assert (c[1].batch, c[1].ctx, c[1].dtype, c[1].threshold) == (1, 4096, "f16", 0.90)
    assert (c[2].batch, c[2].ctx, c[2].threshold, c[2].frac_per) == (8, 32768, 0.95, "kv_head")
    assert (c[3].layers, c[3].batch, c[3].ctx, c[3].dtype, c[3].random_table) == (32, 4, 131072, "bf16", True)
    assert (c[4].batch, c[4].num_q_heads, c[4].group, c[4].ctx_min, c[4].threshold) == (64, 64, 8, 4096, 0.98)
    assert (c[5].planted, c[5].batch, c[5].ctx, c[5].extra_thresholds) == (False, 16, 65536, (0.99,))


def test_deterministic_and_layout():
    cfg = get_config(4).scaled(batch=3, ctx=700, ctx_min=100)
    a, b = generate_layer(cfg), generate_layer(cfg)
    for x, y in ((a.q, b.q), (a.k_pool, b.k_pool), (a.v_pool, b.v_pool), (a.block_table, b.block_table)):
        assert torch.equal(x.view(torch.int16) if x.is_floating_point() else x,
                           y.view(torch.int16) if y.is_floating_point() else y)
    ctx = a.ctx_lens.numpy()
    assert ctx.min() >= 100 and ctx.max() <= 700
    nblk = (ctx + 15) // 16
    assert a.k_pool.shape == (nblk.sum(), 8, 16, 128) and a.q.shape == (3, 64, 128)
    used = np.concatenate([a.block_table[r, :nblk[r]].numpy() for r in range(3)])
    assert sorted(used.tolist()) == list(range(nblk.sum()))          # a permutation of all pages
    assert not np.array_equal(used, np.arange(nblk.sum()))           # and really shuffled
    pb = _problem(a)
    assert np.array_equal(a.page_fill.numpy(), pb.page_fill())
    other = generate_layer(cfg, seed=7)
    assert not torch.equal(other.q.view(torch.int16), a.q.view(torch.int16))


def test_planted_tokens_carry_the_mass_and_tail_is_poisoned_only_on_request():
    cfg = get_config(1).scaled(ctx=1000)                              # partial last page: 1000 = 62*16 + 8
    li = generate_layer(cfg, poison_tail=True)
    pb = _problem(li)
    last = li.block_table[0, 62].item()
    assert torch.isnan(li.k_pool[last, :, 8:]).all() and not torch.isnan(li.k_pool[last, :, :8]).any()
    assert li.page_fill[last].item() == 8
    s = ref.logits(pb, 0, 0)
    w = np.exp(s - s.max())
    w /= w.sum()
    # the first 16 and last 64 tokens are critical by construction: they hold most of the weight
    assert w[:16].sum() + w[-64:].sum() > 0.5
    clean = generate_layer(cfg)
    assert not torch.isnan(clean.k_pool).any()


def test_uniform_config_has_flat_attention():
    cfg = get_config(5).scaled(batch=1, ctx=2048)
    pb = _problem(generate_layer(cfg))
    s = ref.logits(pb, 0, 0)
    w = np.exp(s - s.max())
    w /= w.sum()
    assert w.max() < 10.0 / len(w)


def test_fraction_draws_follow_the_config():
    from workloads.generator import critical_fractions
    f2 = critical_fractions(get_config(2), 1, 0)
    assert f2.shape == (8, 8) and f2.min() >= 0.005 and f2.max() <= 0.10 and len(np.unique(f2)) > 32
    c3 = get_config(3)
    assert np.all(critical_fractions(c3, 1, 0) == 0.5) and np.all(critical_fractions(c3, 1, 1) == 0.5)
    f3 = [critical_fractions(c3, 1, l) for l in range(2, 32)]
    assert all(len(np.unique(f)) == 1 for f in f3) and len({float(f[0, 0]) for f in f3}) == 30
    assert min(f[0, 0] for f in f3) >= 0.002 and max(f[0, 0] for f in f3) <= 0.20
