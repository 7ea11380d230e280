"""psa_decode_attention_static -- the entry point whose workspace is a static device array inside the library --
against psa_decode_attention through the C ABI: same inputs, same tuning, bit for bit the same outputs; two calls
in a row, the second on a smaller input (the array keeps the first call's contents); the sticky error word; a
shape beyond the array is refused."""
import numpy as np
import pytest
import torch

import gpu_common as gc
from workloads import generate_layer, get_config

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psa():
    import paper_2503_00392_amd as psa
    psa.load_library()
    assert torch.cuda.is_available()
    return psa


def _outputs(cfg, MB, dev="cuda"):
    import paper_2503_00392_amd as psa
    B, Hq, H = cfg.batch, cfg.num_q_heads, cfg.num_kv_heads
    return psa.DecodeOutput(torch.full((B, Hq, 128), float("nan"), dtype=torch.float32, device=dev),
                            torch.full((B, Hq), -7, dtype=torch.int32, device=dev),
                            torch.full((B, Hq), float("nan"), dtype=torch.float32, device=dev),
                            torch.full((B, H), -7, dtype=torch.int32, device=dev),
                            torch.full((B, Hq), float("nan"), dtype=torch.float32, device=dev),
                            torch.full((B, H, MB), -7, dtype=torch.int32, device=dev), None, None)


def _both(psa, cfg, eps, m, layer=0):
    li = generate_layer(cfg, layer=layer, device="cuda", poison_tail=True)
    kv = gc.to_kv(li)
    meta = psa.build_block_metadata(kv, page_fill=li.page_fill)
    want = psa.decode_attention(kv, li.q, meta, eps, m, want_order=True)
    got = _outputs(cfg, li.block_table.shape[1])
    err = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    psa.decode_attention_static(kv, li.q, meta, eps, m, got, device_error=err)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert int(err) == 0
    for name in ("out", "n_selected", "mass_est", "blocks_read", "lse", "order"):
        a, b = getattr(want, name), getattr(got, name)
        assert torch.equal(a.view(torch.int32), b.view(torch.int32)), f"{name} differs from psa_decode_attention"
    # and, like every result of the path, against the oracle
    got.scores = psa.decode_attention(kv, li.q, meta, eps, m, want_scores=True).scores
    rep = gc.check_decode_against_oracle(gc.to_problem(li), got, eps, m)
    rep.assert_accounted()
    return li


def test_static_scratch_matches_the_workspace_entry_point_twice_in_a_row(psa):
    # first a batch of 8 requests x 20K tokens (about 27 MiB of the array), then -- over its leftovers -- one
    # short ragged batch, then the first again
    big = get_config(2).scaled(batch=8, ctx=20000)
    small = get_config(4).scaled(batch=3, ctx=3000, ctx_min=40)
    _both(psa, big, big.threshold, 1)
    _both(psa, small, small.threshold, 4)
    _both(psa, big, 1.0, 1)


def test_static_scratch_reports_device_side_errors(psa):
    cfg = get_config(1).scaled(ctx=1024)
    li = generate_layer(cfg, device="cuda")
    kv = gc.to_kv(li)
    meta = psa.build_block_metadata(kv, page_fill=li.page_fill)
    li.block_table[0, 3] = li.k_pool.shape[0] + 5          # outside the pool: clamped and reported
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    psa.decode_attention_static(kv, li.q, meta, 0.9, 1, _outputs(cfg, li.block_table.shape[1]), device_error=err)
    torch.cuda.synchronize()
    assert int(err) == 1


def test_a_shape_beyond_the_static_scratch_is_refused(psa):
    cfg = get_config(3).scaled(layers=1, batch=8)        # eight requests of 128K tokens: about 117 MiB of workspace
    B, MB = cfg.batch, cfg.ctx // 16
    # a descriptor only: nothing this large is allocated, the call must return before it looks at any buffer
    tiny = torch.zeros((1, cfg.num_kv_heads, 16, 128), dtype=torch.bfloat16, device="cuda")
    kv = psa.KvCache(tiny, tiny, torch.zeros((B, MB), dtype=torch.int32, device="cuda"),
                     torch.zeros(B, dtype=torch.int32, device="cuda"), cfg.num_q_heads)
    assert psa.decode_workspace_bytes(kv) > psa.binding.STATIC_SCRATCH_BYTES
    q = torch.zeros((B, cfg.num_q_heads, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(psa.PsaError) as e:
        psa.decode_attention_static(kv, q, tiny, 0.9, 1, _outputs(cfg, MB))
    assert "WORKSPACE_TOO_SMALL" in str(e.value)
