"""Two-tier block store on the GPU (Sec. 3.1, 3.4) through the C ABI.

The pools of a tiered cache are pinned host tensors; a pool of slots on the GPU, shared by the layers,
caches (page, KV head) slices.  Checked here:
  * attention over a tiered cache gives bit for bit what the same kernels give over the same bytes in
    device memory, whatever part of the slices is cached (none, some, all) -- and that one is compared
    with the oracle elsewhere; one case here is compared with the oracle directly;
  * after every update the library's tables (slice -> slot, slot -> slice, stamps, clock) and the update's
    counts equal, entry by entry, what the model in oracle/tier_oracle.py gives for the same sequence of
    used slices, evictions and the busy range included;
  * a cached slice holds the bytes of its host copy, also after tokens were appended;
  * with a staging buffer the same holds, and the slices the attention read from host memory reach their slots
    from the staging buffer (counted), as far as the buffer has room.
"""
import numpy as np
import pytest
import torch

import gpu_common as gc
from oracle import psa_oracle as po
from oracle.tier_oracle import TierModel, used_slices
from workloads import add_headroom, generate_layer, get_config, step_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psa():
    import paper_2503_00392_amd as psa
    psa.load_library()
    assert torch.cuda.is_available()
    return psa


class Layer:
    """One layer twice: `dev` in device memory (the reference), `host` tiered, same bytes."""

    def __init__(self, psa, li, tier, slice_base):
        self.li = li
        self.dev = gc.to_kv(li)
        self.k_host = li.k_pool.cpu().pin_memory()
        self.v_host = li.v_pool.cpu().pin_memory()
        self.ctx_host_side = li.ctx_lens.clone()
        self.host = psa.KvCache(self.k_host, self.v_host, li.block_table, self.ctx_host_side, li.cfg.num_q_heads,
                                tier=tier, slice_base=slice_base)
        fill = torch.from_numpy(gc.to_problem(li).page_fill()).cuda()
        self.meta_dev = psa.build_block_metadata(self.dev, page_fill=fill)
        self.meta_host = self.meta_dev.clone()
        self.slice_base = slice_base
        self.n_slices = li.k_pool.shape[0] * li.k_pool.shape[1]


def _same(a, b):
    for name in ("out", "n_selected", "mass_est", "blocks_read", "lse", "order"):
        x, y = getattr(a, name), getattr(b, name)
        assert torch.equal(x, y), f"{name} differs between the tiered and the single-tier call"


def _check_tables(tier, model, layers):
    slot_of, owner, stamp, clock = tier.tables()
    assert clock == model.clock
    assert np.array_equal(slot_of, model.slot_of)
    assert np.array_equal(owner, model.owner)
    assert np.array_equal(stamp, model.stamp)
    # a cached slice holds the bytes of its host copy
    pool = tier.slot_pool.cpu().numpy().view(np.uint16)                    # [slots][2][16][128]
    for L in layers:
        k = L.k_host.view(torch.int16).numpy().view(np.uint16).reshape(-1, 16, 128)       # [pages * H][16][128]
        v = L.v_host.view(torch.int16).numpy().view(np.uint16).reshape(-1, 16, 128)
        ids = np.nonzero(slot_of[L.slice_base:L.slice_base + L.n_slices] >= 0)[0]
        slots = slot_of[L.slice_base + ids]
        assert np.array_equal(pool[slots, 0], k[ids]) and np.array_equal(pool[slots, 1], v[ids])


def _update(psa, L, out, tier, model, busy=(0, 0)):
    stats = psa.tier_update(L.host, out.order, out.blocks_read, busy[0], busy[1])
    torch.cuda.synchronize()
    H = L.li.k_pool.shape[1]
    ids = used_slices(L.li.block_table.cpu().numpy(), out.order.cpu().numpy(), out.blocks_read.cpu().numpy(), H,
                      L.slice_base)
    want = model.update(ids, busy[0], busy[1])
    assert stats.tolist()[:4] == [want.hits, want.misses, want.promoted, want.evicted]
    want.from_staging = int(stats[4])
    return want


@pytest.mark.parametrize("staging_slices", [0, 1 << 14, 37])
@pytest.mark.parametrize("slots_share", [1.0, 0.3, 0.02])
def test_cold_then_warm_single_layer(psa, slots_share, staging_slices):
    cfg = get_config(3).scaled(batch=2, ctx=4096, layers=1)
    li = generate_layer(cfg, layer=5, device="cuda")
    n_slices = li.k_pool.shape[0] * li.k_pool.shape[1]
    num_slots = max(int(n_slices * slots_share), 1)
    tier = psa.Tier(n_slices, num_slots)
    model = TierModel(n_slices, num_slots)
    L = Layer(psa, li, tier, 0)
    if staging_slices:
        L.host.staging = psa.Tier.staging_buffer(staging_slices)
    ref = psa.decode_attention(L.dev, li.q, L.meta_dev, cfg.threshold, 1, want_order=True)
    for step in range(3):
        got = psa.decode_attention(L.host, li.q, L.meta_host, cfg.threshold, 1, want_order=True)
        torch.cuda.synchronize()
        assert psa.read_device_error(got._workspace) == 0
        _same(got, ref)
        st = _update(psa, L, got, tier, model)
        _check_tables(tier, model, [L])
        if step == 0:
            assert st.hits == 0 and st.misses == int(ref.blocks_read.sum())
        elif slots_share >= 1.0:
            assert st.misses == 0 and st.hits == int(ref.blocks_read.sum())
        # every slice placed was read from host memory by the attention kernels first: it comes from the staging
        # buffer as far as that had room (entries also go to keys read ahead of the stop, which no update places)
        if staging_slices >= (1 << 14):
            assert st.from_staging == st.promoted
        elif staging_slices:
            assert st.from_staging <= min(st.promoted, staging_slices)
        else:
            assert st.from_staging == 0
    assert model.clock == 3
    if slots_share < 0.05:      # fewer slots than the call uses: the pool is full and stays as it is
        assert (model.owner >= 0).all()
    # and against the oracle itself, with part of the slices cached
    got = psa.decode_attention(L.host, li.q, L.meta_host, cfg.threshold, 1, want_order=True, want_scores=True,
                               want_traffic=True)
    torch.cuda.synchronize()
    rep = gc.check_decode_against_oracle(gc.to_problem(li), got, cfg.threshold, 1)
    rep.assert_accounted()


def test_two_layers_share_a_small_pool_over_a_decode_loop(psa):
    """Two layers, one pool too small for both: drifting queries, a token appended per step, the other
    layer named busy in every update.  Outputs equal the single-tier run's; tables equal the model's."""
    steps = 5
    cfgs = [get_config(3).scaled(batch=2, ctx=3000, layers=2), get_config(3).scaled(batch=2, ctx=3000, layers=2)]
    lis = [add_headroom(generate_layer(cfgs[i], layer=3 + i, device="cuda"), steps) for i in range(2)]
    sizes = [li.k_pool.shape[0] * li.k_pool.shape[1] for li in lis]
    bases = [0, sizes[0]]
    total = sum(sizes)
    num_slots = total // 16
    tier = psa.Tier(total, num_slots)
    model = TierModel(total, num_slots)
    layers = [Layer(psa, lis[i], tier, bases[i]) for i in range(2)]
    for i, L in enumerate(layers):
        L.host.staging = psa.Tier.staging_buffer(4096)
    evicted = staged = 0
    for t in range(1, steps + 1):
        for i, L in enumerate(layers):
            q, k_new, v_new = step_inputs(L.li, t)
            psa.append_kv(L.dev, k_new, v_new, L.meta_dev)
            psa.append_kv(L.host, k_new, v_new, L.meta_host)
            ref = psa.decode_attention(L.dev, q, L.meta_dev, 0.9, 1, want_order=True)
            got = psa.decode_attention(L.host, q, L.meta_host, 0.9, 1, want_order=True)
            torch.cuda.synchronize()
            assert torch.equal(L.meta_dev.view(torch.int16), L.meta_host.view(torch.int16))
            assert torch.equal(L.li.ctx_lens, L.ctx_host_side)
            _same(got, ref)
            other = layers[1 - i]
            st = _update(psa, L, got, tier, model, busy=(other.slice_base, other.n_slices))
            evicted += st.evicted
            staged += st.from_staging
            assert st.from_staging == st.promoted
            _check_tables(tier, model, layers)
    assert evicted > 0, "the pool was meant to be too small"
    assert staged > 0
    # the appended tokens reached host memory as well
    for L in layers:
        assert torch.equal(L.k_host.view(torch.int16), L.li.k_pool.cpu().view(torch.int16))
        assert torch.equal(L.v_host.view(torch.int16), L.li.v_pool.cpu().view(torch.int16))


def test_fixed_budget_and_ragged_batch_with_a_tier(psa):
    cfg = get_config(4).scaled(batch=5, ctx=3000, ctx_min=40)
    li = generate_layer(cfg, device="cuda", poison_tail=True)
    n_slices = li.k_pool.shape[0] * li.k_pool.shape[1]
    tier = psa.Tier(n_slices + 100, n_slices // 3)
    model = TierModel(n_slices + 100, n_slices // 3)
    L = Layer(psa, li, tier, 100)
    for k in (7, 40):
        ref = psa.topk_attention(L.dev, li.q, L.meta_dev, k, want_order=True)
        got = psa.topk_attention(L.host, li.q, L.meta_host, k, want_order=True)
        torch.cuda.synchronize()
        _same(got, ref)
        _update(psa, L, got, tier, model)
        _check_tables(tier, model, [L])
    ref = psa.decode_attention(L.dev, li.q, L.meta_dev, cfg.threshold, 2, want_order=True)
    got = psa.decode_attention(L.host, li.q, L.meta_host, cfg.threshold, 2, want_order=True)
    torch.cuda.synchronize()
    _same(got, ref)


def test_metadata_builds_read_a_tiered_cache_in_place(psa):
    """Both metadata builds over pools in pinned host memory give the bits they give over the same pools in device
    memory."""
    cfg = get_config(3).scaled(batch=2, ctx=3000, layers=1)
    li = generate_layer(cfg, layer=4, device="cuda", poison_tail=True)
    n_slices = li.k_pool.shape[0] * li.k_pool.shape[1]
    tier = psa.Tier(n_slices, 64)
    L = Layer(psa, li, tier, 0)
    fill = torch.from_numpy(gc.to_problem(li).page_fill()).cuda()
    for build in (psa.build_block_metadata, psa.build_block_means):
        a = build(L.dev, page_fill=fill)
        b = build(L.host, page_fill=fill)
        torch.cuda.synchronize()
        assert b.is_cuda and torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_tier_arguments_are_checked_on_the_host(psa):
    cfg = get_config(1).scaled(ctx=256)
    li = generate_layer(cfg, device="cuda")
    n_slices = li.k_pool.shape[0] * li.k_pool.shape[1]
    tier = psa.Tier(n_slices, 16)
    L = Layer(psa, li, tier, 0)
    out = psa.decode_attention(L.host, li.q, L.meta_host, 0.9, 1, want_order=True)
    torch.cuda.synchronize()
    # an id range that does not fit the tier
    bad = psa.KvCache(L.k_host, L.v_host, li.block_table, li.ctx_lens, cfg.num_q_heads, tier=tier, slice_base=1)
    with pytest.raises(psa.PsaError):
        psa.decode_attention(bad, li.q, L.meta_host, 0.9, 1)
    with pytest.raises(psa.PsaError):
        psa.tier_update(bad, out.order, out.blocks_read)
    # an update of a cache without a tier
    assert psa.tier_update_workspace_bytes(L.dev) == 0
    with pytest.raises(psa.PsaError):
        psa.tier_update(L.dev, out.order, out.blocks_read, workspace=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    # a workspace that is too small
    with pytest.raises(psa.PsaError):
        psa.tier_update(L.host, out.order, out.blocks_read, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert psa.tier_state_bytes(0, 4) == 0 and psa.tier_state_bytes(4, 0) == 0 and psa.tier_state_bytes(1 << 31, 4) == 0


def test_updates_on_a_second_stream_beside_the_next_layer(psa):
    """The overlap protocol of Sec. 3.3 as the benchmark runs it: layer j's update goes to a second stream
    with layer j+1 named busy and runs beside layer j+1's attention; layer j+2 waits for it.  Outputs equal
    the single-tier run's and the tables end up exactly as the model's, which applies the same updates one
    after the other."""
    steps, nl = 4, 3
    cfg = get_config(3).scaled(batch=2, ctx=4096, layers=nl)
    lis = [generate_layer(cfg, layer=2 + i, device="cuda") for i in range(nl)]
    sizes = [li.k_pool.shape[0] * li.k_pool.shape[1] for li in lis]
    bases = [int(sum(sizes[:i])) for i in range(nl)]
    total = int(sum(sizes))
    num_slots = total // 12
    tier = psa.Tier(total, num_slots)
    model = TierModel(total, num_slots)
    layers = [Layer(psa, lis[i], tier, bases[i]) for i in range(nl)]
    main_s, side_s = torch.cuda.current_stream(), torch.cuda.Stream()
    uws = torch.empty(max(psa.tier_update_workspace_bytes(L.host) for L in layers), dtype=torch.uint8, device="cuda")
    stats = torch.zeros((steps, nl, 5), dtype=torch.int32, device="cuda")
    staging = [psa.Tier.staging_buffer(8192) for _ in range(2)]      # consecutive calls alternate between the two
    calls = 0
    done = [None] * nl
    log = []                                  # what each update saw, for the model: (layer, order, blocks_read)
    for t in range(1, steps + 1):
        outs = []
        for j, L in enumerate(layers):
            q = step_inputs(L.li, t)[0]
            if done[(j - 2) % nl] is not None:
                main_s.wait_event(done[(j - 2) % nl])     # (the update two calls back: it used this staging buffer)
            L.host.staging = staging[calls % 2]
            calls += 1
            got = psa.decode_attention(L.host, q, L.meta_host, 0.9, 1, want_order=True)
            ref = psa.decode_attention(L.dev, q, L.meta_dev, 0.9, 1, want_order=True)
            outs.append((got, ref))
            decoded = torch.cuda.Event()
            decoded.record(main_s)
            side_s.wait_event(decoded)
            nxt = (j + 1) % nl
            psa.tier_update(L.host, got.order, got.blocks_read, bases[nxt], sizes[nxt], stats=stats[t - 1, j],
                            workspace=uws, stream=side_s)
            done[j] = torch.cuda.Event()
            done[j].record(side_s)
            log.append((j, got.order, got.blocks_read, nxt))
        main_s.wait_event(done[nl - 1])
        torch.cuda.synchronize()
        for got, ref in outs:
            _same(got, ref)
    got_stats = stats.cpu().numpy().reshape(-1, 5)
    for k, (j, order, read, nxt) in enumerate(log):
        L = layers[j]
        ids = used_slices(L.li.block_table.cpu().numpy(), order.cpu().numpy(), read.cpu().numpy(), L.li.k_pool.shape[1],
                          L.slice_base)
        want = model.update(ids, bases[nxt], sizes[nxt])
        assert got_stats[k].tolist()[:4] == [want.hits, want.misses, want.promoted, want.evicted], f"update {k}"
        assert got_stats[k][4] == want.promoted, f"update {k}: every slice placed comes from the staging buffer"
    _check_tables(tier, model, layers)
    assert got_stats[:, 3].sum() > 0, "the pool was meant to be too small"
