"""GPU parity: the HIP path through the C ABI against the fp64 oracle, element by element, on the
same seeded bytes.  Sizes here are ones the oracle finishes in seconds yet span several chunks,
several tiles of every kernel and ragged tails."""
import numpy as np
import pytest
import torch

import gpu_common as gc
from oracle import psa_oracle as po
from workloads import add_headroom, as_bits, generate_layer, get_config, step_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psa():
    import paper_2503_00392_amd as psa
    psa.load_library()
    assert torch.cuda.is_available()
    return psa


def _small(idx, **kw):
    return get_config(idx).scaled(**kw)


CASES = {
    "c1_full": (get_config(1), {}),
    "c2_small_kvhead_fracs": (_small(2, batch=2, ctx=4096), {}),
    "c3_small_bf16_random_table": (_small(3, batch=2, ctx=8192, layers=1), {"layer": 5}),
    "c3_dense_layer": (_small(3, batch=1, ctx=4096, layers=1), {"layer": 0}),
    # long enough (2500 blocks, 16 streams) for the ranking to be shared by several workgroups per stream
    "c2_ranking_in_parts": (_small(2, batch=2, ctx=40000), {}),
    "c4_ragged_g8": (_small(4, batch=6, ctx=6000, ctx_min=100), {}),
    # group of 8 with a KV-head count the page-by-page scoring does not take (3: scored on the matrix cores) and one
    # it does (2: eight blocks per step)
    "g8_three_kv_heads": (_small(4, batch=2, ctx=5000, ctx_min=900, num_q_heads=24, num_kv_heads=3), {}),
    "g8_two_kv_heads": (_small(4, batch=3, ctx=3000, ctx_min=50, num_q_heads=16, num_kv_heads=2, dtype="bf16"), {}),
    "c5_uniform": (_small(5, batch=2, ctx=4096), {}),
    "mha_g1": (_small(1, num_q_heads=8, num_kv_heads=8, ctx=2000), {}),
    "gqa_g2": (_small(1, num_q_heads=16, num_kv_heads=8, ctx=1500, dtype="bf16"), {}),
    # flat attention goes deep: more chunks than the stop rule folds at a time (64 with one head per KV head, 32
    # with two), so its state is carried from one group of chunks to the next
    "flat_g1_many_chunks": (_small(5, batch=1, ctx=40000, num_q_heads=4, num_kv_heads=4), {}),
    "flat_g2_many_chunks": (_small(5, batch=1, ctx=20000, num_q_heads=8, num_kv_heads=4), {}),
}


@pytest.fixture(scope="module", params=list(CASES))
def case(request):
    cfg, kw = CASES[request.param]
    li = generate_layer(cfg, device="cuda", poison_tail=True, **kw)
    return request.param, cfg, li, gc.to_problem(li)


def test_metadata_bit_exact(psa, case):
    name, cfg, li, pb = case
    kv = gc.to_kv(li)
    meta = psa.build_block_metadata(kv, page_fill=li.page_fill)
    torch.cuda.synchronize()
    got = meta.view(torch.int16).cpu().numpy().view(np.uint16)
    want = po.block_metadata(pb, li.page_fill.cpu().numpy())
    assert np.array_equal(got, want)


def test_dense_matches_oracle(psa, case):
    name, cfg, li, pb = case
    out, lse = psa.dense_attention(gc.to_kv(li), li.q)
    torch.cuda.synchronize()
    assert psa.read_device_error(out._workspace) == 0
    want, wlse = po.dense_attention(pb)
    err = gc.rel_l2(out.cpu().numpy().astype(np.float64), want)
    assert err.max() <= gc.OUT_RTOL, err.max()
    np.testing.assert_allclose(lse.cpu().numpy(), wlse, rtol=0, atol=2e-3)


@pytest.mark.parametrize("m", [1, 4])
def test_decode_matches_oracle(psa, case, m):
    name, cfg, li, pb = case
    for eps in (cfg.threshold,) + tuple(cfg.extra_thresholds):
        gpu = gc.run_gpu_decode(li, eps, m)
        rep = gc.check_decode_against_oracle(pb, gpu, eps, m)
        print(f"\n[{name} eps={eps} m={m}] {rep}")
        assert rep.empty == int((pb.num_blocks() == 0).sum()) * pb.q.shape[1]
        rep.assert_accounted()      # every head in one class; the near-boundary classes are bounded exceptions


def test_threshold_one_is_dense(psa, case):
    """Strict '>' never fires at eps = 1: every block is attended and the result is exact attention."""
    name, cfg, li, pb = case
    gpu = gc.run_gpu_decode(li, 1.0, 1)
    want, _ = po.dense_attention(pb)
    err = gc.rel_l2(gpu.out.cpu().numpy().astype(np.float64), want)
    assert err.max() <= gc.OUT_RTOL
    N = pb.num_blocks()
    G = cfg.group
    assert np.array_equal(gpu.n_selected.cpu().numpy(), np.repeat(N[:, None], cfg.num_q_heads, 1))
    assert np.array_equal(gpu.blocks_read.cpu().numpy(), np.repeat(N[:, None], cfg.num_kv_heads, 1))
    mass = gpu.mass_est.cpu().numpy()
    assert np.all(mass[N > 0] == 1.0)
    tr = gpu.traffic.cpu().numpy()
    assert np.array_equal(tr[..., 0], np.repeat(N[:, None], cfg.num_kv_heads, 1))   # K: everything, once
    assert np.array_equal(tr[..., 1], tr[..., 0])


def test_threshold_zero_takes_one_microbatch(psa, case):
    name, cfg, li, pb = case
    N = pb.num_blocks()
    for m in (1, 5, 40):
        gpu = gc.run_gpu_decode(li, 0.0, m)
        want = np.repeat(np.minimum(m, N)[:, None], cfg.num_q_heads, 1)
        assert np.array_equal(gpu.n_selected.cpu().numpy(), want)
        own = po.attend_prefix(pb, gpu.order.cpu().numpy(), gpu.n_selected.cpu().numpy())
        assert gc.rel_l2(gpu.out.cpu().numpy().astype(np.float64), own).max() <= gc.OUT_RTOL


@pytest.mark.parametrize("chunk,window,spin", [(8, 1, 0), (16, 3, 0), (64, 2, 0), (32, 64, 0), (12, 1, 1)])
def test_result_does_not_depend_on_tuning(psa, case, chunk, window, spin):
    """Chunk size, read-ahead window and the patience of waiting workgroups change traffic and scheduling, not the selection:
    the selected sets are identical and outputs agree to rounding."""
    name, cfg, li, pb = case
    eps = cfg.threshold
    base = gc.run_gpu_decode(li, eps, 1)
    alt = gc.run_gpu_decode(li, eps, 1, tuning=psa.Tuning(chunk_blocks=chunk, window_chunks=window, spin_limit=spin))
    assert torch.equal(base.order, alt.order)
    rep = gc.check_decode_against_oracle(pb, alt, eps, 1)
    rep.assert_accounted()
    same = (base.n_selected == alt.n_selected)
    # a different chunking folds the prefix in a different order: only boundary flips may differ
    assert (~same).sum().item() <= rep.stop_flips + 1
    err = gc.rel_l2(alt.out[same].cpu().numpy().astype(np.float64),
                    base.out[same].cpu().numpy().astype(np.float64))
    assert err.max() <= 1e-4


def test_repeated_calls_are_bitwise_identical(psa, case):
    """Scheduling is dynamic (which chunks are published when the stop rule looks) but every reduction has a fixed order."""
    name, cfg, li, pb = case
    a = gc.run_gpu_decode(li, cfg.threshold, 1)
    b = gc.run_gpu_decode(li, cfg.threshold, 1)
    assert torch.equal(a.out, b.out) and torch.equal(a.n_selected, b.n_selected)
    assert torch.equal(a.mass_est, b.mass_est) and torch.equal(a.order, b.order)


def test_bucket_ranking_equals_bitonic_ranking(psa, case):
    """The two ranking paths of the order kernel implement the same total order."""
    name, cfg, li, pb = case
    a = gc.run_gpu_decode(li, cfg.threshold, 1)
    b = gc.run_gpu_decode(li, cfg.threshold, 1, tuning=psa.Tuning(force_bitonic=1))
    assert torch.equal(a.order, b.order) and torch.equal(a.n_selected, b.n_selected)
    assert torch.equal(a.out, b.out)


def test_degenerate_scores_rank_by_block_index(psa):
    """All keys equal: every score ties, the ranking must be the identity (ties go to the smaller
    logical block) -- this drives the order kernel through its large-bucket fallback -- and the
    result is plain attention over a prefix."""
    cfg = get_config(3).scaled(batch=2, ctx=40000, layers=1)
    li = generate_layer(cfg, device="cuda")
    li.k_pool[...] = li.k_pool[0, 0, 0].clone()
    pb = gc.to_problem(li)
    gpu = gc.run_gpu_decode(li, 0.5, 1)
    N = pb.num_blocks()
    order = gpu.order.cpu().numpy()
    for r in range(2):
        assert np.array_equal(order[r, :, :N[r]], np.tile(np.arange(N[r]), (cfg.num_kv_heads, 1)))
    rep = gc.check_decode_against_oracle(pb, gpu, 0.5, 1)
    # every block weighs the same, so P_acc(n) = n/N lands exactly on the threshold: stop flips are the rule here
    rep.assert_accounted(max_rank_swaps=0, max_stop_flips=rep.heads)
    assert rep.set_tolerated == 0


@pytest.mark.parametrize("k", [1, 7, 32, 100, 10000])
def test_topk_matches_oracle(psa, case, k):
    """Fixed-budget control: same ranking, every head takes min(k, N) blocks, keys are read no
    further than the budget (rounded up to whole chunks)."""
    name, cfg, li, pb = case
    kv = gc.to_kv(li)
    meta = psa.build_block_metadata(kv, page_fill=li.page_fill)
    gpu = psa.topk_attention(kv, li.q, meta, k, want_order=True, want_scores=True, want_traffic=True)
    torch.cuda.synchronize()
    assert psa.read_device_error(gpu._workspace) == 0
    ora = po.topk_attention(pb, k)
    N = pb.num_blocks()
    want_n = np.repeat(np.minimum(k, N)[:, None], cfg.num_q_heads, 1)
    g_n = gpu.n_selected.cpu().numpy()
    assert np.array_equal(g_n, want_n) and np.array_equal(ora.n_selected, want_n)
    assert np.array_equal(gpu.blocks_read.cpu().numpy(), np.repeat(np.minimum(k, N)[:, None], cfg.num_kv_heads, 1))
    g_order = gpu.order.cpu().numpy()
    g_out = gpu.out.cpu().numpy().astype(np.float64)
    own, own_lse = po.attend_prefix(pb, g_order, g_n, want_lse=True)
    assert gc.rel_l2(g_out, own).max() <= gc.OUT_RTOL
    fin = np.isfinite(own_lse)
    assert np.abs(gpu.lse.cpu().numpy()[fin] - own_lse[fin]).max(initial=0.0) <= gc.LSE_ATOL
    G = cfg.group
    for r in range(cfg.batch):
        n = int(want_n[r, 0])
        for h in range(cfg.num_kv_heads):
            sg, so = set(g_order[r, h, :n].tolist()), set(ora.order[r, h, :n].tolist())
            if sg == so:
                sl = slice(h * G, (h + 1) * G)
                assert gc.rel_l2(g_out[r, sl], ora.out[r, sl]).max() <= gc.OUT_RTOL
                np.testing.assert_allclose(gpu.mass_est[r, sl].cpu().numpy(), ora.mass_est[r, sl], atol=1e-4, rtol=0)
            else:
                edge = ora.cs[r, h, ora.order[r, h, n - 1]]
                assert all(abs(ora.cs[r, h, b] - edge) <= gc.SCORE_ATOL for b in sg ^ so)
    chunk = 32
    tr = gpu.traffic.cpu().numpy()
    lim = np.minimum(N, -(-np.minimum(k, N) // chunk) * chunk)
    assert np.array_equal(tr[..., 0], np.repeat(lim[:, None], cfg.num_kv_heads, 1))       # keys: budget, whole chunks
    assert np.array_equal(tr[..., 1], np.repeat(np.minimum(k, N)[:, None], cfg.num_kv_heads, 1))


def test_cuboid_center_scorer_matches_oracle(psa, case):
    """The second scorer: same metadata, the centre of the bounding cuboid instead of its best corner."""
    name, cfg, li, pb = case
    for m in (1, 4):
        gpu = gc.run_gpu_decode(li, cfg.threshold, m, scorer=psa.SCORE_CUBOID_CENTER)
        rep = gc.check_decode_against_oracle(pb, gpu, cfg.threshold, m, scorer=po.CUBOID_CENTER)
        print(f"\n[{name} centre scorer m={m}] {rep}")
        assert rep.empty == int((pb.num_blocks() == 0).sum()) * pb.q.shape[1]
        rep.assert_accounted()
    k = 9
    kv = gc.to_kv(li)
    meta = psa.build_block_metadata(kv, page_fill=li.page_fill)
    top = psa.topk_attention(kv, li.q, meta, k, want_order=True, scorer=psa.SCORE_CUBOID_CENTER)
    torch.cuda.synchronize()
    assert torch.equal(top.order, gpu.order)
    own = po.attend_prefix(pb, top.order.cpu().numpy(), top.n_selected.cpu().numpy())
    assert gc.rel_l2(top.out.cpu().numpy().astype(np.float64), own).max() <= gc.OUT_RTOL


def test_mean_key_metadata_and_scorer_match_oracle(psa, case):
    """The third scorer: one mean vector per block (bit for bit the oracle's exactly rounded means, partly filled
    pages included), scored by the mean key's logit; everything after the score is the same path."""
    name, cfg, li, pb = case
    kv = gc.to_kv(li)
    means = psa.build_block_means(kv, page_fill=li.page_fill)
    torch.cuda.synchronize()
    want = po.block_means(pb, li.page_fill.cpu().numpy())
    assert np.array_equal(means.view(torch.int16).cpu().numpy().view(np.uint16), want)
    # a listed rebuild writes the listed pages only, and the same bits
    listed = torch.arange(0, li.k_pool.shape[0], 3, dtype=torch.int32, device="cuda")
    again = torch.zeros_like(means)
    psa.build_block_means(kv, means=again, page_fill=li.page_fill, page_list=listed)
    torch.cuda.synchronize()
    got = again.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got[::3], want[::3]) and not got[1::3].any()
    for m in (1, 4):
        gpu = gc.run_gpu_decode(li, cfg.threshold, m, meta=means, scorer=psa.SCORE_MEAN_KEY)
        rep = gc.check_decode_against_oracle(pb, gpu, cfg.threshold, m, scorer=po.MEAN_KEY)
        print(f"\n[{name} mean-key scorer m={m}] {rep}")
        assert rep.empty == int((pb.num_blocks() == 0).sum()) * pb.q.shape[1]
        rep.assert_accounted()


@pytest.mark.parametrize("which", ["c1_ragged", "c3_small_bf16"])
def test_incremental_decode_loop(psa, which):
    """Several decode steps in a row: append the step's token (K, V, metadata, length -- all on the GPU),
    then PSA with the step's query.  After every step the cache and the metadata equal, bit for bit,
    what the oracle gets by appending to its own copy and rebuilding the metadata from scratch, and the
    decode result matches the oracle's on that cache.  Lengths are chosen so that pages fill, new
    pages start and a request starts from nothing."""
    if which == "c1_ragged":
        cfg = _small(1, batch=4, ctx=700)             # every request generated at 700 tokens, then cut back
        start = [16 * 9 - 2, 16 * 20, 333, 0]
    else:
        cfg = _small(3, batch=2, ctx=4096, layers=1)
        start = [4096 - 3, 2000]
    steps = 6
    li = add_headroom(generate_layer(cfg, device="cuda", poison_tail=True), steps)
    li.ctx_lens.copy_(torch.tensor(start, dtype=torch.int32))
    kv = gc.to_kv(li)
    fill0 = torch.from_numpy(gc.to_problem(li).page_fill()).cuda()
    meta = psa.build_block_metadata(kv, page_fill=fill0)
    means = psa.build_block_means(kv, page_fill=fill0)      # mean-key metadata: rebuilt for the touched pages each step
    pb = gc.to_problem(li)
    status = torch.full((cfg.batch,), -1, dtype=torch.int32, device="cuda")
    for t in range(1, steps + 1):
        q, k_new, v_new = step_inputs(li, t)
        psa.append_kv(kv, k_new, v_new, meta, status)
        torch.cuda.synchronize()
        pb, want_status = po.append_kv(po.Problem(as_bits(q), pb.k_pool, pb.v_pool, pb.block_table, pb.ctx_lens, pb.dtype),
                                       as_bits(k_new), as_bits(v_new))
        assert np.array_equal(status.cpu().numpy(), want_status) and not want_status.any()
        assert np.array_equal(li.ctx_lens.cpu().numpy(), pb.ctx_lens)
        fill = pb.page_fill()
        want_meta = po.block_metadata(pb, fill)
        got_meta = as_bits(meta)
        used = fill > 0
        assert np.array_equal(got_meta[used], want_meta[used]), f"metadata differs after step {t}"
        # valid tokens of the pools are identical (rows beyond a page's fill may hold the poison)
        gk, gv = as_bits(li.k_pool), as_bits(li.v_pool)
        for page in np.nonzero(used)[0]:
            assert np.array_equal(gk[page, :, :fill[page]], pb.k_pool[page, :, :fill[page]])
            assert np.array_equal(gv[page, :, :fill[page]], pb.v_pool[page, :, :fill[page]])
        out = psa.decode_attention(kv, q, meta, cfg.threshold, 1, want_order=True, want_scores=True, want_traffic=True)
        torch.cuda.synchronize()
        assert psa.read_device_error(out._workspace) == 0
        rep = gc.check_decode_against_oracle(pb, out, cfg.threshold, 1)
        rep.assert_accounted()
        # mean-key metadata is not maintained by the append: the pages that received a token are rebuilt from a list
        touched = torch.tensor([int(pb.block_table[r, (int(pb.ctx_lens[r]) - 1) // 16]) for r in range(cfg.batch)],
                               dtype=torch.int32, device="cuda")
        fill_dev = torch.from_numpy(fill.astype(np.int32)).cuda()
        psa.build_block_means(kv, means=means, page_fill=fill_dev, page_list=touched)
        torch.cuda.synchronize()
        want_means = po.block_means(pb, fill)
        assert np.array_equal(as_bits(means)[used], want_means[used]), f"mean-key metadata differs after step {t}"
    assert np.array_equal(pb.ctx_lens, np.array(start) + steps)


def test_append_reports_a_full_table_row_and_leaves_the_request_alone(psa):
    cfg = _small(1, batch=2, ctx=64)
    li = generate_layer(cfg, device="cuda")          # rows of exactly 4 blocks, both requests full
    li.ctx_lens.copy_(torch.tensor([64, 63], dtype=torch.int32))
    kv = gc.to_kv(li)
    meta = psa.build_block_metadata(kv, page_fill=li.page_fill)
    before_k, before_meta = li.k_pool.clone(), meta.clone()
    q, k_new, v_new = step_inputs(li, 1)
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    psa.append_kv(kv, k_new, v_new, meta, status)
    torch.cuda.synchronize()
    assert status.tolist() == [2, 0] and li.ctx_lens.tolist() == [64, 64]
    page0 = li.block_table[0].long()
    assert torch.equal(li.k_pool[page0], before_k[page0]) and torch.equal(meta[page0].view(torch.int16), before_meta[page0].view(torch.int16))
    last = int(li.block_table[1, 3])
    assert torch.equal(li.k_pool[last, :, 15].view(torch.int16), k_new[1].view(torch.int16))


@pytest.mark.parametrize("kind", ["exact", "zero", "huge", "random"])
def test_depth_hint_changes_traffic_not_results(psa, case, kind):
    """A hint of how deep each stream will go only moves the read-ahead: any hint, right or wrong, gives
    the same selection and the same bits."""
    name, cfg, li, pb = case
    base = gc.run_gpu_decode(li, cfg.threshold, 1)
    B, H = cfg.batch, cfg.num_kv_heads
    if kind == "exact":
        hint = base.blocks_read.clone()
    elif kind == "zero":
        hint = torch.zeros((B, H), dtype=torch.int32, device="cuda")
    elif kind == "huge":
        hint = torch.full((B, H), 1 << 30, dtype=torch.int32, device="cuda")
    else:
        hint = torch.randint(-5, 3000, (B, H), dtype=torch.int32, device="cuda", generator=torch.Generator("cuda").manual_seed(7))
    alt = gc.run_gpu_decode(li, cfg.threshold, 1, tuning=psa.Tuning(depth_hint=hint))
    assert torch.equal(base.out, alt.out) and torch.equal(base.n_selected, alt.n_selected)
    assert torch.equal(base.mass_est, alt.mass_est) and torch.equal(base.order, alt.order)
    if kind == "exact":          # keys are then read no further than whole chunks of what is needed, plus the window
        assert (alt.traffic[..., 0] >= base.blocks_read).all()
