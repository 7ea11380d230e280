"""GPU edge cases through the C ABI: empty and one-token requests inside a batch, lengths around a
page boundary, and inputs only the device can see are wrong (a table entry outside the pool, a length
beyond the table row, a negative length) -- the kernels clamp, say so in the sticky error word, and
leave the other requests' results untouched."""
import numpy as np
import pytest
import torch

import gpu_common as gc
from oracle import psa_oracle as po
from workloads import generate_layer, get_config

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def psa():
    import paper_2503_00392_amd as psa
    psa.load_library()
    assert torch.cuda.is_available()
    return psa


def _layer(batch, ctx):
    return generate_layer(get_config(1).scaled(batch=batch, ctx=ctx), device="cuda", poison_tail=True)


LENGTHS = [0, 1, 15, 16, 17, 0, 300, 33]


def _cut(li, lengths):
    li.ctx_lens.copy_(torch.tensor(lengths, dtype=torch.int32))
    pb = gc.to_problem(li)
    return pb, torch.from_numpy(pb.page_fill()).cuda()


@pytest.mark.parametrize("eps,m", [(0.9, 1), (0.5, 3), (1.0, 1), (0.0, 2)])
def test_empty_tiny_and_page_boundary_requests(psa, eps, m):
    li = _layer(len(LENGTHS), 320)
    pb, fill = _cut(li, LENGTHS)
    kv = gc.to_kv(li)
    meta = psa.build_block_metadata(kv, page_fill=fill)
    gpu = psa.decode_attention(kv, li.q, meta, eps, m, want_order=True, want_scores=True, want_traffic=True)
    torch.cuda.synchronize()
    assert psa.read_device_error(gpu._workspace) == 0
    rep = gc.check_decode_against_oracle(pb, gpu, eps, m)
    empty = [i for i, n in enumerate(LENGTHS) if n == 0]
    assert rep.empty == len(empty) * pb.q.shape[1]
    rep.assert_accounted()
    for r in empty:
        assert not gpu.out[r].any() and not gpu.n_selected[r].any() and not gpu.mass_est[r].any()
        assert torch.isneginf(gpu.lse[r]).all() and not gpu.blocks_read[r].any()
        assert (gpu.order[r] == -1).all()
    one = LENGTHS.index(1)                       # a single token: attention returns its value, estimate 1
    assert (gpu.n_selected[one] == 1).all() and (gpu.mass_est[one] == 1.0).all()
    page = int(li.block_table[one, 0])
    G = li.cfg.group
    for hq in range(li.cfg.num_q_heads):
        assert torch.equal(gpu.out[one, hq], li.v_pool[page, hq // G, 0].float())


def test_dense_and_topk_on_the_same_batch(psa):
    li = _layer(len(LENGTHS), 320)
    pb, fill = _cut(li, LENGTHS)
    kv = gc.to_kv(li)
    out, lse = psa.dense_attention(kv, li.q)
    torch.cuda.synchronize()
    want, wlse = po.dense_attention(pb)
    live = np.array(LENGTHS) > 0
    assert gc.rel_l2(out.cpu().numpy().astype(np.float64), want).max() <= gc.OUT_RTOL
    np.testing.assert_allclose(lse.cpu().numpy()[live], wlse[live], rtol=0, atol=2e-3)
    assert torch.isneginf(lse[~torch.from_numpy(live).cuda()]).all() and not out[~torch.from_numpy(live).cuda()].any()
    meta = psa.build_block_metadata(kv, page_fill=fill)
    top = psa.topk_attention(kv, li.q, meta, 2, want_order=True)
    torch.cuda.synchronize()
    nb = pb.num_blocks()
    assert np.array_equal(top.n_selected.cpu().numpy(), np.repeat(np.minimum(2, nb)[:, None], li.cfg.num_q_heads, 1))
    own = po.attend_prefix(pb, top.order.cpu().numpy(), top.n_selected.cpu().numpy())
    assert gc.rel_l2(top.out.cpu().numpy().astype(np.float64), own).max() <= gc.OUT_RTOL


def test_inputs_only_the_device_can_see_are_wrong(psa):
    """Request 1 gets a table entry outside the pool, request 2 a length beyond its table row, request
    3 a negative length.  Nothing faults; the error word names both kinds; requests 0 and 4 come out
    exactly as in the clean run."""
    li = _layer(5, 640)
    kv = gc.to_kv(li)
    meta = psa.build_block_metadata(kv, page_fill=li.page_fill)
    clean = psa.decode_attention(kv, li.q, meta, 0.9, 1, want_order=True)
    dclean, _ = psa.dense_attention(kv, li.q)
    torch.cuda.synchronize()
    assert psa.read_device_error(clean._workspace) == 0
    li.block_table[1, 7] = li.k_pool.shape[0] + 12345
    li.ctx_lens[2] = li.block_table.shape[1] * 16 + 999
    li.ctx_lens[3] = -5
    bad = psa.decode_attention(kv, li.q, meta, 0.9, 1, want_order=True)
    torch.cuda.synchronize()
    flags = psa.read_device_error(bad._workspace)
    assert flags == 3, flags
    assert torch.isfinite(bad.out).all()
    for r in (0, 4):
        assert torch.equal(bad.out[r], clean.out[r]) and torch.equal(bad.n_selected[r], clean.n_selected[r])
        assert torch.equal(bad.order[r], clean.order[r])
    assert not bad.out[3].any() and not bad.n_selected[3].any()          # negative length reads as empty
    assert (bad.n_selected[2] <= li.block_table.shape[1]).all()          # clamped to the row
    dbad, _ = psa.dense_attention(kv, li.q)
    torch.cuda.synchronize()
    dflags = psa.read_device_error(dbad._workspace)
    assert dflags & 1 and dflags & 2
    for r in (0, 4):
        assert torch.equal(dbad[r], dclean[r])
    # the next clean call starts from a clean error word
    li.block_table[1, 7] = 0
    li.ctx_lens[2] = 640
    li.ctx_lens[3] = 640
    again = psa.decode_attention(kv, li.q, meta, 0.9, 1, workspace=bad._workspace)
    torch.cuda.synchronize()
    assert psa.read_device_error(again._workspace) == 0


def test_bench_read_probe_sizes_and_alignment(psa):
    """The benchmark's measurement aid (bench_probe.hip) reads and keeps nothing: any size runs (empty, below one
    load, ragged, several workgroups' worth), the source is unchanged, a misaligned source is refused on the host."""
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import bench
    probe = bench.load_read_probe()
    buf = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    before = buf.clone()
    sink = torch.zeros(1, dtype=torch.int64, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    for n in (0, 1, 4, 5, 1000, 2048 * 4 + 12, 1 << 20):
        assert probe(buf.data_ptr(), n * 4, sink.data_ptr(), st) == 0
    assert probe(buf.data_ptr(), buf.numel() * 4, None, st) == 0
    torch.cuda.synchronize()
    assert torch.equal(buf, before)
    assert probe(buf.data_ptr() + 4, 4096, sink.data_ptr(), st) == 1        # 4 bytes past a 16-byte boundary


@pytest.mark.parametrize("bad", ["nan", "inf", "huge"])
def test_non_finite_keys_do_not_disturb_other_requests(psa, bad):
    """Keys that are NaN, infinite or as large as the type allows in one request: the call completes (every
    loop of the kernels is bounded whatever the data), the other request's results are bit for bit those
    of a clean run, and the damaged request still reports a block count within its range."""
    cfg = get_config(1).scaled(batch=2, ctx=3000)
    li = generate_layer(cfg, device="cuda")
    clean = gc.run_gpu_decode(li, 0.9, 1)
    val = {"nan": float("nan"), "inf": float("inf"), "huge": 65504.0}[bad]
    pages = li.block_table[0, :188].long()
    k = li.k_pool.clone()
    k[pages[5], :, 3, :17] = val
    k[pages[100], 2, :, 64] = -val if bad != "nan" else val
    k[pages[187], :, 7, :] = val
    li.k_pool.copy_(k)
    kv = gc.to_kv(li)
    meta = psa.build_block_metadata(kv, page_fill=li.page_fill)
    out = psa.decode_attention(kv, li.q, meta, 0.9, 1, want_order=True)
    dense, _ = psa.dense_attention(kv, li.q)
    torch.cuda.synchronize()
    assert psa.read_device_error(out._workspace) == 0
    for name in ("out", "n_selected", "mass_est", "blocks_read", "lse"):
        assert torch.equal(getattr(out, name)[1], getattr(clean, name)[1]), name
    N0 = (int(li.ctx_lens[0]) + 15) // 16
    assert int(out.n_selected[0].min()) >= 0 and int(out.n_selected[0].max()) <= N0
    o = out.order[0, :, :N0].sort(dim=-1).values
    assert torch.equal(o, torch.arange(N0, device="cuda", dtype=torch.int32).expand_as(o)), "ranking must stay a permutation"
    assert torch.isfinite(dense[1]).all()
