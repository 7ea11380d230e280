"""The decode call enqueues kernels only (no allocation, no synchronisation, no memset node), so a caller
can record it into a HIP graph.  Replayed several times, with eager work and synchronisations between
the replays and with new queries written into the same buffer, every replay must give what the eager
call gives."""
import pytest
import torch

import gpu_common as gc
from workloads import generate_layer, get_config, step_inputs

pytestmark = pytest.mark.gpu


def test_decode_call_replays_from_a_graph():
    import paper_2503_00392_amd as psa
    psa.load_library()
    cfg = get_config(3).scaled(batch=2, ctx=8192, layers=1)
    li = generate_layer(cfg, layer=3, device="cuda")
    kv = gc.to_kv(li)
    meta = psa.build_block_metadata(kv, page_fill=li.page_fill)
    q = li.q.clone()
    first = psa.decode_attention(kv, q, meta, cfg.threshold, 1, want_order=True)      # warm-up outside the graph
    torch.cuda.synchronize()
    ws = first._workspace
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            psa.decode_attention(kv, q, meta, cfg.threshold, 1, workspace=ws, outputs=first,
                                 stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    seen = []
    for step in range(4):
        if step:
            q.copy_(step_inputs(li, step)[0])                   # new query bits in the captured buffer
        eager = psa.decode_attention(kv, q, meta, cfg.threshold, 1, want_order=True)
        torch.cuda.synchronize()
        want = (eager.out.clone(), eager.n_selected.clone(), eager.mass_est.clone(), eager.lse.clone(),
                eager.order.clone())
        first.out.zero_()
        first.n_selected.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert psa.read_device_error(ws) == 0
        got = (first.out, first.n_selected, first.mass_est, first.lse, first.order)
        for a, b in zip(want, got):
            assert torch.equal(a, b), f"replay {step} differs from the eager call"
        seen.append(want[0])
    assert not torch.equal(seen[0], seen[-1])           # the replays really ran on new queries
