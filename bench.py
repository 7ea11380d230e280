#!/usr/bin/env python3
"""Benchmark of the PSA decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]

A "step" is one decode step of the whole model of the chosen workload: for every layer, the
per-step metadata build (the pages that filled at this step), then scoring, ranking, progressive
attention with the on-GPU stop rule, and the final merge -- all through the C ABI of libpsa.so.
Inputs are seeded synthetic KV caches (workloads/generator.py), resident in HBM before timing.
Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class HipEvents:
    """hipEvent_t handles through the HIP runtime directly (the library records them itself)."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.all = []

    def array(self, n):
        arr = (C.c_void_p * n)()
        for i in range(n):
            ev = C.c_void_p()
            assert self.hip.hipEventCreate(C.byref(ev)) == 0
            arr[i] = ev
            self.all.append(ev)
        return arr

    def elapsed_ms(self, a, b) -> float:
        ms = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(ms), a, b)
        assert rc == 0, rc
        return float(ms.value)

    def destroy(self):
        for ev in self.all:
            self.hip.hipEventDestroy(ev)
        self.all = []


def load_read_probe():
    """bench_stream_read_probe of libbench_probe.so (bench_probe.hip, built by __graft_entry__.build())."""
    path = os.path.join(ROOT, "libbench_probe.so")
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is missing: run `python __graft_entry__.py` to build it")
    lib = C.CDLL(path)
    lib.bench_stream_read_probe.restype = C.c_int
    lib.bench_stream_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    return lib.bench_stream_read_probe


KERNEL_SOURCES = {"select_kernel": ["psa_select.hip", "psa_device.h"], "attend_kernel": ["psa_values.hip", "psa_attend.h", "psa_device.h"],
                  "score_kernel": ["psa_score.hip", "psa_device.h"]}


def kernel_source_hash(kernel: str) -> str:
    """sha256 (first 16 hex digits) over the source files a kernel is built from."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES.get(kernel, []):
        with open(os.path.join(ROOT, "paper_2503_00392_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def read_measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel` on `workload` as measured with hardware counters (two
    rocprofv3 --pmc runs, scaled by a plain copy of known size) and recorded in the text summary
    profiles/hbm_traffic_<workload>.md as a line `traffic_bytes_per_launch <kernel> = <number>`, next to a line
    `traffic_source_hash <kernel> = <hash>` of the kernel's sources at the time.  Returns (bytes, stamp): bytes is
    None if there is no such record or the kernel's sources have changed since it was taken (a stale number
    is worse than none)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.md")
    if not os.path.exists(path):
        return None, None
    value = stamp = None
    for line in open(path):
        parts = line.replace("`", "").split()
        if len(parts) >= 4 and parts[1] == kernel and parts[2] == "=":
            if parts[0] == "traffic_bytes_per_launch":
                value = float(parts[3])
            elif parts[0] == "traffic_source_hash":
                stamp = parts[3]
    now = kernel_source_hash(kernel)
    if value is None or stamp != now:
        return None, {"measured_at_source_hash": stamp, "current_source_hash": now,
                      "note": "no counter measurement for the kernel as it is built now"}
    return value, {"measured_at_source_hash": stamp, "current_source_hash": now}


def host_tier_leg(psa, args, cfg, layers, metas, eps, m, tuning_kw, dev):
    """Sec. 3.1 / 3.4 on this machine: the KV pools of a few layers live in pinned host memory, one pool of slots
    on the GPU caches their (page, KV head) slices, least recently used goes first.  Consecutive decode steps
    with slowly drifting queries; attention reads cached slices from HBM and the others over the host link;
    after each layer's attention the pool is updated on a second stream while the next layer computes."""
    import numpy as np
    import torch
    from workloads import step_inputs

    ids = [int(x) for x in args.host_tier_layers.split(",") if int(x) < len(layers)]
    n_steps, Lt = args.host_tier, len(ids)
    if Lt < 3:
        return {"skipped": "the leg needs at least three layers of the workload"}
    B, Hq, H = cfg.batch, cfg.num_q_heads, cfg.num_kv_heads
    per_layer = [layers[i].k_pool.shape[0] * H for i in ids]
    bases = [int(sum(per_layer[:j])) for j in range(Lt)]
    total = int(sum(per_layer))
    num_slots = max(int(total * args.slot_share), 1)
    t0 = time.time()
    tier = psa.Tier(total, num_slots)
    hosts = []
    for j, i in enumerate(ids):
        kh = torch.empty(layers[i].k_pool.shape, dtype=layers[i].k_pool.dtype, pin_memory=True)
        vh = torch.empty(layers[i].v_pool.shape, dtype=layers[i].v_pool.dtype, pin_memory=True)
        kh.copy_(layers[i].k_pool)
        vh.copy_(layers[i].v_pool)
        hosts.append(psa.KvCache(kh, vh, layers[i].block_table, layers[i].ctx_lens, Hq, tier=tier, slice_base=bases[j]))
    devs = [psa.KvCache(layers[i].k_pool, layers[i].v_pool, layers[i].block_table, layers[i].ctx_lens, Hq) for i in ids]
    torch.cuda.synchronize()
    log(f"[bench] host tier: {Lt} layers, {total * 8192 / 2**30:.1f} GiB pinned, {num_slots} slots "
        f"({num_slots * 8192 / 2**30:.1f} GiB) ready in {time.time() - t0:.1f}s")
    qs = [[step_inputs(layers[i], t)[0] for i in ids] for t in range(1, n_steps + 1)]
    MB = layers[ids[0]].block_table.shape[1]

    def new_outs():
        return [psa.DecodeOutput(torch.empty((B, Hq, 128), dtype=torch.float32, device=dev),
                                 torch.empty((B, Hq), dtype=torch.int32, device=dev),
                                 torch.empty((B, Hq), dtype=torch.float32, device=dev),
                                 torch.empty((B, H), dtype=torch.int32, device=dev),
                                 torch.empty((B, Hq), dtype=torch.float32, device=dev),
                                 torch.empty((B, H, MB), dtype=torch.int32, device=dev), None, None) for _ in range(Lt)]

    tun = psa.Tuning(**tuning_kw)
    ws = torch.empty(max(psa.decode_workspace_bytes(kv, tun) for kv in hosts), dtype=torch.uint8, device=dev)
    uws = torch.empty(max(psa.tier_update_workspace_bytes(kv) for kv in hosts), dtype=torch.uint8, device=dev)
    main_s, side_s = torch.cuda.current_stream(), torch.cuda.Stream()
    ev = lambda: torch.cuda.Event(enable_timing=True)

    # staging buffers (the attention kernels leave the slices they read over the host link there, so that the update
    # need not fetch them again): consecutive calls alternate between two, each with room for a cold layer's misses
    staging = [psa.Tier.staging_buffer(1 << 16, device=dev) for _ in range(2)]

    def run(caches, overlap, with_tier, use_hint=True, staged=True):
        outs = new_outs()
        hint = [torch.zeros((B, H), dtype=torch.int32, device=dev) for _ in range(Lt)]
        stats = torch.zeros((n_steps, Lt, 5), dtype=torch.int32, device=dev)
        calls = 0
        marks = [ev() for _ in range(n_steps + 1)]
        done = [None] * Lt                      # event: the last update of layer j has finished
        decoded = [ev() for _ in range(Lt)]
        torch.cuda.synchronize()
        marks[0].record(main_s)
        for t in range(n_steps):
            for j in range(Lt):
                if with_tier and overlap and done[(j - 2) % Lt] is not None:
                    main_s.wait_event(done[(j - 2) % Lt])     # the update that ran beside layer j-1 may have evicted anything else
                # the depth hint of a step is what the same layer read in the step before (a copy: the call rewrites it)
                tn = psa.Tuning(depth_hint=hint[j], **tuning_kw) if (use_hint and t > 0) else tun
                if with_tier:
                    caches[j].staging = staging[calls % 2] if staged else None
                    calls += 1
                psa.decode_attention(caches[j], qs[t][j], metas[ids[j]], eps, m, workspace=ws, outputs=outs[j], tuning=tn)
                if use_hint:
                    hint[j].copy_(outs[j].blocks_read)
                if not with_tier:
                    continue
                if overlap:
                    decoded[j].record(main_s)
                    side_s.wait_event(decoded[j])
                    nxt = (j + 1) % Lt
                    psa.tier_update(caches[j], outs[j].order, outs[j].blocks_read, bases[nxt], per_layer[nxt],
                                    stats=stats[t, j], workspace=uws, stream=side_s)
                    done[j] = ev()
                    done[j].record(side_s)
                    # the next decode of this layer overwrites outs[j]: not before this update has read them
                else:
                    psa.tier_update(caches[j], outs[j].order, outs[j].blocks_read, 0, 0, stats=stats[t, j], workspace=uws)
            if with_tier and overlap:
                main_s.wait_event(done[Lt - 1])               # (also keeps outs[] from being overwritten too early)
            marks[t + 1].record(main_s)
        torch.cuda.synchronize()
        ms = [marks[t].elapsed_time(marks[t + 1]) for t in range(n_steps)]
        return ms, stats.cpu().numpy().astype(np.int64), [o.blocks_read.clone() for o in outs], [o.out.clone() for o in outs]

    hbm_ms, _, hbm_read, hbm_out = run(devs, False, False)
    psa.tier_init(tier)
    ser_ms, ser_stats, ser_read, ser_out = run(hosts, False, True)
    psa.tier_init(tier)
    ovl_ms, ovl_stats, ovl_read, ovl_out = run(hosts, True, True)
    psa.tier_init(tier)
    noh_ms, noh_stats, _, noh_out = run(hosts, True, True, use_hint=False)
    psa.tier_init(tier)
    uns_ms, uns_stats, _, uns_out = run(hosts, True, True, staged=False)
    same = all(torch.equal(a, b) for a, b in zip(hbm_out, ser_out)) and all(torch.equal(a, b) for a, b in zip(hbm_out, ovl_out)) \
        and all(torch.equal(a, b) for a, b in zip(hbm_out, uns_out))
    assert psa.read_device_error(ws) == 0

    def summary(ms, st):
        used = st[..., 0] + st[..., 1]
        half = n_steps // 2
        return {"first_step_ms": ms[0], "steady_ms_per_step": float(np.median(ms[half:])),
                "hit_ratio_first_step": float(st[0, :, 0].sum() / max(used[0].sum(), 1)),
                "hit_ratio_steady": float(st[half:, :, 0].sum() / max(used[half:].sum(), 1)),
                "slices_used_per_step": float(used[half:].sum(1).mean()),
                "host_link_MB_per_step_steady": float((st[half:, :, 1] + st[half:, :, 2] - st[half:, :, 4]).sum(1).mean() * 8192 / 1e6),
                "placed_from_staging_per_step_steady": float(st[half:, :, 4].sum(1).mean()),
                "evicted_per_step_steady": float(st[half:, :, 3].sum(1).mean())}

    return {"layers": ids, "steps": n_steps, "pinned_GiB": total * 8192 / 2**30, "slots": num_slots,
            "slot_pool_GiB": num_slots * 8192 / 2**30, "slot_share": args.slot_share,
            "all_in_hbm_ms_per_step": float(np.median(hbm_ms[n_steps // 2:])),
            "tier_update_on_the_same_stream": summary(ser_ms, ser_stats),
            "tier_update_on_a_second_stream": summary(ovl_ms, ovl_stats),
            "tier_update_on_a_second_stream_no_depth_hint": summary(noh_ms, noh_stats),
            "tier_update_on_a_second_stream_no_staging": summary(uns_ms, uns_stats),
            "outputs_equal_all_in_hbm": bool(same),
            "note": "queries drift from step to step, the cache does not grow; host_link_MB counts slices read in "
                    "place by the attention kernels (misses) plus slices the update fetched from host memory (those "
                    "placed that did not come from the staging buffer)"}


def other_workload(psa, idx, eps, m, steps, dev):
    """One of the other workloads at its full shape: PSA and the dense control on the same inputs, every step
    timed on its own with device events (inputs that would fit the last-level cache twice over are evicted
    between steps by a 1 GiB write, which is not timed)."""
    import numpy as np
    import torch
    from workloads import generate_layer, get_config
    cfg = get_config(idx)
    B, Hq, H = cfg.batch, cfg.num_q_heads, cfg.num_kv_heads
    li = generate_layer(cfg, device=dev)
    kv = psa.KvCache(li.k_pool, li.v_pool, li.block_table, li.ctx_lens, Hq)
    meta = psa.build_block_metadata(kv, page_fill=li.page_fill)
    nblk = (li.ctx_lens.cpu().numpy().astype(np.int64) + 15) // 16
    last_pages = torch.stack([li.block_table[r, max(int(nblk[r]) - 1, 0)] for r in range(B)]).contiguous()
    ws = torch.empty(psa.decode_workspace_bytes(kv), dtype=torch.uint8, device=dev)
    out = psa.DecodeOutput(torch.empty((B, Hq, 128), dtype=torch.float32, device=dev),
                           torch.empty((B, Hq), dtype=torch.int32, device=dev),
                           torch.empty((B, Hq), dtype=torch.float32, device=dev),
                           torch.empty((B, H), dtype=torch.int32, device=dev),
                           torch.empty((B, Hq), dtype=torch.float32, device=dev), None, None,
                           torch.empty((B, H, 2), dtype=torch.int32, device=dev))
    dws = torch.empty(psa.dense_workspace_bytes(kv), dtype=torch.uint8, device=dev)
    dout = torch.empty((B, Hq, 128), dtype=torch.float32, device=dev)
    dlse = torch.empty((B, Hq), dtype=torch.float32, device=dev)
    working_set = kv.k_pool.numel() * 2 * 2 + meta.numel() * 2
    flush = torch.empty(1 << 30, dtype=torch.uint8, device=dev) if working_set < (512 << 20) else None

    def psa_step():
        psa.build_block_metadata(kv, meta, page_fill=li.page_fill, page_list=last_pages)
        psa.decode_attention(kv, li.q, meta, eps, m, workspace=ws, outputs=out)

    def dense_step():
        psa.dense_attention(kv, li.q, workspace=dws, out=dout, lse=dlse)

    def timed(fn):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        for k in range(steps):
            if flush is not None:
                flush.fill_(k & 0xFF)
            ev[k][0].record()
            fn()
            ev[k][1].record()
        torch.cuda.synchronize()
        return float(np.median([a.elapsed_time(b) for a, b in ev]))

    psa_ms, dense_ms = timed(psa_step), timed(dense_step)
    assert psa.read_device_error(ws) == 0
    read = out.blocks_read.cpu().numpy().astype(np.int64)
    Ntot = np.repeat(nblk[:, None], H, 1)
    alg = int((read * 8192 + Ntot * 516).sum() + B * Hq * 256)
    dense_bytes = int((Ntot * 8196).sum() + B * Hq * 256)
    true_mass = torch.exp(out.lse - dlse)
    live = torch.isfinite(dlse)
    return {"workload": cfg.name, "threshold": eps, "check_granularity": m, "kv_dtype": cfg.dtype,
            "query_heads": B * Hq, "psa_ms_per_step": psa_ms, "dense_ms_per_step": dense_ms,
            "psa_query_heads_per_s": B * Hq / (psa_ms * 1e-3), "psa_speedup": dense_ms / psa_ms,
            "kv_reduction_vs_dense": float((Ntot * 8192).sum() / (Ntot * 512 + read * 8192).sum()),
            "mean_selected_fraction": float((read / np.maximum(Ntot, 1)).mean()),
            "algorithmic_bytes_per_step": alg, "hbm_frac": alg / (psa_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "dense_hbm_frac": dense_bytes / (dense_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "true_mass_mean": float(true_mass[live].mean()) if bool(live.any()) else 1.0,
            "timing": "median of the steps, each timed on its own" + (", inputs evicted from the cache between steps" if flush is not None else "")}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (3 = the 128K-context one)")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging)")
    ap.add_argument("--check-granularity", type=int, default=1)
    ap.add_argument("--threshold", type=float, default=-1.0, help="override the workload's threshold (tuning)")
    ap.add_argument("--scorer", type=int, default=0, help="0 = upper bound (default), 1 = cuboid centre")
    ap.add_argument("--chunk-blocks", type=int, default=0)
    ap.add_argument("--window-chunks", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-topk-comparison", action="store_true")
    ap.add_argument("--no-scorer-comparison", action="store_true")
    ap.add_argument("--no-depth-hint", action="store_true")
    ap.add_argument("--decode-loop", type=int, default=8,
                    help="also run this many consecutive decode steps (append a token, drift the queries; 0 = skip), with and "
                         "without the previous step's blocks_read as depth hint")
    ap.add_argument("--cpu-layers", type=str, default="", help="layers the oracle is timed on")
    ap.add_argument("--host-tier", type=int, default=12,
                    help="decode steps of the two-tier leg (KV of a few layers in pinned host memory, a slot pool on "
                         "the GPU); 0 = skip")
    ap.add_argument("--host-tier-layers", type=str, default="2,3,4,5")
    ap.add_argument("--slot-share", type=float, default=0.19, help="slots of the pool / slices of the tiered layers")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the leg that runs the other four workloads (PSA and dense, a few steps each)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
            "(the path shards by request or by KV head with no exchange between the shards)")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2503_00392_amd as psa
    from workloads import generate_layer, get_config

    psa.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = get_config(args.config)
    if args.layers:
        cfg = cfg.scaled(layers=args.layers)
    L, B, Hq, H, G = cfg.layers, cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.group
    eps, m = (args.threshold if args.threshold >= 0 else cfg.threshold), args.check_granularity
    tuning_kw = dict(chunk_blocks=args.chunk_blocks, window_chunks=args.window_chunks)

    # ---- inputs, resident in HBM ---------------------------------------------------------------
    t0 = time.time()
    layers = []
    for l in range(L):
        li = generate_layer(cfg, layer=l, device=dev)
        layers.append(li)
        if l % 8 == 0:
            log(f"[bench] generated layer {l + 1}/{L}  ({time.time() - t0:.1f}s, "
                f"{torch.cuda.memory_allocated() / 2**30:.1f} GiB)")
    kvs = [psa.KvCache(li.k_pool, li.v_pool, li.block_table, li.ctx_lens, Hq) for li in layers]
    nblk = [((li.ctx_lens.cpu().numpy().astype(np.int64) + 15) // 16) for li in layers]
    # the page of each request that fills at this step (its last one): the per-step metadata work
    last_pages = [torch.stack([li.block_table[r, max(int(nblk[i][r]) - 1, 0)] for r in range(B)]).contiguous()
                  for i, li in enumerate(layers)]
    torch.cuda.synchronize()

    # ---- bulk metadata build (once per filled page in a serving system; timed on its own) -------
    metas = [torch.empty((kv.k_pool.shape[0], H, 2, 128), dtype=kv.k_pool.dtype, device=dev) for kv in kvs]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for rep in range(2):
        e0.record()
        for kv, meta, li in zip(kvs, metas, layers):
            psa.build_block_metadata(kv, meta, page_fill=li.page_fill)
        e1.record()
        torch.cuda.synchronize()
    meta_ms = e0.elapsed_time(e1)
    meta_bytes = sum(kv.k_pool.numel() * 2 + mt.numel() * 2 for kv, mt in zip(kvs, metas))

    # ---- buffers of the timed loop: nothing is allocated inside it --------------------------------
    tun = psa.Tuning(**tuning_kw)
    ws_bytes = max(psa.decode_workspace_bytes(kv, tun) for kv in kvs)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    MB = max(kv.block_table.shape[1] for kv in kvs)
    outs = [psa.DecodeOutput(torch.empty((B, Hq, 128), dtype=torch.float32, device=dev),
                             torch.empty((B, Hq), dtype=torch.int32, device=dev),
                             torch.empty((B, Hq), dtype=torch.float32, device=dev),
                             torch.empty((B, H), dtype=torch.int32, device=dev),
                             torch.empty((B, Hq), dtype=torch.float32, device=dev), None, None,
                             torch.empty((B, H, 2), dtype=torch.int32, device=dev)) for _ in range(L)]

    def step(tunings=None):
        for i in range(L):
            psa.build_block_metadata(kvs[i], metas[i], page_fill=layers[i].page_fill, page_list=last_pages[i])
            psa.decode_attention(kvs[i], layers[i].q, metas[i], eps, m, workspace=ws, outputs=outs[i],
                                 tuning=tunings[i] if tunings else tun, scorer=args.scorer)

    # one plain 1 GiB device copy: the known-size kernel that hardware-counter runs are scaled by
    cal_src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    # streaming-read ceiling: a plain kernel reads 4 GiB once (the cache holds 256 MB); 2 untimed + 7 timed
    probe = torch.empty(4 << 30, dtype=torch.uint8, device=dev).fill_(0x5A)
    sink = torch.zeros(1, dtype=torch.int64, device=dev)
    probe_ms = []
    read_probe = load_read_probe()
    for rep in range(9):
        e0.record()
        assert read_probe(probe.data_ptr(), probe.numel(), sink.data_ptr(), torch.cuda.current_stream().cuda_stream) == 0
        e1.record()
        torch.cuda.synchronize()
        if rep >= 2:
            probe_ms.append(e0.elapsed_time(e1))
    ceiling_gbs = probe.numel() / (float(np.median(probe_ms)) * 1e-3) / 1e9
    read_ceiling = {"GBps": ceiling_gbs, "GBps_best": probe.numel() / (min(probe_ms) * 1e-3) / 1e9,
                    "frac_of_peak": ceiling_gbs / HBM_PEAK_GBS, "bytes": probe.numel(), "runs": len(probe_ms),
                    "kernel": "bench_stream_read_probe (16-byte non-temporal loads, one pass)"}
    del probe
    log(f"[bench] streaming-read ceiling {ceiling_gbs:.0f} GB/s")

    # inputs smaller than twice the 256 MB last-level cache would be timed cache-warm: evict them between
    # steps with a 1 GiB write, and time every step on its own so that the eviction is not counted
    working_set = sum(kv.k_pool.numel() * 2 * 2 + mt.numel() * 2 for kv, mt in zip(kvs, metas))
    flush = torch.empty(1 << 30, dtype=torch.uint8, device=dev) if working_set < (512 << 20) else None

    log(f"[bench] inputs ready in {time.time() - t0:.1f}s; warmup")
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert psa.read_device_error(ws) == 0

    # ---- timed region: exactly K steps -------------------------------------------------------------
    step_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    e0.record()
    for k in range(args.steps):
        if flush is not None:
            flush.fill_(k & 0xFF)
        step_ev[k][0].record()
        step()
        step_ev[k][1].record()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_start) * 1e3
    gpu_ms = e0.elapsed_time(e1)
    step_ms = [a.elapsed_time(b) for a, b in step_ev]
    if flush is None:
        ms_per_step = max(wall_ms, gpu_ms) / args.steps          # the whole bracket, host clock included
        timing = "K steps back to back between two synchronisations; max of host clock and device events"
    else:
        ms_per_step = float(np.sum(step_ms)) / args.steps        # the evictions between the steps are not the path's
        timing = ("inputs fit the last-level cache: 1 GiB written between steps to evict them, every step timed "
                  "on its own with device events, evictions excluded")
    q_heads_per_step = L * B * Hq
    value = q_heads_per_step / (ms_per_step * 1e-3)

    # ---- selection statistics and bytes (from the outputs of the last step) -------------------------
    blocks_read = np.stack([o.blocks_read.cpu().numpy().astype(np.int64) for o in outs])      # [L][B][H]
    traffic = np.stack([o.traffic.cpu().numpy().astype(np.int64) for o in outs])              # [L][B][H][2]
    n_sel = np.stack([o.n_selected.cpu().numpy().astype(np.int64) for o in outs])
    N_total = np.stack([np.repeat(nb[:, None], H, 1) for nb in nblk])                          # [L][B][H]
    page_bytes = blocks_read * 8192
    meta_read = N_total * 512
    table_read = N_total * 4
    q_bytes = L * B * Hq * 256
    alg_bytes = int(page_bytes.sum() + meta_read.sum() + table_read.sum() + q_bytes)
    dense_bytes = int((N_total * 8192).sum() + table_read.sum() + q_bytes)
    kv_reduction = float((N_total * 8192).sum() / (meta_read.sum() + page_bytes.sum()))
    spec_k_bytes = int(((traffic[..., 0] - blocks_read) * 4096).sum())
    eff_gbs = alg_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- the same step with a depth hint per (request, KV head): the blocks the previous step read.  The
    # steps of this benchmark are identical, so the hint is exact -- the upper bound of what the similarity
    # of consecutive decode queries can give; `value` above is measured without any hint. ------------------
    hinted = None
    if not args.no_depth_hint:
        hints = [o.blocks_read.clone() for o in outs]
        hinted_tun = [psa.Tuning(depth_hint=hints[i], **tuning_kw) for i in range(L)]
        step(hinted_tun)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            step(hinted_tun)
        e1.record()
        torch.cuda.synchronize()
        hint_ms = e0.elapsed_time(e1) / args.steps
        hint_same = all(torch.equal(o.blocks_read, h) for o, h in zip(outs, hints))
        hinted = {"ms_per_step": hint_ms, "query_heads_per_s": q_heads_per_step / (hint_ms * 1e-3),
                  "same_selection_as_without_hint": bool(hint_same),
                  "hint": "blocks_read of an identical previous step (exact: an upper bound for real decode loops)"}

    # ---- per-kernel durations, live, with HIP events recorded by the library around its kernels ----
    hev = HipEvents()
    ev_sets = [[hev.array(6) for _ in range(L)] for _ in range(args.steps)]
    for k in range(args.steps):
        step([psa.Tuning(phase_events=ev_sets[k][i], **tuning_kw) for i in range(L)])
    torch.cuda.synchronize()
    names = ["score", "order", "select", "attend", "finalize"]
    phase_ms = {n: [] for n in names}
    for k in range(args.steps):
        for i in range(L):
            ev = ev_sets[k][i]
            for j, n in enumerate(names):
                phase_ms[n].append(hev.elapsed_ms(ev[j], ev[j + 1]))
    hev.destroy()
    phase_avg = {n: float(np.mean(v)) for n, v in phase_ms.items()}
    # algorithmic bytes per launch: the selection kernel must move the key
    # slices of the blocks read and their page ids, the attention kernel the value slices and page ids,
    # the scoring kernel the metadata and the block table.  Scratch the implementation adds (stored
    # logits, partials) is not counted.
    kern_bytes = {"select_kernel": float(blocks_read.sum() * (4096 + 8) / L),
                  "attend_kernel": float(blocks_read.sum() * (4096 + 8) / L),
                  "score_kernel": float((meta_read.sum() + table_read.sum()) / L)}
    kern_ms = {"select_kernel": phase_avg["select"], "attend_kernel": phase_avg["attend"],
               "score_kernel": phase_avg["score"]}
    dom = max(kern_ms, key=kern_ms.get)
    dom_gbs = kern_bytes[dom] / (kern_ms[dom] * 1e-3) / 1e9
    kern_gbs = {k: kern_bytes[k] / (kern_ms[k] * 1e-3) / 1e9 for k in kern_ms}
    per_layer = {n: np.array(phase_ms[n]).reshape(args.steps, L).mean(0) for n in names}

    # ---- dense control on the same inputs -------------------------------------------------------------
    dense = None
    if not args.no_dense:
        dws = torch.empty(max(psa.dense_workspace_bytes(kv) for kv in kvs), dtype=torch.uint8, device=dev)
        dout = torch.empty((B, Hq, 128), dtype=torch.float32, device=dev)
        dlse = torch.empty((B, Hq), dtype=torch.float32, device=dev)
        for rep in range(1 + args.steps):
            if rep == 1:
                e0.record()
            for i in range(L):
                psa.dense_attention(kvs[i], layers[i].q, workspace=dws, out=dout, lse=dlse)
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1) / args.steps
        dense = {"ms_per_step": dense_ms, "query_heads_per_s": q_heads_per_step / (dense_ms * 1e-3),
                 "bytes": dense_bytes, "GBps": dense_bytes / (dense_ms * 1e-3) / 1e9,
                 "hbm_frac": dense_bytes / (dense_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "frac_of_read_ceiling": dense_bytes / (dense_ms * 1e-3) / 1e9 / ceiling_gbs,
                 "psa_speedup": dense_ms / ms_per_step, "kv_reduction_implied": kv_reduction}

    # ---- fixed-budget control: the smallest uniform k that gives every query head at least the true
    # attention mass PSA's selection holds for it (the adaptive-budget claim of Sec. 1 / Sec. 5.2 on
    # these inputs).  True mass of a selection = exp(lse of the selection - lse of dense attention).
    topk = None
    if not args.no_topk_comparison:
        dws2 = torch.empty(max(psa.dense_workspace_bytes(kv) for kv in kvs), dtype=torch.uint8, device=dev)
        dout2 = torch.empty((B, Hq, 128), dtype=torch.float32, device=dev)
        tout = psa.DecodeOutput(torch.empty((B, Hq, 128), dtype=torch.float32, device=dev),
                                torch.empty((B, Hq), dtype=torch.int32, device=dev),
                                torch.empty((B, Hq), dtype=torch.float32, device=dev),
                                torch.empty((B, H), dtype=torch.int32, device=dev),
                                torch.empty((B, Hq), dtype=torch.float32, device=dev), None, None, None)
        k_layer, mass_min, mass_mean = [], [], []
        for i in range(L):
            dlse_i = torch.empty((B, Hq), dtype=torch.float32, device=dev)
            psa.dense_attention(kvs[i], layers[i].q, workspace=dws2, out=dout2, lse=dlse_i)
            live = torch.isfinite(dlse_i)
            target = torch.exp(outs[i].lse - dlse_i)
            mass_min.append(float(target[live].min()) if bool(live.any()) else 1.0)
            mass_mean.append(float(target[live].mean()) if bool(live.any()) else 1.0)
            lo, hi = 1, max(int(nblk[i].max()), 1)
            while lo < hi:
                mid = (lo + hi) // 2
                psa.topk_attention(kvs[i], layers[i].q, metas[i], mid, workspace=ws, outputs=tout, tuning=tun)
                reached = torch.exp(tout.lse - dlse_i) >= target * (1.0 - 1e-5)
                if bool((reached | ~live).all()):
                    hi = mid
                else:
                    lo = mid + 1
            k_layer.append(lo)
        k_all = max(k_layer)
        for rep in range(1 + args.steps):
            if rep == 1:
                e0.record()
            for i in range(L):
                psa.topk_attention(kvs[i], layers[i].q, metas[i], k_all, workspace=ws, outputs=tout, tuning=tun)
        e1.record()
        torch.cuda.synchronize()
        assert psa.read_device_error(ws) == 0
        topk_ms = e0.elapsed_time(e1) / args.steps
        uni_all = np.minimum(N_total, k_all).sum()
        uni_layer = sum(np.minimum(N_total[i], k_layer[i]).sum() for i in range(L))
        topk = {"definition": "smallest k such that top-k attention gives every query head at least the true "
                              "attention mass of PSA's selection for that head",
                "uniform_k_all_layers": k_all, "uniform_k_per_layer": k_layer,
                "psa_blocks_read_per_stream_mean": float(blocks_read.mean()),
                "psa_true_mass_min": float(min(mass_min)), "psa_true_mass_mean": float(np.mean(mass_mean)),
                "blocks_uniform_k_over_psa": float(uni_all / max(blocks_read.sum(), 1)),
                "blocks_per_layer_k_over_psa": float(uni_layer / max(blocks_read.sum(), 1)),
                "topk_ms_per_step_at_uniform_k": topk_ms, "psa_speedup_over_uniform_k": topk_ms / ms_per_step}
        log(f"[bench] uniform top-k matching PSA's true mass on every head: k = {k_all} "
            f"(per layer {k_layer}); PSA reads {blocks_read.mean():.0f} blocks per stream on average")

    # ---- ranking quality of the two scorers over the same metadata: how many blocks PSA reads with each,
    # what share of the true attention mass the selection then holds, how far the rule's own estimate
    # P_acc overshoots it (the estimate is only a bound under an ideal ranking, Sec. 3.2) -------------------
    scorers = None
    if not args.no_scorer_comparison:
        dws3 = torch.empty(max(psa.dense_workspace_bytes(kv) for kv in kvs), dtype=torch.uint8, device=dev)
        dout3 = torch.empty((B, Hq, 128), dtype=torch.float32, device=dev)
        dlses = []
        for i in range(L):
            dl = torch.empty((B, Hq), dtype=torch.float32, device=dev)
            psa.dense_attention(kvs[i], layers[i].q, workspace=dws3, out=dout3, lse=dl)
            dlses.append(dl)
        so = psa.DecodeOutput(torch.empty((B, Hq, 128), dtype=torch.float32, device=dev),
                              torch.empty((B, Hq), dtype=torch.int32, device=dev),
                              torch.empty((B, Hq), dtype=torch.float32, device=dev),
                              torch.empty((B, H), dtype=torch.int32, device=dev),
                              torch.empty((B, Hq), dtype=torch.float32, device=dev), None, None, None)
        scorers = {}
        # mean-key metadata: one vector per block, half the bytes of the cuboid (built here, outside the timed steps)
        mean_metas = [psa.build_block_means(kvs[i], page_fill=layers[i].page_fill) for i in range(L)]
        for name, code in (("upper_bound", psa.SCORE_UPPER_BOUND), ("cuboid_center", psa.SCORE_CUBOID_CENTER),
                           ("mean_key", psa.SCORE_MEAN_KEY)):
            use = mean_metas if code == psa.SCORE_MEAN_KEY else metas
            read, true_mass, gap, short = [], [], [], []
            for rep in range(2):
                if rep == 1:
                    e0.record()
                for i in range(L):
                    psa.decode_attention(kvs[i], layers[i].q, use[i], eps, m, workspace=ws, outputs=so,
                                         tuning=tun, scorer=code)
                    if rep == 0:
                        live = torch.isfinite(dlses[i])
                        tm = torch.exp(so.lse - dlses[i])[live]
                        read.append(so.blocks_read.double().mean().item())
                        true_mass.append(tm.double().mean().item())
                        gap.append((so.mass_est[live] - tm).double().mean().item())
                        short.append((tm < eps).double().mean().item())
            e1.record()
            torch.cuda.synchronize()
            scorers[name] = {"blocks_read_per_stream_mean": float(np.mean(read)),
                             "true_mass_mean": float(np.mean(true_mass)),
                             "estimate_minus_true_mass_mean": float(np.mean(gap)),
                             "heads_with_true_mass_below_threshold": float(np.mean(short)),
                             "metadata_bytes_per_block": 256 if code == psa.SCORE_MEAN_KEY else 512,
                             "ms_per_step": e0.elapsed_time(e1)}
            log(f"[bench] scorer {name}: {scorers[name]}")
        assert psa.read_device_error(ws) == 0
        del mean_metas

    # ---- the oracle on the host cores, bounded sample ----------------------------------------------------
    cpu = parity = None
    if not args.no_cpu_baseline:
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import gpu_common as gc
        from oracle import psa_oracle as po
        if args.cpu_layers:
            sample = [int(x) for x in args.cpu_layers.split(",")]
        else:
            sample = list(range(L))          # the whole step: about 10-20 s of oracle time for config 3
        reqs = list(range(B))
        t_cpu, heads = 0.0, 0
        same_n = out_ok = 0
        for l in sample:
            pb = gc.to_problem(layers[l])
            sub = po.Problem(pb.q[reqs], pb.k_pool, pb.v_pool, pb.block_table[reqs], pb.ctx_lens[reqs], pb.dtype)
            meta_bits = po.block_metadata(sub, sub.page_fill())     # the oracle's own, not timed (bulk step)
            t1 = time.perf_counter()
            res = po.psa_decode(sub, eps, m, meta=meta_bits)
            t_cpu += time.perf_counter() - t1
            heads += len(reqs) * Hq
            g_n = outs[l].n_selected.cpu().numpy()[reqs]
            eq = g_n == res.n_selected
            same_n += int(eq.sum())
            # where both took the same number of blocks the outputs must agree (heads that stop elsewhere are the
            # near-boundary classes the parity tests examine block by block)
            err = gc.rel_l2(outs[l].out.cpu().numpy().astype(np.float64)[reqs], res.out)
            out_ok += int((err[eq] <= gc.OUT_RTOL).sum())
            log(f"[bench] oracle layer {l}: {len(reqs) * Hq} heads, n_selected equal on "
                f"{eq.mean() * 100:.1f}% of heads, cumulative {t_cpu:.1f}s")
            del pb, sub
        parity = {"heads": heads, "n_selected_equal": same_n, "frac": same_n / max(heads, 1),
                  "outputs_within_tolerance_where_equal": out_ok, "tolerance": gc.OUT_RTOL,
                  "ok": bool(same_n >= 0.99 * heads and out_ok >= 0.995 * same_n),
                  "what": "the timed step's results against the oracle on the cpu_baseline sample: heads that stop at "
                          "the same block count, and how many of those have outputs within the tolerance (the rest are "
                          "heads whose last blocks tie in score, which the element-by-element rule of "
                          "tests/gpu_common.py examines block by block); fails below 99 % / 99.5 %"}
        cpu = {"value": heads / t_cpu, "unit": "query-heads/s", "cores": po.num_threads(), "kind": "oracle",
               "sample": f"config {cfg.index}, layers {sample}, requests {reqs}, all {Hq} query heads, "
                         f"scoring+ranking+progressive loop in fp64 ({t_cpu:.1f}s of CPU time)"}
        # the same code on one thread, on the middle layer of the sample and as many of its requests as about
        # 8 s of work cover (estimated from the run above)
        threads = po.num_threads()
        l1 = sample[len(sample) // 2]
        est_layer = t_cpu / len(sample) * threads
        n1 = int(min(B, max(1, B * 8.0 / max(est_layer, 1e-9))))
        reqs1 = list(range(n1))
        pb = gc.to_problem(layers[l1])
        sub = po.Problem(pb.q[reqs1], pb.k_pool, pb.v_pool, pb.block_table[reqs1], pb.ctx_lens[reqs1], pb.dtype)
        meta_bits = po.block_metadata(sub, sub.page_fill())
        log(f"[bench] oracle on one thread: layer {l1}, requests {reqs1}")
        po.set_num_threads(1)
        t1 = time.perf_counter()
        po.psa_decode(sub, eps, m, meta=meta_bits)
        t_one = time.perf_counter() - t1
        po.set_num_threads(threads)
        cpu["single_thread"] = {"value": n1 * Hq / t_one, "unit": "query-heads/s", "cores": 1,
                                "sample": f"config {cfg.index}, layer {l1}, requests {reqs1}, all query heads ({t_one:.1f}s)"}
        log(f"[bench] oracle on one thread: {t_one:.1f}s")
        del pb, sub

    tier_leg = None
    if args.host_tier > 0:
        try:
            tier_leg = host_tier_leg(psa, args, cfg, layers, metas, eps, m, tuning_kw, dev)
        except Exception as exc:                      # e.g. no pinned memory to be had: the leg is an extra
            tier_leg = {"error": f"{type(exc).__name__}: {exc}"}
        log(f"[bench] host tier: {tier_leg}")

    # ---- consecutive decode steps: every step appends one token per request to every layer's cache
    # (K, V, metadata, length: psa_append_kv) and decodes with queries that drifted a little; the depth
    # hint of a step is what the same layer read in the step before -------------------------------------
    loop = None
    if args.decode_loop > 0:
        from workloads import step_inputs
        n_steps = args.decode_loop
        # room for the appended tokens: the loop starts from contexts cut back by whole pages (at 128K the
        # block table is full), and refills those pages -- in place, this is the last leg of the run
        cut = 16 * ((n_steps + 15) // 16)
        roomy, kvs2, metas2, ws2 = layers, kvs, metas, ws
        inputs = [[step_inputs(roomy[i], t) for i in range(L)] for t in range(1, n_steps + 1)]
        ctx0 = [torch.clamp(li.ctx_lens - cut, min=0) for li in roomy]
        # two sets of outputs used in turn: a step's hint is the other set's blocks_read, written one step
        # earlier -- no copy, no extra kernel inside the timed loop
        louts2 = [[psa.DecodeOutput(torch.empty((B, Hq, 128), dtype=torch.float32, device=dev),
                                    torch.empty((B, Hq), dtype=torch.int32, device=dev),
                                    torch.empty((B, Hq), dtype=torch.float32, device=dev),
                                    torch.empty((B, H), dtype=torch.int32, device=dev),
                                    torch.empty((B, Hq), dtype=torch.float32, device=dev), None, None, None) for _ in range(L)]
                  for _ in range(2)]
        loop = {"steps": n_steps}
        for mode in ("warm_up", "without_hint", "with_previous_step_hint"):
            for i in range(L):
                roomy[i].ctx_lens.copy_(ctx0[i])
            read = []
            tunings = [[psa.Tuning(depth_hint=louts2[k][i].blocks_read, **tuning_kw) for i in range(L)] for k in range(2)]
            torch.cuda.synchronize()
            e0.record()
            for t in range(1 if mode == "warm_up" else n_steps):     # (the first append loads its kernel: not timed)
                cur, old = louts2[t % 2], tunings[(t + 1) % 2]
                for i in range(L):
                    qt, kt, vt = inputs[t][i]
                    psa.append_kv(kvs2[i], kt, vt, metas2[i])
                    tn = old[i] if (mode == "with_previous_step_hint" and t > 0) else tun
                    psa.decode_attention(kvs2[i], qt, metas2[i], eps, m, workspace=ws2, outputs=cur[i], tuning=tn,
                                         scorer=args.scorer)
            e1.record()
            torch.cuda.synchronize()
            read = [o.blocks_read.double().mean().item() for o in cur]
            assert psa.read_device_error(ws2) == 0
            if mode != "warm_up":
                loop[mode] = {"ms_per_step": e0.elapsed_time(e1) / n_steps,
                              "blocks_read_per_stream_mean_last_step": float(np.mean(read))}
        log(f"[bench] decode loop: {loop}")

    # ---- the other workloads, each at its full shape (beside the headline's inputs: 288 GB hold both) -----
    others = None
    if not args.no_other_configs:
        others = []
        for idx, th in ((1, None), (2, None), (4, None), (5, 0.95), (5, 0.99)):
            if idx == cfg.index:
                continue
            try:
                rec = other_workload(psa, idx, get_config(idx).threshold if th is None else th, m, max(args.steps, 10), dev)
            except Exception as exc:
                rec = {"workload": get_config(idx).name, "error": f"{type(exc).__name__}: {exc}"}
            log(f"[bench] other workload: {rec}")
            others.append(rec)
            torch.cuda.empty_cache()

    traffic, traffic_stamp = read_measured_traffic(cfg.name, dom)

    result = {
        "metric": "psa_decode_query_heads_per_s", "value": value, "unit": "query-heads/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_median": float(np.median(step_ms)), "ms_per_step_min": float(np.min(step_ms)), "timing": timing,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "accumulate": "f32", "contraction": f"{cfg.dtype} x {cfg.dtype} -> f32 on the matrix cores",
        "data": "synthetic",
        "config": {"workload": cfg.name, "layers": L, "batch": B, "num_q_heads": Hq, "num_kv_heads": H,
                   "ctx": cfg.ctx, "kv_dtype": cfg.dtype, "threshold": eps, "check_granularity": m,
                   "scorer": ["upper_bound", "cuboid_center"][args.scorer],
                   "chunk_blocks": args.chunk_blocks or 32, "parallelism": "1 GPU"},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": dom_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": dom_gbs / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_measured_at": traffic_stamp,
                     "frac_of_read_ceiling": dom_gbs / ceiling_gbs,
                     "avg_launch_ms": kern_ms[dom], "algorithmic_bytes_per_launch": kern_bytes[dom]},
        "cpu_baseline": cpu,
        "parity": parity,
        "read_ceiling": read_ceiling,
        "whole_path": {"algorithmic_bytes_per_step": alg_bytes, "GBps": eff_gbs, "hbm_frac": eff_gbs / HBM_PEAK_GBS,
                       "frac_of_read_ceiling": eff_gbs / ceiling_gbs,
                       "speculative_k_bytes_per_step": spec_k_bytes,
                       "GBps_with_speculative_reads": (alg_bytes + spec_k_bytes) / (ms_per_step * 1e-3) / 1e9,
                       "hbm_frac_with_speculative_reads": (alg_bytes + spec_k_bytes) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "kv_reduction_vs_dense": kv_reduction,
                       "mean_selected_fraction": float((blocks_read / np.maximum(N_total, 1)).mean()),
                       "phase_avg_ms_per_layer": phase_avg,
                       "kernel_GBps": kern_gbs},
        "with_depth_hint": hinted,
        "decode_loop": loop,
        "dense_control": dense,
        "topk_control": topk,
        "scorer_comparison": scorers,
        "host_tier": tier_leg,
        "other_configs": others,
        "metadata_bulk_build": {"ms": meta_ms, "GBps": meta_bytes / (meta_ms * 1e-3) / 1e9},
    }
    for n in ("select", "attend"):
        log(f"[bench] per-layer {n} ms: " + " ".join(f"{x:.3f}" for x in per_layer[n]))
    log("[bench] per-layer blocks read, min/mean/max over the (request, KV head) pairs: " +
        " ".join(f"{int(x.min())}/{int(x.mean())}/{int(x.max())}" for x in blocks_read.reshape(L, -1)))
    log("[bench] per-layer selected fraction: " +
        " ".join(f"{x:.3f}" for x in (blocks_read / np.maximum(N_total, 1)).mean((1, 2))))
    print(json.dumps(result), flush=True)
    if parity is not None and not parity["ok"]:
        log(f"[bench] PARITY FAILED against the oracle: {parity}")
        sys.exit(3)


if __name__ == "__main__":
    main()
