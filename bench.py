#!/usr/bin/env python3
"""Benchmark of the KV offloading hot path on one MI355X.

One step = one pass of the whole path over a synthetic KV cache already resident in HBM:
  offload  (plan lookups, pack kernels, chunked D2H, page-cache-path memcpy hop) of every layer, then
  reload   (memcpy hop, chunked H2D, unpack kernels) + decode attention of every layer.
Prints one JSON line: offload+reload GB/s over the step, with the dominant kernel's roofline, the
measured host-link ceiling, decode-attention microseconds per layer and a CPU baseline (the plain
checker timed on a bounded sample of the same workload).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measure_link(torch, total_bytes: int, piece: int = 64 << 20):
    """Back-to-back pinned copies in >= 64 MiB pieces, each direction, no kernels: the host-link ceiling."""
    n = max(1, total_bytes // piece)
    host = torch.empty(piece, dtype=torch.uint8, pin_memory=True)
    host.fill_(1)
    dev = torch.empty(piece, dtype=torch.uint8, device="cuda")
    out = {}
    for name, (dst, src) in {"h2d": (dev, host), "d2h": (host, dev)}.items():
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        out[name] = n * piece / (time.perf_counter() - t0) / 1e9
    return out


def cpu_baseline(cfg, W, budget_s: float = 20.0):
    """The CPU checker (one thread, as it stands) on whole layers of the same workload until about
    budget_s seconds of its own work: pack K and V into extent images, unpack them back, one decode
    attention.  Only the checker's calls are timed, not the input generation."""
    import numpy as np
    from oracle import kv_oracle as o
    lens = W.seq_lens(cfg)
    plan = o.layout_plan(cfg.n_layers, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, lens, 2, cfg.sector_bytes,
                         cfg.extent_mode == W.PER_SEQ, cfg.pc_budget_bytes, cfg.lba_start)
    nbytes = plan.n_blocks_tensor * plan.lba_size
    moved, layers, move_s, attn_s = 0, 0, 0.0, 0.0
    for layer in range(cfg.n_layers):
        K = W.bhsd_layer(cfg, layer, 0, "cpu")
        V = W.bhsd_layer(cfg, layer, 1, "cpu")
        q = W.query(cfg, layer, "cpu")
        src = o.bhsd_source(K.shape)
        ext = np.empty(nbytes, dtype=np.uint8)
        back = np.empty_like(o.u16(K))
        t0 = time.perf_counter()
        for t in (K, V):
            o.pack(src, o.u16(t), plan.per_seq, lens, plan.seq_base, plan.n_blocks_tensor, plan.lba_size, ext)
            o.unpack(src, back, plan.per_seq, lens, plan.seq_base, plan.lba_size, ext)
            moved += 2 * nbytes  # once out, once back
        t1 = time.perf_counter()
        o.attention(src, o.u16(K), o.u16(V), o.u16(q), cfg.dtype == W.BF16, lens, cfg.n_q_heads)
        t2 = time.perf_counter()
        move_s += t1 - t0
        attn_s += t2 - t1
        layers += 1
        if (move_s + attn_s) * (layers + 1) / layers > budget_s:
            break
    total = move_s + attn_s
    return {"value": round(moved / total / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{layers} of {cfg.n_layers} layers of the same workload: pack+unpack of K and V and one decode "
                      f"attention per layer, plain C checker, 1 thread, {total:.1f} s",
            "pack_unpack_GBps": round(2 * moved / move_s / 1e9, 3),
            "decode_attn_us_per_layer": round(attn_s / layers * 1e6, 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="llama8b_32k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--host-workers", type=int, default=0)
    ap.add_argument("--span-chunks", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2604_26557_amd import binding as kv
    from paper_2604_26557_amd import workloads as W
    from kvcase import native_plan

    kv.lib()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    cfg = W.config(args.config)
    lens = W.seq_lens(cfg)
    plan = native_plan(cfg, lens)
    info = plan.info
    L = cfg.n_layers
    log(f"[bench] {cfg.name}: L={L} H={cfg.n_kv_heads} Hq={cfg.n_q_heads} D={cfg.head_dim} B={cfg.batch} "
        f"lens={lens if len(set(lens)) > 1 else lens[0]} chunk={cfg.chunk_tokens} depth={cfg.depth} "
        f"pagecache_layers={info.n_pagecache_layers}")

    # ---- synthetic KV resident in HBM (seeded N(0,1) in the config's 16-bit dtype)
    if cfg.layout == W.PAGED:
        table, n_pool = W.block_table(cfg, lens)
        table_dev = table.cuda()
        k = [W.paged_layer(cfg, l, 0, n_pool, "cuda") for l in range(L)]
        v = [W.paged_layer(cfg, l, 1, n_pool, "cuda") for l in range(L)]
        lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
        mk = lambda kk, vv: kv.paged_view(kk, vv, table_dev, lens, lens_dev)
    else:
        k = [W.bhsd_layer(cfg, l, 0, "cuda") for l in range(L)]
        v = [W.bhsd_layer(cfg, l, 1, "cuda") for l in range(L)]
        lens_dev = torch.tensor(lens, dtype=torch.int32, device="cuda")
        mk = lambda kk, vv: kv.bhsd_view(kk, vv, lens, lens_dev)
    src_view = mk(k, v)
    k2 = [torch.zeros_like(t) for t in k]
    v2 = [torch.zeros_like(t) for t in v]
    dst_view = mk(k2, v2)
    qs = [W.query(cfg, l, "cuda") for l in range(L)]
    outs = [torch.zeros((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=torch.float32, device="cuda") for _ in range(L)]

    # ---- storage model: pinned LBA region (direct path) + pageable arena (page-cache path)
    region = torch.empty(max(int(info.region_bytes_needed), 1), dtype=torch.uint8, pin_memory=True)
    region.zero_()
    arena = np.zeros(max(int(info.pageable_bytes_needed), 1), dtype=np.uint8)
    arena[::4096] = 1  # touch every page before timing
    torch.cuda.synchronize()

    payload = 2 * L * int(info.tensor_blocks) * cfg.sector_bytes  # bytes over the link per direction

    def step(timed: bool):
        a = kv.kv_pipeline_run(plan, kv.KV_DIR_OFFLOAD, 0, L, src_view, region, arena, depth=cfg.depth,
                               span_chunks=args.span_chunks, host_workers=args.host_workers, time_kernels=timed)
        b = kv.kv_pipeline_run(plan, kv.KV_DIR_RELOAD_ATTN, 0, L, dst_view, region, arena, depth=cfg.depth,
                               q_layers=qs, out_layers=outs, span_chunks=args.span_chunks,
                               host_workers=args.host_workers, time_kernels=timed)
        return a, b

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    stats = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        stats.append(step(True))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    value = 2 * payload * args.steps / elapsed / 1e9

    # round trip must be exact (cheap on-device check of the timed work's result)
    for l in (0, L - 1):
        assert torch.equal(k[l].view(torch.int16), k2[l].view(torch.int16)), "reload differs from source"
        assert torch.equal(v[l].view(torch.int16), v2[l].view(torch.int16)), "reload differs from source"

    off_s = sum(a.wall_s for a, _ in stats) / args.steps
    rel_s = sum(b.wall_s for _, b in stats) / args.steps

    def kstat(kind, which):
        ms = sum(s[which].kernel_ms[kind] for s in stats)
        n = sum(s[which].kernel_launches[kind] for s in stats)
        return (ms / n * 1e3 if n else 0.0), n  # microseconds per launch

    tensor_payload = int(info.tensor_payload_bytes)
    tensor_image = int(info.tensor_blocks) * cfg.sector_bytes
    pack_us, pack_n = kstat(kv.KV_KERNEL_PACK, 0)
    unpack_us, unpack_n = kstat(kv.KV_KERNEL_UNPACK, 1)
    attn_us, attn_n = kstat(kv.KV_KERNEL_ATTN_PARTIAL, 1)
    launches_per_tensor_pack = pack_n / (2 * L * args.steps)
    launches_per_tensor_unpack = unpack_n / (2 * L * args.steps)
    rooflines = []
    for name, us, per_launch in (
            ("kv_layout_kernel<pack>", pack_us, (tensor_payload + tensor_image) / launches_per_tensor_pack),
            ("kv_layout_kernel<unpack>", unpack_us, 2 * tensor_payload / launches_per_tensor_unpack),
            ("kv_attn_partial_kernel+combine", attn_us, 2 * tensor_payload)):
        ach = per_launch / (us * 1e-6) / 1e9 if us > 0 else 0.0
        rooflines.append({"kernel": name, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS,
                          "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None,
                          "us_per_launch": round(us, 2), "bytes_per_launch": int(per_launch)})
    totals = [pack_us * pack_n, unpack_us * unpack_n, attn_us * attn_n]
    dominant = rooflines[max(range(3), key=lambda i: totals[i])]

    link = measure_link(torch, min(payload, 2 << 30))
    off_gbps = payload / off_s / 1e9
    rel_gbps = payload / rel_s / 1e9

    # per-path throughput (outside the timed region): page-cache-path layers and direct-path layers alone
    n1 = int(info.n_pagecache_layers)
    per_path = {}
    for label, lo, hi in (("pagecache", 0, n1), ("direct", n1, L)):
        if hi > lo:
            a = kv.kv_pipeline_run(plan, kv.KV_DIR_OFFLOAD, lo, hi, src_view, region, arena, depth=cfg.depth,
                                   span_chunks=args.span_chunks, host_workers=args.host_workers)
            b = kv.kv_pipeline_run(plan, kv.KV_DIR_RELOAD, lo, hi, dst_view, region, arena, depth=cfg.depth,
                                   span_chunks=args.span_chunks, host_workers=args.host_workers)
            nb = (a.bytes_direct + a.bytes_pagecache)
            per_path[label] = {"offload_GBps": round(nb / a.wall_s / 1e9, 2), "reload_GBps": round(nb / b.wall_s / 1e9, 2),
                               "offload_frac_of_link": round(nb / a.wall_s / 1e9 / link["d2h"], 3),
                               "reload_frac_of_link": round(nb / b.wall_s / 1e9 / link["h2d"], 3)}

    # overlap: how much of everything that is not link time was hidden behind the link
    kern_s = (pack_us * pack_n + unpack_us * unpack_n + attn_us * attn_n) * 1e-6 / args.steps
    t_link = payload / (link["d2h"] * 1e9) + payload / (link["h2d"] * 1e9)
    t_pipe = off_s + rel_s
    overlap = None
    if n1 == 0 and kern_s > 0:
        overlap = round(max(0.0, min(1.0, (t_link + kern_s - t_pipe) / kern_s)), 3)

    res = {
        "metric": "KV offload+reload GB/s and decode-attn us/layer, 8B-shape KV at 32K ctx",
        "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {L} layers, {cfg.n_kv_heads} KV heads, {cfg.n_q_heads} query heads, "
                               f"head_dim {cfg.head_dim}, batch {cfg.batch}, context {max(lens)}, {cfg.dtype} K/V, "
                               f"{cfg.sector_bytes} B sectors",
                   "chunk_tokens": cfg.chunk_tokens, "depth": cfg.depth, "pagecache_layers": n1,
                   "span_chunks": args.span_chunks, "layout": cfg.layout, "extent_mode": cfg.extent_mode},
        "offload_GBps": round(off_gbps, 2), "reload_attn_GBps": round(rel_gbps, 2),
        "decode_attn_us_per_layer": round(attn_us, 2),
        "host_link": {"h2d_GBps": round(link["h2d"], 2), "d2h_GBps": round(link["d2h"], 2),
                      "offload_frac": round(off_gbps / link["d2h"], 3), "reload_frac": round(rel_gbps / link["h2d"], 3),
                      "how": "back-to-back pinned 64 MiB copies, no kernels"},
        "per_path": per_path,
        "overlap_fraction": overlap,
        "roofline": {k2_: dominant[k2_] for k2_ in ("bound", "achieved", "peak", "unit", "frac", "traffic")} | {"kernel": dominant["kernel"]},
        "rooflines": rooflines,
    }

    if not args.no_cpu_baseline and cfg.layout == W.BHSD:
        log("[bench] timing the CPU checker on a bounded sample ...")
        res["cpu_baseline"] = cpu_baseline(cfg, W)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
