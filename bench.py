#!/usr/bin/env python3
"""Benchmark of the Eigen Attention decode path on one MI355X.

Workload (the paper's Introduction example, compressed to rank 80): a Llama-2-7B-shaped
model, 32 attention layers, d_model 4096, 32 heads, d_head 128, r_k = r_v = 80, batch 16,
32768 cached tokens per sequence; all 32 layers' rank-80 bf16 K/V pools (about 172 GB) are
resident in HBM.  One step = one generated token = for every layer: fused low-rank QKV
projection + cache append, decode attention over the 32768 cached tokens, output
projection -- 32 x 3 library calls back to back on one stream.

Prints ONE JSON line.  `value` is the algorithmic HBM traffic of the whole step divided by
its duration; `roofline` is for the dominant kernel (decode attention), timed live with
events on the launch stream; `cpu_baseline` times the fp64 oracle on host cores on a
bounded sample of the same attention workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--layers", type=int, default=32, help="resident layers (32 = the full model)")
    ap.add_argument("--page-tokens", type=int, default=64)
    ap.add_argument("--n-splits", type=int, default=0, help="0 = library default")
    ap.add_argument("--no-fullrank", action="store_true", help="skip the d_h = 128 full-rank comparison")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 4 GiB device copy, so that a rocprofv3 --pmc run of this command has a "
                         "kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--cpu-streams", type=int, default=512, help="(sequence, head) streams the oracle is timed on")
    return ap.parse_args()


def traffic_from_profiles():
    """HBM bytes per decode-attention launch measured with rocprofv3 --pmc (committed summary), or None."""
    path = os.path.join(ROOT, "profiles", "decode_attn_cfg3_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_oracle_baseline(n_streams: int, n_ctx: int, r: int, d_head: int):
    """The fp64 oracle's decode attention on `n_streams` (sequence, head) streams of the bench
    workload's shape, single-threaded BLAS, host-generated inputs with the same distribution."""
    import numpy as np
    from oracle import eigen_attention as ora
    from paper_2408_05646_amd import synth
    try:
        from threadpoolctl import threadpool_limits
    except Exception:       # pragma: no cover
        threadpool_limits = None
    g = synth.rng(3, 777)
    heads = 32
    n_seq = max(1, n_streams // heads)
    # one sequence's worth of data, referenced by every sampled sequence (timing does not depend on values)
    K1 = synth.round_to_bf16(g.standard_normal((heads, n_ctx, r), dtype=np.float32)).astype(np.float64)
    V1 = synth.round_to_bf16(g.standard_normal((heads, n_ctx, r), dtype=np.float32)).astype(np.float64)
    K, V = [K1] * n_seq, [V1] * n_seq
    q = g.standard_normal((n_seq, heads, r))
    cache = ora.RankCache.from_arrays(K, V)

    def run():
        t0 = time.perf_counter()
        ora.decode_attention(q, cache, d_head)
        return time.perf_counter() - t0

    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            run()
            dt = min(run(), run())
    else:                   # pragma: no cover
        run()
        dt = min(run(), run())
    cache_bytes = n_seq * heads * n_ctx * 2 * r * 2          # what the GPU kernel would stream (bf16)
    return {"value": cache_bytes / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"{n_seq * heads} of 512 (sequence, head) streams of one layer (n={n_ctx}, r={r}), "
                      f"fp64 numpy, {dt:.2f} s; one full 32-layer step would take {dt * 512 / (n_seq * heads) * 32:.0f} s",
            "seconds": dt}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2408_05646_amd as ea
    from paper_2408_05646_amd import synth

    ea.load_library()                      # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    dev = "cuda"
    s = synth.CFG3
    L, B, n, P = args.layers, s.batch, s.n_ctx, args.page_tokens
    H, Hkv, r_k, r_v, d = s.n_heads, s.n_kv_heads, s.r_k, s.r_v, s.d_model
    desc = ea.LayerDesc(d, H, Hkv, s.d_head, r_k, r_v, ea.EA_BF16, P)
    max_pages = n // P
    pool_pages = B * max_pages
    n_qkv = H * r_k + Hkv * (r_k + r_v)

    free, _total = torch.cuda.mem_get_info()
    lay = ea.cache_layout_query(desc)
    need = L * pool_pages * (lay.k_page_elems + lay.v_page_elems) * 2
    if need + (12 << 30) > free:
        print(f"bench.py: {L} layers need {need / 2**30:.0f} GiB of HBM, only {free / 2**30:.0f} GiB free",
              file=sys.stderr)
        sys.exit(3)

    # ---- synthetic, seeded inputs, generated on the device (172 GB cannot be staged from the host).
    # Cached rank-space rows z.M + 0.05 eps.U with orthogonal M are N(0, (1 + 0.0025) I): fill the pools with that.
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED + 3)
    layers = []
    t_fill = time.perf_counter()
    for l in range(L):
        k_pool, v_pool = ea.alloc_pools(desc, pool_pages, zero=False)
        k_pool.normal_(0.0, 1.00125, generator=gen)
        v_pool.normal_(0.0, 1.00125, generator=gen)
        perm = torch.randperm(pool_pages, generator=gen, device=dev).to(torch.int32)   # pages in seeded random order
        layers.append(dict(
            k_pool=k_pool, v_pool=v_pool, page_table=perm.reshape(B, max_pages).contiguous(),
            wqkv_t=ea.pack_weight((torch.randn((n_qkv, d), generator=gen, device=dev) * d ** -0.5).to(torch.bfloat16)),
            wo_t=ea.pack_weight((torch.randn((d, H * r_v), generator=gen, device=dev) * d ** -0.5).to(torch.bfloat16)),
            x=torch.randn((B, d), generator=gen, device=dev).to(torch.bfloat16),
            y=torch.empty((B, d), dtype=torch.bfloat16, device=dev)))
    torch.cuda.synchronize()
    t_fill = time.perf_counter() - t_fill

    seq_before = torch.full((B,), n - 1, dtype=torch.int32, device=dev)    # the step appends token n-1 ...
    seq_after = torch.full((B,), n, dtype=torch.int32, device=dev)         # ... and attends over n tokens
    q_r = torch.empty((B, H, r_k), dtype=torch.float32, device=dev)
    o = torch.empty((B, H, r_v), dtype=torch.float32, device=dev)
    S = args.n_splits or ea.decode_auto_splits(desc, B, n)
    ws_bytes = ea.decode_workspace_bytes(desc, B, S)
    ws = torch.empty(max(ws_bytes // 4, 4), dtype=torch.float32, device=dev)

    def step(events=None):
        for l, lay_ in enumerate(layers):
            ea.project_qkv(desc, lay_["x"], lay_["wqkv_t"], q_r, lay_["k_pool"], lay_["v_pool"], lay_["page_table"],
                           seq_before, 1)
            if events is not None:
                events[l][0].record()
            ea.decode_attn(desc, q_r, lay_["k_pool"], lay_["v_pool"], lay_["page_table"], seq_after, o, n_splits=S,
                           ws=ws)
            if events is not None:
                events[l][1].record()
            ea.out_proj(desc, o.view(B, -1), lay_["wo_t"], lay_["y"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[[torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)] for _ in range(L)]
          for _ in range(args.steps)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for k in range(args.steps):
        step(ev[k])
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = e0.elapsed_time(e1) / args.steps
    attn_us = [a.elapsed_time(b_) * 1e3 for k in range(args.steps) for (a, b_) in ev[k]]
    attn_us_avg = sum(attn_us) / len(attn_us)

    # ---- algorithmic bytes (what the method itself must move), per layer
    cache_bytes = B * Hkv * n * (r_k + r_v) * 2
    attn_bytes = cache_bytes + B * H * r_k * 4 + B * H * r_v * 4 + B * max_pages * 4
    proj_bytes = n_qkv * d * 2 + B * d * 2 + B * H * r_k * 4 + B * Hkv * (r_k + r_v) * 2
    out_bytes = H * r_v * d * 2 + B * H * r_v * 4 + B * d * 2
    step_bytes = L * (attn_bytes + proj_bytes + out_bytes)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    attn_gbps = attn_bytes / (attn_us_avg * 1e-6) / 1e9

    result = {
        "metric": "low-rank decode attn: achieved HBM GB/s over the whole decode step (B=16, n=32k, r=80)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg3 long-context decode: Llama-2-7B-shaped, {L} layers resident, B={B}, n={n}, "
                               f"H={H}, d_h={s.d_head}, r_k=r_v={r_k}, bf16 paged cache (page {P} tokens, "
                               f"pages in random order), project_qkv + decode_attn + out_proj per layer",
                   "layers": L, "batch": B, "n_ctx": n, "r_k": r_k, "r_v": r_v, "page_tokens": P, "n_splits": S},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "us_per_step": round(ms_per_step * 1e3, 1),
        "tokens_per_s": round(B / (ms_per_step * 1e-3), 1),
        "decode_attn_us_per_layer": round(attn_us_avg, 1),
        "step_algorithmic_bytes": step_bytes,
        "fill_seconds": round(t_fill, 1), "timed_wall_seconds": round(wall, 3),
        "roofline": {"bound": "hbm", "achieved": round(attn_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(attn_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic_from_profiles(),
                     "kernel": "ea_decode_attn (split kernel + merge)", "bytes_per_launch": attn_bytes,
                     "us_per_launch": round(attn_us_avg, 2)},
    }

    # ---- the same kernel at full rank (standard attention, d_h = 128) on one layer-sized buffer
    if not args.no_fullrank:
        fdesc = ea.LayerDesc(d, H, Hkv, s.d_head, s.d_head, s.d_head, ea.EA_BF16, P)
        fk, fv = ea.alloc_pools(fdesc, pool_pages, zero=False)
        fk.normal_(generator=gen); fv.normal_(generator=gen)
        fq = torch.randn((B, H, s.d_head), generator=gen, device=dev)
        fo = torch.empty((B, H, s.d_head), dtype=torch.float32, device=dev)
        fS = args.n_splits or ea.decode_auto_splits(fdesc, B, n)
        fws = torch.empty(max(ea.decode_workspace_bytes(fdesc, B, fS) // 4, 4), dtype=torch.float32, device=dev)
        pt = layers[0]["page_table"]
        for _ in range(3):
            ea.decode_attn(fdesc, fq, fk, fv, pt, seq_after, fo, n_splits=fS, ws=fws)
        torch.cuda.synchronize()
        f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 16
        f0.record()
        for _ in range(reps):
            ea.decode_attn(fdesc, fq, fk, fv, pt, seq_after, fo, n_splits=fS, ws=fws)
        f1.record()
        torch.cuda.synchronize()
        full_us = f0.elapsed_time(f1) * 1e3 / reps
        full_bytes = B * Hkv * n * 2 * s.d_head * 2
        result["fullrank_baseline"] = {
            "decode_attn_us_per_layer": round(full_us, 1), "achieved_GBps": round(full_bytes / full_us / 1e3, 1),
            "latency_ratio_lowrank_over_fullrank": round(attn_us_avg / full_us, 4),
            "ratio_predicted_by_rank": round(r_k / s.d_head, 4),
            "note": "same kernel, r_k = r_v = d_h = 128, same B, n and page table, one 8.6 GB layer buffer"}
        del fk, fv

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.float32, device=dev).normal_(generator=gen)     # 4 GiB
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["calibration_copy_bytes_each_way"] = src.numel() * 4

    if not args.no_cpu:
        result["cpu_baseline"] = cpu_oracle_baseline(args.cpu_streams, n, r_k, s.d_head)

    print(json.dumps(result))


if __name__ == "__main__":
    main()
