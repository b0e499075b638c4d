#!/usr/bin/env python3
"""Benchmark of the Eigen Attention hot path on one MI355X.

Default workload (`--workload cfg3`, the headline): the paper's Introduction example compressed to
rank 80 -- a Llama-2-7B-shaped model, 32 attention layers, d_model 4096, 32 heads, d_head 128,
r_k = r_v = 80, batch 16, 32768 cached tokens per sequence; all 32 layers' rank-80 bf16 K/V pools
(about 172 GB) are resident in HBM.  One step = one generated token = for every layer: fused low-rank
QKV projection + cache append, decode attention over the 32768 cached tokens, output projection --
32 x 3 library calls back to back on one stream.

Other workloads (same step, other shapes): `cfg2` (n = 4096), `cfg5` (grouped-query attention, 32 query
heads on 8 kv heads, B = 8, n = 16384, per-layer ranks drawn from {48,...,112}); `cfg4` is the causal
prefill of B = 4 sequences of 8192 tokens at r = 64 (project_qkv + prefill_attn + out_proj of one layer).
`cfgN-rope` is the variant for models with rotary positions (Sec. 4.3); `cfgN-q4` keeps all pages but the newest
of every sequence in the 4-bit group-quantised form the paper combines the method with (quantisation paragraph
of the results) and attends with ea_decode_attn_q4.

Prints ONE JSON line.  `value` is the algorithmic HBM traffic of the whole step divided by its duration
(decode workloads) or the step's TFLOP/s (prefill); `roofline` is for the dominant kernel, timed live
with events on the launch stream; `cpu_baseline` times the fp64 oracle on host cores on a bounded sample.
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
ROPE_BASE = 10000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# The paper's own figures (other hardware, whole PyTorch / Hugging Face models): context, not the target.
PAPER_CONTEXT = {
    "kv_cache_reduction": "up to 40 % (cache at 0.6x) across OPT, MPT and Llama models (abstract)",
    "attention_latency": "average latency per attention layer during generation, 2x NVIDIA A100-80GB, 2048-token "
                         "prompt, 128 generated tokens, KV cache at 0.6x (latency table): OPT-66b 1.57 -> 0.62 ms "
                         "(-60 %), Llama-2-70b 0.79 -> 0.77 ms (-3 %), Llama-3-70b 0.74 -> 0.80 ms (+8 %, RoPE variant)",
    "memory_example": "Llama-2-7B, batch 16, 32k tokens, 16 bit: 14 GB of weights, 256 GB of KV cache (Introduction); "
                      "at rank 80 of 128 the cache is 160 GiB",
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--q4-key-group", type=int, default=64, choices=[64, 128],
                    help="-q4 workloads: tokens that share a key scale (128 needs --page-tokens 128 or more)")
    ap.add_argument("--q4-bits", type=int, default=4, choices=[4, 3], help="-q4 workloads: width of a code")
    ap.add_argument("--workload", default="cfg3", choices=["cfg2", "cfg3", "cfg4", "cfg5", "cfg3-rope", "cfg5-rope", "cfg4-rope", "cfg2-q4", "cfg3-q4",
                             "cfg5-q4", "cfg3-rope-q4", "cfg2-h2o", "cfg3-h2o", "cfg2-rope-h2o", "cfg3-rope-h2o", "cfg4-q4"])
    ap.add_argument("--prefill-chunk", type=int, default=2048,
                    help="cfg4-q4: tokens per sequence that are prefilled (and then quantised) at a time")
    ap.add_argument("--q4-staged", action="store_true",
                    help="cfg4-q4: attend through ea_prefill_attn_q4_staged (codes dequantised into 16-bit stage pools "
                         "inside the workspace, then the 16-bit prefill kernel) instead of ea_prefill_attn_q4")
    ap.add_argument("--layers", type=int, default=32, help="resident layers (32 = the full model)")
    ap.add_argument("--page-tokens", type=int, default=64)
    ap.add_argument("--n-splits", type=int, default=0, help="0 = library default")
    ap.add_argument("--no-fullrank", action="store_true", help="skip the d_h = 128 full-rank comparison")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-graph", action="store_true", help="skip the extra timing of the step replayed as a HIP graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 4 GiB device copy, so that a rocprofv3 --pmc run of this command has a "
                         "kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--cpu-streams", type=int, default=64,
                    help="(sequence, kv head) streams of the first layer copied back for the oracle timing")
    ap.add_argument("--no-parity", action="store_true", help="skip the oracle check of the timed step")
    ap.add_argument("--parity-samples", type=int, default=64,
                    help="(layer, sequence, kv head) triples of the timed step compared with the oracle")
    return ap.parse_args()


def source_stamp(files=None) -> str:
    """First 16 hex digits of the SHA-256 over library sources (names and contents, in sorted order): the named
    files of csrc/ and include/, or all of them.  A committed profile summary lists the sources of the kernels it
    measured and carries their stamp, so that a figure taken from it can be told apart from one that no longer
    belongs to the kernels being timed."""
    import hashlib
    h = hashlib.sha256()
    found = {}
    for d in (os.path.join(ROOT, "paper_2408_05646_amd", "csrc"), os.path.join(ROOT, "include")):
        for name in os.listdir(d):
            if name.endswith((".hip", ".h")):
                found[name] = os.path.join(d, name)
    names = sorted(found) if files is None else sorted(files)
    for name in names:
        h.update(name.encode())
        h.update(open(found[name], "rb").read() if name in found else b"<missing>")
    return h.hexdigest()[:16]


def traffic_from_profiles(workload: str):
    """(HBM bytes per decode-attention launch measured with rocprofv3 --pmc, where that figure comes from), read
    from the committed summary of that measurement; (None, None) if there is none for this workload.  The
    counters cannot be read from inside this process, so the figure is only as fresh as its file: the summary
    names the kernel sources it was measured on and carries their stamp, and `stale` says whether they have
    changed since."""
    name = {"cfg3": "decode_attn_cfg3_hbm_traffic.txt", "cfg3-rope": "decode_attn_rope_cfg3_hbm_traffic.txt",
            "cfg3-q4": "decode_attn_q4_cfg3_hbm_traffic.txt", "cfg3-q4-3bit": "decode_attn_q3_cfg3_hbm_traffic.txt",
            "cfg3-h2o": "decode_attn_mass_cfg3_hbm_traffic.txt",
            "cfg2": "decode_attn_cfg2_hbm_traffic.txt", "cfg5": "decode_attn_cfg5_hbm_traffic.txt",
            "cfg3-rope-h2o": "decode_attn_mass_rope_pos_cfg3_hbm_traffic.txt"}.get(workload)
    if name is None:
        return None, None
    path = os.path.join(ROOT, "profiles", name)
    traffic, stamp, files = None, None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
            if line.startswith("kernel_sources:"):
                files = line.split(":")[1].split()
            if line.startswith("kernel_sources_sha16:"):
                stamp = line.split(":")[1].strip()
    except OSError:
        return None, None
    if traffic is None:
        return None, None
    now = source_stamp(files)
    return traffic, {"file": "profiles/" + name, "kernel_sources": files, "measured_on_sources": stamp,
                     "sources_now": now, "stale": stamp != now}


def _timed_single_thread(fn):
    try:
        from threadpoolctl import threadpool_limits
    except Exception:       # pragma: no cover
        threadpool_limits = None

    def run():
        t0 = time.perf_counter()
        fn()
        return time.perf_counter() - t0

    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            run()
            return min(run(), run())
    run()                   # pragma: no cover
    return min(run(), run())


def usable_cores() -> int:
    """Host cores this process may use for the oracle timing: its affinity mask, capped by the thread count the
    environment grants (OMP_NUM_THREADS on a shared box)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:      # pragma: no cover
        n = os.cpu_count() or 1
    cap = os.environ.get("OMP_NUM_THREADS", "")
    if cap.isdigit() and int(cap) > 0:
        n = min(n, int(cap))
    return max(1, n)


def oracle_worker_main(path: str, d_head: int, rope_base: float, reps: int) -> None:
    """One host core's share of the all-core oracle timing; runs in a fresh process of its own
    (`bench.py --oracle-worker ...`): loads its streams, says "ready", waits for "go" on stdin, runs the fp64
    oracle's decode attention over its streams `reps` times (single-threaded BLAS), prints the seconds it took."""
    import numpy as np
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)
    except Exception:       # pragma: no cover
        limiter = None
    from oracle import eigen_attention as ora
    from paper_2408_05646_amd import synth
    z = np.load(path)
    K = synth.bf16_bits_to_f32(z["k"]).astype(np.float64)          # [streams, n, r_k]
    V = synth.bf16_bits_to_f32(z["v"]).astype(np.float64)
    q = z["q"].astype(np.float64)                                  # [streams, G, q_dim]
    U = z["u"].astype(np.float64) if "u" in z.files else None
    caches = [ora.RankCache.from_arrays([K[i][None]], [V[i][None]]) for i in range(K.shape[0])]
    print("ready", flush=True)
    if sys.stdin.readline().strip() != "go":
        return
    t0 = time.perf_counter()
    for _ in range(reps):
        for i, c in enumerate(caches):
            if U is None:
                ora.decode_attention(q[i][None], c, d_head)
            else:
                ora.decode_attention_rope(q[i][None], c, U, d_head, rope_base)
    print(f"done {time.perf_counter() - t0:.6f}", flush=True)
    del limiter


def cpu_oracle_decode(streams, d_head, rope_u=None, h2o=False, positions=None):
    """The fp64 oracle's decode attention timed on host cores, on cache slices copied back from the device.
    `streams` = list of (K bits [n, r_k] uint16, V bits [n, r_v] uint16, q [G, q_dim] float32): the bfloat16 contents
    of (sequence, kv head) streams of the first resident layer, exactly as the GPU kernel reads them.  Timed twice:
    on one core, and on every core this process may use (one fresh single-threaded process per core over disjoint
    streams).  positions (rotary + h2o: the cache of a pruned sequence) = list, per stream, of (position of the token
    in every slot [n], position of the query)."""
    import tempfile

    import numpy as np
    from oracle import eigen_attention as ora
    from paper_2408_05646_amd import synth
    if h2o:
        from oracle import eviction as oe
    n_ctx, r_k = streams[0][0].shape
    r_v = streams[0][1].shape[1]
    G = streams[0][2].shape[0]
    bytes_per_stream = n_ctx * (r_k + r_v) * 2                     # what the GPU kernel streams for it (bf16)
    U = None if rope_u is None else rope_u.astype(np.float64)

    # ---- one core
    caches = [ora.RankCache.from_arrays([synth.bf16_bits_to_f32(k).astype(np.float64)[None]],
                                        [synth.bf16_bits_to_f32(v).astype(np.float64)[None]]) for k, v, _ in streams]
    qs = [q.astype(np.float64)[None] for _, _, q in streams]

    def one_pass():
        for i, (c, q) in enumerate(zip(caches, qs)):
            if positions is not None:
                oe.attention_mass_rope_positions(q, [positions[i][1]], c, [positions[i][0]], U, d_head, ROPE_BASE)
                oe.decode_attention_rope_positions(q, [positions[i][1]], c, [positions[i][0]], U, d_head, ROPE_BASE)
            elif U is None:
                ora.decode_attention(q, c, d_head)
                if h2o:
                    oe.attention_mass(q, c, d_head)
            else:
                ora.decode_attention_rope(q, c, U, d_head, ROPE_BASE)

    t_probe = _timed_single_thread(one_pass)
    reps1 = max(1, int(round(2.0 / max(t_probe, 1e-4))))           # about two seconds per timing

    def work():
        for _ in range(reps1):
            one_pass()

    dt1 = _timed_single_thread(work) / reps1
    single = len(streams) * bytes_per_stream / dt1 / 1e9
    del caches

    # ---- all cores: one fresh process per core, each with its own share of the streams
    cores = min(usable_cores(), len(streams))
    multi, dt_all, reps_all = None, None, None
    note = None
    if cores > 1 and not h2o:
        import subprocess
        tmp = tempfile.mkdtemp(prefix="ea_oracle_", dir="/dev/shm" if os.path.isdir("/dev/shm") else None)
        shares = [streams[i::cores] for i in range(cores)]
        per_worker = max(len(sh) for sh in shares)
        reps_all = max(1, int(round(3.0 / max(dt1 / len(streams) * per_worker, 1e-4))))      # about three seconds
        procs = []
        try:
            for i, sh in enumerate(shares):
                path = os.path.join(tmp, f"share{i}.npz")
                arrays = dict(k=np.stack([k for k, _, _ in sh]), v=np.stack([v for _, v, _ in sh]),
                              q=np.stack([q for _, _, q in sh]))
                if U is not None:
                    arrays["u"] = U
                np.savez(path, **arrays)
                procs.append(subprocess.Popen(
                    [sys.executable, "-u", os.path.abspath(__file__), "--oracle-worker", path, str(d_head),
                     repr(ROPE_BASE), str(reps_all)], stdin=subprocess.PIPE, stdout=subprocess.PIPE, text=True, cwd=ROOT))
            if all(pr.stdout.readline().strip() == "ready" for pr in procs):     # every worker holds its data in fp64
                t0 = time.perf_counter()
                for pr in procs:
                    pr.stdin.write("go\n")
                    pr.stdin.flush()
                done = [pr.stdout.readline().split() for pr in procs]
                dt_wall = time.perf_counter() - t0
                if all(len(dn) == 2 and dn[0] == "done" for dn in done):
                    dt_all = dt_wall / reps_all
                    multi = sum(len(sh) for sh in shares) * bytes_per_stream / dt_all / 1e9
                else:
                    note = "an oracle worker process ended early: all-core figure not available"
            else:
                note = "an oracle worker process did not start: all-core figure not available"
        finally:
            for pr in procs:
                try:
                    pr.stdin.close()
                    pr.wait(timeout=30)
                except Exception:
                    pr.kill()
            for f in os.listdir(tmp):
                os.remove(os.path.join(tmp, f))
            os.rmdir(tmp)
    what = ("rotary " if U is not None else "") + "decode attention" + \
        (" and attention mass per cached token" if h2o else "") + \
        (" over a pruned cache (explicit positions)" if positions is not None else "")
    res = {"value": round(multi if multi is not None else single, 3), "unit": "GB/s",
           "cores": cores if multi is not None else 1, "kind": "oracle",
           "sample": f"{what} of {len(streams)} (sequence, kv head) streams of the first resident layer (n={n_ctx}, "
                     f"r_k={r_k}, r_v={r_v}, {G} query head(s) each), their bfloat16 cache slices and the step's queries "
                     f"copied back from the device; fp64 numpy; GB/s = the bf16 bytes the GPU kernel streams for these "
                     f"streams per second of oracle time",
           "single_core": {"value": round(single, 3), "unit": "GB/s", "cores": 1,
                           "seconds_per_pass": round(dt1, 4), "passes_timed": reps1},
           "seconds": round(dt_all if dt_all is not None else dt1, 4)}
    if note:
        res["note"] = note
    if multi is not None:
        res["all_cores"] = {"value": round(multi, 3), "unit": "GB/s", "cores": cores,
                            "seconds_per_pass": round(dt_all, 4), "passes_timed": reps_all,
                            "how": "one fresh single-threaded process per core over disjoint streams, started "
                                   "together, timed from the common start to the last one's end"}
    return res


def cpu_oracle_decode_q4(n_streams: int, n_ctx: int, r: int, d_head: int, page_tokens: int, rope: bool = False,
                         key_group: int = 64, bits: int = 4):
    """The oracle of the quantised-cache step on `n_streams` (sequence, head) streams: codes and scales are
    prepared outside the timed region (they are the cache's content); timed is what a generation step does with
    them, dequantisation of the 4-bit part and fp64 attention over it and the 16-bit newest page."""
    import numpy as np
    from oracle import eigen_attention as ora
    from oracle import quant_cache as oq
    from paper_2408_05646_amd import synth
    g = synth.rng(3, 778)
    heads = 32
    n_seq = max(1, n_streams // heads)
    nq = n_ctx - page_tokens
    K1 = synth.round_to_bf16(g.standard_normal((heads, n_ctx, r), dtype=np.float32)).astype(np.float64)
    V1 = synth.round_to_bf16(g.standard_normal((heads, n_ctx, r), dtype=np.float32)).astype(np.float64)
    kq = [oq.quantize_keys(K1[h, :nq], key_group, bits) for h in range(heads)]
    vq = [oq.quantize_values(V1[h, :nq], bits) for h in range(heads)]
    q = g.standard_normal((n_seq, heads, d_head if rope else r))
    U = synth.orthonormal_basis(g, d_head, r) if rope else None

    def work():
        Kd = np.stack([np.concatenate([oq.dequantize_keys(*kq[h]), K1[h, nq:]]) for h in range(heads)])
        Vd = np.stack([np.concatenate([oq.dequantize_values(*vq[h]), V1[h, nq:]]) for h in range(heads)])
        cache = ora.RankCache.from_arrays([Kd] * n_seq, [Vd] * n_seq)
        if rope:
            ora.decode_attention_rope(q, cache, U, d_head, ROPE_BASE)
        else:
            ora.decode_attention(q, cache, d_head)

    dt = _timed_single_thread(work)
    tiles = nq // 64
    cache_bytes = n_seq * heads * (tiles * (2 * 8 * bits * ((r + 15) // 16 * 16) + 128 * ((r + 31) // 32) * 64 // key_group + 256)
                                   + page_tokens * 2 * r * 2)      # what the GPU kernels would stream
    return {"value": round(cache_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": f"dequantisation and {'rotary ' if rope else ''}decode attention of {n_seq * heads} of one layer's 512 (sequence, head) "
                      f"streams (n={n_ctx}, r={r}, all but the last {page_tokens} tokens in 4 bits), fp64 numpy, "
                      f"{dt:.2f} s per pass, timed three times (best kept)",
            "seconds": round(dt, 3)}


def cpu_oracle_prefill(n_rows: int, n_ctx: int, r: int, d_head: int):
    """The fp64 oracle's causal attention for the last `n_rows` query rows of one (sequence, head)."""
    from oracle import eigen_attention as ora
    from paper_2408_05646_amd import synth
    g = synth.rng(4, 777)
    K = g.standard_normal((1, n_ctx, r))
    V = g.standard_normal((1, n_ctx, r))
    q = g.standard_normal((1, n_rows, 1, r))
    cache = ora.RankCache.from_arrays([K], [V])
    dt = _timed_single_thread(lambda: ora.prefill_attention(q, cache, d_head))
    flops = sum(2 * (n_ctx - n_rows + j + 1) * 2 * r for j in range(n_rows))
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
            "sample": f"causal attention of the last {n_rows} query rows of one (sequence, head) of the workload "
                      f"(n={n_ctx}, r={r}), fp64 numpy, {dt:.2f} s",
            "seconds": round(dt, 3)}


# ---- the bf16 cache layout, undone on the host (index arithmetic from the header's description of the layout):
# what the oracle is handed never passes through the library
def _k_tiles_to_rows(tiles, r_pad):
    """[n_tiles, 64 * r_pad] K tiles -> [n_tiles * 64, r_pad]; a tile is [4 blocks][r_pad/8 chunks][16 tokens][8 channels]."""
    t = tiles.reshape(-1, 4, r_pad // 8, 16, 8)
    return t.transpose(0, 1, 3, 2, 4).reshape(-1, r_pad)


def _v_tiles_to_rows(tiles, r_pad):
    """V tile = [2 groups][r_pad/16 blocks][4 quads][16 channels][8 slots], slot j of quad q = token 16*(j/4) + 4*q + j%4."""
    t = tiles.reshape(-1, 2, r_pad // 16, 4, 16, 2, 4)            # tile, group, block, quad, channel, j/4, j%4
    return t.transpose(0, 1, 5, 3, 6, 2, 4).reshape(-1, r_pad)


def _stream_bits(torch, pool, page_table_row, head, n_kv_heads, r, r_pad, rows_fn, page_tokens, n):
    """bfloat16 bit patterns [n, r] (uint16) of one (sequence, kv head) stream, read from raw pool memory."""
    slab = page_tokens * r_pad
    view = pool.view(torch.int16).view(pool.shape[0], n_kv_heads, slab)
    got = view[page_table_row.long(), head].cpu().numpy().view("uint16")        # [pages, slab]
    return rows_fn(got.reshape(-1, 64 * r_pad), r_pad)[:n, :r].copy()


def check_step_parity(torch, ea, synth, layers, s, B, n, P, rope, n_samples, seed, slot_pos=None, q_pos=None):
    """The resident step that was just timed, against the fp64 oracle: sampled (layer, sequence, kv head) triples
    spread over all layers for the attention (cache slices and the step's own queries copied back from the device),
    and, for the first and last layer, the projection (queries of all heads, the appended key and value rows of the
    sampled heads) and the output projection (all of y)."""
    import numpy as np
    from oracle import eigen_attention as ora
    L, H, Hkv, d_h = len(layers), s.n_heads, s.n_kv_heads, s.d_head
    G = H // Hkv
    g = synth.rng(33, seed)
    triples = [(0, 0, 0), (L - 1, B - 1, Hkv - 1)]
    while len(triples) < n_samples:
        li = (len(triples) - 2) % L
        triples.append((li, int(g.integers(B)), int(g.integers(Hkv))))
    worst, where, errs = 0.0, None, []
    streams0 = {}
    for li, b, kvh in triples:
        l = layers[li]
        dc = l["desc"]
        lay = ea.cache_layout_query(dc)
        Kb = _stream_bits(torch, l["k_pool"], l["page_table"][b], kvh, Hkv, dc.r_k, lay.r_k_pad, _k_tiles_to_rows, P, n)
        Vb = _stream_bits(torch, l["v_pool"], l["page_table"][b], kvh, Hkv, dc.r_v, lay.r_v_pad, _v_tiles_to_rows, P, n)
        heads = list(range(kvh * G, (kvh + 1) * G))
        q = l["q_r"][b, heads].cpu().numpy()
        if li == 0:
            streams0[(b, kvh)] = (Kb, Vb, q)
        cache = ora.RankCache.from_arrays([synth.bf16_bits_to_f32(Kb).astype(np.float64)[None]],
                                          [synth.bf16_bits_to_f32(Vb).astype(np.float64)[None]])
        if rope and slot_pos is not None:
            from oracle import eviction as oe
            ref = oe.decode_attention_rope_positions(q[None].astype(np.float64), [int(q_pos[b])], cache,
                                                     [slot_pos[b, :n].cpu().numpy()], l["u_k"].float().cpu().numpy(),
                                                     d_h, ROPE_BASE)
        elif rope:
            ref = ora.decode_attention_rope(q[None].astype(np.float64), cache, l["u_k"].float().cpu().numpy(), d_h,
                                            ROPE_BASE)
        else:
            ref = ora.decode_attention(q[None].astype(np.float64), cache, d_h)
        got = l["o"][b, heads].cpu().numpy()[None]
        if not np.isfinite(got).all():
            return {"samples": len(errs), "worst_rel_l2": float("inf"), "where": f"non-finite output, layer {li}"}, streams0
        e = ora.rel_l2(got, ref)
        errs.append(e)
        if e > worst:
            worst, where = e, f"layer {li}, sequence {b}, kv head {kvh}"
    res = {"samples": len(errs), "worst_rel_l2": float(f"{worst:.3e}"), "mean_rel_l2": float(f"{np.mean(errs):.3e}"),
           "where_worst": where, "bar": 1e-2,
           "what": "decode attention outputs of the timed resident step vs the fp64 oracle on the same bfloat16 "
                   "cache slices and queries (copied back from the device), sampled over all resident layers"}
    # ---- first and last layer: projection + append + output projection of the same step
    proj = {}
    for li in sorted({0, L - 1}):
        l = layers[li]
        if "wqkv_raw" not in l:
            continue
        dc = l["desc"]
        q_dim = d_h if rope else dc.r_k
        x = l["x"].float().cpu().numpy().astype(np.float64)
        w = l["wqkv_raw"].float().cpu().numpy().astype(np.float64)                  # [N_qkv, d], out-major
        nq, nk = H * q_dim, Hkv * dc.r_k
        Wq = [w[i * q_dim:(i + 1) * q_dim].T for i in range(H)]
        Wk = [w[nq + i * dc.r_k:nq + (i + 1) * dc.r_k].T for i in range(Hkv)]
        Wv = [w[nq + nk + i * dc.r_v:nq + nk + (i + 1) * dc.r_v].T for i in range(Hkv)]
        q_ref, k_ref, v_ref = ora.project_qkv(x, Wq, Wk, Wv)
        e_q = ora.rel_l2(l["q_r"].cpu().numpy(), q_ref)
        lay = ea.cache_layout_query(dc)
        e_kv = 0.0
        for b, kvh in ((0, 0), (B - 1, Hkv - 1)):
            Kb = _stream_bits(torch, l["k_pool"], l["page_table"][b], kvh, Hkv, dc.r_k, lay.r_k_pad, _k_tiles_to_rows, P, n)
            Vb = _stream_bits(torch, l["v_pool"], l["page_table"][b], kvh, Hkv, dc.r_v, lay.r_v_pad, _v_tiles_to_rows, P, n)
            e_kv = max(e_kv, ora.rel_l2(synth.bf16_bits_to_f32(Kb[n - 1]), k_ref[b, kvh]),
                       ora.rel_l2(synth.bf16_bits_to_f32(Vb[n - 1]), v_ref[b, kvh]))
        wo = l["wo_raw"].float().cpu().numpy().astype(np.float64)                   # [d, H * r_v], out-major
        Wo = np.stack([wo[:, i * dc.r_v:(i + 1) * dc.r_v].T for i in range(H)])
        y_ref = ora.out_proj(l["o"].cpu().numpy().astype(np.float64), Wo)
        e_y = ora.rel_l2(l["y"].float().cpu().numpy(), y_ref)
        proj[f"layer_{li}"] = {"q_rel_l2": float(f"{e_q:.3e}"), "appended_kv_rel_l2": float(f"{e_kv:.3e}"),
                               "y_rel_l2": float(f"{e_y:.3e}")}
        worst = max(worst, e_q, e_kv, e_y)
    res["projections"] = proj
    res["worst_rel_l2"] = float(f"{worst:.3e}")
    res["ok"] = bool(np.isfinite(worst) and worst <= 1e-2)
    return res, streams0


def check_step_parity_q4(torch, ea, synth, layers, s, B, n, P, rope, n_samples, seed, bits, key_group):
    """The timed step over the group-quantised cache against the fp64 oracle: for sampled (layer, sequence, kv head)
    triples the codes, scales and zeros of the stream are gathered from raw pool memory at the positions the
    library's host reference functions give (ea_q4_*_pos / ea_q3_*_pos), dequantised by the oracle, joined with the
    bfloat16 newest page, and attended by the oracle with the step's own queries."""
    import numpy as np
    from oracle import eigen_attention as ora
    from oracle import quant_cache as oq
    L, H, Hkv, d_h = len(layers), s.n_heads, s.n_kv_heads, s.d_head
    G = H // Hkv
    g = synth.rng(34, seed)
    triples = [(0, 0, 0), (L - 1, B - 1, Hkv - 1)]
    while len(triples) < n_samples:
        triples.append(((len(triples) - 2) % L, int(g.integers(B)), int(g.integers(Hkv))))
    n_q = n - P                                   # tokens held as codes; the newest page is bfloat16
    pages_q = n_q // P
    pos_cache = {}

    def positions(dc, kvh):
        """Bit offsets of the codes and byte offsets of the scales of one (page 0, kv head) tile run: [P, r] each."""
        key = (dc.r_k, dc.r_v, kvh)
        if key not in pos_cache:
            out = {}
            for name, r, code_pos3, code_pos4, scale_pos in (
                    ("k", dc.r_k, ea.q3_k_code_pos, ea.q4_k_code_pos, lambda t, c: ea.q4_k_scale_pos(dc, 0, kvh, t, c)),
                    ("v", dc.r_v, ea.q3_v_code_pos, ea.q4_v_code_pos, lambda t, c: ea.q4_v_scale_pos(dc, 0, kvh, t))):
                cp = np.zeros((bits if bits == 3 else 1, P, r), np.int64)
                sp = np.zeros((P, r), np.int64)
                for t in range(P):
                    for c in range(r):
                        if bits == 3:
                            cp[:, t, c] = code_pos3(dc, 0, kvh, t, c)
                        else:
                            cp[0, t, c] = code_pos4(dc, 0, kvh, t, c)
                        sp[t, c] = scale_pos(t, c)
                assert (cp >= 0).all() and (sp >= 0).all()
                out[name] = (cp, sp)
            pos_cache[key] = out
        return pos_cache[key]

    def gather(pool, page_ids, cp, sp, zero_off):
        """codes uint8 [pages * P, r], scale and zero fp16 [pages * P, r] of the pages, from raw pool bytes."""
        flat = pool.reshape(-1)
        base = (page_ids.long() * pool.shape[1])[:, None, None]                       # byte offset of each page
        codes = torch.zeros((page_ids.numel(),) + cp.shape[1:], dtype=torch.uint8, device=pool.device)
        for bit in range(cp.shape[0]):
            cpt = torch.from_numpy(cp[bit]).to(pool.device)
            byte = flat[(base + cpt[None] // 8).reshape(-1)].reshape(codes.shape)
            sh = (cpt % 8).to(torch.uint8)[None]
            if cp.shape[0] == 1:
                codes = (byte >> sh) & 15
            else:
                codes |= ((byte >> sh) & 1) << bit
        spt = torch.from_numpy(sp).to(pool.device)
        half = flat.view(torch.float16)

        def halves(off):
            return half[((base + spt[None] + off) // 2).reshape(-1)].reshape(codes.shape).cpu().numpy()

        r = cp.shape[2]
        return codes.reshape(-1, r).cpu().numpy(), halves(0).reshape(-1, r), halves(zero_off).reshape(-1, r)

    worst, where, errs = 0.0, None, []
    for li, b, kvh in triples:
        l = layers[li]
        dc = l["desc"]
        lay = ea.cache_layout_query(dc)
        pos = positions(dc, kvh)
        pids = l["page_table"][b, :pages_q]
        kc, ks, kz = gather(l["kq_pool"], pids, *pos["k"], 16)
        vc, vs, vz = gather(l["vq_pool"], pids, *pos["v"], 128)
        # one key scale per channel and group of `key_group` tokens (every token of a group names the same one), one
        # value scale per token (every channel names the same one)
        assert (ks.reshape(-1, key_group, dc.r_k) == ks.reshape(-1, key_group, dc.r_k)[:, :1]).all()
        Kq = oq.dequantize_keys(kc, ks[::key_group], kz[::key_group])
        Vq = oq.dequantize_values(vc, vs[:, 0], vz[:, 0])
        Kt = _stream_bits(torch, l["k_pool"], l["tail_table"][b], kvh, Hkv, dc.r_k, lay.r_k_pad, _k_tiles_to_rows, P, P)
        Vt = _stream_bits(torch, l["v_pool"], l["tail_table"][b], kvh, Hkv, dc.r_v, lay.r_v_pad, _v_tiles_to_rows, P, P)
        K = np.concatenate([Kq, synth.bf16_bits_to_f32(Kt).astype(np.float64)])
        V = np.concatenate([Vq, synth.bf16_bits_to_f32(Vt).astype(np.float64)])
        cache = ora.RankCache.from_arrays([K[None]], [V[None]])
        heads = list(range(kvh * G, (kvh + 1) * G))
        q = l["q_r"][b, heads].cpu().numpy()[None].astype(np.float64)
        if rope:
            ref = ora.decode_attention_rope(q, cache, l["u_k"].float().cpu().numpy(), d_h, ROPE_BASE)
        else:
            ref = ora.decode_attention(q, cache, d_h)
        got = l["o"][b, heads].cpu().numpy()[None]
        if not np.isfinite(got).all():
            return {"samples": len(errs), "worst_rel_l2": float("inf"), "ok": False,
                    "where": f"non-finite output, layer {li}"}
        e = ora.rel_l2(got, ref)
        errs.append(e)
        if e > worst:
            worst, where = e, f"layer {li}, sequence {b}, kv head {kvh}"
    return {"samples": len(errs), "worst_rel_l2": float(f"{worst:.3e}"), "mean_rel_l2": float(f"{np.mean(errs):.3e}"),
            "where_worst": where, "bar": 1e-2, "ok": bool(np.isfinite(worst) and worst <= 1e-2),
            "what": f"decode attention outputs of the timed resident step over the {bits}-bit cache vs the fp64 oracle: "
                    "codes, scales and zeros gathered from raw pool memory at the positions the host reference "
                    "functions give, dequantised by the oracle, joined with the bfloat16 newest page; the step's own "
                    "queries; sampled over all resident layers"}


def bench_decode(args, torch, ea, synth):
    dev = "cuda"
    base_name, rope = args.workload.split("-")[0], "-rope" in args.workload
    q4 = args.workload.endswith("-q4")       # all pages but the newest of every sequence held in 4 bits
    h2o = args.workload.endswith("-h2o")     # the step also accumulates the attention mass every cached token receives
    pruned = rope and h2o                    # rotary + eviction: every cache slot carries the position its token had
    s = {"cfg2": synth.CFG2, "cfg3": synth.CFG3, "cfg5": synth.CFG5}[base_name]
    L, B, n, P = args.layers, s.batch, s.n_ctx, args.page_tokens
    H, Hkv, d = s.n_heads, s.n_kv_heads, s.d_model
    ranks = synth.cfg5_layer_ranks(L) if base_name == "cfg5" else tuple((s.r_k, s.r_v) for _ in range(L))
    descs = [ea.LayerDesc(d, H, Hkv, s.d_head, rk, rv, ea.EA_BF16, P, args.q4_key_group if q4 else 0,
                          args.q4_bits if q4 else 0) for rk, rv in ranks]
    max_pages = n // P
    pool_pages = B * max_pages

    free, _total = torch.cuda.mem_get_info()
    if q4:
        need = sum(pool_pages * (ea.q4_layout_query(dc).k_page_bytes + ea.q4_layout_query(dc).v_page_bytes)
                   for dc in descs)
    else:
        need = sum(pool_pages * (ea.cache_layout_query(dc).k_page_elems + ea.cache_layout_query(dc).v_page_elems) * 2
                   for dc in descs)
    if need + (12 << 30) > free:
        print(f"bench.py: {L} layers need {need / 2**30:.0f} GiB of HBM, only {free / 2**30:.0f} GiB free",
              file=sys.stderr)
        sys.exit(3)

    # ---- synthetic, seeded inputs, generated on the device (172 GB cannot be staged from the host).
    # Cached rank-space rows z.M + 0.05 eps.U with orthogonal M are N(0, (1 + 0.0025) I): fill the pools with that.
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED + int(base_name[-1]))
    layers = []
    t_fill = time.perf_counter()
    for li, dc in enumerate(descs):
        q_dim = s.d_head if rope else dc.r_k          # the rotary variant keeps the query at full rank (Sec. 4.3)
        n_qkv = H * q_dim + Hkv * (dc.r_k + dc.r_v)
        extra = {}
        if q4:
            # The first n - P tokens of every sequence are in the 4-bit pools: uniformly random codes, and scales /
            # zeros as unit-variance groups have them (range of 64 samples ~ 4.7 sigma -> step ~ 0.31, zero ~ -2.3).
            # The newest page (P tokens once the step's token is appended) is in the bfloat16 pools.
            lay = ea.q4_layout_query(dc)
            tpp = P // 64
            kq_pool, vq_pool = ea.alloc_q4_pools(dc, pool_pages, zero=False)
            # a unit = what repeats inside a kv head's part of a page: a tile block, or (key groups of 128 tokens) a
            # pair of K tile blocks, [codes][the pair's scales][codes]
            tpg = 2 if dc.q4_key_group == 128 else 1
            k_scales = 128 * ((lay.r_k_pad + 31) // 32)
            k_codes = lay.k_tile_bytes - k_scales
            for pool, unit_bytes, units, sc_off, sc_bytes in (
                    (kq_pool, tpg * k_codes + k_scales, Hkv * tpp // tpg, k_codes, k_scales),
                    (vq_pool, lay.v_tile_bytes, Hkv * tpp, lay.v_tile_bytes - 256, 256)):
                pool.random_(0, 256, generator=gen)
                blocks = pool.view(pool_pages, units, unit_bytes)
                sz = torch.empty((pool_pages, units, sc_bytes // 2), dtype=torch.float16, device=dev)
                grp = 8 if pool is kq_pool else 64              # run length of scales before their zeros
                szv = sz.view(pool_pages, units, -1, 2, grp)
                szv[:, :, :, 0].uniform_(0.28, 0.34, generator=gen)
                szv[:, :, :, 1].normal_(-2.3, 0.3, generator=gen)
                blocks[:, :, sc_off:sc_off + sc_bytes] = sz.view(torch.uint8)
            k_pool, v_pool = ea.alloc_pools(dc, B, zero=False)
            extra = dict(kq_pool=kq_pool, vq_pool=vq_pool,
                         tail_table=torch.arange(B, dtype=torch.int32, device=dev).reshape(B, 1).contiguous())
        else:
            k_pool, v_pool = ea.alloc_pools(dc, pool_pages, zero=False)
        k_pool.normal_(0.0, 1.00125, generator=gen)
        v_pool.normal_(0.0, 1.00125, generator=gen)
        perm = torch.randperm(pool_pages, generator=gen, device=dev).to(torch.int32)   # pages in seeded random order
        layers.append(dict(
            **extra,
            desc=dc, k_pool=k_pool, v_pool=v_pool, page_table=perm.reshape(B, max_pages).contiguous(),
            S=args.n_splits or (ea.decode_auto_splits(dc, B, n) if (q4 or not rope) else
                                ea.decode_rope_auto_splits(dc, B, n)),
            wqkv_raw=(torch.randn((n_qkv, d), generator=gen, device=dev) * d ** -0.5).to(torch.bfloat16),
            wo_raw=(torch.randn((d, H * dc.r_v), generator=gen, device=dev) * d ** -0.5).to(torch.bfloat16),
            x=torch.randn((B, d), generator=gen, device=dev).to(torch.bfloat16),
            q_r=torch.empty((B, H, q_dim), dtype=torch.float32, device=dev),
            # rotary variant: ONE key basis for all heads of the layer, orthonormal columns (QR of a Gaussian)
            u_k=(torch.linalg.qr(torch.randn((s.d_head, dc.r_k), generator=gen, device=dev))[0].contiguous()
                 .to(torch.bfloat16) if rope else None),
            o=torch.empty((B, H, dc.r_v), dtype=torch.float32, device=dev),
            mass=torch.zeros((B, Hkv, n), dtype=torch.float32, device=dev) if h2o else None,
            y=torch.empty((B, d), dtype=torch.bfloat16, device=dev)))
        l = layers[-1]
        l["wqkv"], l["wo"] = ea.pack_weight(l["wqkv_raw"]), ea.pack_weight(l["wo_raw"])
        if li not in (0, L - 1):          # the unpacked weights of the first and last layer stay for the parity check
            del l["wqkv_raw"], l["wo_raw"]
    torch.cuda.synchronize()
    t_fill = time.perf_counter() - t_fill

    slot_pos, q_pos = None, None
    if pruned:
        # what is left of a text four times as long: n kept tokens per sequence, in whatever slot eviction left them
        gp = torch.Generator(device=dev)
        gp.manual_seed(20240805 + 77)
        slot_pos = torch.stack([torch.randperm(4 * n, generator=gp, device=dev)[:n] for _ in range(B)]).to(torch.int32)
        slot_pos = slot_pos.contiguous()
        q_pos = torch.full((B,), 4 * n, dtype=torch.int32, device=dev)
    seq_before = torch.full((B,), n - 1, dtype=torch.int32, device=dev)    # the step appends token n-1 ...
    seq_after = torch.full((B,), n, dtype=torch.int32, device=dev)         # ... and attends over n tokens
    if h2o:
        ws_bytes = max(ea.decode_attn_mass_workspace_bytes(l["desc"], B, max_pages, l["S"]) for l in layers)
    else:
        ws_bytes = max((ea.decode_q4_workspace_bytes if q4 else ea.decode_workspace_bytes)(l["desc"], B, l["S"])
                       for l in layers)
    q4_len = torch.full((B,), n - P, dtype=torch.int32, device=dev)
    tail_before = torch.full((B,), P - 1, dtype=torch.int32, device=dev)
    tail_after = torch.full((B,), P, dtype=torch.int32, device=dev)
    ws = torch.empty(max(ws_bytes // 4, 4), dtype=torch.float32, device=dev)

    def step(events=None):
        for li, l in enumerate(layers):
            if q4:
                (ea.project_qkv_rope if rope else ea.project_qkv)(
                    l["desc"], l["x"], l["wqkv"], l["q_r"], l["k_pool"], l["v_pool"], l["tail_table"], tail_before, 1)
            else:
                (ea.project_qkv_rope if rope else ea.project_qkv)(
                    l["desc"], l["x"], l["wqkv"], l["q_r"], l["k_pool"], l["v_pool"], l["page_table"], seq_before, 1)
            if events is not None:
                events[li][0].record()
            if q4 and rope:
                ea.decode_attn_rope_q4(l["desc"], l["q_r"], l["u_k"], ROPE_BASE, l["kq_pool"], l["vq_pool"],
                                       l["page_table"], q4_len, l["k_pool"], l["v_pool"], l["tail_table"], tail_after,
                                       l["o"], l["S"], ws)
            elif q4:
                ea.decode_attn_q4(l["desc"], l["q_r"], l["kq_pool"], l["vq_pool"], l["page_table"], q4_len,
                                  l["k_pool"], l["v_pool"], l["tail_table"], tail_after, l["o"], l["S"], ws)
            elif pruned:
                ea.decode_attn_mass_rope_pos(l["desc"], l["q_r"], l["u_k"], ROPE_BASE, l["k_pool"], l["v_pool"],
                                             l["page_table"], seq_after, slot_pos, q_pos, l["o"], l["mass"], l["S"], ws)
            elif h2o:
                ea.decode_attn_mass(l["desc"], l["q_r"], l["k_pool"], l["v_pool"], l["page_table"], seq_after, l["o"],
                                    l["mass"], l["S"], ws)
            elif rope:
                ea.decode_attn_rope(l["desc"], l["q_r"], l["u_k"], ROPE_BASE, l["k_pool"], l["v_pool"], l["page_table"],
                                    seq_after, l["o"], n_splits=l["S"], ws=ws)
            else:
                ea.decode_attn(l["desc"], l["q_r"], l["k_pool"], l["v_pool"], l["page_table"], seq_after, l["o"],
                               n_splits=l["S"], ws=ws)
            if events is not None:
                events[li][1].record()
            ea.out_proj(l["desc"], l["o"].view(B, -1), l["wo"], l["y"])

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

    # ---- the same step captured once in a HIP graph and replayed (launch gaps shrink; reported beside the
    # eager figure, which stays the headline because its per-kernel events are what the roofline uses)
    ms_per_step_graph = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(args.steps):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        ms_per_step_graph = g0.elapsed_time(g1) / args.steps

    # ---- the same step with ONE library call per layer (ea_decode_layer: q_r and o stay in its workspace)
    ms_per_step_layer = None
    if not q4 and not h2o:
        lws = torch.empty(max(ea.decode_layer_workspace_bytes(l["desc"], B, l["S"], rope) for l in layers) // 4,
                          dtype=torch.float32, device=dev)

        def layer_step():
            for l in layers:
                ea.decode_layer(l["desc"], l["x"], l["wqkv"], l["wo"], l["k_pool"], l["v_pool"], l["page_table"],
                                seq_before, l["y"], l["S"], lws, u_k=l["u_k"], rope_base=ROPE_BASE)

        for _ in range(max(args.warmup, 1)):
            layer_step()
        torch.cuda.synchronize()
        l0, l1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        l0.record()
        for _ in range(args.steps):
            layer_step()
        l1.record()
        torch.cuda.synchronize()
        ms_per_step_layer = l0.elapsed_time(l1) / args.steps
        step()                              # leaves q_r / o / y of the separate calls in place for the parity check
        torch.cuda.synchronize()

    # ---- the same step in TWO launches per layer (ea_decode_layer_fused: projection + append, then attention, split
    # merge and output projection in one launch), eager and as a HIP-graph replay; its y against the separate calls'
    fused = None
    if not q4 and not h2o and B <= 16:
        y_sep = [l["y"].clone() for l in layers]
        fws = torch.empty(max(ea.decode_layer_fused_workspace_bytes(l["desc"], B, l["S"], rope) for l in layers) // 4,
                          dtype=torch.float32, device=dev)
        fstatus = torch.zeros(1, dtype=torch.int32, device=dev)

        def fused_step():
            for l in layers:
                ea.decode_layer(l["desc"], l["x"], l["wqkv"], l["wo"], l["k_pool"], l["v_pool"], l["page_table"],
                                seq_before, l["y"], l["S"], fws, u_k=l["u_k"], rope_base=ROPE_BASE, status=fstatus,
                                fused=True)

        for _ in range(max(args.warmup, 1)):
            fused_step()
        torch.cuda.synchronize()
        f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        f0.record()
        for _ in range(args.steps):
            fused_step()
        f1.record()
        torch.cuda.synchronize()
        ms_fused = f0.elapsed_time(f1) / args.steps
        worst = max(float((l["y"].float() - ys.float()).norm() / ys.float().norm()) for l, ys in zip(layers, y_sep))
        ms_fused_graph = None
        if not args.no_graph:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                fused_step()
            torch.cuda.current_stream().wait_stream(side)
            fgraph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(fgraph):
                fused_step()
            fgraph.replay()
            torch.cuda.synchronize()
            f0.record()
            for _ in range(args.steps):
                fgraph.replay()
            f1.record()
            torch.cuda.synchronize()
            ms_fused_graph = f0.elapsed_time(f1) / args.steps
        fused = {
            "ms_per_step": round(ms_fused, 4),             "hip_graph_replay_ms_per_step": None if ms_fused_graph is None else round(ms_fused_graph, 4),
            "y_rel_l2_vs_separate_calls": round(worst, 6), "status_word": int(fstatus.item()),
            "what": "the same step through ea_decode_layer_fused" + ("_rope" if rope else "") +
                    ": two launches per layer (o rounded to bfloat16 once before the output projection)"}
        if fused["status_word"] != 0 or not worst < 6e-3:
            print(f"bench.py: two-launch step disagrees with the separate calls ({fused})", file=sys.stderr)
            fused["ok"] = False
        else:
            fused["ok"] = True
        step()
        torch.cuda.synchronize()

    # ---- algorithmic bytes (what the method itself must move)
    attn_bytes_sum, step_bytes = 0, 0
    for dc in descs:
        q_dim = s.d_head if rope else dc.r_k
        n_qkv = H * q_dim + Hkv * (dc.r_k + dc.r_v)
        if q4:
            lay = ea.q4_layout_query(dc)
            cache_bytes = B * ((n - P) // P) * (lay.k_page_bytes + lay.v_page_bytes) + \
                B * Hkv * P * (dc.r_k + dc.r_v) * 2
        else:
            cache_bytes = B * Hkv * n * (dc.r_k + dc.r_v) * 2
        attn = cache_bytes + B * H * q_dim * 4 + B * H * dc.r_v * 4 + B * max_pages * 4 + \
            (s.d_head * dc.r_k * 2 if rope else 0) + \
            (B * Hkv * n * 8 if h2o else 0) + \
            (B * n * 4 if pruned else 0)           # the accumulator, read and written (the staged scores are overhead); the positions
        proj = n_qkv * d * 2 + B * d * 2 + B * H * q_dim * 4 + B * Hkv * (dc.r_k + dc.r_v) * 2
        outp = H * dc.r_v * d * 2 + B * H * dc.r_v * 4 + B * d * 2
        attn_bytes_sum += attn
        step_bytes += attn + proj + outp
    attn_bytes = attn_bytes_sum / L
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    attn_gbps = attn_bytes / (attn_us_avg * 1e-6) / 1e9
    splits = sorted(set(l["S"] for l in layers))
    kern = "decode_bf16_kernel" + (" (rotary variant)" if rope else "") + \
        ("" if splits == [1] else " + merge_splits_kernel") + \
        (" (one ea_decode_attn_rope call)" if rope else " (one ea_decode_attn call)")
    if q4:
        kern = (f"decode_q4_kernel ({args.q4_bits}-bit part and, in its last grid slices, the bf16 newest page) + merge_splits_kernel "
                "(one ea_decode_attn_q4 call)")
    if h2o:
        kern = ("decode_bf16_kernel (score-storing form) + merge_splits_kernel + mass_from_scores_kernel "
                "(one ea_decode_attn_mass call)")
    if q4 and rope:
        kern = ("decode_rope_q4_kernel + decode_bf16_kernel (rotary variant, newest page) + merge_splits_kernel "
                "(one ea_decode_attn_rope_q4 call)")
    if pruned:
        kern = ("decode_bf16_kernel (rotary variant with explicit positions, score-storing form) + merge_splits_kernel + "
                "mass_from_scores_kernel (one ea_decode_attn_mass_rope_pos call)")

    # (a figure belongs to one cache format: 64-token key groups, and one summary per code width)
    key = args.workload
    if q4:
        key = None if args.q4_key_group != 64 else (key + "-3bit" if args.q4_bits == 3 else key)
    traffic, traffic_src = traffic_from_profiles(key)
    if traffic_src is not None and traffic_src["stale"]:
        print(f"bench.py: {traffic_src['file']} was measured on other kernel sources "
              f"({traffic_src['measured_on_sources']} != {traffic_src['sources_now']}): roofline.traffic may be out of date",
              file=sys.stderr)
    if traffic is not None and not 0.95 <= traffic / attn_bytes <= 1.5:
        # (a summary whose counters were scaled wrongly, not a property of the kernel: say so rather than report it)
        print(f"bench.py: {traffic_src['file']} holds {traffic:.0f} bytes per launch against {attn_bytes:.0f} algorithmic: "
              "not a plausible HBM traffic for this kernel, left out", file=sys.stderr)
        traffic_src["implausible_bytes"] = traffic
        traffic = None
    rank_note = f"r_k=r_v={s.r_k}" if base_name != "cfg5" else "per-layer (r_k, r_v) drawn from {48,64,80,96,112}"
    result = {
        "metric": "low-rank decode attn: achieved HBM GB/s over the whole decode step"
                  + (" (B=16, n=32k, r=80)" if args.workload == "cfg3" else f" ({args.workload})"),
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload} decode: Llama-2-7B-shaped, {L} layers resident, B={B}, n={n}, "
                               f"H={H}, H_kv={Hkv}, d_h={s.d_head}, {rank_note}, "
                               + (f"cache in {args.q4_bits}-bit groups (keys per channel over {args.q4_key_group} tokens, values per token; fp16 "
                                  "scales and zeros) except the newest page of each sequence, which is bf16; "
                                  if q4 else "bf16 ") +
                               f"paged cache (page {P} tokens, pages in random order), "
                               + ("rotary position variant (Sec. 4.3): project_qkv_rope + decode_attn_rope_q4 + out_proj "
                                  "per layer, query at position n-1, base 10000" if (q4 and rope) else
                                  "project_qkv + decode_attn_q4 + out_proj per layer" if q4 else
                                  "rotary model after token pruning (Sec. 4.3 with H2O): project_qkv_rope + "
                                  "decode_attn_mass_rope_pos + out_proj per layer; the n cached tokens of a sequence are "
                                  "a random subset of a text of 4n tokens, each at its original position, in random slot "
                                  "order; query at position 4n, base 10000" if pruned else
                                  "project_qkv + decode_attn_mass (attention output and, for an H2O-style eviction "
                                  "policy, the attention mass of every cached token added to a per-layer accumulator) "
                                  "+ out_proj per layer" if h2o else
                                  "rotary position variant (Sec. 4.3): project_qkv_rope + decode_attn_rope + out_proj "
                                  "per layer, query at position n-1, base 10000" if rope else
                                  "project_qkv + decode_attn + out_proj per layer"),
                   "layers": L, "batch": B, "n_ctx": n, "page_tokens": P, "n_splits": splits},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "us_per_step": round(ms_per_step * 1e3, 1),
        "tokens_per_s": round(B / (ms_per_step * 1e-3), 1),
        "decode_attn_us_per_layer": round(attn_us_avg, 1),
        "hip_graph_replay": None if ms_per_step_graph is None else {
            "ms_per_step": round(ms_per_step_graph, 4),
            "GBps": round(step_bytes / (ms_per_step_graph * 1e-3) / 1e9, 1)},
        "one_call_per_layer": None if ms_per_step_layer is None else {
            "ms_per_step": round(ms_per_step_layer, 4),
            "GBps": round(step_bytes / (ms_per_step_layer * 1e-3) / 1e9, 1),
            "what": "the same step through ea_decode_layer" + ("_rope" if rope else "") + " (one call per layer)"},
        "two_launches_per_layer": None if fused is None else dict(
            fused, GBps=round(step_bytes / (fused["ms_per_step"] * 1e-3) / 1e9, 1)),
        "step_algorithmic_bytes": step_bytes,
        "fill_seconds": round(t_fill, 1), "timed_wall_seconds": round(wall, 3),
        "paper_context": PAPER_CONTEXT,
        "roofline": {"bound": "hbm", "achieved": round(attn_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(attn_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": kern, "bytes_per_launch": round(attn_bytes), "us_per_launch": round(attn_us_avg, 2)},
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
        mean_rank = sum(rk + rv for rk, rv in ranks) / (2 * L)
        result["fullrank_baseline"] = {
            "decode_attn_us_per_layer": round(full_us, 1), "achieved_GBps": round(full_bytes / full_us / 1e3, 1),
            "latency_ratio_lowrank_over_fullrank": round(attn_us_avg / full_us, 4),
            "ratio_predicted_by_rank": round(mean_rank / s.d_head, 4),
            "note": "position-free kernel, r_k = r_v = d_h = 128, same B, n and page table, one layer-sized buffer"
                    + ("; this is also what standard attention with rotary positions costs per step, since its cache "
                       "holds keys that are already rotated" if rope else "")}
        del fk, fv

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.float32, device=dev).normal_(generator=gen)     # 4 GiB
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        torch.cuda.synchronize()
        result["calibration_copy_bytes_each_way"] = src.numel() * 4

    # ---- what was timed, checked: sampled outputs of the resident step against the oracle (outside the timed region)
    streams0 = {}
    if not q4 and not args.no_parity:
        result["parity"], streams0 = check_step_parity(torch, ea, synth, layers, s, B, n, P, rope,
                                                       max(args.parity_samples, 2), int(base_name[-1]),
                                                       slot_pos=slot_pos, q_pos=q_pos)
    elif q4 and not args.no_parity:
        result["parity"] = check_step_parity_q4(torch, ea, synth, layers, s, B, n, P, rope,
                                                max(min(args.parity_samples, 16), 2), int(base_name[-1]),
                                                args.q4_bits, args.q4_key_group)

    if not args.no_cpu and q4:
        result["cpu_baseline"] = cpu_oracle_decode_q4(512 // (32 if rope else 8), n, ranks[0][0], s.d_head,
                                                      P, rope=rope, key_group=args.q4_key_group, bits=args.q4_bits)
    elif not args.no_cpu:
        # streams of the first resident layer, copied back from the device (those the parity check already holds first)
        l = layers[0]
        dc = l["desc"]
        lay = ea.cache_layout_query(dc)
        G = H // Hkv
        want = max(1, min(args.cpu_streams // (4 if rope else 1), B * Hkv))
        keys = list(streams0.keys())
        for b in range(B):
            for kvh in range(Hkv):
                if len(keys) < want and (b, kvh) not in streams0:
                    keys.append((b, kvh))
        streams = []
        positions = ([(slot_pos[b, :n].cpu().numpy(), int(q_pos[b])) for b, _ in keys[:want]] if pruned else None)
        for b, kvh in keys[:want]:
            if (b, kvh) in streams0:
                streams.append(streams0[(b, kvh)])
                continue
            Kb = _stream_bits(torch, l["k_pool"], l["page_table"][b], kvh, Hkv, dc.r_k, lay.r_k_pad, _k_tiles_to_rows, P, n)
            Vb = _stream_bits(torch, l["v_pool"], l["page_table"][b], kvh, Hkv, dc.r_v, lay.r_v_pad, _v_tiles_to_rows, P, n)
            streams.append((Kb, Vb, l["q_r"][b, kvh * G:(kvh + 1) * G].cpu().numpy()))
        result["cpu_baseline"] = cpu_oracle_decode(streams, s.d_head,
                                                   rope_u=l["u_k"].float().cpu().numpy() if rope else None, h2o=h2o,
                                                   positions=positions)
    return result


def bench_prefill(args, torch, ea, synth):
    dev = "cuda"
    s = synth.CFG4
    B, n, P = s.batch, s.n_ctx, args.page_tokens
    H, d, r = s.n_heads, s.d_model, s.r_k
    desc = ea.LayerDesc(d, H, H, s.d_head, r, r, ea.EA_BF16, P)
    max_pages = n // P
    pool_pages = B * max_pages
    rope = args.workload.endswith("-rope")
    q_dim = s.d_head if rope else r                  # the rotary variant keeps the query at full rank (Sec. 4.3)
    n_qkv = H * q_dim + 2 * H * r
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED + 4)
    k_pool, v_pool = ea.alloc_pools(desc, pool_pages)
    pt = torch.randperm(pool_pages, generator=gen, device=dev).to(torch.int32).reshape(B, max_pages).contiguous()
    seq0 = torch.zeros((B,), dtype=torch.int32, device=dev)
    seq1 = torch.full((B,), n, dtype=torch.int32, device=dev)
    x = torch.randn((B * n, d), generator=gen, device=dev).to(torch.bfloat16)
    wqkv_raw = (torch.randn((n_qkv, d), generator=gen, device=dev) * d ** -0.5).to(torch.bfloat16)
    wo_raw = (torch.randn((d, H * r), generator=gen, device=dev) * d ** -0.5).to(torch.bfloat16)
    wqkv, wo = ea.pack_weight(wqkv_raw), ea.pack_weight(wo_raw)
    q_r = torch.empty((B * n, H, q_dim), dtype=torch.bfloat16, device=dev)
    o = torch.empty((B, n, H, r), dtype=torch.bfloat16, device=dev)
    y = torch.empty((B * n, d), dtype=torch.bfloat16, device=dev)
    if rope:
        u_k = torch.linalg.qr(torch.randn((s.d_head, r), generator=gen, device=dev))[0].contiguous().to(torch.bfloat16)
        ws = torch.empty((ea.prefill_rope_workspace_bytes(desc, B, n, max_pages) // 2,), dtype=torch.bfloat16, device=dev)

    def step(events=None):
        if events is not None:
            events[0].record()
        (ea.project_qkv_rope if rope else ea.project_qkv)(desc, x, wqkv, q_r, k_pool, v_pool, pt, seq0, n)
        if events is not None:
            events[1].record()
        if rope:
            ea.prefill_attn_rope(desc, q_r.view(B, n, H, q_dim), u_k, ROPE_BASE, k_pool, v_pool, pt, seq1, o, ws=ws)
        else:
            ea.prefill_attn(desc, q_r.view(B, n, H, r), k_pool, v_pool, pt, seq1, o)
        if events is not None:
            events[2].record()
        ea.out_proj(desc, o.view(B * n, H * r), wo, y)
        if events is not None:
            events[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for k in range(args.steps):
        step(ev[k])
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    t = [sum(ev[k][i].elapsed_time(ev[k][i + 1]) for k in range(args.steps)) / args.steps for i in range(3)]
    f_proj = 2 * B * n * d * n_qkv
    # causal-counted: 2 * (n^2 / 2) * (score width + r_v) per (sequence, head); the rotary variant scores at d_h
    # channels and brings every cached key back to d_h channels once (2 * n * r * d_h per sequence and head)
    f_attn = B * H * n * n * (q_dim + r) + (2 * B * H * n * r * s.d_head if rope else 0)
    f_out = 2 * B * n * H * r * d
    flops = f_proj + f_attn + f_out

    def tf(f, ms):
        return f / (ms * 1e-3) / 1e12

    # the dominant kernel = the longest of the three calls (causal-counted flops for the attention)
    calls = [("gemm_bf16_async_kernel (ea_project_qkv" + ("_rope" if rope else "") + ")", f_proj, t[0]),
             ("prefill_bf16_direct_kernel (ea_prefill_attn" + ("_rope: expand + rotate + attention" if rope else "") +
              ", flops counted below the causal diagonal only)", f_attn, t[1]),
             ("gemm_bf16_async_kernel (ea_out_proj)", f_out, t[2])]
    dom = max(calls, key=lambda c: c[2])
    roofline = {"bound": "mfma", "achieved": round(tf(dom[1], dom[2]), 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(tf(dom[1], dom[2]) / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                "kernel": dom[0] + ", the longest of the three calls", "flops_per_launch": dom[1],
                "us_per_launch": round(dom[2] * 1e3, 1)}
    result = {
        "metric": f"low-rank causal prefill: TFLOP/s of project_qkv + prefill_attn + out_proj ({args.workload})",
        "value": round(tf(flops, ms_per_step), 1), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload} causal prefill: one Llama-2-7B-shaped layer, B={B}, n={n}, H={H}, "
                               f"d_h={s.d_head}, r_k=r_v={r}, bf16, cache written to a paged pool (page {P} tokens, "
                               f"random order)" + (", rotary positions (Sec. 4.3): project_qkv_rope + "
                                                   "prefill_attn_rope + out_proj" if rope else ""),
                   "batch": B, "n_ctx": n, "r_k": r, "r_v": r, "page_tokens": P},
        "tokens_per_s": round(B * n / (ms_per_step * 1e-3), 1),
        "kernels": {"project_qkv": {"ms": round(t[0], 4), "tflops": round(tf(f_proj, t[0]), 1)},
                    "prefill_attn": {"ms": round(t[1], 4), "tflops_causal_counted": round(tf(f_attn, t[1]), 1),
                                     "tflops_dense_counted": round(tf(2 * f_attn, t[1]), 1)},
                    "out_proj": {"ms": round(t[2], 4), "tflops": round(tf(f_out, t[2]), 1)}},
        "roofline": roofline,
    }
    # ---- what was timed, checked: sampled query rows of the step's attention output and rows of its projections
    # against the oracle, on the cache contents and queries the step itself produced (copied back from the device)
    if not args.no_parity:
        import numpy as np
        from oracle import eigen_attention as ora
        lay = ea.cache_layout_query(desc)
        g = synth.rng(44, int(rope))
        worst, errs = 0.0, []
        u_host = u_k.float().cpu().numpy().astype(np.float64) if rope else None
        picks = [(0, 0, 64), (B - 1, H - 1, n)] + [(int(g.integers(B)), int(g.integers(H)), int(g.integers(65, n)))
                                                    for _ in range(max(args.parity_samples // 8, 2))]
        for b, h, m in picks:                         # the 64 queries that end at position m - 1 of (sequence b, head h)
            Kb = _stream_bits(torch, k_pool, pt[b], h, H, r, lay.r_k_pad, _k_tiles_to_rows, P, m)
            Vb = _stream_bits(torch, v_pool, pt[b], h, H, r, lay.r_v_pad, _v_tiles_to_rows, P, m)
            cache = ora.RankCache.from_arrays([synth.bf16_bits_to_f32(Kb).astype(np.float64)[None]],
                                              [synth.bf16_bits_to_f32(Vb).astype(np.float64)[None]])
            qrows = q_r.view(B, n, H, q_dim)[b, m - 64:m, h].float().cpu().numpy().astype(np.float64)[None, :, None, :]
            if rope:
                ref = ora.prefill_attention_rope(qrows, cache, u_host, s.d_head, ROPE_BASE)
            else:
                ref = ora.prefill_attention(qrows, cache, s.d_head)
            got = o[b, m - 64:m, h].float().cpu().numpy()[None, :, None, :]
            e = ora.rel_l2(got, ref) if np.isfinite(got).all() else float("inf")
            errs.append(e)
            worst = max(worst, e)
        # projection and output projection on 64 sampled rows
        rows = np.sort(g.choice(B * n, size=64, replace=False))
        xr = x[torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
        w = wqkv_raw.float().cpu().numpy().astype(np.float64)
        q_ref = xr @ w[:H * q_dim].T
        e_q = ora.rel_l2(q_r.view(B * n, H * q_dim)[torch.from_numpy(rows).cuda()].float().cpu().numpy(), q_ref)
        orows = o.view(B * n, H * r)[torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
        wo_h = wo_raw.float().cpu().numpy().astype(np.float64)
        e_y = ora.rel_l2(y[torch.from_numpy(rows).cuda()].float().cpu().numpy(), orows @ wo_h.T)
        worst = max(worst, e_q, e_y)
        result["parity"] = {"samples": len(errs), "worst_rel_l2": float(f"{worst:.3e}"),
                            "attention_mean_rel_l2": float(f"{np.mean(errs):.3e}"),
                            "q_rel_l2": float(f"{e_q:.3e}"), "y_rel_l2": float(f"{e_y:.3e}"), "bar": 1e-2,
                            "ok": bool(np.isfinite(worst) and worst <= 1e-2),
                            "what": "blocks of 64 query rows of the timed step's attention output (first rows, last rows, "
                                    "seeded random positions) and 64 rows of its two projections vs the fp64 oracle, on "
                                    "the cache slices and queries the step produced"}
    if not args.no_cpu and not rope:
        result["cpu_baseline"] = cpu_oracle_prefill(512, n, r, s.d_head)
    return result


def bench_prefill_q4(args, torch, ea, synth):
    """cfg4-q4: the config-4 prompt prefilled chunk by chunk, every finished chunk quantised to 4 bits at once, so that
    only one chunk per sequence ever exists in 16 bits.  A step = the whole prompt through one layer: per chunk
    project_qkv (into the same few bfloat16 pages), ea_prefill_attn_q4 (the chunk causally, all earlier chunks as
    codes), ea_quantize_pages_q4, out_proj."""
    import numpy as np
    dev = "cuda"
    s = synth.CFG4
    B, n, P, C = s.batch, s.n_ctx, args.page_tokens, args.prefill_chunk
    H, d, r = s.n_heads, s.d_model, s.r_k
    group = args.q4_key_group
    if C % P or n % C or P % group:
        raise SystemExit("cfg4-q4: the chunk must be whole pages, the prompt whole chunks, a page whole key groups")
    desc = ea.LayerDesc(d, H, H, s.d_head, r, r, ea.EA_BF16, P, group, args.q4_bits)
    n_qkv = 3 * H * r
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED + 4)
    cpp = C // P                                         # pages per chunk and sequence
    k_pool, v_pool = ea.alloc_pools(desc, B * cpp)       # the only bfloat16 cache there is: one chunk per sequence
    stage = torch.randperm(B * cpp, generator=gen, device=dev).to(torch.int32).reshape(B, cpp).contiguous()
    q4_pages = B * (n // P)
    kq, vq = ea.alloc_q4_pools(desc, q4_pages)
    q4_table = torch.randperm(q4_pages, generator=gen, device=dev).to(torch.int32).reshape(B, n // P).contiguous()
    x = torch.randn((B, n, d), generator=gen, device=dev).to(torch.bfloat16)
    wqkv_raw = (torch.randn((n_qkv, d), generator=gen, device=dev) * d ** -0.5).to(torch.bfloat16)
    wo_raw = (torch.randn((d, H * r), generator=gen, device=dev) * d ** -0.5).to(torch.bfloat16)
    wqkv, wo = ea.pack_weight(wqkv_raw), ea.pack_weight(wo_raw)
    q_r = torch.empty((B, n, H, r), dtype=torch.bfloat16, device=dev)         # kept whole for the parity check
    o = torch.empty((B, n, H, r), dtype=torch.bfloat16, device=dev)
    y = torch.empty((B, n, d), dtype=torch.bfloat16, device=dev)
    xc = [x[:, c0:c0 + C].contiguous().view(B * C, d) for c0 in range(0, n, C)]
    qc = torch.empty((B * C, H, r), dtype=torch.bfloat16, device=dev)
    oc = torch.empty((B, C, H, r), dtype=torch.bfloat16, device=dev)
    yc = torch.empty((B * C, d), dtype=torch.bfloat16, device=dev)
    staged = bool(args.q4_staged)
    ws_bytes = (ea.prefill_q4_staged_workspace_bytes(desc, B, C, n // P, cpp) if staged
                else ea.prefill_q4_workspace_bytes(desc, B, C))
    ws = torch.empty(ws_bytes // 4, dtype=torch.float32, device=dev)
    zero = torch.zeros((B,), dtype=torch.int32, device=dev)
    full = torch.full((B,), C, dtype=torch.int32, device=dev)
    q4_lens = [torch.full((B,), c0, dtype=torch.int32, device=dev) for c0 in range(0, n, C)]
    src_pages = stage.reshape(-1).contiguous()
    dst_pages = [q4_table[:, c0 // P:(c0 + C) // P].reshape(-1).contiguous() for c0 in range(0, n, C)]
    n_chunks = n // C

    def step(events=None, keep=False):
        for c in range(n_chunks):
            e = events[c] if events is not None else None
            if e: e[0].record()
            ea.project_qkv(desc, xc[c], wqkv, qc, k_pool, v_pool, stage, zero, C)
            if e: e[1].record()
            ea.prefill_attn_q4(desc, qc.view(B, C, H, r), kq, vq, q4_table, q4_lens[c], k_pool, v_pool, stage, full, oc, ws,
                               staged=staged)
            if e: e[2].record()
            ea.quantize_pages_q4(desc, k_pool, v_pool, src_pages, kq, vq, dst_pages[c])
            if e: e[3].record()
            ea.out_proj(desc, oc.view(B * C, H * r), wo, yc)
            if e: e[4].record()
            if keep:
                q_r[:, c * C:(c + 1) * C] = qc.view(B, C, H, r)
                o[:, c * C:(c + 1) * C] = oc
                y[:, c * C:(c + 1) * C] = yc.view(B, C, d)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(n_chunks)] for _ in range(args.steps)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for k in range(args.steps):
        step(ev[k])
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    t = [sum(ev[k][c][i].elapsed_time(ev[k][c][i + 1]) for k in range(args.steps) for c in range(n_chunks)) / args.steps
         for i in range(4)]
    attn_per_chunk = [sum(ev[k][c][1].elapsed_time(ev[k][c][2]) for k in range(args.steps)) / args.steps
                      for c in range(n_chunks)]
    f_proj, f_attn, f_out = 2 * B * n * d * n_qkv, B * H * n * n * 2 * r, 2 * B * n * H * r * d
    flops = f_proj + f_attn + f_out

    def tf(f, ms):
        return f / (ms * 1e-3) / 1e12

    lay, lay16 = ea.q4_layout_query(desc), ea.cache_layout_query(desc)
    result = {
        "metric": f"low-rank causal prefill over a {args.q4_bits}-bit cache: TFLOP/s of the whole prompt, chunk by chunk (cfg4-q4)",
        "value": round(tf(flops, ms_per_step), 1), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg4-q4 causal prefill: one Llama-2-7B-shaped layer, B={B}, n={n}, H={H}, d_h={s.d_head}, "
                               f"r_k=r_v={r}, in chunks of {C} tokens per sequence; per chunk project_qkv (into the same "
                               f"{B * cpp} bfloat16 pages) + {'prefill_attn_q4_staged' if staged else 'prefill_attn_q4'} (the chunk causally, earlier chunks as {args.q4_bits}-bit "
                               f"codes, key groups of {group} tokens) + quantize_pages_q4 + out_proj; pages of {P} tokens "
                               f"in random order",
                   "batch": B, "n_ctx": n, "r_k": r, "r_v": r, "page_tokens": P, "chunk": C},
        "tokens_per_s": round(B * n / (ms_per_step * 1e-3), 1),
        "kernels": {"project_qkv": {"ms": round(t[0], 4), "tflops": round(tf(f_proj, t[0]), 1)},
                    ("prefill_attn_q4_staged" if staged else "prefill_attn_q4"): {"ms": round(t[1], 4), "tflops_causal_counted": round(tf(f_attn, t[1]), 1),
                                        "ms_per_chunk": [round(v, 4) for v in attn_per_chunk]},
                    "quantize_pages_q4": {"ms": round(t[2], 4)},
                    "out_proj": {"ms": round(t[3], 4), "tflops": round(tf(f_out, t[3]), 1)}},
        "cache_bytes": {"bf16_resident": int(B * cpp * (lay16.k_page_elems + lay16.v_page_elems) * 2),
                        "workspace_of_the_attention_call": int(ws_bytes),
                        "q4_after_the_prompt": int(q4_pages * (lay.k_page_bytes + lay.v_page_bytes)),
                        "bf16_if_the_prompt_were_kept_in_16_bits": int(B * (n // P) * (lay16.k_page_elems + lay16.v_page_elems) * 2)},
        "roofline": {"bound": "mfma", "achieved": round(tf(f_attn, t[1]), 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(tf(f_attn, t[1]) / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                     "kernel": ("stage_lists_kernel + dequantize_q4_kernel + copy_pages_kernel + prefill_bf16_direct_kernel: all "
                                "ea_prefill_attn_q4_staged calls of the prompt, flops counted below the causal diagonal only"
                                if staged else
                                "prefill_bf16_direct_kernel (the chunk itself) + prefill_q4_kernel (earlier chunks) + "
                                "merge_prefill_parts_kernel: all ea_prefill_attn_q4 calls of the prompt, flops counted below "
                                "the causal diagonal only"), "flops_per_launch": f_attn, "us_per_launch": round(t[1] * 1e3, 1)},
    }
    if not args.no_parity:
        from oracle import eigen_attention as ora
        from oracle import quant_cache as oq
        step(keep=True)
        # the keys and values as the step's projection produced them, once more into pools that hold the whole prompt
        # (for the check only), so that the oracle can quantise the same bfloat16 values
        kf, vf = ea.alloc_pools(desc, B * (n // P))
        ptf = torch.arange(B * (n // P), dtype=torch.int32, device=dev).reshape(B, n // P).contiguous()
        qtmp = torch.empty((B * C, H, r), dtype=torch.bfloat16, device=dev)
        for c in range(n_chunks):
            ea.project_qkv(desc, xc[c], wqkv, qtmp, kf, vf, ptf, q4_lens[c], C)
        torch.cuda.synchronize()
        g = synth.rng(45)
        picks = [(0, 0, 64), (B - 1, H - 1, n), (0, 1, C + 64)] + \
                [(int(g.integers(B)), int(g.integers(H)), int(g.integers(65, n))) for _ in range(max(args.parity_samples // 8, 2))]
        worst, errs = 0.0, []
        for b, h, m in picks:
            Kb = _stream_bits(torch, kf, ptf[b], h, H, r, lay16.r_k_pad, _k_tiles_to_rows, P, m)
            Vb = _stream_bits(torch, vf, ptf[b], h, H, r, lay16.r_v_pad, _v_tiles_to_rows, P, m)
            K1 = synth.bf16_bits_to_f32(Kb).astype(np.float64)[None]
            V1 = synth.bf16_bits_to_f32(Vb).astype(np.float64)[None]
            lo = max(m - 64, (m - 1) // C * C)               # the block's rows that lie in the chunk of row m - 1
            qrows = q_r[b, lo:m, h].float().cpu().numpy().astype(np.float64)[None, :, None, :]
            ref = oq.prefill_attention_quantized(qrows, [K1], [V1], [(m - 1) // C * C], s.d_head, group_tokens=group,
                                                 bits=args.q4_bits)
            got = o[b, lo:m, h].float().cpu().numpy()[None, :, None, :]
            e = ora.rel_l2(got, ref) if np.isfinite(got).all() else float("inf")
            errs.append(e)
            worst = max(worst, e)
        result["parity"] = {"samples": len(errs), "worst_rel_l2": float(f"{worst:.3e}"),
                            "attention_mean_rel_l2": float(f"{np.mean(errs):.3e}"), "bar": 1e-2,
                            "ok": bool(np.isfinite(worst) and worst <= 1e-2),
                            "what": "blocks of up to 64 query rows of the step's attention output (first rows, last rows, "
                                    "the first rows of the second chunk, seeded random positions) vs the fp64 oracle's causal "
                                    "attention over the same keys and values with the earlier chunks quantised"}
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_oracle_prefill(512, n, r, s.d_head)
    return result


def main():
    if len(sys.argv) >= 6 and sys.argv[1] == "--oracle-worker":       # a child of cpu_oracle_decode: no GPU, no torch
        oracle_worker_main(sys.argv[2], int(sys.argv[3]), float(sys.argv[4]), int(sys.argv[5]))
        return
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
    if args.workload == "cfg4-q4":
        result = bench_prefill_q4(args, torch, ea, synth)
    elif args.workload.startswith("cfg4"):
        result = bench_prefill(args, torch, ea, synth)
    else:
        result = bench_decode(args, torch, ea, synth)
    print(json.dumps(result))
    par = result.get("parity")
    if isinstance(par, dict) and par.get("ok") is False:
        print(f"bench.py: the timed step does not match the oracle: {par}", file=sys.stderr)
        sys.exit(4)
    two = result.get("two_launches_per_layer")
    if isinstance(two, dict) and two.get("ok") is False:
        sys.exit(4)


if __name__ == "__main__":
    main()
