#!/usr/bin/env python3
"""KCache decode-attention benchmark on one MI355X.

A step is one decode step of the whole hot path over one batch: for every
layer, the new token's K/V rows are stored (T = 1) and kcache_decode_attention
runs (K scan over the full context, softmax, top-N, V pull from pinned host
memory, weighted sum).  All inputs are synthetic, seeded, and already resident
(K in HBM, V in pinned host memory) when the timed region starts.  By default the
step is issued as one launch of a HIP graph captured from kcache_decode_step (the
same kernels in the same order on one stream); --step-mode selects the eager forms.

Prints one JSON line: tokens/s for the whole job, the HBM roofline of the K-scan
kernel (HIP events around every launch, taken live in a second timed pass of
the same steps), the host-link figures of the V pull, and the CPU oracle timed
on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import kcache_inputs as ki  # noqa: E402

HBM_PEAK_GBPS = 8000.0
K_FP8_EXP = -5   # cache exponent of the 8-bit K variant: covers |K| < 14 of the synthetic workloads


def algorithmic_bytes(wl, lens, k_elem_bytes=2):
    """Bytes one layer of a decode step has to move, whatever the implementation (Table 1):
    the K rows of every cached position from HBM (the 2bnhs term of the S~ row) and the N
    kept V rows of every query head over the host link (the 2bNd term of the A~ row)."""
    lens = np.asarray(lens, dtype=np.int64)
    k_bytes = int(lens.sum()) * wl.Hkv * wl.d * k_elem_bytes
    v_bytes = int(np.minimum(lens, wl.N).sum()) * wl.H * wl.d * 2
    return k_bytes, v_bytes


def eq4_break_even(bw_gpu, bw_h2d, overlapped=False):
    """s/N above which KCache is no slower than a conventional KV cache (section 3.2,
    equation (4)): Bandwidth_GPU / Bandwidth_H2D when the V pull follows the K scan; half of
    it when the two overlap (N rows over the link then only have to beat 2 s rows from HBM)."""
    return bw_gpu / bw_h2d / (2.0 if overlapped else 1.0)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="workload of BASELINE.json (1-5); 6 = the shape of the paper's Table 4 "
                         "headline row (batch 5, 16k context, N 128), for context")
    ap.add_argument("--layers", type=int, default=0, help="debug: use fewer layers (invalid as a result)")
    ap.add_argument("--parts", type=int, default=0, help="pipeline parts per layer (0 = library default)")
    ap.add_argument("--gather", choices=["zerocopy", "staged"], default="zerocopy")
    ap.add_argument("--rows", type=int, default=0, help="fused kernel: positions per workgroup (0 = auto)")
    ap.add_argument("--unfused", action="store_true",
                    help="separate scan / select / gather launches instead of the fused kernel")
    ap.add_argument("--cpu-units", type=int, default=64, help="units in the CPU-oracle sample")
    ap.add_argument("--cpu-passes", type=int, default=6, help="oracle passes over the sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true")
    ap.add_argument("--prefill", action="store_true",
                    help="also time kcache_prefill_store of one layer's whole context (K to HBM, "
                         "V device-to-host), reported under \"prefill_store\"")
    ap.add_argument("--step-mode", choices=["graph", "step", "calls"], default="graph",
                    help="how a decode step is issued: one captured HIP graph launch (default), "
                         "one kcache_decode_step call, or per-layer store + attention calls")
    ap.add_argument("--lanes", type=int, default=1,
                    help="streams a step is spread over (kcache_decode_step)")
    ap.add_argument("--split", choices=["sequences", "layers"], default="sequences",
                    help="what the lanes hold: a share of the batch each, run through all layers "
                         "in order (keeps every dependency of a real decode step), or whole "
                         "layers dealt round-robin (only meaningful for the attention in "
                         "isolation)")
    ap.add_argument("--no-overlap-leg", action="store_true",
                    help="skip the extra timed passes with two lanes reported under lanes_2")
    ap.add_argument("--hbm-layers", type=int, default=0,
                    help="the first L layers keep their V cache in HBM and run conventional "
                         "attention (the method's second knob, section 3.1 / Table 2); -1 = every "
                         "layer, i.e. the conventional KV-cache baseline")
    ap.add_argument("--gqa-dedup", action="store_true",
                    help="grouped queries: pull the union of a group's V rows once")
    ap.add_argument("--shared-pivots", action="store_true",
                    help="synthetic variant of the workload in which the heads of a group share "
                         "their pivotal positions (what --gqa-dedup is for)")
    ap.add_argument("--k-fp8", action="store_true",
                    help="variant: 8-bit K cache (E4M3 codes, cache exponent -5); halves the bytes "
                         "of the K scan")
    ap.add_argument("--crossover", action="store_true",
                    help="also time, on one layer of this workload's shape, the KCache launch "
                         "against conventional attention with V in HBM over a grid of context "
                         "lengths and N (section 3.2, equations (3)-(4)), reported under "
                         "\"crossover\"")
    return ap.parse_args()


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the method's (sequence, head) units are "
              "independent and would shard by head or by sequence without any exchange); "
              "--gpus %d is not supported" % a.gpus, file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    import paper_2404_18057_amd as kc

    wl = ki.config(a.config)
    if a.shared_pivots:
        wl = wl.replace(shared_pivots=True, name=wl.name + "_shared_pivots")
    L = a.layers if a.layers > 0 else wl.L
    Lh = L if a.hbm_layers < 0 else min(a.hbm_layers, L)   # layers with V in HBM
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    ctx = kc.Context(0, kc.workspace_bytes(wl.B, wl.H, wl.S_cap, wl.N))
    ctx.set_pipeline_parts(a.parts)
    ctx.set_fused(not a.unfused)
    ctx.set_fused_rows(a.rows)
    ctx.set_gqa_dedup(a.gqa_dedup)
    mode = kc.GATHER_ZEROCOPY if a.gather == "zerocopy" else kc.GATHER_STAGED
    dt = ki.torch_dtype(wl.dtype)
    lens = wl.seq_lens()
    lens_dev = torch.from_numpy(lens).to(dev)
    pos_last = torch.from_numpy(lens - 1).to(dev)

    # ---- resident state: K in HBM, V in pinned host memory, placed by the store path
    t0 = time.time()
    caches, qs, k_tok, v_tok = [], [], [], []
    shape = (wl.B, wl.Hkv, wl.S_cap, wl.d)
    T_chunk = min(wl.S_cap, 8192)
    hks = list(range(wl.Hkv))
    # one pinned allocation for every layer's V (torch rounds each pinned request up to a
    # power of two: per-layer requests of 1.25 GiB would pin 2 GiB each)
    layer_elems = int(np.prod(shape))
    v_all = torch.empty(max(L - Lh, 1) * layer_elems, dtype=dt, pin_memory=True)
    for layer in range(L):
        k_cache = torch.empty(shape, dtype=torch.uint8 if a.k_fp8 else dt, device=dev)
        if layer < Lh:
            v_cache = torch.empty(shape, dtype=dt, device=dev)
        else:
            v_cache = v_all[(layer - Lh) * layer_elems:(layer - Lh + 1) * layer_elems].view(shape)
        cache = kc.LayerCache(k_cache, v_cache, k_exp=K_FP8_EXP)
        kt = torch.empty((wl.B, 1, wl.Hkv, wl.d), dtype=dt, device=dev)
        vt = torch.empty((wl.B, 1, wl.Hkv, wl.d), dtype=dt, device=dev)
        for b in range(wl.B):
            k, v = ki.gen_kv_units(wl, layer, b, hks, wl.S_cap, dev)
            sub = kc.LayerCache(k_cache[b:b + 1], v_cache[b:b + 1], k_exp=K_FP8_EXP)
            zero = torch.zeros(1, dtype=torch.int32, device=dev)
            alive = []   # the V half runs on the library's side stream: inputs must outlive it
            for t in range(0, wl.S_cap, T_chunk):
                kn = k[:, t:t + T_chunk].permute(1, 0, 2).unsqueeze(0).contiguous()
                vn = v[:, t:t + T_chunk].permute(1, 0, 2).unsqueeze(0).contiguous()
                pos = zero + t
                ctx.prefill_store(sub, kn, vn, pos)
                alive.append((kn, vn, pos))
            kt[b, 0] = k[:, lens[b] - 1]
            vt[b, 0] = v[:, lens[b] - 1]
            ctx.synchronize()
            torch.cuda.synchronize()
            del alive
        caches.append(cache)
        qs.append(ki.gen_q(wl, layer, dev))
        k_tok.append(kt)
        v_tok.append(vt)
    ctx.device_check()
    setup_s = time.time() - t0

    outs = [torch.empty((wl.B, wl.H, wl.d), dtype=torch.float32, device=dev) for _ in range(L)]
    idxs = [torch.empty((wl.B, wl.H, wl.N), dtype=torch.int32, device=dev) for _ in range(L)]
    ws = [torch.empty((wl.B, wl.H, wl.N), dtype=torch.float32, device=dev) for _ in range(L)]

    step_layers = [dict(cache=caches[l], k_new=k_tok[l], v_new=v_tok[l], q=qs[l], out=outs[l],
                        idx_out=idxs[l], w_out=ws[l]) for l in range(L)]
    plain = mode == kc.GATHER_ZEROCOPY and not a.unfused   # what the step calls implement
    step_mode = a.step_mode if plain else "calls"
    ctx.set_step_lanes(a.lanes, split_sequences=(a.split == "sequences"))
    graph = ctx.step_graph(step_layers, wl.H, pos_last, lens_dev, wl.N) \
        if step_mode == "graph" else None

    def step_calls():
        for l in range(L):
            ctx.prefill_store(caches[l], k_tok[l], v_tok[l], pos_last)
            if l < Lh:
                ctx.full_attention(caches[l], qs[l], lens_dev, out=outs[l])
            else:
                ctx.decode_attention(caches[l], qs[l], lens_dev, wl.N, out=outs[l],
                                     idx_out=idxs[l], w_out=ws[l], gather_mode=mode)

    def step_eager():
        ctx.decode_step(step_layers, wl.H, pos_last, lens_dev, wl.N)

    step = {"graph": (lambda: graph.launch()), "step": step_eager, "calls": step_calls}[step_mode]

    def timed(n):
        torch.cuda.synchronize()
        ctx.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            step()
        ctx.synchronize()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / n

    for _ in range(a.warmup):
        step()
    sec_per_step = timed(a.steps)

    # ---- optional: the same step spread over two streams, both ways
    overlap = None
    if plain and not a.no_overlap_leg and a.lanes == 1 and L > 1:
        if graph is not None:
            graph.close()
            graph = None
        keep = step
        overlap = {}
        for what in ("sequences", "layers"):
            if what == "sequences" and wl.B < 2:
                continue
            ctx.set_step_lanes(2, split_sequences=(what == "sequences"))
            g2 = ctx.step_graph(step_layers, wl.H, pos_last, lens_dev, wl.N)
            step = lambda: g2.launch()
            for _ in range(a.warmup):
                step()
            sec2 = timed(a.steps)
            g2.close()
            overlap[what] = {"ms_per_step": sec2 * 1e3, "tokens_per_s": wl.B / sec2}
        ctx.set_step_lanes(1)
        step = keep
        overlap["note"] = ("two streams, so that the K scan of one launch hides the merge / V-pull "
                           "tail of another.  sequences: each stream takes half of the batch "
                           "through the layers in order, which keeps every dependency of a real "
                           "decode step; layers: whole layers alternate between the streams, "
                           "which is only meaningful for the attention in isolation.  Neither is "
                           "the headline value: their launches overlap, so no per-launch "
                           "roofline can be quoted for them")

    # ---- second pass of the same steps with HIP events around every kernel launch
    # (eager launches: events are not part of a captured graph)
    if step_mode == "graph":
        step = step_eager
    ctx.set_step_lanes(1)   # one launch at a time: its duration is the kernel's own
    ctx.set_profile(True)
    ctx.profile_reset()
    sec_per_step_prof = timed(a.steps)
    prof = {k: ctx.profile_read(k) for k in kc.KERNELS}
    ctx.set_profile(False)
    ctx.device_check()

    units_per_layer = wl.B * wl.H
    k_bytes_layer, v_bytes_layer = algorithmic_bytes(wl, lens, 1 if a.k_fp8 else 2)
    fused_path = prof["fused"][1] > 0 or Lh == L
    scan_ms, scan_n = prof["fused"] if fused_path else prof["kscan"]
    full_ms, full_n = prof["full"]
    gat_ms, gat_n = prof["fused"] if fused_path else prof["gather"]
    sel_ms, sel_n = prof["select"]
    Lk = L - Lh                       # layers on the KCache path
    scan_gbps = k_bytes_layer * Lk * a.steps / (scan_ms * 1e-3) / 1e9 if scan_ms else 0.0
    gather_gbps = v_bytes_layer * Lk * a.steps / (gat_ms * 1e-3) / 1e9 if gat_ms else 0.0
    full_gbps = 2 * k_bytes_layer * Lh * a.steps / (full_ms * 1e-3) / 1e9 if full_ms else 0.0

    # ---- measured denominators
    probes = {}
    if not a.no_probes:
        kflat = caches[0].k.view(-1)
        probes["hbm_stream_read_GBps"] = ctx.probe_read(kflat, iters=5)
    if not a.no_probes and Lk > 0:
        vflat = caches[-1].v.view(-1)
        n1g = min(vflat.numel(), (1 << 30) // 2)
        stage = torch.empty(n1g, dtype=dt, device=dev)
        # the boxes pin little more than the 64 GiB of V that config 2 needs (a 66th GiB is
        # refused): the device-to-host probe gets by with a 256 MiB target
        n256m = min(n1g, (1 << 28) // 2)
        pinned = torch.empty(n256m, dtype=dt, pin_memory=True)
        probes["h2d_pinned_copy_GBps"] = ctx.probe_copy(stage, vflat[:n1g], iters=5)
        probes["d2h_pinned_copy_GBps"] = ctx.probe_copy(pinned, stage[:n256m], iters=20)
        probes["zerocopy_stream_read_GBps"] = ctx.probe_read(vflat[:n1g], iters=3)
        probes["zerocopy_row_read_GBps"] = ctx.probe_rows(vflat, 1 << 20, iters=3)
        del stage, pinned

    # HBM traffic per launch measured offline with rocprofv3 counters (null if this
    # workload / path has no committed counter run)
    traffic = None
    try:
        tj = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
        path = "conventional" if Lh == L else "fused" if fused_path else "unfused"
        ent = tj.get("%s/%s" % (wl.name, path))
        if ent and L == wl.L and Lh in (0, L) and not a.k_fp8:
            traffic = ent["fetch_bytes_per_launch"] + ent["write_bytes_per_launch"]
    except (OSError, ValueError, KeyError):
        traffic = None

    if Lh == L:   # the conventional baseline: the dominant kernel is the K + V stream
        roofline = {"bound": "hbm", "kernel": "full_kernel", "achieved": full_gbps,
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": full_gbps / HBM_PEAK_GBPS,
                    "traffic": traffic, "bytes_per_launch": 2.0 * k_bytes_layer,
                    "avg_launch_ms": full_ms / max(full_n, 1), "launches": full_n}
    else:
        roofline = {
            "bound": "hbm", "kernel": "fused_kernel" if fused_path else "kscan_kernel",
            "achieved": scan_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": scan_gbps / HBM_PEAK_GBPS,
            "traffic": traffic,
            "bytes_per_launch": k_bytes_layer * Lk * a.steps / max(scan_n, 1),
            "avg_launch_ms": scan_ms / max(scan_n, 1), "launches": scan_n,
        }
    result = {
        "metric": "KCache decode-attn tokens/s" if Lh < L else
                  "conventional KV-cache decode-attn tokens/s",
        "value": wl.B / sec_per_step,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": sec_per_step * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": wl.name, "layers": L, "batch": wl.B, "q_heads": wl.H,
                   "kv_heads": wl.Hkv, "head_dim": wl.d, "context": int(lens.max()), "top_n": wl.N,
                   "gather": a.gather, "path": "fused" if fused_path else "unfused",
                   "k_cache": "e4m3, exponent %d" % K_FP8_EXP if a.k_fp8 else wl.dtype,
                   "gqa_dedup": a.gqa_dedup,
                   "pipeline_parts": a.parts, "v_in_hbm_layers": Lh, "step_mode": step_mode,
                   "lanes": a.lanes, "lane_split": a.split if a.lanes > 1 else None,
                   "k_cache_GiB": L * np.prod(shape) * (1 if a.k_fp8 else 2) / 2 ** 30, "setup_s": round(setup_s, 1)},
        "roofline": roofline,
        "v_gather": {
            "kernel": "fused_kernel (whole launch)" if fused_path else "gather_kernel",
            "achieved": gather_gbps, "unit": "GB/s", "bytes_per_step": v_bytes_layer * Lk,
            "avg_launch_ms": gat_ms / max(gat_n, 1), "launches": gat_n,
            "peak_measured_h2d": probes.get("h2d_pinned_copy_GBps"),
            "frac_of_measured": (gather_gbps / probes["h2d_pinned_copy_GBps"]
                                 if probes.get("h2d_pinned_copy_GBps") else None),
            "link_busy_frac_of_step": (v_bytes_layer * Lk / sec_per_step / 1e9 /
                                       probes["h2d_pinned_copy_GBps"]
                                       if probes.get("h2d_pinned_copy_GBps") else None),
        },
        "select": {"avg_launch_ms": sel_ms / max(sel_n, 1), "launches": sel_n},
        "ms_per_step_with_event_profiling": sec_per_step_prof * 1e3,
        "hbm_GBps_of_step": k_bytes_layer * (Lk + 2 * Lh) / sec_per_step / 1e9,
        "full_attention": {"layers": Lh, "kernel": "full_kernel", "achieved": full_gbps,
                           "unit": "GB/s", "bytes_per_launch": 2.0 * k_bytes_layer,
                           "avg_launch_ms": full_ms / max(full_n, 1), "launches": full_n},
        "probes": probes,
        "lanes_2": overlap,
    }

    if a.prefill:
        result["prefill_store"] = prefill_leg(ctx, kc, wl, caches[0], dev, dt)

    if a.crossover and Lk > 0:
        result["crossover"] = crossover_leg(ctx, kc, wl, caches[-1], qs[-1], dev, probes)

    if not a.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, L, Lh, a.cpu_units, a.cpu_passes, outs, idxs, ws,
                                              a.k_fp8)
    print(json.dumps(result))


def prefill_leg(ctx, kc, wl, cache, dev, dt, reps=3):
    """Store of one layer's full context through kcache_prefill_store, timed as a whole
    (wall clock, K and V halves overlapped) and per half (HIP events around each kernel).
    The rows written are the ones already in the cache, so its contents do not change."""
    T = wl.S_cap
    k_new = cache.k.permute(0, 2, 1, 3).contiguous()
    v_new = cache.v.to(dev).permute(0, 2, 1, 3).contiguous()
    pos = torch.zeros(wl.B, dtype=torch.int32, device=dev)
    nbytes = k_new.numel() * k_new.element_size()
    ctx.prefill_store(cache, k_new, v_new, pos)          # warm-up
    ctx.synchronize()
    torch.cuda.synchronize()
    ctx.set_profile(True)
    ctx.profile_reset()
    t = time.perf_counter()
    for _ in range(reps):
        ctx.prefill_store(cache, k_new, v_new, pos)
    ctx.synchronize()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t) / reps
    k_ms, k_n = ctx.profile_read("store_k")
    v_ms, v_n = ctx.profile_read("store_v")
    ctx.set_profile(False)
    return {"tokens_per_layer": wl.B * T, "bytes_each_of_K_and_V": nbytes,
            "ms_per_layer": wall * 1e3,
            "k_to_hbm_GBps": nbytes * k_n / (k_ms * 1e-3) / 1e9 if k_ms else None,
            "v_to_host_GBps": nbytes * v_n / (v_ms * 1e-3) / 1e9 if v_ms else None,
            "note": "K half reads and writes HBM (2 x bytes of traffic); V half is posted PCIe "
                    "writes from the store kernel into the mapped host cache"}


def crossover_leg(ctx, kc, wl, cache, q, dev, probes, reps=10):
    """Break-even of section 3.2: the KCache launch (K from HBM, N rows of V over the host
    link) against conventional attention (K and V from HBM) on one layer of this workload's
    shape, every sequence at length s, for a grid of s and N.  Times are HIP-event averages
    per launch.  Equation (4) predicts KCache to be no slower once s/N exceeds
    BW_HBM / BW_H2D when the two transfers follow each other; a launch that overlaps them
    breaks even at half that ratio."""
    hbm_layer = kc.LayerCache(cache.k, cache.v.to(dev))
    B, H = wl.B, wl.H
    s_grid = [s for s in (1024, 1536, 2048, 3072, 4096, 6144, 8192, 12288, 16384, 24576, 32768,
                          49152, 65536) if s <= wl.S_cap]
    n_grid = [32, 64, 128, 256, 512, 1024]
    out = torch.empty((B, H, wl.d), dtype=torch.float32, device=dev)
    rows = []
    ctx.set_profile(True)
    for s in s_grid:
        lens_dev = torch.full((B,), s, dtype=torch.int32, device=dev)
        ctx.full_attention(hbm_layer, q, lens_dev, out=out)      # warm-up
        ctx.profile_reset()
        for _ in range(reps):
            ctx.full_attention(hbm_layer, q, lens_dev, out=out)
        ms, n = ctx.profile_read("full")
        t_full = ms / n * 1e3
        k_bytes = B * wl.Hkv * s * wl.d * 2
        row = {"s": s, "full_us": round(t_full, 1),
               "full_GBps": round(2 * k_bytes / (t_full * 1e-6) / 1e9, 1), "kcache_us": {}}
        for N in n_grid:
            if N > s:
                continue
            ctx.decode_attention(cache, q, lens_dev, N, out=out)  # warm-up (workspace growth)
            ctx.profile_reset()
            for _ in range(reps):
                ctx.decode_attention(cache, q, lens_dev, N, out=out)
            ms, n = ctx.profile_read("fused")
            row["kcache_us"][str(N)] = round(ms / n * 1e3, 1)
        rows.append(row)
    ctx.set_profile(False)
    ctx.device_check()
    # per N: the ratio s/N at which the two times cross (linear interpolation in s between
    # the neighbouring grid points; None when they do not cross inside the grid)
    wins = {}
    for N in n_grid:
        pts = [(r["s"], r["kcache_us"][str(N)] - r["full_us"]) for r in rows
               if str(N) in r["kcache_us"]]
        wins[str(N)] = None
        for (s0, d0), (s1, d1) in zip(pts, pts[1:]):
            if d0 > 0 >= d1:
                wins[str(N)] = round((s0 + (s1 - s0) * d0 / (d0 - d1)) / N, 1)
                break
    hbm, link = probes.get("hbm_stream_read_GBps"), probes.get("zerocopy_row_read_GBps")
    return {"shape": {"B": B, "H": H, "Hkv": wl.Hkv, "dtype": wl.dtype}, "grid": rows,
            "break_even_s_over_N": wins,
            "eq4_ratio_measured_bandwidths": eq4_break_even(hbm, link) if hbm and link else None,
            "eq4_ratio_with_overlap": (eq4_break_even(hbm, link, overlapped=True)
                                       if hbm and link else None)}


def cpu_baseline(wl, L, Lh, n_units, passes, outs, idxs, ws, k_fp8=False):
    """The CPU oracle, as it stands, on a seeded sample of this workload's units,
    one thread per available core; its results double as a spot check of the GPU
    outputs of the last timed step."""
    import oracle
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from harness import check_unit, dtype_code   # the acceptance rule of the parity tests
    cores = len(os.sched_getaffinity(0))
    rng = np.random.default_rng(wl.seed)
    lens = wl.seq_lens()
    n_units = min(n_units, L * wl.B * wl.H)
    picks = []
    while len(picks) < n_units:
        l, b, h = int(rng.integers(L)), int(rng.integers(wl.B)), int(rng.integers(wl.H))
        if (l, b, h) not in picks:
            picks.append((l, b, h))
    s_max = int(max(lens[b] for _, b, _ in picks))
    q = np.zeros((n_units, 1, wl.d), np.uint16)
    K = np.zeros((n_units, 1, s_max, wl.d), np.uint16)
    V = np.zeros((n_units, 1, s_max, wl.d), np.uint16)
    sl = np.zeros(n_units, np.int32)
    for i, (l, b, h) in enumerate(picks):
        qb, kb, vb = ki.gen_unit(wl, l, b, h)
        q[i, 0], sl[i] = qb, kb.shape[0]
        K[i, 0, :sl[i]], V[i, 0, :sl[i]] = kb, vb
    code = dtype_code(wl)
    t = time.perf_counter()
    for _ in range(passes):
        oracle.decode_attention(q, K, V, code, sl, wl.N, nthreads=cores)
    wall = time.perf_counter() - t
    units_per_step = L * wl.B * wl.H
    step_s = wall / (n_units * passes) * units_per_step
    # the same oracle on one thread, on a few of the same units
    n1 = min(4, n_units)
    t = time.perf_counter()
    oracle.decode_attention(q[:n1], K[:n1], V[:n1], code, sl[:n1], wl.N, nthreads=1)
    wall1 = time.perf_counter() - t
    step_s1 = wall1 / n1 * units_per_step
    # spot check of the GPU results against the oracle's, same acceptance rule as the tests
    checked = identical = 0
    failures = []
    for i, (l, b, h) in enumerate(picks[:16]):
        if l < Lh:   # a layer with V in HBM ran conventional attention
            ref = oracle.full_unit(q[i, 0], K[i, 0, :sl[i]], V[i, 0, :sl[i]], code)
            err = np.abs(outs[l][b, h].cpu().numpy().astype(np.float64) - ref)
            if (err <= 1e-3 + 2e-3 * np.abs(ref)).all():
                checked += 1
                identical += 1
            else:
                failures.append("%s: conventional attention max err %g" % ((l, b, h), err.max()))
            continue
        if k_fp8:
            codes = oracle.e4m3_quantise(K[i, 0, :sl[i]], code, K_FP8_EXP)
            r = oracle.decode_unit_k8(q[i, 0], codes, K_FP8_EXP, V[i, 0, :sl[i]], code, wl.N,
                                      want_scores=True)
        else:
            r = oracle.decode_unit(q[i, 0], K[i, 0, :sl[i]], V[i, 0, :sl[i]], code, wl.N,
                                   want_scores=True)
        r["v"] = oracle.decode16(V[i, 0, :sl[i]], code)
        try:
            identical += check_unit(r, wl.N, outs[l][b, h].cpu().numpy(),
                                    idxs[l][b, h].cpu().numpy(), ws[l][b, h].cpu().numpy())
            checked += 1
        except AssertionError as e:
            failures.append("%s: %s" % ((l, b, h), e))
    return {"value": wl.B / step_s, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "single_thread_value": wl.B / step_s1,
            "sample": "%d of %d (layer, sequence, head) units of %s, regenerated on the host, "
                      "fp64 oracle with %d threads, %d passes, %.2f s wall (%.1f core-seconds); scaled to "
                      "a full step" % (n_units, units_per_step, wl.name, cores, passes, wall,
                                       wall * cores),
            "extrapolated": True,
            "gpu_spot_check": {"units": checked, "index_sets_identical": identical,
                               "failures": failures}}


if __name__ == "__main__":
    main()
