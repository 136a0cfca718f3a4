#!/usr/bin/env python3
"""KCache decode-attention benchmark on one MI355X.

A step is one decode step of the whole hot path over one batch: for every
layer, the new token's K/V rows are stored (T = 1) and KCache attention runs
(K scan over the full context, softmax, top-N, V pull from pinned host memory,
weighted sum).  All inputs are synthetic, seeded, and already resident (K in
HBM, V in pinned host memory) when the timed region starts.  A step is issued
the way the library issues it by default: one launch of a HIP graph captured
from kcache_decode_step, spread over the lanes that KC_OPT_STEP_LANES = 0
chooses (two lanes with half of the batch each where the batch allows it; every
dependency of a real decode step is kept).

Prints one JSON line.  `value` is the whole-job tokens/s of the headline workload
(config 2 unless --config says otherwise).  `roofline` is the HBM roofline of the
dominant kernel, one launch at a time (HIP events around every launch in a second,
eager, single-lane pass of the same steps), with the step-level rates and the
host-link side next to it.  A default run then frees the headline workload and
measures the other four named workloads (`workloads`), the N x pivot-fraction
sweep of the ragged workload (`config4_sweep`) and the prefill store of config 5.
The CPU oracle is timed on a bounded sample of the headline workload.
"""
import argparse
import hashlib
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
SWEEP_N = (32, 64, 128, 256, 512)
SWEEP_FRAC = (0.001, 0.01, 0.05)


def algorithmic_bytes(wl, lens, k_elem_bytes=2, N=None):
    """Bytes one layer of a decode step has to move, whatever the implementation (Table 1):
    the K rows of every cached position from HBM (the 2bnhs term of the S~ row) and the N
    kept V rows of every query head over the host link (the 2bNd term of the A~ row)."""
    lens = np.asarray(lens, dtype=np.int64)
    N = wl.N if N is None else N
    k_bytes = int(lens.sum()) * wl.Hkv * wl.d * k_elem_bytes
    v_bytes = int(np.minimum(lens, N).sum()) * wl.H * wl.d * 2
    return k_bytes, v_bytes


def eq4_break_even(bw_gpu, bw_h2d, overlapped=False, G=1):
    """s/N above which KCache is no slower than a conventional KV cache (section 3.2,
    equation (4)): Bandwidth_GPU / Bandwidth_H2D when the V pull follows the K scan; half of
    it when the two overlap (N rows over the link then only have to beat 2 s rows from HBM).
    G query heads per KV head (the paper writes the condition for G = 1): the HBM side reads a
    position once per group while every query head pulls its own N rows, so the ratio grows
    G-fold."""
    return G * bw_gpu / bw_h2d / (2.0 if overlapped else 1.0)


def launch_floor_us(wl, lens, N, hbm_gbps, link_gbps, k_elem_bytes=2):
    """Lower bound of one layer's launch when the two transfers overlap perfectly: the larger
    of K bytes / HBM rate and V-row bytes / link rate (section 3.2, equation (3), read with
    overlap).  Returns (floor_us, hbm_us, link_us)."""
    k_bytes, v_bytes = algorithmic_bytes(wl, lens, k_elem_bytes, N)
    t_hbm = k_bytes / (hbm_gbps * 1e9) * 1e6
    t_link = v_bytes / (link_gbps * 1e9) * 1e6
    return max(t_hbm, t_link), t_hbm, t_link


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="headline workload of BASELINE.json (1-5); 6 = the shape of "
                         "the paper's Table 4 headline row (batch 5, 16k context, N 128), 7 = grouped queries "
                         "where the K scan binds (config 3's model, batch 32, 32k context, N 32); both for context")
    ap.add_argument("--only", action="store_true",
                    help="measure the headline workload only (no other workloads, no sweep)")
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
                         "V device-to-host) alone and under a concurrent decode launch, reported "
                         "under \"prefill_store\" (always on for config 5 in a default run)")
    ap.add_argument("--sweep", action="store_true",
                    help="config 4: time one layer over N in {32..512} x pivot fraction in "
                         "{0.1, 1, 5} %%, reported under \"config4_sweep\" (always on in a default run)")
    ap.add_argument("--step-mode", choices=["graph", "step", "calls"], default="graph",
                    help="how a decode step is issued: one captured HIP graph launch (default), "
                         "one kcache_decode_step call, or per-layer store + attention calls")
    ap.add_argument("--lanes", type=int, default=0,
                    help="streams a step is spread over; 0 = the library's own choice (default)")
    ap.add_argument("--split", choices=["sequences", "layers"], default="sequences",
                    help="what explicitly requested lanes hold: a share of the batch each, run through "
                         "all layers in order (keeps every dependency of a real decode step), or "
                         "whole layers dealt round-robin (only meaningful for the attention in isolation)")
    ap.add_argument("--no-overlap-leg", action="store_true",
                    help="skip the extra timed passes with other lane counts reported under lane_modes")
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


class PinnedPool:
    """One pinned host allocation shared by the workloads of a run.  The GPU machines pin little
    more than 65 GiB, and torch rounds each pinned request up to a power of two, so the V
    caches of all layers of a workload are views into one buffer that later workloads reuse."""

    def __init__(self):
        self.buf = None

    def get(self, n_elems, dtype):
        need = n_elems * 2
        if self.buf is None:
            self.buf = torch.empty(need // 2, dtype=torch.int16, pin_memory=True)
        if self.buf.numel() * 2 < need:
            raise RuntimeError("pinned pool of %d bytes is smaller than the %d bytes asked for; "
                               "run the largest workload first" % (self.buf.numel() * 2, need))
        return self.buf[:n_elems].view(dtype)


class Workload:
    """Resident state of one workload: per layer K cache (HBM), V cache (pinned host, or HBM for
    the first Lh layers), q, the new token's rows and the outputs."""

    def __init__(self, ctx, kc, wl, L, Lh, pool, dev, k_fp8=False):
        self.wl, self.L, self.Lh, self.k_fp8 = wl, L, Lh, k_fp8
        dt = ki.torch_dtype(wl.dtype)
        self.dt = dt
        self.lens = wl.seq_lens()
        self.lens_dev = torch.from_numpy(self.lens).to(dev)
        self.pos_last = torch.from_numpy(self.lens - 1).to(dev)
        t0 = time.time()
        self.caches, self.qs, self.k_tok, self.v_tok = [], [], [], []
        shape = (wl.B, wl.Hkv, wl.S_cap, wl.d)
        self.shape = shape
        T_chunk = min(wl.S_cap, 8192)
        hks = list(range(wl.Hkv))
        layer_elems = int(np.prod(shape))
        v_all = pool.get(max(L - Lh, 1) * layer_elems, dt)
        for layer in range(L):
            k_cache = torch.empty(shape, dtype=torch.uint8 if k_fp8 else dt, device=dev)
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
                kt[b, 0] = k[:, self.lens[b] - 1]
                vt[b, 0] = v[:, self.lens[b] - 1]
                ctx.synchronize()
                torch.cuda.synchronize()
                del alive
            self.caches.append(cache)
            self.qs.append(ki.gen_q(wl, layer, dev))
            self.k_tok.append(kt)
            self.v_tok.append(vt)
        ctx.device_check()
        self.setup_s = time.time() - t0
        self.alloc_outputs(wl.N, dev)

    def alloc_outputs(self, N, dev):
        wl, L = self.wl, self.L
        self.outs = [torch.empty((wl.B, wl.H, wl.d), dtype=torch.float32, device=dev) for _ in range(L)]
        self.idxs = [torch.empty((wl.B, wl.H, N), dtype=torch.int32, device=dev) for _ in range(L)]
        self.ws = [torch.empty((wl.B, wl.H, N), dtype=torch.float32, device=dev) for _ in range(L)]
        self.step_layers = [dict(cache=self.caches[l], k_new=self.k_tok[l], v_new=self.v_tok[l],
                                 q=self.qs[l], out=self.outs[l], idx_out=self.idxs[l],
                                 w_out=self.ws[l]) for l in range(L)]

    def release(self):
        for name in ("caches", "qs", "k_tok", "v_tok", "outs", "idxs", "ws", "step_layers"):
            setattr(self, name, None)
        torch.cuda.empty_cache()


def reserve_for(ctx, kc, st, N, mode):
    """Sizes the context for everything the timed passes of this workload call (the library
    refuses to grow inside a call unless told to): single-layer calls and whole steps at
    every lane setting the benchmark uses."""
    wl = st.wl
    for lanes, seqs in ((0, True), (1, True), (2, True), (2, False)):
        ctx.set_step_lanes(lanes, split_sequences=seqs)
        for cache in {id(c): c for c in (st.caches[0], st.caches[-1])}.values():
            ctx.reserve(cache, wl.H, N, gather_mode=mode, step_layers=st.L)
    ctx.set_step_lanes(0, split_sequences=True)


def measure(ctx, kc, st, a, probes, dev, headline):
    """Times the decode step of one resident workload.  Returns the result dict (the keys of the
    JSON line for the headline workload; a compact subset is taken from it for the others)."""
    wl, L, Lh, lens = st.wl, st.L, st.Lh, st.lens
    mode = kc.GATHER_ZEROCOPY if a.gather == "zerocopy" else kc.GATHER_STAGED
    plain = mode == kc.GATHER_ZEROCOPY and not a.unfused   # what the step calls implement
    step_mode = a.step_mode if plain else "calls"
    reserve_for(ctx, kc, st, wl.N, mode)
    allocs_before = ctx.stat(kc.STAT_REALLOCS)

    def set_lanes(lanes, split="sequences"):
        ctx.set_step_lanes(lanes, split_sequences=(split == "sequences"))

    def step_calls():
        for l in range(L):
            ctx.prefill_store(st.caches[l], st.k_tok[l], st.v_tok[l], st.pos_last)
            if l < Lh:
                ctx.full_attention(st.caches[l], st.qs[l], st.lens_dev, out=st.outs[l])
            else:
                ctx.decode_attention(st.caches[l], st.qs[l], st.lens_dev, wl.N, out=st.outs[l],
                                     idx_out=st.idxs[l], w_out=st.ws[l], gather_mode=mode)

    def step_eager():
        ctx.decode_step(st.step_layers, wl.H, st.pos_last, st.lens_dev, wl.N)

    def timed(step, n):
        torch.cuda.synchronize()
        ctx.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            step()
        ctx.synchronize()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / n

    def time_mode(lanes, split):
        """Seconds per step with the step issued in `step_mode` at this lane setting."""
        set_lanes(lanes, split)
        used = ctx.step_lanes_for(st.caches[-1], L, wl.H)
        if step_mode == "graph":
            g = ctx.step_graph(st.step_layers, wl.H, st.pos_last, st.lens_dev, wl.N)
            step = g.launch
        else:
            g = None
            step = step_eager if step_mode == "step" else step_calls
        for _ in range(a.warmup):
            step()
        sec = timed(step, a.steps)
        if g is not None:
            g.close()
        return sec, used

    # ---- other lane settings, for comparison (timed first: they also bring the part to its
    # steady clocks before the headline pass)
    lane_modes = None
    if plain and not a.no_overlap_leg and a.lanes == 0 and step_mode != "calls":
        lane_modes = {}
        sec1, _ = time_mode(1, "sequences")
        lane_modes["one_lane"] = {"ms_per_step": sec1 * 1e3, "tokens_per_s": wl.B / sec1}
        if headline and L > 1:
            sec2, _ = time_mode(2, "layers")
            lane_modes["two_lanes_layers_alternating"] = {
                "ms_per_step": sec2 * 1e3, "tokens_per_s": wl.B / sec2,
                "note": "whole layers alternate between two streams: only meaningful for the "
                        "attention in isolation (in a model layer l+1's query depends on layer l)"}
        if wl.B >= 4 and headline:
            sec4, used4 = time_mode(4, "sequences")
            lane_modes["four_lanes_sequences"] = {"ms_per_step": sec4 * 1e3,
                                                  "tokens_per_s": wl.B / sec4}

    # ---- the headline timing: the library's default issue of a step
    sec_per_step, lanes_used = time_mode(a.lanes, a.split)

    # ---- second pass of the same steps, one lane, eager, with HIP events around every
    # kernel launch (events are not part of a captured graph; one launch at a time, so a
    # launch's duration is the kernel's own)
    set_lanes(1)
    ctx.set_profile(True)
    ctx.profile_reset()
    sec_per_step_prof = timed(step_eager if plain else step_calls, a.steps)
    prof = {k: ctx.profile_read(k) for k in kc.KERNELS}
    ctx.set_profile(False)
    set_lanes(0)
    ctx.device_check()
    grown = ctx.stat(kc.STAT_REALLOCS) - allocs_before

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

    # ---- measured denominators (taken once per run, on the first workload that can)
    if not a.no_probes and "hbm_stream_read_GBps" not in probes and \
            st.caches[0].k.numel() * st.caches[0].k.element_size() >= (1 << 28):
        probes["hbm_stream_read_GBps"] = ctx.probe_read(st.caches[0].k.view(-1), iters=5)
    if not a.no_probes and Lk > 0 and "h2d_pinned_copy_GBps" not in probes and \
            st.caches[-1].v.numel() >= (1 << 27):
        vflat = st.caches[-1].v.view(-1)
        n1g = min(vflat.numel(), (1 << 30) // 2)
        stage = torch.empty(n1g, dtype=st.dt, device=dev)
        # the boxes pin little more than the 64 GiB of V that config 2 needs (a 66th GiB is
        # refused): the device-to-host probe gets by with a 256 MiB target
        n256m = min(n1g, (1 << 28) // 2)
        pinned = torch.empty(n256m, dtype=st.dt, pin_memory=True)
        probes["h2d_pinned_copy_GBps"] = ctx.probe_copy(stage, vflat[:n1g], iters=5)
        probes["d2h_pinned_copy_GBps"] = ctx.probe_copy(pinned, stage[:n256m], iters=20)
        probes["zerocopy_stream_read_GBps"] = ctx.probe_read(vflat[:n1g], iters=3)
        probes["zerocopy_row_read_GBps"] = ctx.probe_rows(vflat, 1 << 20, iters=3)
        del stage, pinned
    h2d = probes.get("h2d_pinned_copy_GBps")

    # HBM traffic per launch from the committed rocprofv3 counter runs: an OFFLINE figure,
    # valid for the kernel source it was measured on (null when the source has changed)
    traffic, traffic_src = None, None
    try:
        tj = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
        path = "conventional" if Lh == L else "fused" if fused_path else "unfused"
        ent = tj.get("%s/%s" % (wl.name, path))
        if ent and L == wl.L and Lh in (0, L) and not a.k_fp8:
            traffic_src = {"summary": ent.get("summary"), "kernel_source_sha16": ent.get("kernel_source_sha16"),
                           "current_kernel_source_sha16": kernel_source_hash()}
            if ent.get("kernel_source_sha16") == kernel_source_hash():
                traffic = ent["fetch_bytes_per_launch"] + ent["write_bytes_per_launch"]
    except (OSError, ValueError, KeyError):
        traffic = None

    k_step, v_step = k_bytes_layer * (Lk + 2 * Lh), v_bytes_layer * Lk
    step_hbm_gbps = k_step / sec_per_step / 1e9
    step_link_gbps = v_step / sec_per_step / 1e9
    floor_us, hbm_us, link_us = launch_floor_us(wl, lens, wl.N, HBM_PEAK_GBPS, h2d or 57.0,
                                                1 if a.k_fp8 else 2)
    binding = "hbm" if hbm_us >= link_us or Lk == 0 else "host_link"
    avg_launch_ms = (full_ms / max(full_n, 1)) if Lh == L else (scan_ms / max(scan_n, 1))
    link_part = {
        "achieved": gather_gbps, "peak": h2d, "unit": "GB/s",
        "frac": gather_gbps / h2d if h2d else None,
        "note": "V-row bytes of a launch / the same launch duration, against the pinned "
                "host-to-device copy rate measured in this run"}
    if wl.G > 1 and Lk > 0 and fused_path:
        # heads of a group that keep the same position: the caches can serve the repeats, so
        # the link carries between the distinct rows and all rows
        ix = st.idxs[L - 1].view(wl.B, wl.Hkv, wl.G * wl.N).to(torch.int64)
        srt = torch.sort(ix, dim=-1).values
        distinct = ((srt[..., 1:] != srt[..., :-1]) & (srt[..., 1:] >= 0)).sum() + (srt[..., 0] >= 0).sum()
        kept = (ix >= 0).sum()
        uf = float(distinct) / max(int(kept), 1)
        link_part["distinct_row_frac"] = uf
        link_part["achieved_distinct_rows"] = gather_gbps * uf
        link_part["frac_distinct_rows"] = gather_gbps * uf / h2d if h2d else None
        link_part["note"] += ("; distinct_row_frac: distinct positions among the rows the heads of a "
                              "group keep (last layer of the last step); a repeat may be served by the "
                              "caches, so the link carried between achieved_distinct_rows and achieved")
    if Lh == L:   # the conventional baseline: the dominant kernel is the K + V stream
        roofline = {"bound": "hbm", "kernel": "full_kernel", "achieved": full_gbps,
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": full_gbps / HBM_PEAK_GBPS,
                    "traffic": traffic, "traffic_offline": traffic_src,
                    "bytes_per_launch": 2.0 * k_bytes_layer,
                    "avg_launch_ms": avg_launch_ms, "launches": full_n}
    else:
        roofline = {
            "bound": "hbm", "kernel": "fused_kernel" if fused_path else "kscan_kernel",
            "achieved": scan_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": scan_gbps / HBM_PEAK_GBPS,
            "traffic": traffic, "traffic_offline": traffic_src,
            "bytes_per_launch": k_bytes_layer * Lk * a.steps / max(scan_n, 1),
            "avg_launch_ms": avg_launch_ms, "launches": scan_n,
            "how": "one launch at a time: single-lane eager pass, HIP events on the launch stream",
            "host_link": link_part,
            "binding_resource": binding,
            "binding_note": "floors of one launch at the published HBM peak and the measured link "
                            "rate: K %.0f us, V rows %.0f us; the larger one names the resource that "
                            "binds this workload" % (hbm_us, link_us),
            "step": {"hbm_achieved": step_hbm_gbps, "hbm_frac": step_hbm_gbps / HBM_PEAK_GBPS,
                     "link_achieved": step_link_gbps,
                     "link_frac": step_link_gbps / h2d if h2d else None,
                     "how": "bytes of a whole step / ms_per_step of the timed (default-issue) pass: "
                            "K bytes %d, V-row bytes %d" % (k_step, v_step)},
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
                   "lanes": lanes_used, "lanes_requested": a.lanes,
                   "lane_split": "sequences" if a.lanes == 0 else a.split,
                   "k_cache_GiB": L * np.prod(st.shape) * (1 if a.k_fp8 else 2) / 2 ** 30,
                   "setup_s": round(st.setup_s, 1)},
        "roofline": roofline,
        "v_gather": {
            "kernel": "fused_kernel (whole launch)" if fused_path else "gather_kernel",
            "achieved": gather_gbps, "unit": "GB/s", "bytes_per_step": v_step,
            "avg_launch_ms": gat_ms / max(gat_n, 1), "launches": gat_n,
            "peak_measured_h2d": h2d,
            "frac_of_measured": gather_gbps / h2d if h2d else None,
            "link_busy_frac_of_step": step_link_gbps / h2d if h2d else None,
        },
        "select": {"avg_launch_ms": sel_ms / max(sel_n, 1), "launches": sel_n},
        "ms_per_step_with_event_profiling": sec_per_step_prof * 1e3,
        "hbm_GBps_of_step": step_hbm_gbps,
        "full_attention": {"layers": Lh, "kernel": "full_kernel", "achieved": full_gbps,
                           "unit": "GB/s", "bytes_per_launch": 2.0 * k_bytes_layer,
                           "avg_launch_ms": full_ms / max(full_n, 1), "launches": full_n},
        "probes": dict(probes),
        "lane_modes": lane_modes,
        "context_growth_inside_timed_calls": grown,
    }
    return result


_KHASH = None


def kernel_source_hash():
    """Hash of the kernel sources an offline counter run belongs to."""
    global _KHASH
    if _KHASH is None:
        h = hashlib.sha256()
        csrc = os.path.join(ROOT, "paper_2404_18057_amd", "csrc")
        for name in ("decode_fused.hip", "full_attention.hip", "attn_common.h", "topn.h",
                     "kc_internal.h"):
            h.update(open(os.path.join(csrc, name), "rb").read())
        _KHASH = h.hexdigest()[:16]
    return _KHASH


def compact(r, spot):
    """What the line keeps of a non-headline workload."""
    rf = r["roofline"]
    bound = rf.get("binding_resource", "hbm")
    link = rf.get("host_link") or {}
    return {
        "ms_per_step": r["ms_per_step"], "tokens_per_s": r["value"],
        "lanes": r["config"]["lanes"], "layers": r["config"]["layers"], "dtype": r["dtype"],
        "one_lane_ms_per_step": (r["lane_modes"] or {}).get("one_lane", {}).get("ms_per_step"),
        "kernel": rf["kernel"], "kernel_us_per_launch": rf["avg_launch_ms"] * 1e3,
        "k_bytes_per_launch": rf["bytes_per_launch"],
        "K_GBps_per_launch": rf["achieved"], "V_row_GBps_per_launch": link.get("achieved"),
        "bound": bound,
        # grouped queries: the link carried at least the distinct rows of every group (a repeat
        # may come from the caches), so the lower bound is the figure that cannot overstate
        "frac_of_bound": (rf["frac"] if bound == "hbm" else
                          link.get("frac_distinct_rows") or link.get("frac")),
        "hbm_frac": rf["frac"], "link_frac": link.get("frac"),
        "distinct_row_frac": link.get("distinct_row_frac"),
        "link_frac_distinct_rows": link.get("frac_distinct_rows"),
        "step_hbm_frac": rf.get("step", {}).get("hbm_frac"),
        "step_link_frac": rf.get("step", {}).get("link_frac"),
        "binding_note": rf.get("binding_note"),
        "context_growth_inside_timed_calls": r["context_growth_inside_timed_calls"],
        "setup_s": r["config"]["setup_s"],
        "oracle_spot_check": spot,
    }


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

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    # the context is sized with kcache_reserve before the timed passes; with auto_grow off the
    # library refuses (rather than synchronises) should a timed call still need more
    ctx = kc.Context(0, auto_grow=False)
    ctx.set_pipeline_parts(a.parts)
    ctx.set_fused(not a.unfused)
    ctx.set_fused_rows(a.rows)
    ctx.set_gqa_dedup(a.gqa_dedup)
    pool = PinnedPool()
    probes = {}

    wl = ki.config(a.config)
    if a.shared_pivots:
        wl = wl.replace(shared_pivots=True, name=wl.name + "_shared_pivots")
    L = a.layers if a.layers > 0 else wl.L
    Lh = L if a.hbm_layers < 0 else min(a.hbm_layers, L)   # layers with V in HBM
    variant = a.unfused or a.gather != "zerocopy" or a.k_fp8 or a.hbm_layers != 0 or a.layers > 0 \
        or a.shared_pivots or a.gqa_dedup or a.rows or a.parts or a.lanes != 0 or a.step_mode != "graph"
    all_workloads = a.config == 2 and not a.only and not variant

    st = Workload(ctx, kc, wl, L, Lh, pool, dev, a.k_fp8)
    result = measure(ctx, kc, st, a, probes, dev, headline=True)
    if a.prefill:
        result["prefill_store"] = prefill_leg(ctx, kc, st, dev)
    if a.sweep and a.config == 4:
        result["config4_sweep"] = sweep_leg(ctx, kc, a, pool, dev, probes, first=st)
    if a.crossover and L - Lh > 0:
        ctx.set_option(9, 1)   # this leg walks over many shapes: let the context follow (KC_OPT_AUTO_GROW)
        result["crossover"] = crossover_leg(ctx, kc, wl, st.caches[-1], st.qs[-1], dev, probes)
        ctx.set_option(9, 0)
    if not a.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, L, Lh, a.cpu_units, a.cpu_passes, st.outs, st.idxs,
                                              st.ws, a.k_fp8)

    if all_workloads:
        st.release()
        others = {}
        for cfg in (1, 3, 4, 5):
            w2 = ki.config(cfg)
            t0 = time.time()
            s2 = Workload(ctx, kc, w2, w2.L, 0, pool, dev)
            r2 = measure(ctx, kc, s2, a, probes, dev, headline=False)
            spot = spot_check(w2, w2.L, s2.outs, s2.idxs, s2.ws, 16)
            ent = compact(r2, spot)
            if cfg == 5:
                ent["prefill_store"] = prefill_leg(ctx, kc, s2, dev)
            if cfg == 4:
                result["config4_sweep"] = sweep_leg(ctx, kc, a, pool, dev, probes, first=s2)
            ent["wall_s"] = round(time.time() - t0, 1)
            others[w2.name] = ent
            s2.release()
        result["workloads"] = others
        # not one of the named workloads: grouped queries where the K scan binds (the named
        # grouped-query workload, config 3, is bound by the host link), so that the line also
        # holds the grouped-query kernel against the HBM roofline
        w7 = ki.config(7)
        t0 = time.time()
        s7 = Workload(ctx, kc, w7, w7.L, 0, pool, dev)
        r7 = measure(ctx, kc, s7, a, probes, dev, headline=False)
        ent = compact(r7, spot_check(w7, w7.L, s7.outs, s7.idxs, s7.ws, 16))
        ent["wall_s"] = round(time.time() - t0, 1)
        result["context_workloads"] = {w7.name: ent}
        s7.release()
        result["probes"] = dict(probes)
    print(json.dumps(result))


def prefill_leg(ctx, kc, st, dev, reps=3):
    """Store of one layer's full context (Figure 1, upper half: K rows to the HBM cache, V rows
    device-to-host) in both forms the library offers - kcache_prefill_store (positions in device
    memory, V half by a kernel that writes into the mapped host cache) and
    kcache_prefill_store_at (positions on the host, V half by the copy engine) - each timed
      alone      as a whole (wall clock, K and V halves overlapped) and per half (HIP events);
      together   with attention launches of another layer running on a second context and
                 stream while the V half is in flight: section 3.2, equations (1)-(2), asks
                 that layer i's device-to-host copy hides under layer i+1's work, so neither
                 may slow the other down.
    The rows written are the ones already in the cache, so its contents do not change."""
    wl, cache = st.wl, st.caches[0]
    T = wl.S_cap
    k_new = cache.k.permute(0, 2, 1, 3).contiguous()
    v_new = cache.v.to(dev).permute(0, 2, 1, 3).contiguous()
    pos = torch.zeros(wl.B, dtype=torch.int32, device=dev)
    pos_host = [0] * wl.B
    nbytes = k_new.numel() * k_new.element_size()
    # for scale: a plain device-to-device copy of the same bytes (read + write traffic of the
    # same size as the K half, no relayout)
    scratch = torch.empty_like(k_new)
    d2d = ctx.probe_copy(scratch, k_new, iters=5)
    del scratch
    out = {"tokens_per_layer": wl.B * T, "bytes_each_of_K_and_V": nbytes,
           "plain_device_copy_GBps": d2d}
    if st.L > 1:
        other = st.caches[-1]
        q, lens = st.qs[-1], st.lens_dev
        o = torch.empty((wl.B, wl.H, wl.d), dtype=torch.float32, device=dev)
        other_hbm = kc.LayerCache(other.k, other.v.to(dev))
        ctx2 = kc.Context(0, auto_grow=False)
        ctx2.reserve(other, wl.H, wl.N)
        ctx2.reserve(other_hbm, wl.H, wl.N)
        side = torch.cuda.Stream()
        legs = {
            # HBM-heavy work with no host traffic: stands in for the next layer's compute
            "with_concurrent_hbm_attention": (
                "full", lambda: ctx2.full_attention(other_hbm, q, lens, out=o, stream=side),
                "conventional attention of another layer (K and V rows streamed from HBM, no "
                "host traffic) on a second stream: the stand-in for layer i+1's compute"),
            # the KCache decode launch also pulls V rows host-to-device while the store pushes
            # rows device-to-host
            "with_concurrent_kcache_decode": (
                "fused", lambda: ctx2.decode_attention(other, q, lens, wl.N, out=o, stream=side),
                "fused KCache launches of another layer (K scan from HBM + V-row pulls "
                "host-to-device) on a second stream: what a decode step of other sequences "
                "would add while a prompt is being stored"),
        }
    else:
        legs = {}
    forms = {"kernel_store": lambda: ctx.prefill_store(cache, k_new, v_new, pos),
             "copy_engine_store": lambda: ctx.prefill_store_at(cache, k_new, v_new, pos_host)}
    for form, store in forms.items():
        store()                                              # warm-up
        ctx.synchronize()
        torch.cuda.synchronize()
        ctx.set_profile(True)
        ctx.profile_reset()
        t = time.perf_counter()
        for _ in range(reps):
            store()
            ctx.synchronize()                                # one store at a time
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t) / reps
        k_ms, k_n = ctx.profile_read("store_k")
        v_ms, v_n = ctx.profile_read("store_v")
        ent = {"ms_per_layer": wall * 1e3,
               "k_to_hbm_GBps": nbytes * k_n / (k_ms * 1e-3) / 1e9 if k_ms else None,
               "v_to_host_GBps": nbytes * v_n / (v_ms * 1e-3) / 1e9 if v_ms else None}
        store_v_ms = v_ms / max(v_n, 1)
        for name, (kern, launch, what) in legs.items():
            ctx2.set_profile(True)
            for _ in range(3):
                launch()
            ctx2.profile_reset()
            for _ in range(20):
                launch()
            ms, n = ctx2.profile_read(kern)
            alone_us = ms / n * 1e3
            # both at once: the store first, then launches for about 80 % of its V half
            n_att = max(8, int(0.8 * store_v_ms / (alone_us * 1e-3)))
            ctx.profile_reset()
            ctx2.profile_reset()
            store()
            for _ in range(n_att):
                launch()
            ctx.synchronize()
            ctx2.synchronize()
            torch.cuda.synchronize()
            k2_ms, k2_n = ctx.profile_read("store_k")
            v2_ms, v2_n = ctx.profile_read("store_v")
            d_ms, d_n = ctx2.profile_read(kern)
            ctx2.set_profile(False)
            ent[name] = {
                "launches": d_n,
                "attention_us_alone": alone_us, "attention_us_together": d_ms / d_n * 1e3,
                "v_to_host_GBps_together": nbytes * v2_n / (v2_ms * 1e-3) / 1e9 if v2_ms else None,
                "k_to_hbm_GBps_together": nbytes * k2_n / (k2_ms * 1e-3) / 1e9 if k2_ms else None,
                "what": "V half of one layer's store together with " + what}
        ctx.set_profile(False)
        out[form] = ent
    if legs:
        ctx2.close()
    out["note"] = ("K half reads and writes HBM (2 x bytes of traffic).  kernel_store: V half as "
                   "posted PCIe writes from a store kernel into the mapped host cache; "
                   "copy_engine_store: V half as one strided device-to-host copy per (sequence, "
                   "KV head) issued to the copy engine")
    return out


def sweep_leg(ctx, kc, a, pool, dev, probes, first=None, reps=10):
    """Config 4 (64 ragged sequences, one layer): one launch timed for every N in {32..512} and
    pivot fraction in {0.1, 1, 5} % (HIP events, average of `reps` launches after a warm-up).
    Table 4 of the paper shows throughput falling as N grows; here the launch time follows the
    larger of the K-scan floor (independent of N) and the V-row floor (proportional to N)."""
    rows = []
    base = ki.config(4)
    h2d = probes.get("h2d_pinned_copy_GBps") or 57.0
    # the resident workload first: the others are placed into the same pinned memory
    fracs = sorted(SWEEP_FRAC, key=lambda f: not (first is not None and first.wl.pivot_frac == f))
    for frac in fracs:
        wl = base.replace(pivot_frac=frac)
        if first is not None and first.wl.pivot_frac == frac:
            st, own = first, False
        else:
            st, own = Workload(ctx, kc, wl, 1, 0, pool, dev), True
        cache, q, lens_dev = st.caches[0], st.qs[0], st.lens_dev
        for N in SWEEP_N:
            ctx.reserve(cache, wl.H, N)
            out = torch.empty((wl.B, wl.H, wl.d), dtype=torch.float32, device=dev)
            for _ in range(10):      # warm-up (the first launches over a new cache run slower)
                ctx.decode_attention(cache, q, lens_dev, N, out=out)
            ctx.set_profile(True)
            ctx.profile_reset()
            for _ in range(reps):
                ctx.decode_attention(cache, q, lens_dev, N, out=out)
            ms, n = ctx.profile_read("fused")
            ctx.set_profile(False)
            us = ms / n * 1e3
            k_bytes, v_bytes = algorithmic_bytes(wl, st.lens, 2, N)
            floor, hbm_us, link_us = launch_floor_us(wl, st.lens, N, HBM_PEAK_GBPS, h2d)
            rows.append({"pivot_frac": frac, "N": N, "kernel_us": round(us, 1),
                         "tokens_per_s": round(wl.B / (us * 1e-6), 1),
                         "K_GBps": round(k_bytes / us / 1e3, 1), "V_row_GBps": round(v_bytes / us / 1e3, 2),
                         "floor_us": round(floor, 1),
                         "bound": "hbm" if hbm_us >= link_us else "host_link"})
        ctx.device_check()
        if own:
            st.release()
    rows.sort(key=lambda r: (r["pivot_frac"], r["N"]))
    return {"workload": base.name, "layers": 1, "batch": base.B, "reps": reps, "rows": rows,
            "note": "one fused launch (one layer) per cell; tokens_per_s = batch / launch time"}


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
                                       if hbm and link else None),
            "eq4_ratio_with_overlap_for_this_group_size": (
                eq4_break_even(hbm, link, overlapped=True, G=wl.G) if hbm and link else None)}


def pick_units(wl, L, n_units):
    rng = np.random.default_rng(wl.seed)
    n_units = min(n_units, L * wl.B * wl.H)
    picks = []
    while len(picks) < n_units:
        l, b, h = int(rng.integers(L)), int(rng.integers(wl.B)), int(rng.integers(wl.H))
        if (l, b, h) not in picks:
            picks.append((l, b, h))
    return picks


def spot_check(wl, L, outs, idxs, ws, n_units):
    """Oracle check of n_units seeded (layer, sequence, head) units of the last timed step,
    with the acceptance rule of the parity tests; units are regenerated on the host."""
    import concurrent.futures as cf
    import oracle
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from harness import check_unit, dtype_code
    picks = pick_units(wl, L, n_units)
    code = dtype_code(wl)
    host = {}
    for l in {l for l, _, _ in picks}:
        host[l] = (outs[l].cpu().numpy(), idxs[l].cpu().numpy(), ws[l].cpu().numpy())

    def one(p):
        l, b, h = p
        qb, kb, vb = ki.gen_unit(wl, l, b, h)
        r = oracle.decode_unit(qb, kb, vb, code, wl.N, want_scores=True)
        r["v"] = oracle.decode16(vb, code)
        o, i, w = host[l]
        try:
            return check_unit(r, wl.N, o[b, h], i[b, h], w[b, h]), None
        except AssertionError as e:
            return False, "%s: %s" % (p, e)

    with cf.ThreadPoolExecutor(max_workers=max(1, min(16, len(os.sched_getaffinity(0))))) as ex:
        res = list(ex.map(one, picks))
    failures = [f for _, f in res if f]
    return {"units": len(picks) - len(failures), "index_sets_identical": sum(1 for s, f in res if s and not f),
            "failures": failures}


def cpu_baseline(wl, L, Lh, n_units, passes, outs, idxs, ws, k_fp8=False):
    """The CPU oracle, as it stands, on a seeded sample of this workload's units,
    one thread per available core; its results double as a spot check of the GPU
    outputs of the last timed step."""
    import oracle
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from harness import check_unit, dtype_code   # the acceptance rule of the parity tests
    cores = len(os.sched_getaffinity(0))
    lens = wl.seq_lens()
    picks = pick_units(wl, L, n_units)
    n_units = len(picks)
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
