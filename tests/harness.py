"""Shared helpers of the GPU parity tests: cache set-up through the C ABI and the
acceptance rule that compares the GPU result of a unit with the CPU oracle."""
import numpy as np
import torch

import kcache_inputs as ki
import oracle

TIE_BAND = 1e-3      # scaled-score units: below this gap several top-N sets are correct
ABS_TOL, REL_TOL = 1e-3, 2e-3


def dtype_code(wl):
    return oracle.F16 if wl.dtype == "f16" else oracle.BF16


def pinned_like(t):
    return torch.empty(t.shape, dtype=t.dtype, pin_memory=True)


def build_layer(ctx, wl, layer, device="cuda:0", chunk_T=None):
    """Generates one layer on the GPU and places it with kcache_prefill_store:
    K into a device cache, V into a pinned host cache.  Returns
    (LayerCache, q, seq_lens_dev, k_generated_dev, v_generated_dev)."""
    import paper_2404_18057_amd as kc
    q, k, v, lens = ki.gen_layer(wl, layer, device)
    k_cache = torch.zeros_like(k)
    v_cache = pinned_like(v)
    v_cache.zero_()
    cache = kc.LayerCache(k_cache, v_cache)
    T = wl.S_cap if chunk_T is None else chunk_T
    for t0 in range(0, wl.S_cap, T):
        t1 = min(wl.S_cap, t0 + T)
        k_new = k[:, :, t0:t1].permute(0, 2, 1, 3).contiguous()
        v_new = v[:, :, t0:t1].permute(0, 2, 1, 3).contiguous()
        pos = torch.full((wl.B,), t0, dtype=torch.int32, device=device)
        ctx.prefill_store(cache, k_new, v_new, pos)
        ctx.synchronize()
        torch.cuda.synchronize()
    lens_dev = torch.from_numpy(lens).to(device)
    return cache, q, lens_dev, k, v


def oracle_unit(wl, layer, b, h, N, bits=None):
    qb, kb, vb = bits if bits is not None else ki.gen_unit(wl, layer, b, h)
    r = oracle.decode_unit(qb, kb, vb, dtype_code(wl), N, want_scores=True)
    r["v"] = oracle.decode16(vb, dtype_code(wl))
    return r


def check_unit(r, N, out_gpu, idx_gpu, w_gpu, tag=""):
    """Acceptance rule for one (sequence, head) unit.  r: oracle result with z, p, v.

    - positions ascending, -1 padded beyond N_eff, weights 0 there;
    - the index set equals the oracle's wherever the gap between the N-th and the
      (N+1)-th largest score exceeds TIE_BAND; otherwise every position in the
      symmetric difference must lie within TIE_BAND of the N-th largest score;
    - weights within REL_TOL of the oracle's softmax values at the GPU's positions;
    - out within ABS_TOL + REL_TOL*|ref| of the oracle's sum evaluated on the
      GPU's index set (equal to the oracle's own output when the sets agree).
    Returns True when the sets were identical."""
    z, p = r["z"], r["p"]
    s = len(z)
    n_eff = min(N, s)
    idx_gpu = np.asarray(idx_gpu)
    kept = idx_gpu[:n_eff]
    assert (idx_gpu[n_eff:] == -1).all(), tag + " padding of idx"
    assert (np.asarray(w_gpu)[n_eff:] == 0).all(), tag + " padding of weights"
    assert (kept >= 0).all() and (kept < s).all(), tag + " position outside the sequence"
    assert (np.diff(kept) > 0).all(), tag + " positions not strictly ascending"
    o_set, g_set = set(r["idx"][:n_eff].tolist()), set(kept.tolist())
    same = o_set == g_set
    if not same:
        zs = np.sort(z)[::-1]
        z_n = zs[n_eff - 1]
        gap = z_n - zs[n_eff] if n_eff < s else np.inf
        assert gap <= TIE_BAND, "%s index set differs although the boundary gap is %g" % (tag, gap)
        for t in o_set ^ g_set:
            assert abs(z[t] - z_n) <= TIE_BAND, \
                "%s position %d (score %g) is outside the tie band around %g" % (tag, t, z[t], z_n)
    w_ref = p[kept]
    assert np.allclose(np.asarray(w_gpu)[:n_eff], w_ref, rtol=REL_TOL, atol=1e-7), tag + " weights"
    ref = r["out"] if same else w_ref @ r["v"][kept]
    err = np.abs(np.asarray(out_gpu, dtype=np.float64) - ref)
    bound = ABS_TOL + REL_TOL * np.abs(ref)
    assert (err <= bound).all(), "%s out: max err %g (bound %g)" % (tag, err.max(), bound.min())
    return same


def sample_units(wl, count, seed=0):
    """Seeded sample of (b, h) pairs that always contains the first and last head
    of the first and last sequence."""
    rng = np.random.default_rng(seed)
    must = {(0, 0), (0, wl.H - 1), (wl.B - 1, 0), (wl.B - 1, wl.H - 1)}
    total = wl.B * wl.H
    if count >= total:
        return [(b, h) for b in range(wl.B) for h in range(wl.H)]
    pick = rng.choice(total, size=count, replace=False)
    units = must | {(int(u) // wl.H, int(u) % wl.H) for u in pick}
    return sorted(units)[:max(count, len(must))]


def check_units_parallel(wl, layer, units, N, out_h, idx_h, w_h, tag="", workers=None):
    """Oracle + acceptance rule for many units, spread over host threads (the unit generator
    and the C oracle both release the interpreter lock).  Returns the number of units whose
    index sets were identical; raises the first failure."""
    import concurrent.futures as cf
    import os
    workers = workers or max(1, min(16, len(os.sched_getaffinity(0))))

    def one(u):
        b, h = u
        r = oracle_unit(wl, layer, b, h, N)
        return check_unit(r, N, out_h[b, h], idx_h[b, h], w_h[b, h],
                          tag="%s %s layer %d unit (%d,%d) N=%d" % (tag, wl.name, layer, b, h, N))

    if workers == 1 or len(units) < 4:
        return sum(one(u) for u in units)
    with cf.ThreadPoolExecutor(max_workers=workers) as ex:
        return sum(ex.map(one, units))


def run_and_check(ctx, wl, layer, cache, q, lens_dev, units, N=None, gather_mode=0, tag=""):
    """One kcache_decode_attention call checked against the oracle on `units`."""
    N = wl.N if N is None else N
    dev = q.device
    idx = torch.full((wl.B, wl.H, N), -7, dtype=torch.int32, device=dev)
    w = torch.full((wl.B, wl.H, N), -7.0, dtype=torch.float32, device=dev)
    out = torch.full((wl.B, wl.H, wl.d), float("nan"), dtype=torch.float32, device=dev)
    ctx.decode_attention(cache, q, lens_dev, N, out=out, idx_out=idx, w_out=w,
                         gather_mode=gather_mode)
    torch.cuda.synchronize()
    ctx.device_check()
    out_h, idx_h, w_h = out.cpu().numpy(), idx.cpu().numpy(), w.cpu().numpy()
    identical = check_units_parallel(wl, layer, units, N, out_h, idx_h, w_h, tag=tag)
    return identical, len(units), (out_h, idx_h, w_h)
