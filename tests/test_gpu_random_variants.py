"""Seeded random configurations through the fused path and conventional attention: head
dimension, group size, batch, capacity, ragged lengths, N, dtype, 8-bit K cache, V in HBM,
renormalised weights, forced chunk sizes, pivot density - each checked against the oracle."""
import numpy as np
import pytest
import torch

import kcache_inputs as ki
import oracle
from harness import ABS_TOL, REL_TOL, check_unit, pinned_like

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
K_EXP = -5


@pytest.fixture(scope="module")
def kc():
    import paper_2404_18057_amd as kc
    return kc


@pytest.fixture(scope="module")
def ctx(kc):
    c = kc.Context(0)
    yield c
    c.close()


def draw(case):
    rng = np.random.default_rng(7000 + case)
    c = dict(
        d=int(rng.choice([64, 128, 128, 128, 256])),
        G=int(rng.choice([1, 1, 2, 4, 8, 16, 32])),
        Hkv=int(rng.integers(1, 4)), B=int(rng.integers(1, 5)),
        S=int(rng.choice([1, 2, 63, 64, 65, 511, 512, 513, 1023, 1024, 1025, 2047, 2049, 3000,
                          4096, 8191, 12000, 20000])),
        N=int(rng.choice([1, 2, 3, 31, 64, 100, 256, 300, 512, 1000, 1024, 1025, 3000])),
        dt="f16" if rng.integers(2) else "bf16")
    c["k8"] = bool(c["d"] == 128 and rng.integers(4) == 0)
    c["hbm"] = bool(rng.integers(4) == 0)
    c["renorm"] = bool(rng.integers(5) == 0)
    c["full"] = bool(c["hbm"] and not c["k8"] and rng.integers(2))
    c["rows"] = int(rng.choice([0, 0, 0, 512, 1024, 2048]))
    c["frac"] = float(rng.choice([0.0005, 0.01, 0.2]))
    c["lens"] = [int(rng.integers(1, c["S"] + 1)) for _ in range(c["B"])]
    c["lens"][0] = c["S"]
    c["pick"] = rng
    return c


@pytest.mark.parametrize("case", range(48))
def test_random_configuration(kc, ctx, case):
    c = draw(case)
    B, G, Hkv, S, N, d = c["B"], c["G"], c["Hkv"], c["S"], c["N"], c["d"]
    H = Hkv * G
    wl = ki.config(1, B=B, H=H, Hkv=Hkv, S_cap=S, N=N, d=d, dtype=c["dt"], seed=7000 + case,
                   pivot_frac=c["frac"])
    tag = "case %d %s" % (case, {k: v for k, v in c.items() if k != "pick"})
    q, k, v, _ = ki.gen_layer(wl, 0, DEV)
    k_cache = torch.zeros(k.shape, dtype=torch.uint8, device=DEV) if c["k8"] else torch.zeros_like(k)
    v_cache = torch.zeros_like(v) if c["hbm"] else pinned_like(v)
    cache = kc.LayerCache(k_cache, v_cache, k_exp=K_EXP)
    ctx.prefill_store(cache, k.permute(0, 2, 1, 3).contiguous(), v.permute(0, 2, 1, 3).contiguous(),
                      torch.zeros(B, dtype=torch.int32, device=DEV))
    ctx.synchronize()
    torch.cuda.synchronize()
    lens = c["lens"]
    lens_dev = torch.tensor(lens, dtype=torch.int32, device=DEV)
    code = oracle.F16 if c["dt"] == "f16" else oracle.BF16
    renorm = c["renorm"] and not c["full"]
    ctx.set_fused_rows(c["rows"] if c["rows"] * min(G, 8) <= 8192 else 0)
    ctx.set_renormalize(renorm)
    try:
        if c["full"]:
            out = ctx.full_attention(cache, q, lens_dev).cpu().numpy()
        else:
            idx = torch.empty((B, H, N), dtype=torch.int32, device=DEV)
            w = torch.empty((B, H, N), dtype=torch.float32, device=DEV)
            out = ctx.decode_attention(cache, q, lens_dev, N, idx_out=idx, w_out=w).cpu().numpy()
            idx, w = idx.cpu().numpy(), w.cpu().numpy()
        torch.cuda.synchronize()
        ctx.device_check()
    finally:
        ctx.set_renormalize(False)
        ctx.set_fused_rows(0)
    units = [(b, h) for b in range(B) for h in range(H)]
    if len(units) > 6:
        units = [units[i] for i in c["pick"].choice(len(units), 6, replace=False)]
    for (b, h) in units:
        qb, kb, vb = ki.gen_unit(wl, 0, b, h)
        s = lens[b]
        if c["full"]:
            ref = oracle.full_unit(qb, kb[:s], vb[:s], code)
            err = np.abs(out[b, h] - ref)
            assert (err <= ABS_TOL + REL_TOL * np.abs(ref)).all(), "%s: max err %g" % (tag, err.max())
            continue
        if c["k8"]:
            r = oracle.decode_unit_k8(qb, oracle.e4m3_quantise(kb[:s], code, K_EXP), K_EXP, vb[:s],
                                      code, N, want_scores=True)
        else:
            r = oracle.decode_unit(qb, kb[:s], vb[:s], code, N, want_scores=True)
        r["v"] = oracle.decode16(vb[:s], code)
        if not renorm:
            check_unit(r, N, out[b, h], idx[b, h], w[b, h], tag=tag)
            continue
        # renormalised variant: same selection rule, weights divided by the kept mass
        n_eff = min(N, s)
        kept = idx[b, h, :n_eff]
        p_kept = r["p"][kept]
        plain_w = np.concatenate([p_kept, np.zeros(N - n_eff)])
        check_unit(r, N, p_kept @ r["v"][kept], idx[b, h], plain_w, tag=tag + " (selection)")
        assert np.allclose(w[b, h, :n_eff], p_kept / p_kept.sum(), rtol=3e-3, atol=1e-7), tag
        ref = (p_kept / p_kept.sum()) @ r["v"][kept]
        assert (np.abs(out[b, h] - ref) <= ABS_TOL + REL_TOL * np.abs(ref)).all(), tag
