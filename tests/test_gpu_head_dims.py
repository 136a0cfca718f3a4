"""GPU parity for head dimensions 64 and 256 (128 is what every other GPU test uses):
store, KCache decode (fused path), conventional attention with V in HBM, step graph."""
import numpy as np
import pytest
import torch

import kcache_inputs as ki
import oracle
from harness import ABS_TOL, REL_TOL, check_unit, dtype_code, oracle_unit, pinned_like, sample_units

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def kc():
    import paper_2404_18057_amd as kc
    return kc


@pytest.fixture(scope="module")
def ctx(kc):
    c = kc.Context(0)
    yield c
    c.close()


def build(kc, ctx, wl, layer, hbm_v=False, chunk_T=None):
    q, k, v, lens = ki.gen_layer(wl, layer, DEV)
    v_cache = torch.zeros_like(v) if hbm_v else pinned_like(v)
    if not hbm_v:
        v_cache.zero_()
    cache = kc.LayerCache(torch.zeros_like(k), v_cache)
    T = wl.S_cap if chunk_T is None else chunk_T
    for t0 in range(0, wl.S_cap, T):
        t1 = min(wl.S_cap, t0 + T)
        k_new = k[:, :, t0:t1].permute(0, 2, 1, 3).contiguous()
        v_new = v[:, :, t0:t1].permute(0, 2, 1, 3).contiguous()
        pos = torch.full((wl.B,), t0, dtype=torch.int32, device=DEV)
        ctx.prefill_store(cache, k_new, v_new, pos)
        ctx.synchronize()
        torch.cuda.synchronize()
    return cache, q, torch.from_numpy(lens).to(DEV), k, v


@pytest.mark.parametrize("d", [64, 256])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_store_is_bit_exact(kc, ctx, d, dtype):
    wl = ki.config(1, B=2, H=5, Hkv=5, S_cap=777, d=d, dtype=dtype)
    cache, q, lens, k, v = build(kc, ctx, wl, 0, chunk_T=301)
    assert torch.equal(cache.k.view(torch.int16), k.view(torch.int16))
    assert torch.equal(cache.v.view(torch.int16), v.cpu().view(torch.int16))


@pytest.mark.parametrize("d", [64, 256])
@pytest.mark.parametrize("G,dtype", [(1, "f16"), (2, "bf16"), (4, "f16"), (8, "bf16"), (16, "f16")])
def test_kcache_decode_matches_oracle(kc, ctx, d, G, dtype):
    wl = ki.config(1, B=3, H=2 * G, Hkv=2, S_cap=5000, N=70, d=d, dtype=dtype)
    cache, q, _, _, _ = build(kc, ctx, wl, 1, chunk_T=2048)
    lens_list = [5000, 1, 2049]
    lens = torch.tensor(lens_list, dtype=torch.int32, device=DEV)
    idx = torch.empty((wl.B, wl.H, wl.N), dtype=torch.int32, device=DEV)
    w = torch.empty((wl.B, wl.H, wl.N), dtype=torch.float32, device=DEV)
    out = ctx.decode_attention(cache, q, lens, wl.N, idx_out=idx, w_out=w)
    torch.cuda.synchronize()
    ctx.device_check()
    out_h, idx_h, w_h = out.cpu().numpy(), idx.cpu().numpy(), w.cpu().numpy()
    code = dtype_code(wl)
    for b, s in enumerate(lens_list):
        for h in range(wl.H):
            qb, kb, vb = ki.gen_unit(wl, 1, b, h)
            r = oracle.decode_unit(qb, kb[:s], vb[:s], code, wl.N, want_scores=True)
            r["v"] = oracle.decode16(vb[:s], code)
            check_unit(r, wl.N, out_h[b, h], idx_h[b, h], w_h[b, h],
                       tag="d=%d G=%d (%d,%d)" % (d, G, b, h))


@pytest.mark.parametrize("d", [64, 256])
def test_long_context_many_chunks(kc, ctx, d):
    # enough positions for several workgroups per unit at either row size
    wl = ki.config(1, B=2, H=4, Hkv=4, S_cap=20000, N=256, d=d)
    cache, q, lens, _, _ = build(kc, ctx, wl, 0, chunk_T=8192)
    idx = torch.empty((wl.B, wl.H, wl.N), dtype=torch.int32, device=DEV)
    w = torch.empty((wl.B, wl.H, wl.N), dtype=torch.float32, device=DEV)
    out = ctx.decode_attention(cache, q, lens, wl.N, idx_out=idx, w_out=w)
    torch.cuda.synchronize()
    out_h, idx_h, w_h = out.cpu().numpy(), idx.cpu().numpy(), w.cpu().numpy()
    for (b, h) in sample_units(wl, 8):
        r = oracle_unit(wl, 0, b, h, wl.N)
        check_unit(r, wl.N, out_h[b, h], idx_h[b, h], w_h[b, h], tag="d=%d (%d,%d)" % (d, b, h))


@pytest.mark.parametrize("d", [64, 256])
@pytest.mark.parametrize("G,dtype", [(1, "bf16"), (4, "f16"), (8, "f16")])
def test_conventional_attention_matches_oracle(kc, ctx, d, G, dtype):
    wl = ki.config(1, B=2, H=2 * G, Hkv=2, S_cap=4100, d=d, dtype=dtype)
    cache, q, _, k, v = build(kc, ctx, wl, 0, hbm_v=True)
    lens_list = [4100, 1300]
    # rows beyond the length must not reach the result
    cache.v[1, :, 1300:] = float("inf")
    lens = torch.tensor(lens_list, dtype=torch.int32, device=DEV)
    out = ctx.full_attention(cache, q, lens)
    torch.cuda.synchronize()
    ctx.device_check()
    out_h = out.cpu().numpy()
    assert np.isfinite(out_h).all()
    code = dtype_code(wl)
    for b, s in enumerate(lens_list):
        for h in range(wl.H):
            qb, kb, vb = ki.gen_unit(wl, 0, b, h)
            ref = oracle.full_unit(qb, kb[:s], vb[:s], code)
            err = np.abs(out_h[b, h].astype(np.float64) - ref)
            assert (err <= ABS_TOL + REL_TOL * np.abs(ref)).all(), (d, G, b, h, err.max())


@pytest.mark.parametrize("d", [64, 256])
def test_step_graph_with_split_lanes(kc, ctx, d):
    wl = ki.config(1, B=4, H=4, Hkv=2, S_cap=3000, N=33, d=d)
    layers = []
    for l in range(2):
        cache, q, lens, k, v = build(kc, ctx, wl, l, hbm_v=(l == 0))
        layers.append(dict(cache=cache, q=q,
                           k_new=k[:, :, wl.S_cap - 1].unsqueeze(1).contiguous(),
                           v_new=v[:, :, wl.S_cap - 1].unsqueeze(1).contiguous(),
                           out=torch.zeros((wl.B, wl.H, wl.d), dtype=torch.float32, device=DEV),
                           idx_out=torch.zeros((wl.B, wl.H, wl.N), dtype=torch.int32, device=DEV),
                           w_out=torch.zeros((wl.B, wl.H, wl.N), dtype=torch.float32, device=DEV)))
        cache.k[:, :, wl.S_cap - 1] = 0
        cache.v[:, :, wl.S_cap - 1] = 0
    pos = (lens - 1).to(torch.int32)
    ctx.set_step_lanes(2, split_sequences=True)
    try:
        g = ctx.step_graph(layers, wl.H, pos, lens, wl.N)
        g.launch()
        ctx.synchronize()
        g.close()
    finally:
        ctx.set_step_lanes(1)
    torch.cuda.synchronize()
    ctx.device_check()
    code = dtype_code(wl)
    o0 = layers[0]["out"].cpu().numpy()
    y = layers[1]
    o1, i1, w1 = y["out"].cpu().numpy(), y["idx_out"].cpu().numpy(), y["w_out"].cpu().numpy()
    for b in range(wl.B):
        for h in (0, wl.H - 1):
            qb, kb, vb = ki.gen_unit(wl, 0, b, h)
            ref = oracle.full_unit(qb, kb, vb, code)
            assert (np.abs(o0[b, h] - ref) <= ABS_TOL + REL_TOL * np.abs(ref)).all()
            r = oracle_unit(wl, 1, b, h, wl.N)
            check_unit(r, wl.N, o1[b, h], i1[b, h], w1[b, h], tag="d=%d step (%d,%d)" % (d, b, h))


def test_unsupported_combinations(kc, ctx):
    wl = ki.config(1, d=64)
    q, k, v, lens = ki.gen_layer(wl, 0, DEV)
    lens_dev = torch.from_numpy(lens).to(DEV)
    cache = kc.LayerCache(k, pinned_like(v))
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_attention(cache, q, lens_dev, 8, gather_mode=kc.GATHER_STAGED)
    assert e.value.status == -2
    ctx.set_fused(False)
    try:
        with pytest.raises(kc.KCacheError) as e:
            ctx.decode_attention(cache, q, lens_dev, 8)
        assert e.value.status == -2
    finally:
        ctx.set_fused(True)
    k8 = torch.zeros(k.shape, dtype=torch.uint8, device=DEV)
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_attention(kc.LayerCache(k8, pinned_like(v), k_exp=-5), q, lens_dev, 8)
    assert e.value.status == -2
