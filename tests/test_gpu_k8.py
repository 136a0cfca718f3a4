"""GPU parity of the variant with an 8-bit K cache (OCP FP8 E4M3 codes with a power-of-two
cache exponent): the store must produce exactly the oracle's codes, and the decode must match
the oracle run on those codes, with the acceptance rule of the 16-bit parity tests."""
import numpy as np
import pytest
import torch

import kcache_inputs as ki
import oracle
from harness import check_unit, dtype_code, pinned_like, sample_units

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
K_EXP = -5      # |K| of the synthetic workloads stays below 448 * 2^-5 = 14


@pytest.fixture(scope="module")
def kc():
    import paper_2404_18057_amd as kc
    return kc


@pytest.fixture(scope="module")
def ctx(kc):
    c = kc.Context(0)
    yield c
    c.close()


def build_k8_layer(kc, ctx, wl, layer, k_exp=K_EXP, chunk_T=None, hbm_v=False):
    q, k, v, lens = ki.gen_layer(wl, layer, DEV)
    k8 = torch.zeros(k.shape, dtype=torch.uint8, device=DEV)
    v_cache = torch.zeros_like(v) if hbm_v else pinned_like(v)
    cache = kc.LayerCache(k8, v_cache, k_exp=k_exp)
    assert cache.k_fp8
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


def check_k8_units(ctx, wl, layer, cache, q, lens, units, N, k_exp=K_EXP, tag=""):
    idx = torch.full((wl.B, wl.H, N), -7, dtype=torch.int32, device=DEV)
    w = torch.full((wl.B, wl.H, N), -7.0, dtype=torch.float32, device=DEV)
    out = ctx.decode_attention(cache, q, lens, N, idx_out=idx, w_out=w)
    torch.cuda.synchronize()
    ctx.device_check()
    out_h, idx_h, w_h = out.cpu().numpy(), idx.cpu().numpy(), w.cpu().numpy()
    G = wl.H // wl.Hkv
    for (b, h) in units:
        qb, kb, vb = ki.gen_unit(wl, layer, b, h)
        code = dtype_code(wl)
        codes = oracle.e4m3_quantise(kb, code, k_exp)
        # the cache holds exactly these codes
        s = kb.shape[0]
        got = cache.k[b, h // G, :s].cpu().numpy()
        assert np.array_equal(got, codes), "%s stored codes of unit (%d,%d)" % (tag, b, h)
        r = oracle.decode_unit_k8(qb, codes, k_exp, vb, code, N, want_scores=True)
        r["v"] = oracle.decode16(vb, code)
        check_unit(r, N, out_h[b, h], idx_h[b, h], w_h[b, h],
                   tag="%s k8 %s layer %d unit (%d,%d)" % (tag, wl.name, layer, b, h))


def test_store_quantises_every_fp16_value_exactly(kc, ctx):
    # all 65536 fp16 bit patterns through the store kernel, three exponents
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    k_new = torch.from_numpy(allbits.view(np.int16)).view(torch.float16).reshape(1, 512, 1, 128)
    for k_exp in (0, -5, 3):
        k8 = torch.full((1, 1, 512, 128), 0x55, dtype=torch.uint8, device=DEV)
        v = torch.zeros((1, 1, 512, 128), dtype=torch.float16, device=DEV)
        cache = kc.LayerCache(k8, v, k_exp=k_exp)
        pos = torch.zeros(1, dtype=torch.int32, device=DEV)
        ctx.prefill_store(cache, k_new.to(DEV), k_new.to(DEV), pos)
        ctx.synchronize()
        torch.cuda.synchronize()
        want = oracle.e4m3_quantise(allbits, oracle.F16, k_exp).reshape(512, 128)
        got = k8[0, 0].cpu().numpy()
        bad = np.nonzero(got != want)
        assert bad[0].size == 0, "k_exp %d: first mismatch at fp16 bits 0x%04x: got 0x%02x want 0x%02x" % (
            k_exp, allbits[bad[0][0] * 128 + bad[1][0]], got[bad[0][0], bad[1][0]],
            want[bad[0][0], bad[1][0]])
        assert torch.equal(v.view(torch.int16), k_new.to(DEV).view(torch.int16).reshape(1, 1, 512, 128))


def test_config1_every_unit(kc, ctx):
    wl = ki.config(1)
    cache, q, lens, _, _ = build_k8_layer(kc, ctx, wl, 0)
    check_k8_units(ctx, wl, 0, cache, q, lens, sample_units(wl, 10 ** 9), wl.N)


def test_bf16_store_quantises_every_bit_pattern_exactly(kc, ctx):
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    k_new = torch.from_numpy(allbits.view(np.int16)).view(torch.bfloat16).reshape(1, 512, 1, 128)
    k8 = torch.zeros((1, 1, 512, 128), dtype=torch.uint8, device=DEV)
    v = torch.zeros((1, 1, 512, 128), dtype=torch.bfloat16, device=DEV)
    cache = kc.LayerCache(k8, v, k_exp=-4)
    ctx.prefill_store(cache, k_new.to(DEV), k_new.to(DEV), torch.zeros(1, dtype=torch.int32, device=DEV))
    ctx.synchronize()
    torch.cuda.synchronize()
    want = oracle.e4m3_quantise(allbits, oracle.BF16, -4).reshape(512, 128)
    assert np.array_equal(k8[0, 0].cpu().numpy(), want)


def test_bf16_gqa_layer(kc, ctx):
    # config 3's per-layer shape (GQA group of 4, bf16) with an 8-bit K cache
    wl = ki.config(3)
    cache, q, lens, _, _ = build_k8_layer(kc, ctx, wl, 7, chunk_T=4096)
    check_k8_units(ctx, wl, 7, cache, q, lens, sample_units(wl, 16, seed=3), wl.N)


@pytest.mark.parametrize("cfg,layer,count", [(2, 3, 10), (5, 0, 6)])
def test_full_shapes_sampled_units(kc, ctx, cfg, layer, count):
    wl = ki.config(cfg)
    cache, q, lens, _, _ = build_k8_layer(kc, ctx, wl, layer, chunk_T=8192)
    check_k8_units(ctx, wl, layer, cache, q, lens, sample_units(wl, count, seed=cfg), wl.N)
    del cache
    torch.cuda.empty_cache()


@pytest.mark.parametrize("G", [2, 4, 8, 16])
def test_group_sizes_ragged_lengths_and_hbm_v(kc, ctx, G):
    wl = ki.config(1, B=3, H=2 * G, Hkv=2, S_cap=2600, N=40)
    cache, q, lens, _, _ = build_k8_layer(kc, ctx, wl, 0, chunk_T=1000, hbm_v=(G == 4))
    lens = torch.tensor([2600, 1, 1029], dtype=torch.int32, device=DEV)
    idx = torch.empty((wl.B, wl.H, wl.N), dtype=torch.int32, device=DEV)
    w = torch.empty((wl.B, wl.H, wl.N), dtype=torch.float32, device=DEV)
    out = ctx.decode_attention(cache, q, lens, wl.N, idx_out=idx, w_out=w)
    torch.cuda.synchronize()
    ctx.device_check()
    out_h, idx_h, w_h = out.cpu().numpy(), idx.cpu().numpy(), w.cpu().numpy()
    for b, s in enumerate([2600, 1, 1029]):
        for h in range(wl.H):
            qb, kb, vb = ki.gen_unit(wl, 0, b, h)
            codes = oracle.e4m3_quantise(kb[:s], oracle.F16, K_EXP)
            r = oracle.decode_unit_k8(qb, codes, K_EXP, vb[:s], oracle.F16, wl.N, want_scores=True)
            r["v"] = oracle.decode16(vb[:s], oracle.F16)
            check_unit(r, wl.N, out_h[b, h], idx_h[b, h], w_h[b, h], tag="G=%d (%d,%d)" % (G, b, h))


def test_append_then_decode_and_step_graph(kc, ctx):
    wl = ki.config(1, B=2, S_cap=1500)
    cache, q, lens, k, v = build_k8_layer(kc, ctx, wl, 0)
    # wipe the newest position, let the step's append restore (and quantise) it
    cache.k[:, :, wl.S_cap - 1] = 0
    cache.v[:, :, wl.S_cap - 1] = 0
    layer = dict(cache=cache, q=q, k_new=k[:, :, wl.S_cap - 1].unsqueeze(1).contiguous(),
                 v_new=v[:, :, wl.S_cap - 1].unsqueeze(1).contiguous(),
                 out=torch.zeros((wl.B, wl.H, wl.d), dtype=torch.float32, device=DEV),
                 idx_out=torch.zeros((wl.B, wl.H, wl.N), dtype=torch.int32, device=DEV),
                 w_out=torch.zeros((wl.B, wl.H, wl.N), dtype=torch.float32, device=DEV))
    pos = (lens - 1).to(torch.int32)
    graph = ctx.step_graph([layer], wl.H, pos, lens, wl.N)
    graph.launch()
    ctx.synchronize()
    torch.cuda.synchronize()
    graph.close()
    out, idx, w = layer["out"].cpu().numpy(), layer["idx_out"].cpu().numpy(), layer["w_out"].cpu().numpy()
    for (b, h) in sample_units(wl, 6):
        qb, kb, vb = ki.gen_unit(wl, 0, b, h)
        codes = oracle.e4m3_quantise(kb, oracle.F16, K_EXP)
        assert np.array_equal(cache.k[b, h, wl.S_cap - 1].cpu().numpy(), codes[-1])
        r = oracle.decode_unit_k8(qb, codes, K_EXP, vb, oracle.F16, wl.N, want_scores=True)
        r["v"] = oracle.decode16(vb, oracle.F16)
        check_unit(r, wl.N, out[b, h], idx[b, h], w[b, h], tag="k8 step (%d,%d)" % (b, h))


def test_error_paths(kc, ctx):
    wl = ki.config(1)
    q, k, v, lens = ki.gen_layer(wl, 0, DEV)
    lens_dev = torch.from_numpy(lens).to(DEV)
    k8 = torch.zeros(k.shape, dtype=torch.uint8, device=DEV)
    cache = kc.LayerCache(k8, pinned_like(v), k_exp=-5)
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_attention(cache, q, lens_dev, 8, gather_mode=kc.GATHER_STAGED)
    assert e.value.status == -2
    ctx.set_fused(False)
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_attention(cache, q, lens_dev, 8)
    assert e.value.status == -2
    ctx.set_fused(True)
    hbm = kc.LayerCache(k8, torch.zeros_like(v), k_exp=-5)
    with pytest.raises(kc.KCacheError) as e:
        ctx.full_attention(hbm, q, lens_dev)
    assert e.value.status == -2
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_attention(kc.LayerCache(k8, pinned_like(v), k_exp=99), q, lens_dev, 8)
    assert e.value.status == -1
