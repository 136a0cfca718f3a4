"""GPU parity of the layers that keep V in HBM: conventional attention
(kcache_full_attention) and the cache store / KCache selection with a device V
cache, against the CPU oracle through the C ABI."""
import numpy as np
import pytest
import torch

import kcache_inputs as ki
import oracle
from harness import ABS_TOL, REL_TOL, check_unit, dtype_code, oracle_unit, sample_units

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


def build_hbm_layer(kc, ctx, wl, layer, chunk_T=None):
    """One generated layer placed with kcache_prefill_store, V cache in HBM."""
    q, k, v, lens = ki.gen_layer(wl, layer, DEV)
    cache = kc.LayerCache(torch.zeros_like(k), torch.zeros_like(v))
    assert cache.v_in_hbm
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


def check_full(out_gpu, ref, tag):
    err = np.abs(np.asarray(out_gpu, dtype=np.float64) - ref)
    bound = ABS_TOL + REL_TOL * np.abs(ref)
    assert (err <= bound).all(), "%s: max err %g" % (tag, err.max())


def run_full(ctx, wl, layer, cache, q, lens, units, tag=""):
    out = torch.full((wl.B, wl.H, wl.d), float("nan"), dtype=torch.float32, device=DEV)
    ctx.full_attention(cache, q, lens, out=out)
    torch.cuda.synchronize()
    ctx.device_check()
    out_h = out.cpu().numpy()
    assert np.isfinite(out_h).all()
    for (b, h) in units:
        qb, kb, vb = ki.gen_unit(wl, layer, b, h)
        ref = oracle.full_unit(qb, kb, vb, dtype_code(wl))
        check_full(out_h[b, h], ref, "%s %s layer %d unit (%d,%d)" % (tag, wl.name, layer, b, h))
    return out_h


def manual_full(kc, ctx, q, K, V, lens, dtype=torch.float16):
    qt = torch.from_numpy(np.asarray(q, np.float32)).to(dtype)
    kt = torch.from_numpy(np.asarray(K, np.float32)).to(dtype)
    vt = torch.from_numpy(np.asarray(V, np.float32)).to(dtype)
    cache = kc.LayerCache(kt.to(DEV), vt.to(DEV))
    lens_dev = torch.tensor(lens, dtype=torch.int32, device=DEV)
    out = ctx.full_attention(cache, qt.to(DEV), lens_dev)
    torch.cuda.synchronize()
    ctx.device_check()
    code = oracle.F16 if dtype == torch.float16 else oracle.BF16
    ref = oracle.full_attention(ki.as_bits(qt), ki.as_bits(kt), ki.as_bits(vt), code,
                                np.asarray(lens, np.int32), nthreads=4)
    return out.cpu().numpy(), ref


# ------------------------------------------------------------------ named configurations
def test_config1_every_unit(kc, ctx):
    wl = ki.config(1)
    cache, q, lens, _, _ = build_hbm_layer(kc, ctx, wl, 0)
    run_full(ctx, wl, 0, cache, q, lens, sample_units(wl, 10 ** 9))


def test_store_to_hbm_v_cache_is_bit_exact(kc, ctx):
    wl = ki.config(1, B=2, H=4, Hkv=4, S_cap=700)
    cache, q, lens, k, v = build_hbm_layer(kc, ctx, wl, 0, chunk_T=300)
    assert torch.equal(cache.k, k) and torch.equal(cache.v, v)


@pytest.mark.parametrize("cfg,layer,count", [(2, 0, 24), (2, 31, 12), (3, 5, 32), (5, 39, 12)])
def test_full_shapes_sampled_units(kc, ctx, cfg, layer, count):
    # the per-layer shapes of the large workloads, as the benchmark launches them
    wl = ki.config(cfg)
    cache, q, lens, _, _ = build_hbm_layer(kc, ctx, wl, layer, chunk_T=8192)
    run_full(ctx, wl, layer, cache, q, lens, sample_units(wl, count, seed=cfg))
    del cache
    torch.cuda.empty_cache()


def test_config4_ragged_lengths(kc, ctx):
    wl = ki.config(4, B=16)
    cache, q, lens, _, _ = build_hbm_layer(kc, ctx, wl, 0, chunk_T=8192)
    run_full(ctx, wl, 0, cache, q, lens, sample_units(wl, 24, seed=4))


# ------------------------------------------------------------------ edge cases
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("G", [1, 2, 4, 8, 16, 32])
def test_group_sizes_and_ragged_tails(kc, ctx, dtype, G):
    rng = np.random.default_rng(40 + G)
    B, Hkv, S, d = 3, 2, 2500, 128
    H = Hkv * G
    q = rng.standard_normal((B, H, d))
    K = rng.standard_normal((B, Hkv, S, d))
    V = rng.standard_normal((B, Hkv, S, d))
    lens = [2500, 1, 1027]
    # rows beyond the length must not be read into the result: make them poisonous
    for b in range(B):
        K[b, :, lens[b]:] = 300.0
        V[b, :, lens[b]:] = np.inf
    out, ref = manual_full(kc, ctx, q, K, V, lens, dtype)
    for b in range(B):
        for h in range(H):
            check_full(out[b, h], ref[b, h], "G=%d (%d,%d)" % (G, b, h))


def test_uniform_scores_give_the_mean_of_v(kc, ctx):
    rng = np.random.default_rng(41)
    B, H, S, d = 1, 2, 3000, 128
    q = rng.standard_normal((B, H, d))
    K = np.tile(rng.standard_normal((1, 1, 1, d)), (B, H, S, 1))
    V = np.round(rng.standard_normal((B, H, S, d)) * 8) / 8
    out, ref = manual_full(kc, ctx, q, K, V, [S])
    assert np.allclose(ref, V.mean(2), atol=1e-12)   # the oracle's closed form
    check_full(out[0, 0], ref[0, 0], "uniform")
    check_full(out[0, 1], ref[0, 1], "uniform")


def test_large_scores_do_not_overflow(kc, ctx):
    # scores of a few hundred: the chunk maxima differ by far more than exp can hold
    rng = np.random.default_rng(42)
    B, H, S, d = 1, 1, 5000, 128
    q = rng.standard_normal((B, H, d)) * 6
    K = rng.standard_normal((B, H, S, d)) * 6
    V = rng.standard_normal((B, H, S, d))
    out, ref = manual_full(kc, ctx, q, K, V, [S])
    check_full(out[0, 0], ref[0, 0], "large scores")


def test_capacity_one_and_length_one(kc, ctx):
    rng = np.random.default_rng(43)
    q = rng.standard_normal((2, 1, 128))
    K = rng.standard_normal((2, 1, 1, 128))
    V = rng.standard_normal((2, 1, 1, 128))
    out, ref = manual_full(kc, ctx, q, K, V, [1, 1])
    check_full(out[0, 0], ref[0, 0], "S_cap=1")
    check_full(out[1, 0], ref[1, 0], "S_cap=1")


def test_rows_per_workgroup_do_not_change_the_result_beyond_rounding(kc, ctx):
    wl = ki.config(1, B=2, S_cap=6000)
    cache, q, lens, _, _ = build_hbm_layer(kc, ctx, wl, 0)
    outs = []
    for rows in (512, 1024, 4096, 0):
        ctx.set_fused_rows(rows)
        outs.append(run_full(ctx, wl, 0, cache, q, lens, sample_units(wl, 6), tag="rows %d" % rows))
    ctx.set_fused_rows(0)
    again = run_full(ctx, wl, 0, cache, q, lens, [])
    assert np.array_equal(outs[-1], again)   # same launch shape: bit-identical


def test_kcache_selection_with_v_in_hbm_matches_oracle(kc, ctx):
    # a layer with V in HBM may still run the top-N path; its rows then come from HBM
    wl = ki.config(1, B=2, S_cap=5000)
    cache, q, lens, _, _ = build_hbm_layer(kc, ctx, wl, 0)
    N = wl.N
    idx = torch.empty((wl.B, wl.H, N), dtype=torch.int32, device=DEV)
    w = torch.empty((wl.B, wl.H, N), dtype=torch.float32, device=DEV)
    out = ctx.decode_attention(cache, q, lens, N, idx_out=idx, w_out=w)
    torch.cuda.synchronize()
    out_h, idx_h, w_h = out.cpu().numpy(), idx.cpu().numpy(), w.cpu().numpy()
    for (b, h) in sample_units(wl, 8):
        r = oracle_unit(wl, 0, b, h, N)
        check_unit(r, N, out_h[b, h], idx_h[b, h], w_h[b, h], tag="v in hbm (%d,%d)" % (b, h))


def test_full_attention_equals_kcache_with_n_equal_s(kc, ctx):
    # section 3.1: nothing is dropped when N covers the context
    wl = ki.config(1, B=1, S_cap=900)
    cache, q, lens, _, _ = build_hbm_layer(kc, ctx, wl, 0)
    a = ctx.full_attention(cache, q, lens).cpu().numpy()
    b = ctx.decode_attention(cache, q, lens, 900).cpu().numpy()
    assert np.allclose(a, b, rtol=REL_TOL, atol=ABS_TOL)


# ------------------------------------------------------------------ error paths
def test_error_paths(kc, ctx):
    wl = ki.config(1)
    q, k, v, lens = ki.gen_layer(wl, 0, DEV)
    lens_dev = torch.from_numpy(lens).to(DEV)
    v_host = torch.empty(v.shape, dtype=v.dtype, pin_memory=True)
    host_layer = kc.LayerCache(k, v_host)
    with pytest.raises(kc.KCacheError) as e:
        ctx.full_attention(host_layer, q, lens_dev)
    assert e.value.status == -1
    hbm_layer = kc.LayerCache(k, v)
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_attention(hbm_layer, q, lens_dev, 8, gather_mode=kc.GATHER_STAGED)
    assert e.value.status == -2
    # a host pointer declared as HBM is refused before anything is launched
    lying = kc.LayerCache(k, v)
    lying.c.v_host = v_host.data_ptr()
    with pytest.raises(kc.KCacheError) as e:
        ctx.full_attention(lying, q, lens_dev)
    assert e.value.status == -3
    # a length outside the cache is flagged by the kernel, which stays in bounds
    bad = torch.tensor([wl.S_cap + 5], dtype=torch.int32, device=DEV)
    ctx.full_attention(hbm_layer, q, bad)
    with pytest.raises(kc.KCacheError) as e:
        ctx.device_check()
    assert e.value.status == -6
    ctx.device_check()
