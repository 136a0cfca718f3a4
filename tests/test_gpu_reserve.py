"""A context sized with kcache_reserve never allocates (and so never synchronises) inside the
store / attention / step calls; without KC_OPT_AUTO_GROW an unsized context refuses the call."""
import copy

import pytest
import torch

import kcache_inputs as ki

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def kc():
    import paper_2404_18057_amd as kc
    return kc


def hbm_layer(kc, wl):
    """A layer of the workload's per-layer shape with random K rows; the V cache is the same
    device tensor (v_in_hbm), which both attention calls accept."""
    dt = ki.torch_dtype(wl.dtype)
    g = torch.Generator(device=DEV).manual_seed(wl.seed)
    k = torch.randn((wl.B, wl.Hkv, wl.S_cap, wl.d), dtype=dt, device=DEV, generator=g)
    return kc.LayerCache(k, k)


def host_shape(cache):
    """The same shape with the V cache declared in host memory (kcache_reserve reads no pointer)."""
    shape = copy.copy(cache)
    shape.c = type(cache.c).from_buffer_copy(cache.c)
    shape.c.v_in_hbm = 0
    return shape


def test_reserved_context_never_reallocates_on_the_five_workload_shapes(kc):
    c = kc.Context(0, auto_grow=False)
    try:
        layers = {}
        for cfg in (1, 2, 3, 4, 5):
            wl = ki.config(cfg)
            cache = hbm_layer(kc, wl)
            layers[cfg] = (wl, cache)
            c.reserve(cache, wl.H, wl.N, step_layers=2)               # V in HBM: both attention calls
            c.reserve(host_shape(cache), wl.H, wl.N, step_layers=2)   # V on the host: the KCache launch
        base = c.stat(kc.STAT_REALLOCS)
        assert base >= 1
        for cfg, (wl, cache) in layers.items():
            print("reserved shape: %s" % wl.name, flush=True)
            q = torch.randn((wl.B, wl.H, wl.d), dtype=cache.k.dtype, device=DEV)
            lens = torch.from_numpy(wl.seq_lens()).to(DEV)
            out = torch.empty((wl.B, wl.H, wl.d), dtype=torch.float32, device=DEV)
            c.decode_attention(cache, q, lens, wl.N, out=out)
            c.full_attention(cache, q, lens, out=out)
            step = [dict(cache=cache, q=q, out=out), dict(cache=cache, q=q, out=out)]
            pos = (lens - 1).to(torch.int32)
            c.decode_step(step, wl.H, pos, lens, wl.N)
            g = c.step_graph(step, wl.H, pos, lens, wl.N)
            g.launch()
            c.synchronize()
            g.close()
            assert c.stat(kc.STAT_REALLOCS) == base, "%s made the context grow" % wl.name
            assert torch.isfinite(out).all()
        c.device_check()
    finally:
        c.close()


def test_unsized_context_refuses_instead_of_growing(kc):
    c = kc.Context(0, auto_grow=False)
    try:
        wl = ki.config(1)
        cache = hbm_layer(kc, wl)
        q = torch.randn((wl.B, wl.H, wl.d), dtype=cache.k.dtype, device=DEV)
        lens = torch.from_numpy(wl.seq_lens()).to(DEV)
        with pytest.raises(kc.KCacheError) as e:
            c.decode_attention(cache, q, lens, wl.N)
        assert e.value.status == -4 and "kcache_reserve" in str(e.value)
        assert c.stat(kc.STAT_REALLOCS) == 0
        c.reserve(cache, wl.H, wl.N)
        n = c.stat(kc.STAT_REALLOCS)
        c.decode_attention(cache, q, lens, wl.N)
        # a larger N needs more: refused again, and allowed once auto-grow is switched on
        with pytest.raises(kc.KCacheError) as e:
            c.decode_attention(cache, q, lens, 8 * wl.N)
        assert e.value.status == -4
        c.set_option(9, 1)      # KC_OPT_AUTO_GROW
        c.decode_attention(cache, q, lens, 8 * wl.N)
        assert c.stat(kc.STAT_REALLOCS) > n
        c.synchronize()
        c.device_check()
    finally:
        c.close()


def test_reserve_covers_the_staged_gather_and_the_unfused_launches(kc):
    c = kc.Context(0, auto_grow=False)
    try:
        wl = ki.config(1)
        q, k, v, lens = ki.gen_layer(wl, 0, DEV)
        v_pin = torch.empty(v.shape, dtype=v.dtype, pin_memory=True)
        v_pin.copy_(v)
        cache = kc.LayerCache(k, v_pin)
        lens_dev = torch.from_numpy(lens).to(DEV)
        c.reserve(cache, wl.H, wl.N, gather_mode=kc.GATHER_STAGED)
        base = c.stat(kc.STAT_REALLOCS)
        a = c.decode_attention(cache, q, lens_dev, wl.N, gather_mode=kc.GATHER_STAGED).clone()
        c.set_fused(False)
        b = c.decode_attention(cache, q, lens_dev, wl.N).clone()
        c.set_fused(True)
        torch.cuda.synchronize()
        assert c.stat(kc.STAT_REALLOCS) == base
        assert torch.equal(a, b)     # same kernels on both sides
        c.device_check()
    finally:
        c.close()


def test_lanes_chosen_from_the_shape(kc):
    c = kc.Context(0)
    try:
        want = {1: 1, 2: 2, 3: 2, 4: 2, 5: 2}    # config 1 has a single sequence
        for cfg, lanes in want.items():
            wl = ki.config(cfg)
            k = torch.empty((1, 1, 1, wl.d), dtype=ki.torch_dtype(wl.dtype), device=DEV)
            shape = kc.LayerCache(k, k)
            shape.c.B, shape.c.Hkv, shape.c.S_cap = wl.B, wl.Hkv, wl.S_cap
            assert c.step_lanes_for(shape, wl.L, wl.H) == lanes, wl.name
        c.set_step_lanes(1)
        assert c.step_lanes_for(shape, 40, 40) == 1
        c.set_step_lanes(4, split_sequences=True)
        assert c.step_lanes_for(shape, 40, 40) == 2      # config 5 has two sequences to split
        c.set_step_lanes(4, split_sequences=False)
        assert c.step_lanes_for(shape, 40, 40) == 4
    finally:
        c.close()
