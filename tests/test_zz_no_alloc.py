"""The entry point that allocates nothing (kcache_decode_attention_static) against
kcache_decode_attention: same kernels, scratch in the library's static device array."""
import numpy as np
import pytest
import torch

import kcache_inputs as ki
from harness import build_layer, check_unit, oracle_unit, sample_units

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(kc, ctx, wl, cache, q, lens_dev, N):
    """Runs the existing entry point, then the static one, on the same inputs."""
    res = []
    for static in (False, True):
        idx = torch.full((wl.B, wl.H, N), -7, dtype=torch.int32, device=DEV)
        w = torch.full((wl.B, wl.H, N), -7.0, dtype=torch.float32, device=DEV)
        out = torch.full((wl.B, wl.H, wl.d), float("nan"), dtype=torch.float32, device=DEV)
        if static:
            ctx.decode_attention_static(cache, q, lens_dev, N, out, idx_out=idx, w_out=w)
        else:
            ctx.decode_attention(cache, q, lens_dev, N, out=out, idx_out=idx, w_out=w)
        torch.cuda.synchronize()
        ctx.device_check()
        res.append((out.cpu().numpy(), idx.cpu().numpy(), w.cpu().numpy()))
    return res


def test_static_scratch_entry_point_matches_the_allocating_one():
    import paper_2404_18057_amd as kc
    ctx = kc.Context(0)
    assert kc.static_scratch_bytes() == 48 << 20
    # two calls in a row on the same device array, the second with a smaller input:
    # a ragged batch with grouped lengths first, then the single small sequence of config 1
    for cfg, kw in ((4, dict(B=6, N=200)), (1, {})):
        wl = ki.config(cfg, **kw)
        print("static entry point: %s B=%d N=%d" % (wl.name, wl.B, wl.N), flush=True)
        cache, q, lens_dev, _, _ = build_layer(ctx, wl, 0)
        (out_a, idx_a, w_a), (out_s, idx_s, w_s) = _both(kc, ctx, wl, cache, q, lens_dev, wl.N)
        assert np.array_equal(idx_a, idx_s), "positions differ"
        assert np.array_equal(w_a, w_s), "weights differ"
        assert np.array_equal(out_a, out_s), "outputs differ"
        for (b, h) in sample_units(wl, 6):      # and both agree with the oracle
            r = oracle_unit(wl, 0, b, h, wl.N)
            check_unit(r, wl.N, out_s[b, h], idx_s[b, h], w_s[b, h], tag="static (%d,%d)" % (b, h))
    # grouped queries in bf16 go through the same scratch
    wl = ki.config(3, B=2, S_cap=3000)
    cache, q, lens_dev, _, _ = build_layer(ctx, wl, 0)
    (out_a, idx_a, w_a), (out_s, idx_s, w_s) = _both(kc, ctx, wl, cache, q, lens_dev, wl.N)
    assert np.array_equal(idx_a, idx_s) and np.array_equal(w_a, w_s) and np.array_equal(out_a, out_s)
    ctx.close()


def test_static_scratch_rejects_shapes_beyond_its_size():
    import paper_2404_18057_amd as kc
    ctx = kc.Context(0)
    # 64 sequences x 32 heads x 16 chunks x 512 candidates x 8 bytes = 128 MiB of candidates
    B, H, S, N = 64, 32, 16384, 512
    k = torch.zeros((B, H, S, 128), dtype=torch.float16, device=DEV)
    cache = kc.LayerCache(k, k)      # V in HBM too: every address is valid whatever the call does
    q = torch.zeros((B, H, 128), dtype=torch.float16, device=DEV)
    lens = torch.full((B,), S, dtype=torch.int32, device=DEV)
    out = torch.zeros((B, H, 128), dtype=torch.float32, device=DEV)
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_attention_static(cache, q, lens, N, out)
    assert e.value.status == -4 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    ctx.device_check()
    ctx.close()
