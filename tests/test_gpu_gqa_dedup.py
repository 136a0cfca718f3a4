"""GPU parity of the de-duplicated V pull for grouped queries (KC_OPT_GQA_DEDUP): same
selection and, up to summation order, the same outputs as the per-head pull; checked against
the oracle on workloads whose heads share pivot positions (so that the union is smaller
than the sum) and on ones where they do not."""
import numpy as np
import pytest
import torch

import kcache_inputs as ki
from harness import build_layer, check_unit, oracle_unit, sample_units

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


def run(ctx, wl, cache, q, lens, dedup):
    idx = torch.full((wl.B, wl.H, wl.N), -7, dtype=torch.int32, device=DEV)
    w = torch.full((wl.B, wl.H, wl.N), -7.0, dtype=torch.float32, device=DEV)
    out = torch.full((wl.B, wl.H, wl.d), float("nan"), dtype=torch.float32, device=DEV)
    ctx.set_gqa_dedup(dedup)
    try:
        ctx.decode_attention(cache, q, lens, wl.N, out=out, idx_out=idx, w_out=w)
        torch.cuda.synchronize()
        ctx.device_check()
    finally:
        ctx.set_gqa_dedup(False)
    return out.cpu().numpy(), idx.cpu().numpy(), w.cpu().numpy()


@pytest.mark.parametrize("shared", [True, False])
@pytest.mark.parametrize("G,N,dtype,d", [(2, 128, "f16", 128), (4, 128, "bf16", 128), (4, 100, "f16", 64),
                                         (8, 32, "f16", 128), (2, 500, "bf16", 256)])
def test_union_pull_matches_oracle_and_per_head_pull(kc, ctx, shared, G, N, dtype, d):
    wl = ki.config(3, B=3, H=2 * G, Hkv=2, S_cap=6000, N=N, dtype=dtype, d=d,
                   shared_pivots=shared, len_range=(1, 6000))
    cache, q, lens, _, _ = build_layer(ctx, wl, 2)
    plain = run(ctx, wl, cache, q, lens, False)
    union = run(ctx, wl, cache, q, lens, True)
    assert np.array_equal(plain[1], union[1]) and np.array_equal(plain[2], union[2])
    assert np.allclose(plain[0], union[0], rtol=1e-4, atol=1e-5)
    for (b, h) in sample_units(wl, 10, seed=G):
        r = oracle_unit(wl, 2, b, h, N)
        check_unit(r, N, union[0][b, h], union[1][b, h], union[2][b, h],
                   tag="dedup G=%d shared=%s (%d,%d)" % (G, shared, b, h))


def test_shared_pivots_make_the_union_smaller(kc, ctx):
    # what the option is for: the heads of a group keep mostly the same rows
    wl = ki.config(3, B=1, S_cap=8192, shared_pivots=True)
    cache, q, lens, _, _ = build_layer(ctx, wl, 0)
    _, idx, _ = run(ctx, wl, cache, q, lens, True)
    G = wl.G
    for hk in range(wl.Hkv):
        rows = [set(idx[0, hk * G + g].tolist()) for g in range(G)]
        union = set().union(*rows)
        assert len(union) < 0.6 * sum(len(r) for r in rows)


def test_falls_back_when_the_group_does_not_fit(kc, ctx):
    # (H/Hkv)^2 * N beyond the table: the per-head pull runs, results unchanged
    wl = ki.config(3, B=1, H=8, Hkv=2, S_cap=3000, N=400)
    cache, q, lens, _, _ = build_layer(ctx, wl, 0)
    a = run(ctx, wl, cache, q, lens, False)
    b = run(ctx, wl, cache, q, lens, True)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
