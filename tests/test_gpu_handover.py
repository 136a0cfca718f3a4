"""The hand-over between workgroups of one launch (chunk results to the workgroup that finishes
a unit) must not depend on where the workgroups run or on timing: the same results with the
chunks of a unit dealt over all XCDs, and bit-identical results over many launches."""
import numpy as np
import pytest
import torch

import kcache_inputs as ki
from harness import build_layer, run_and_check, sample_units, pinned_like, check_unit
import oracle

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
    c.set_xcd_spread(False)
    c.close()


def decode(ctx, wl, cache, q, lens, N):
    idx = torch.empty((wl.B, wl.H, N), dtype=torch.int32, device=DEV)
    w = torch.empty((wl.B, wl.H, N), dtype=torch.float32, device=DEV)
    out = ctx.decode_attention(cache, q, lens, N, idx_out=idx, w_out=w)
    return out, idx, w


@pytest.mark.parametrize("cfg,kw", [(1, {}), (4, dict(B=12)), (3, dict(B=3, S_cap=5000))])
def test_chunks_dealt_over_all_xcds_give_the_same_results(kc, ctx, cfg, kw):
    wl = ki.config(cfg, **kw)
    cache, q, lens, _, _ = build_layer(ctx, wl, 0)
    ctx.set_xcd_spread(False)
    a = [t.clone() for t in decode(ctx, wl, cache, q, lens, wl.N)]
    ctx.set_xcd_spread(True)
    try:
        _, n, (out_h, idx_h, w_h) = run_and_check(ctx, wl, 0, cache, q, lens, sample_units(wl, 12))
    finally:
        ctx.set_xcd_spread(False)
    assert np.array_equal(out_h, a[0].cpu().numpy())
    assert np.array_equal(idx_h, a[1].cpu().numpy())
    assert np.array_equal(w_h, a[2].cpu().numpy())


def test_many_chunks_per_unit_across_xcds(kc, ctx):
    # 600 000 positions: 586 chunks of one unit spread over every XCD, merged by one workgroup
    rng = np.random.default_rng(32)
    S, N = 600_000, 8
    q = torch.from_numpy(rng.standard_normal((1, 1, 128)).astype(np.float32)).half()
    K = torch.from_numpy(rng.standard_normal((1, 1, S, 128)).astype(np.float32)).half()
    V = torch.from_numpy(rng.standard_normal((1, 1, S, 128)).astype(np.float32)).half()
    v_host = pinned_like(V)
    v_host.copy_(V)
    cache = kc.LayerCache(K.to(DEV), v_host)
    lens = torch.tensor([S], dtype=torch.int32, device=DEV)
    idx = torch.empty((1, 1, N), dtype=torch.int32, device=DEV)
    w = torch.empty((1, 1, N), dtype=torch.float32, device=DEV)
    ctx.set_xcd_spread(True)
    try:
        out = ctx.decode_attention(cache, q.to(DEV), lens, N, idx_out=idx, w_out=w)
        torch.cuda.synchronize()
        ctx.device_check()
    finally:
        ctx.set_xcd_spread(False)
    r = oracle.decode_unit(ki.as_bits(q)[0, 0], ki.as_bits(K)[0, 0], ki.as_bits(V)[0, 0], oracle.F16, N,
                           want_scores=True)
    r["v"] = oracle.decode16(ki.as_bits(V)[0, 0], oracle.F16)
    check_unit(r, N, out[0, 0].cpu().numpy(), idx[0, 0].cpu().numpy(), w[0, 0].cpu().numpy())


@pytest.mark.parametrize("cfg,kw,spread", [(5, {}, False), (3, dict(B=4), False), (5, dict(B=1), True)])
def test_two_hundred_launches_are_bit_identical(kc, ctx, cfg, kw, spread):
    """Config 5's per-layer shape (single heads, 32 chunks a unit, the pruned merge) and a
    grouped-query shape (four heads a unit): launch 0 is checked against the oracle on a
    sample, every later launch must reproduce it bit for bit."""
    wl = ki.config(cfg, **kw)
    cache, q, lens, _, _ = build_layer(ctx, wl, 0, chunk_T=16384)
    ctx.set_xcd_spread(spread)
    try:
        _, _, first = run_and_check(ctx, wl, 0, cache, q, lens, sample_units(wl, 8))
        ref = [torch.from_numpy(x).to(DEV) for x in first]
        for i in range(1, 200):
            out, idx, w = decode(ctx, wl, cache, q, lens, wl.N)
            same = torch.equal(out, ref[0]) and torch.equal(idx, ref[1]) and torch.equal(w, ref[2])
            assert same, "launch %d differs from launch 0" % i
        ctx.device_check()
    finally:
        ctx.set_xcd_spread(False)
