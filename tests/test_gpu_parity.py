"""GPU parity: libkcache (through the C ABI) against the CPU oracle, unit by unit."""
import numpy as np
import pytest
import torch

import kcache_inputs as ki
import oracle
from harness import (build_layer, check_unit, dtype_code, oracle_unit, pinned_like, run_and_check,
                     sample_units)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def kc():
    import paper_2404_18057_amd as kc
    return kc


@pytest.fixture(scope="module", params=["fused", "unfused"])
def ctx(kc, request):
    """Every test runs on both decode paths: the fused single launch (default)
    and the separate scan / select / gather launches."""
    c = kc.Context(0)
    c.set_fused(request.param == "fused")
    c.fused_default = request.param == "fused"
    yield c
    c.close()


def bits_t(a, dtype=torch.float16):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dtype)


def manual_case(kc, ctx, q, K, V, lens, N, dtype=torch.float16, parts=0, gather_mode=0):
    """q [B][H][d], K/V [B][Hkv][S][d] float arrays -> GPU result + oracle result."""
    qt, kt, vt = bits_t(q, dtype), bits_t(K, dtype), bits_t(V, dtype)
    B, H, d = qt.shape
    k_dev = kt.to(DEV)
    v_host = pinned_like(vt)
    v_host.copy_(vt)
    cache = kc.LayerCache(k_dev, v_host)
    lens_dev = torch.tensor(lens, dtype=torch.int32, device=DEV)
    idx = torch.empty((B, H, N), dtype=torch.int32, device=DEV)
    w = torch.empty((B, H, N), dtype=torch.float32, device=DEV)
    ctx.set_pipeline_parts(parts)
    out = ctx.decode_attention(cache, qt.to(DEV), lens_dev, N, idx_out=idx, w_out=w,
                               gather_mode=gather_mode)
    torch.cuda.synchronize()
    ctx.set_pipeline_parts(0)
    ctx.device_check()
    code = oracle.F16 if dtype == torch.float16 else oracle.BF16
    return (out.cpu().numpy(), idx.cpu().numpy(), w.cpu().numpy(),
            (ki.as_bits(qt), ki.as_bits(kt), ki.as_bits(vt), code))


def check_manual(res, lens, N, G=1):
    out, idx, w, (qb, kb, vb, code) = res
    B, H, _ = qb.shape
    for b in range(B):
        s = int(lens[b])
        for h in range(H):
            r = oracle.decode_unit(qb[b, h], kb[b, h // G, :s], vb[b, h // G, :s], code, N,
                                   want_scores=True)
            r["v"] = oracle.decode16(vb[b, h // G, :s], code)
            check_unit(r, N, out[b, h], idx[b, h], w[b, h], tag="manual (%d,%d)" % (b, h))


# ------------------------------------------------------------------ named configurations
def test_config1_every_unit(kc, ctx):
    wl = ki.config(1)
    cache, q, lens, _, _ = build_layer(ctx, wl, 0)
    same, n, _ = run_and_check(ctx, wl, 0, cache, q, lens, sample_units(wl, 10 ** 9))
    assert n == 8


@pytest.mark.parametrize("parts", [1, 3])
def test_config1_pipelined_parts_give_identical_results(kc, ctx, parts):
    wl = ki.config(1)
    cache, q, lens, _, _ = build_layer(ctx, wl, 0)
    ctx.set_fused(False)            # parts only exist on the unfused path
    ctx.set_pipeline_parts(1)
    _, _, base = run_and_check(ctx, wl, 0, cache, q, lens, [(0, 0)])
    ctx.set_pipeline_parts(parts)
    _, _, got = run_and_check(ctx, wl, 0, cache, q, lens, sample_units(wl, 10 ** 9))
    ctx.set_pipeline_parts(0)
    ctx.set_fused(ctx.fused_default)
    for a, b in zip(base, got):
        assert np.array_equal(a, b)


def spread_layers(wl):
    """First, last and two interior layers."""
    return (0, wl.L // 3, (2 * wl.L) // 3, wl.L - 1)


def big_sample(ctx, per_layer):
    """The full sample on the default (fused) path; the unfused launches, which every other
    test also covers, check a smaller one."""
    return per_layer if ctx.fused_default else max(8, per_layer // 8)


def test_config3_shape_gqa_bf16_four_layers(kc, ctx):
    # full per-layer shape of config 3 (B 16, 32 query / 8 KV heads, 8192, N 128, bf16):
    # 4 x 64 = 256 sampled units over the first, two interior and the last layer
    wl = ki.config(3)
    for layer in spread_layers(wl):
        cache, q, lens, _, _ = build_layer(ctx, wl, layer)
        run_and_check(ctx, wl, layer, cache, q, lens, sample_units(wl, big_sample(ctx, 64), seed=layer))
        del cache


def test_config2_shape_four_layers(kc, ctx):
    # full per-layer shape of config 2 (B 8, 32 heads, 32768, N 256, fp16): 4 x 64 = 256 units
    wl = ki.config(2)
    for layer in spread_layers(wl):
        cache, q, lens, _, _ = build_layer(ctx, wl, layer, chunk_T=8192)
        run_and_check(ctx, wl, layer, cache, q, lens, sample_units(wl, big_sample(ctx, 64), seed=layer))
        del cache


def test_config5_shape_four_layers(kc, ctx):
    # full per-layer shape of config 5 (B 2, 40 heads, 65536, N 512, fp16): 4 x 64 = 256 of
    # the 4 x 80 units of the first, two interior and the last layer
    wl = ki.config(5)
    for layer in spread_layers(wl):
        cache, q, lens, _, _ = build_layer(ctx, wl, layer, chunk_T=16384)
        run_and_check(ctx, wl, layer, cache, q, lens, sample_units(wl, big_sample(ctx, 64), seed=layer))
        del cache


@pytest.mark.parametrize("frac", [0.001, 0.01, 0.05])
def test_config4_ragged_sweeps(kc, ctx, frac):
    # 64 ragged sequences, N swept over {32..512}, pivot fraction over {0.1, 1, 5} %
    wl = ki.config(4, pivot_frac=frac)
    cache, q, lens, _, _ = build_layer(ctx, wl, 0)
    for N in (32, 64, 128, 256, 512):
        run_and_check(ctx, wl, 0, cache, q, lens, sample_units(wl, 24, seed=N), N=N)


# ------------------------------------------------------------------ edge cases
def test_uniform_scores_break_ties_towards_lower_positions(kc, ctx):
    rng = np.random.default_rng(0)
    B, H, S, d, N = 2, 2, 700, 128, 37
    q = rng.standard_normal((B, H, d))
    K = np.tile(rng.standard_normal((B, H, 1, d)), (1, 1, S, 1))     # identical rows
    V = rng.standard_normal((B, H, S, d))
    lens = [700, 123]
    out, idx, w, _ = res = manual_case(kc, ctx, q, K, V, lens, N)
    for b in range(B):
        for h in range(H):
            assert idx[b, h].tolist() == list(range(N))
            assert np.allclose(w[b, h], 1.0 / lens[b], rtol=1e-5)
    check_manual(res, lens, N)


def test_partial_ties_at_the_boundary(kc, ctx):
    # 3 distinct score levels; the boundary falls inside the middle level
    rng = np.random.default_rng(1)
    S, d, N = 300, 128, 50
    base = rng.standard_normal(d)
    q = base[None, None, :]
    level = rng.choice([0.0, 0.5, 1.0], size=S, p=[0.6, 0.3, 0.1])
    K = (level[:, None] * base[None, :] / 4.0)[None, None]
    V = rng.standard_normal((1, 1, S, d))
    out, idx, w, _ = res = manual_case(kc, ctx, q, K, V, [S], N)
    hi = np.flatnonzero(level == 1.0)
    mid = np.flatnonzero(level == 0.5)
    want = sorted(hi.tolist() + mid[:N - len(hi)].tolist())
    assert len(hi) < N < len(hi) + len(mid)
    assert idx[0, 0].tolist() == want
    check_manual(res, [S], N)


@pytest.mark.parametrize("S_cap,lens,N", [
    (1, [1], 4),                 # a single cached position
    (1000, [1000, 1, 63], 64),   # capacity not a multiple of any tile, N > s
    (1029, [1029, 1025], 1),     # N = 1, ragged tail of one row past a block
    (4100, [4100, 2049], 4100),  # N = s: full attention
])
def test_small_shapes_and_ragged_tails(kc, ctx, S_cap, lens, N):
    rng = np.random.default_rng(S_cap)
    B, H, d = len(lens), 3, 128
    q = rng.standard_normal((B, H, d))
    K = rng.standard_normal((B, H, S_cap, d))
    V = rng.standard_normal((B, H, S_cap, d))
    for b in range(B):          # padding must be ignored: make it attractive
        K[b, :, lens[b]:] = 4 * q[b][:, None, :]
    res = manual_case(kc, ctx, q, K, V, lens, N)
    check_manual(res, lens, N)


@pytest.mark.parametrize("G", [2, 8, 16, 32])
def test_other_group_sizes(kc, ctx, G):
    # 16 and 32 (e.g. 32 query heads over 2 KV groups, or multi-query attention) run as
    # several launch units of 8 heads per KV head
    rng = np.random.default_rng(G)
    B, Hkv, S, d, N = 2, 2, 1500, 128, 20
    H = Hkv * G
    q = rng.standard_normal((B, H, d))
    K = rng.standard_normal((B, Hkv, S, d))
    V = rng.standard_normal((B, Hkv, S, d))
    res = manual_case(kc, ctx, q, K, V, [1500, 400], N, dtype=torch.bfloat16)
    check_manual(res, [1500, 400], N, G=G)


def test_staged_gather_matches_zero_copy(kc, ctx):
    wl = ki.config(1)
    cache, q, lens, _, _ = build_layer(ctx, wl, 0)
    ctx.set_fused(False)            # same kernels on both sides: results must be bit-equal
    _, _, a = run_and_check(ctx, wl, 0, cache, q, lens, sample_units(wl, 10 ** 9))
    ctx.set_fused(ctx.fused_default)
    for threads in (1, 4):
        ctx.set_staged_threads(threads)
        _, _, b = run_and_check(ctx, wl, 0, cache, q, lens, sample_units(wl, 10 ** 9),
                                gather_mode=kc.GATHER_STAGED)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)


def test_results_are_deterministic(kc, ctx):
    wl = ki.config(4, B=8)
    cache, q, lens, _, _ = build_layer(ctx, wl, 0)
    _, _, a = run_and_check(ctx, wl, 0, cache, q, lens, [(0, 0)])
    _, _, b = run_and_check(ctx, wl, 0, cache, q, lens, [(7, 31)])
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_fused_and_unfused_paths_agree(kc, ctx):
    # same index sets wherever neither is in a tie band (checked against the oracle by
    # the other tests); here: positions identical, weights and outputs to fp32 rounding
    wl = ki.config(4, B=6, N=200)
    cache, q, lens, _, _ = build_layer(ctx, wl, 0)
    res = {}
    for fused in (True, False):
        ctx.set_fused(fused)
        _, _, res[fused] = run_and_check(ctx, wl, 0, cache, q, lens, sample_units(wl, 12))
    ctx.set_fused(ctx.fused_default)
    assert np.array_equal(res[True][1], res[False][1])
    assert np.allclose(res[True][2], res[False][2], rtol=1e-5, atol=1e-9)
    assert np.allclose(res[True][0], res[False][0], rtol=1e-4, atol=1e-6)


def test_fused_counters_are_clean_between_calls_of_different_shapes(kc, ctx):
    # the ticket counters return to zero after every launch: alternate shapes on one context
    for cfg, kw in ((1, {}), (4, dict(B=5, N=48)), (1, dict(S_cap=3000, N=700)), (3, dict(B=3, S_cap=1500))):
        wl = ki.config(cfg, **kw)
        cache, q, lens, _, _ = build_layer(ctx, wl, 0)
        for _ in range(2):
            run_and_check(ctx, wl, 0, cache, q, lens, sample_units(wl, 6))


# ------------------------------------------------------------------ cache store
@pytest.mark.parametrize("T,S_cap,pos,host_pos", [
    (37, 100, [0, 63, 11], False),       # a small store: one launch for both halves
    (37, 100, [0, 63, 11], True),
    (600, 700, [0, 100, 37], False),     # a large one: V half on the side stream, by the kernel
    (600, 700, [0, 100, 37], True),      # ... and by the copy engine (positions on the host)
])
def test_prefill_store_matches_oracle_bit_for_bit(kc, ctx, T, S_cap, pos, host_pos):
    rng = np.random.default_rng(5)
    B, Hkv, d = 3, 5, 128
    k_new = bits_t(rng.standard_normal((B, T, Hkv, d)))
    v_new = bits_t(rng.standard_normal((B, T, Hkv, d)))
    pos = np.array(pos, np.int32)
    k_cache = torch.full((B, Hkv, S_cap, d), 9.0, dtype=torch.float16)
    v_cache = torch.full((B, Hkv, S_cap, d), -9.0, dtype=torch.float16)
    k_ref, v_ref = ki.as_bits(k_cache).copy(), ki.as_bits(v_cache).copy()
    oracle.store(k_ref, v_ref, ki.as_bits(k_new), ki.as_bits(v_new), pos)
    k_dev = k_cache.to(DEV)
    v_host = pinned_like(v_cache)
    v_host.copy_(v_cache)
    cache = kc.LayerCache(k_dev, v_host)
    done = torch.cuda.Event()
    if host_pos:
        ctx.prefill_store_at(cache, k_new.to(DEV), v_new.to(DEV), pos, done_event=done)
    else:
        ctx.prefill_store(cache, k_new.to(DEV), v_new.to(DEV), torch.from_numpy(pos).to(DEV),
                          done_event=done)
    done.synchronize()
    assert np.array_equal(ki.as_bits(v_host), v_ref)
    torch.cuda.synchronize()
    assert np.array_equal(ki.as_bits(k_dev), k_ref)
    ctx.device_check()


def test_append_one_token_then_decode_sees_it(kc, ctx):
    # decode flow: the new token's K/V rows are stored (T = 1), then attention runs
    wl = ki.config(1, S_cap=600, N=16, seed=5)
    q, k, v, _ = ki.gen_layer(wl, 0, DEV)
    s0 = 555
    k_cache = k.clone()
    v_host = pinned_like(v)
    v_host.copy_(v)
    cache = kc.LayerCache(k_cache, v_host)
    # the appended token is a strong match for every head's query, with a marker V row
    k_tok = (q.float() * 3).to(q.dtype).reshape(wl.B, 1, wl.Hkv, wl.d).contiguous()
    v_tok = torch.full((wl.B, 1, wl.Hkv, wl.d), 2.5, dtype=q.dtype, device=DEV)
    pos = torch.full((wl.B,), s0, dtype=torch.int32, device=DEV)
    ctx.prefill_store(cache, k_tok, v_tok, pos)
    lens = torch.full((wl.B,), s0 + 1, dtype=torch.int32, device=DEV)
    idx = torch.empty((wl.B, wl.H, wl.N), dtype=torch.int32, device=DEV)
    w = torch.empty((wl.B, wl.H, wl.N), dtype=torch.float32, device=DEV)
    out = ctx.decode_attention(cache, q, lens, wl.N, idx_out=idx, w_out=w)
    torch.cuda.synchronize()
    kb, vb = ki.as_bits(k_cache), ki.as_bits(v_host)
    qb = ki.as_bits(q)
    for h in range(wl.H):
        assert s0 in idx[0, h].tolist()
        r = oracle.decode_unit(qb[0, h], kb[0, h, :s0 + 1], vb[0, h, :s0 + 1], dtype_code(wl),
                               wl.N, want_scores=True)
        r["v"] = oracle.decode16(vb[0, h, :s0 + 1], dtype_code(wl))
        check_unit(r, wl.N, out[0, h].cpu().numpy(), idx[0, h].cpu().numpy(),
                   w[0, h].cpu().numpy(), tag="append head %d" % h)


def test_generator_bits_are_identical_on_cpu_and_gpu(kc):
    for cfg, layer in ((1, 0), (3, 5)):
        wl = ki.config(cfg).replace(B=2) if cfg == 3 else ki.config(cfg)
        q, k, v, _ = ki.gen_layer(wl, layer, DEV)
        qc, kc_, vc, _ = ki.gen_layer(wl, layer, "cpu")
        assert torch.equal(q.cpu(), qc) and torch.equal(k.cpu(), kc_) and torch.equal(v.cpu(), vc)


# ------------------------------------------------------------------ error paths (every kernel still exits normally)
def test_bad_arguments_are_reported_not_fatal(kc, ctx):
    wl = ki.config(1)
    q, k, v, lens = ki.gen_layer(wl, 0, DEV)
    v_pin = pinned_like(v)
    cache = kc.LayerCache(k, v_pin)
    lens_dev = torch.from_numpy(lens).to(DEV)
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_attention(cache, q, lens_dev, 0)
    assert e.value.status == -1
    # pageable (not pinned) V cache
    bad = kc.LayerCache(k, v.cpu())
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_attention(bad, q, lens_dev, 8)
    assert e.value.status == -3
    # a sequence length outside the cache is clamped by the kernels and flagged
    wrong = torch.tensor([wl.S_cap + 5], dtype=torch.int32, device=DEV)
    ctx.decode_attention(cache, q, wrong, 8)
    with pytest.raises(kc.KCacheError) as e:
        ctx.device_check()
    assert e.value.status == -6
    ctx.device_check()      # the flag is cleared by the failing check
    # a store position outside the cache is skipped and flagged
    k_new = k[:, :, :4].permute(0, 2, 1, 3).contiguous()
    pos = torch.tensor([wl.S_cap - 2], dtype=torch.int32, device=DEV)
    ctx.prefill_store(cache, k_new, k_new, pos)
    with pytest.raises(kc.KCacheError) as e:
        ctx.device_check()
    assert e.value.status == -6
    # with the positions on the host the same mistake is refused before anything is enqueued
    with pytest.raises(kc.KCacheError) as e:
        ctx.prefill_store_at(cache, k_new, k_new, [wl.S_cap - 2])
    assert e.value.status == -1
    ctx.device_check()


def test_non_finite_scores_never_leave_the_sequence(kc, ctx):
    """A NaN in q makes every score of that head NaN; NaN rows in K make some scores of another
    head NaN (enough of them in one chunk to turn its pruning edge into NaN).  The results of
    those units are unspecified, but every kept position must lie inside the sequence, exactly
    N_eff of them are kept, no row outside the cache is read (device check clean), and the
    heads that saw only finite values still match the oracle."""
    rng = np.random.default_rng(123)
    B, H, S, d, N = 2, 4, 9000, 128, 64     # 9 chunks of 1024: the pruned merge runs
    q = rng.standard_normal((B, H, d)).astype(np.float32)
    K = rng.standard_normal((B, H, S, d)).astype(np.float32)
    V = rng.standard_normal((B, H, S, d)).astype(np.float32)
    q[0, 1, 5] = np.nan                      # head (0, 1): all scores NaN
    K[0, 2, 2048:2048 + 40, 7] = np.nan      # head (0, 2): 40 NaN scores in the third chunk
    K[1, 0, 100, 0] = np.inf                 # head (1, 0): one infinite score
    lens = [S, 4500]
    out, idx, w, (qb, kb, vb, code) = manual_case(kc, ctx, q, K, V, lens, N)   # runs device_check
    for b in range(B):
        s = lens[b]
        for h in range(H):
            kept = idx[b, h]
            assert ((kept >= 0) & (kept < s)).all(), "position outside the sequence at (%d,%d)" % (b, h)
            assert len(set(kept.tolist())) == N, "positions not distinct at (%d,%d)" % (b, h)
            if (b, h) in ((0, 1), (0, 2), (1, 0)):
                continue
            r = oracle.decode_unit(qb[b, h], kb[b, h, :s], vb[b, h, :s], code, N, want_scores=True)
            r["v"] = oracle.decode16(vb[b, h, :s], code)
            check_unit(r, N, out[b, h], idx[b, h], w[b, h], tag="finite head (%d,%d)" % (b, h))
    # the same launch shape with finite inputs afterwards: nothing was left behind
    q[0, 1, 5] = 0.5
    K[0, 2, 2048:2048 + 40, 7] = 0.25
    K[1, 0, 100, 0] = 1.0
    res = manual_case(kc, ctx, q, K, V, lens, N)
    check_manual(res, lens, N)


# ------------------------------------------------------------------ renormalised variant
@pytest.mark.parametrize("gather_mode", [0, 1])
def test_renormalised_variant_matches_its_oracle(kc, ctx, gather_mode):
    """KC_OPT_RENORMALIZE divides the kept weights by their sum (the alternative reading of
    the paper's remark that TopN regularises the softmax); same selection, same tolerance."""
    if gather_mode == 1 and ctx.fused_default:
        pytest.skip("the staged gather runs on the unfused path")
    rng = np.random.default_rng(77)
    B, H, S, d = 2, 3, 3000, 128
    q = rng.standard_normal((B, H, d))
    K = rng.standard_normal((B, H, S, d))
    V = rng.standard_normal((B, H, S, d))
    lens = [3000, 700]
    ctx.set_renormalize(True)
    try:
        for N in (1, 40, 1500):   # 1500 > the 1024 entries the fused kernel stages in LDS
            out, idx, w, (qb, kb, vb, code) = manual_case(kc, ctx, q, K, V, lens, N,
                                                          gather_mode=gather_mode)
            for b in range(B):
                s = lens[b]
                for h in range(H):
                    r = oracle.decode_unit(qb[b, h], kb[b, h, :s], vb[b, h, :s], code, N,
                                           want_scores=True, renormalise=True)
                    n_eff = min(N, s)
                    assert set(idx[b, h, :n_eff].tolist()) == set(r["idx"][:n_eff].tolist())
                    assert abs(float(w[b, h].sum()) - 1.0) < 1e-4
                    assert np.allclose(w[b, h], r["w"], rtol=2e-3, atol=1e-7)
                    err = np.abs(out[b, h].astype(np.float64) - r["out"])
                    assert (err <= 1e-3 + 2e-3 * np.abs(r["out"])).all()
    finally:
        ctx.set_renormalize(False)
    # and the default is untouched afterwards: kept weights sum to less than one again
    out, idx, w, _ = manual_case(kc, ctx, q, K, V, lens, 40)
    assert float(w[0, 0].sum()) < 0.999


# ------------------------------------------------------------------ seeded random shapes
@pytest.mark.parametrize("case", range(12))
def test_seeded_random_shapes(kc, ctx, case):
    """Shapes drawn from a seeded stream: batch, KV heads, group size, capacity, ragged
    lengths (including 1 and the full capacity), N from 1 to beyond the longest sequence,
    both dtypes, with a few duplicated K rows so that exact ties occur."""
    rng = np.random.default_rng(1000 + case)
    B = int(rng.integers(1, 4))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 4, 8, 16]))
    S = int(rng.choice([1, 63, 512, 513, 1500, 2048, 4097, 6000]))
    N = int(rng.choice([1, 2, 17, 64, 300, 1025, 2000]))
    dtype = torch.float16 if rng.integers(2) else torch.bfloat16
    H = Hkv * G
    lens = [int(rng.integers(1, S + 1)) for _ in range(B)]
    lens[0] = S
    if B > 1:
        lens[1] = 1
    q = rng.standard_normal((B, H, 128))
    K = rng.standard_normal((B, Hkv, S, 128))
    V = rng.standard_normal((B, Hkv, S, 128))
    if S >= 64:                      # exact ties: some rows repeat an earlier row
        for _ in range(8):
            a_, b_ = sorted(int(x) for x in rng.integers(0, S, size=2))
            K[:, :, b_] = K[:, :, a_]
    res = manual_case(kc, ctx, q, K, V, lens, N, dtype=dtype)
    check_manual(res, lens, N, G=G)


def test_many_tied_candidates_defeat_the_pruning(kc, ctx):
    """40 000 positions, N = 512, two score levels: 100 scattered positions score high, all the
    others tie.  The unit brings 20 x 512 candidates, more than the merging workgroup's LDS
    buffer holds; every chunk reports the tied score as its edge, so nothing can be dropped
    and the selection has to run over the lists in memory, breaking the tie by position."""
    rng = np.random.default_rng(77)
    S, d, N = 40_000, 128, 512
    base = rng.standard_normal(d)
    q = base[None, None, :]
    hi = np.sort(rng.choice(S, size=100, replace=False))
    level = np.zeros(S)
    level[hi] = 1.0
    K = ((0.25 + level[:, None]) * base[None, :] / 4.0)[None, None]
    V = rng.standard_normal((1, 1, S, d))
    out, idx, w, _ = res = manual_case(kc, ctx, q, K, V, [S], N)
    rest = np.setdiff1d(np.arange(S), hi)[:N - len(hi)]
    assert idx[0, 0].tolist() == sorted(hi.tolist() + rest.tolist())
    check_manual(res, [S], N)


def test_more_chunks_than_threads_in_the_merging_workgroup(kc, ctx):
    """600 000 positions with N = 8: 586 chunks of 1024 rows, more than the 512 threads that
    each fetch one chunk's partials and edge in the first round."""
    rng = np.random.default_rng(32)
    S, N = 600_000, 8
    q = rng.standard_normal((1, 1, 128)).astype(np.float32)
    K = rng.standard_normal((1, 1, S, 128)).astype(np.float32)
    V = rng.standard_normal((1, 1, S, 128)).astype(np.float32)
    K[0, 0, 599_990] = K[0, 0, 5]                       # an exact tie between the ends
    res = manual_case(kc, ctx, q, K, V, [S], N)
    check_manual(res, [S], N)


def test_context_too_long_for_the_merge_buffer(kc, ctx):
    """300 000 positions with N = 256: even at the largest chunk size the unit's candidates
    (37 x 256) exceed the merging workgroup's LDS buffer; they are judged against the chunks'
    edges in registers, and only the survivors are selected from.  Two heads, one of them
    with duplicated rows across distant chunks."""
    rng = np.random.default_rng(31)
    S, N = 300_000, 256
    q = rng.standard_normal((1, 2, 128))
    K = rng.standard_normal((1, 2, S, 128)).astype(np.float32)
    V = rng.standard_normal((1, 2, S, 128)).astype(np.float32)
    K[0, 1, 250_000:250_040] = K[0, 1, 10:50]          # exact ties far apart
    K[0, :, ::997] += 2.5 * q[0][:, None, :] / np.linalg.norm(q[0], axis=-1)[:, None, None] * 11.3
    res = manual_case(kc, ctx, q, K, V, [S], N)
    check_manual(res, [S], N)
