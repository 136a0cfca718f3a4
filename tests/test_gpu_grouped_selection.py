"""GPU parity for grouped-query units, whose heads are selected side by side (one wavefront
per head): ties, degenerate score distributions, non-finite scores, several merge rounds."""
import numpy as np
import pytest
import torch

import oracle
from harness import check_unit
from test_gpu_parity import check_manual, manual_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kc():
    import paper_2404_18057_amd as kc
    return kc


@pytest.fixture(scope="module")
def ctx(kc):
    c = kc.Context(0)
    c.fused_default = True
    yield c
    c.close()


@pytest.mark.parametrize("G", [2, 4, 8])
def test_equal_scores_keep_the_first_positions(kc, ctx, G):
    rng = np.random.default_rng(G)
    B, Hkv, S, d, N = 2, 2, 5000, 128, 37
    q = rng.standard_normal((B, Hkv * G, d))
    K = np.tile(rng.standard_normal((B, Hkv, 1, d)), (1, 1, S, 1))     # identical rows
    V = rng.standard_normal((B, Hkv, S, d))
    lens = [5000, 123]
    out, idx, w, _ = res = manual_case(kc, ctx, q, K, V, lens, N)
    for b in range(B):
        for h in range(Hkv * G):
            assert idx[b, h].tolist() == list(range(N))
            assert np.allclose(w[b, h], 1.0 / lens[b], rtol=1e-5)
    check_manual(res, lens, N, G=G)


@pytest.mark.parametrize("G", [2, 4, 8])
def test_boundary_inside_a_level_of_equal_scores(kc, ctx, G):
    """Three score levels; the boundary falls inside the middle one, which holds far more
    entries than the exact list of the selection takes: the radix path decides it."""
    rng = np.random.default_rng(10 + G)
    S, d, N = 6000, 128, 700 if G == 2 else 200
    base = rng.standard_normal(d)
    q = (np.arange(1, G + 1)[:, None] * base[None, :] / G)[None]          # positive multiples
    level = rng.choice([0.0, 0.5, 1.0], size=S, p=[0.6, 0.38, 0.02])
    K = (level[:, None] * base[None, :] / 4.0)[None, None]
    V = rng.standard_normal((1, 1, S, d))
    out, idx, w, _ = res = manual_case(kc, ctx, q, K, V, [S], N)
    hi = np.flatnonzero(level == 1.0)
    mid = np.flatnonzero(level == 0.5)
    assert len(hi) < N < len(hi) + len(mid)
    want = sorted(hi.tolist() + mid[:N - len(hi)].tolist())
    for g in range(G):
        assert idx[0, g].tolist() == want
    check_manual(res, [S], N, G=G)


@pytest.mark.parametrize("G,S,N", [(4, 9000, 1), (4, 9000, 64), (4, 9000, 256), (4, 9000, 300),
                                   (8, 40000, 64), (2, 70000, 128), (8, 2500, 2500)])
def test_random_scores_with_repeated_rows(kc, ctx, G, S, N):
    """Random scores with rows repeated inside and across chunks, so that exact ties land in
    the exactly ranked list; (8, 40000, 64) merges its heads in three rounds, 300 and 2500
    kept rows take the merge of the whole workgroup."""
    rng = np.random.default_rng(S + N)
    B, Hkv, d = 2, 2, 128
    q = rng.standard_normal((B, Hkv * G, d))
    K = rng.standard_normal((B, Hkv, S, d))
    src = rng.integers(0, S, size=200)
    dst = rng.integers(0, S, size=200)
    K[:, :, dst] = K[:, :, src]
    V = rng.standard_normal((B, Hkv, S, d))
    lens = [S, S // 3 + 1]
    for dtype in (torch.float16, torch.bfloat16):
        res = manual_case(kc, ctx, q, K, V, lens, N, dtype=dtype)
        check_manual(res, lens, N, G=G)


@pytest.mark.parametrize("G,S,N,rows", [(4, 70000, 16, 512), (4, 70000, 200, 512), (8, 70000, 40, 512),
                                        (4, 300000, 24, 512), (2, 150000, 256, 1024)])
def test_many_chunks_per_unit(kc, ctx, G, S, N, rows):
    """Small chunks forced on long contexts: 137, 586 and 147 chunks per unit, i.e. more chunks
    than rows to keep (the unit's pruning bound is then the N-th largest chunk bound, found over
    several bounds per lane, or the smallest one beyond 512 chunks) and fewer (the smallest
    bound).  Repeated rows put exact ties among the candidates."""
    rng = np.random.default_rng(S + N + G)
    B, Hkv, d = 1, 2, 128
    q = rng.standard_normal((B, Hkv * G, d))
    K = rng.standard_normal((B, Hkv, S, d)).astype(np.float32)
    src = rng.integers(0, S, size=300)
    dst = rng.integers(0, S, size=300)
    K[:, :, dst] = K[:, :, src]
    V = rng.standard_normal((B, Hkv, S, d)).astype(np.float32)
    ctx.set_fused_rows(rows)
    try:
        res = manual_case(kc, ctx, q, K, V, [S], N)
    finally:
        ctx.set_fused_rows(0)
    check_manual(res, [S], N, G=G)


def test_renormalised_weights_in_groups(kc, ctx):
    rng = np.random.default_rng(5)
    B, Hkv, G, S, d, N = 2, 2, 4, 7000, 128, 48
    q = rng.standard_normal((B, Hkv * G, d))
    K = rng.standard_normal((B, Hkv, S, d))
    V = rng.standard_normal((B, Hkv, S, d))
    lens = [7000, 2100]
    ctx.set_renormalize(True)
    try:
        out, idx, w, (qb, kb, vb, code) = manual_case(kc, ctx, q, K, V, lens, N)
        for b in range(B):
            s = lens[b]
            for h in range(Hkv * G):
                r = oracle.decode_unit(qb[b, h], kb[b, h // G, :s], vb[b, h // G, :s], code, N,
                                       want_scores=True, renormalise=True)
                assert set(idx[b, h].tolist()) == set(r["idx"][:N].tolist())
                assert abs(float(w[b, h].sum()) - 1.0) < 1e-4
                assert np.allclose(w[b, h], r["w"], rtol=2e-3, atol=1e-7)
                err = np.abs(out[b, h].astype(np.float64) - r["out"])
                assert (err <= 1e-3 + 2e-3 * np.abs(r["out"])).all()
    finally:
        ctx.set_renormalize(False)


def test_non_finite_scores_in_a_group(kc, ctx):
    """NaN in one head's query, NaN and infinite rows of K seen by a whole group: those
    units' results are unspecified, but every kept position lies inside the sequence and is
    distinct, nothing outside the cache is read, and the other groups match the oracle."""
    rng = np.random.default_rng(321)
    B, Hkv, G, S, d, N = 2, 3, 4, 9000, 128, 64
    H = Hkv * G
    q = rng.standard_normal((B, H, d)).astype(np.float32)
    K = rng.standard_normal((B, Hkv, S, d)).astype(np.float32)
    V = rng.standard_normal((B, Hkv, S, d)).astype(np.float32)
    q[0, 1, 5] = np.nan                      # one head of group (0, 0): all scores NaN
    K[0, 1, 2048:2048 + 40, 7] = np.nan      # group (0, 1): 40 NaN scores in one chunk
    K[1, 0, 100, 0] = np.inf                 # group (1, 0): one infinite score per head
    lens = [S, 4500]
    out, idx, w, (qb, kb, vb, code) = manual_case(kc, ctx, q, K, V, lens, N)   # runs device_check
    spoiled = {(0, 1)} | {(0, h) for h in range(G, 2 * G)} | {(1, h) for h in range(G)}
    for b in range(B):
        s = lens[b]
        for h in range(H):
            kept = idx[b, h]
            assert ((kept >= 0) & (kept < s)).all(), "position outside the sequence at (%d,%d)" % (b, h)
            assert len(set(kept.tolist())) == N, "positions not distinct at (%d,%d)" % (b, h)
            if (b, h) in spoiled:
                continue
            r = oracle.decode_unit(qb[b, h], kb[b, h // G, :s], vb[b, h // G, :s], code, N,
                                   want_scores=True)
            r["v"] = oracle.decode16(vb[b, h // G, :s], code)
            check_unit(r, N, out[b, h], idx[b, h], w[b, h], tag="finite head (%d,%d)" % (b, h))
    q[0, 1, 5] = 0.5
    K[0, 1, 2048:2048 + 40, 7] = 0.25
    K[1, 0, 100, 0] = 1.0
    res = manual_case(kc, ctx, q, K, V, lens, N)
    check_manual(res, lens, N, G=G)
