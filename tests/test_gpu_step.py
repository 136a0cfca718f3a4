"""GPU tests of the whole-step calls: kcache_decode_step and its HIP-graph form must give
exactly what the per-layer calls give (same kernels, same launch shapes), including on
replays of the graph with other work in between and with a growing context."""
import numpy as np
import pytest
import torch

import kcache_inputs as ki
from harness import build_layer, oracle_unit, check_unit, sample_units
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
    c.close()


def make_model(kc, ctx, wl, L, hbm_layers=0):
    """L layers of one workload; the first hbm_layers keep V in HBM.  The last cached
    position of every sequence is left for the step's own append."""
    layers, gen = [], []
    for l in range(L):
        cache, q, lens, k, v = build_layer(ctx, wl, l)
        if l < hbm_layers:
            cache = kc.LayerCache(cache.k, cache.v.to(DEV))
        lens_h = lens.cpu().numpy()
        k_tok = torch.stack([k[b, :, lens_h[b] - 1] for b in range(wl.B)]).unsqueeze(1).contiguous()
        v_tok = torch.stack([v[b, :, lens_h[b] - 1] for b in range(wl.B)]).unsqueeze(1).contiguous()
        # wipe the last position so that the append is needed for a correct result
        for b in range(wl.B):
            cache.k[b, :, lens_h[b] - 1] = 0
            cache.v[b, :, lens_h[b] - 1] = 0
        layers.append(dict(cache=cache, q=q, k_new=k_tok, v_new=v_tok,
                           out=torch.zeros((wl.B, wl.H, wl.d), dtype=torch.float32, device=DEV),
                           idx_out=torch.zeros((wl.B, wl.H, wl.N), dtype=torch.int32, device=DEV),
                           w_out=torch.zeros((wl.B, wl.H, wl.N), dtype=torch.float32, device=DEV)))
        gen.append((k, v))
    return layers, lens, gen


def per_layer_reference(ctx, wl, layers, pos, lens):
    outs = []
    for y in layers:
        ctx.prefill_store(y["cache"], y["k_new"], y["v_new"], pos)
        if y["cache"].v_in_hbm:
            o = ctx.full_attention(y["cache"], y["q"], lens)
            outs.append((o.clone(), None, None))
        else:
            idx = torch.empty_like(y["idx_out"])
            w = torch.empty_like(y["w_out"])
            o = ctx.decode_attention(y["cache"], y["q"], lens, wl.N, idx_out=idx, w_out=w)
            outs.append((o.clone(), idx, w))
    torch.cuda.synchronize()
    return outs


def assert_same(layers, ref):
    for y, (o, idx, w) in zip(layers, ref):
        assert torch.equal(y["out"], o)
        if idx is not None:
            assert torch.equal(y["idx_out"], idx) and torch.equal(y["w_out"], w)


def wipe_last(layers, lens):
    """Zeroes the newest cached position again, so that only a working append restores it."""
    lens_h = lens.cpu().numpy()
    for y in layers:
        for b in range(len(lens_h)):
            y["cache"].k[b, :, lens_h[b] - 1] = 0
            y["cache"].v[b, :, lens_h[b] - 1] = 0
    torch.cuda.synchronize()


def clear(layers):
    for y in layers:
        y["out"].fill_(float("nan"))
        y["idx_out"].fill_(-5)
        y["w_out"].fill_(-5.0)


@pytest.mark.parametrize("lanes", [1, 2, 3])
def test_step_equals_per_layer_calls_and_oracle(kc, ctx, lanes):
    wl = ki.config(1, B=2, S_cap=3000)
    L = 5
    layers, lens, _ = make_model(kc, ctx, wl, L, hbm_layers=2)
    pos = (lens - 1).to(torch.int32)
    ref = per_layer_reference(ctx, wl, layers, pos, lens)
    clear(layers)
    wipe_last(layers, lens)
    ctx.set_step_lanes(lanes)
    ctx.decode_step(layers, wl.H, pos, lens, wl.N)
    ctx.synchronize()
    torch.cuda.synchronize()
    ctx.set_step_lanes(1)
    ctx.device_check()
    assert_same(layers, ref)
    # and against the oracle, on a KCache layer, through the step call
    y = layers[3]
    out, idx, w = y["out"].cpu().numpy(), y["idx_out"].cpu().numpy(), y["w_out"].cpu().numpy()
    for (b, h) in sample_units(wl, 6):
        r = oracle_unit(wl, 3, b, h, wl.N)
        check_unit(r, wl.N, out[b, h], idx[b, h], w[b, h], tag="step layer 3 (%d,%d)" % (b, h))


@pytest.mark.parametrize("lanes,graph", [(2, False), (3, False), (2, True), (4, True)])
def test_sequence_split_lanes(kc, ctx, lanes, graph):
    """Lanes that each take a share of the batch through all layers: launches cover fewer
    sequences (and may pick another chunk size), so results are compared to the per-layer
    calls within rounding and to the oracle with the usual rule."""
    wl = ki.config(1, B=5, S_cap=2600, H=4, Hkv=4)
    L = 3
    layers, lens, _ = make_model(kc, ctx, wl, L, hbm_layers=1)
    lens = lens.clone()
    lens[2], lens[4] = 700, 1
    pos = (lens - 1).to(torch.int32)
    # the wiped newest rows sit at S_cap - 1; with shorter lengths the append goes elsewhere
    ref = per_layer_reference(ctx, wl, layers, pos, lens)
    clear(layers)
    wipe_last(layers, lens)
    ctx.set_step_lanes(lanes, split_sequences=True)
    try:
        if graph:
            g = ctx.step_graph(layers, wl.H, pos, lens, wl.N)
            g.launch()
            ctx.synchronize()
            g.close()
        else:
            ctx.decode_step(layers, wl.H, pos, lens, wl.N)
            ctx.synchronize()
    finally:
        ctx.set_step_lanes(1)
    torch.cuda.synchronize()
    ctx.device_check()
    for y, (o, idx, w) in zip(layers, ref):
        assert torch.allclose(y["out"], o, rtol=2e-3, atol=1e-3)
        if idx is not None:
            assert torch.equal(y["idx_out"], idx)
            assert torch.allclose(y["w_out"], w, rtol=2e-3, atol=1e-7)
    lens_h = lens.cpu().numpy()
    y = layers[2]
    out, idx, w = y["out"].cpu().numpy(), y["idx_out"].cpu().numpy(), y["w_out"].cpu().numpy()
    for b in range(wl.B):
        for h in (0, wl.H - 1):
            qb, kb, vb = ki.gen_unit(wl, 2, b, h)
            s = int(lens_h[b])
            # the cache row at s - 1 was replaced by the appended row (generated row S_cap - 1)
            kb, vb = kb[:s].copy(), vb[:s].copy()
            kb[s - 1], vb[s - 1] = ki.gen_unit(wl, 2, b, h)[1][wl.S_cap - 1], \
                ki.gen_unit(wl, 2, b, h)[2][wl.S_cap - 1]
            r = oracle_unit(wl, 2, b, h, wl.N, bits=(qb, kb, vb))
            check_unit(r, wl.N, out[b, h], idx[b, h], w[b, h], tag="split (%d,%d)" % (b, h))


@pytest.mark.parametrize("lanes", [1, 2])
def test_graph_replays_equal_eager_results_with_work_in_between(kc, ctx, lanes):
    wl = ki.config(1, B=2, S_cap=2500)
    L = 4
    layers, lens, gen = make_model(kc, ctx, wl, L, hbm_layers=1)
    lens = lens.clone()
    lens[1] = 1800                      # room to grow
    pos = (lens - 1).to(torch.int32)
    ctx.set_step_lanes(lanes)
    graph = ctx.step_graph(layers, wl.H, pos, lens, wl.N)
    ctx.set_step_lanes(1)
    other = kc.Context(0)               # eager reference on its own workspace
    try:
        for rep in range(4):
            # new token rows for this step: take them from the generated tensors
            lens_h = lens.cpu().numpy()
            for l, y in enumerate(layers):
                k, v = gen[l]
                for b in range(wl.B):
                    y["k_new"][b, 0] = k[b, :, lens_h[b] - 1]
                    y["v_new"][b, 0] = v[b, :, lens_h[b] - 1]
            ref = per_layer_reference(other, wl, layers, pos, lens)
            other.synchronize()
            clear(layers)
            wipe_last(layers, lens)
            graph.launch()
            ctx.synchronize()
            torch.cuda.synchronize()
            assert_same(layers, ref)
            # unrelated eager work of the program between replays
            _ = (layers[0]["q"].float() @ layers[0]["q"].float().transpose(1, 2)).sum().item()
            # the context grows in place: same graph, new lengths
            if rep < 3 and int(lens[1]) < wl.S_cap:
                lens[1] += 1
                pos.copy_(lens - 1)
        ctx.device_check()
    finally:
        graph.close()
        other.close()


def test_workspace_cannot_grow_under_a_live_graph(kc):
    c = kc.Context(0)
    try:
        wl = ki.config(1, B=1, S_cap=1024)
        layers, lens, _ = make_model(kc, c, wl, 1)
        pos = (lens - 1).to(torch.int32)
        graph = c.step_graph(layers, wl.H, pos, lens, wl.N)
        big = ki.config(1, B=4, S_cap=4096)
        cache, q, blens, _, _ = build_layer(kc.Context(0), big, 0)
        with pytest.raises(kc.KCacheError) as e:
            c.decode_attention(cache, q, blens, 512)
        assert e.value.status == -4
        graph.launch()
        c.synchronize()
        graph.close()
        c.decode_attention(cache, q, blens, 512)      # allowed again
        c.synchronize()
    finally:
        c.close()


def test_step_error_paths(kc, ctx):
    wl = ki.config(1)
    layers, lens, _ = make_model(kc, ctx, wl, 2)
    pos = (lens - 1).to(torch.int32)
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_step([], wl.H, pos, lens, wl.N)
    assert e.value.status == -1
    bad = [dict(layers[0]), dict(layers[1])]
    bad[1]["v_new"] = None
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_step(bad, wl.H, pos, lens, wl.N)
    assert e.value.status == -1
    with pytest.raises(kc.KCacheError):
        ctx.set_step_lanes(9)
    with pytest.raises(kc.KCacheError) as e:
        ctx.decode_step(layers, 3, pos, lens, wl.N)   # H not a multiple of Hkv
    assert e.value.status == -1


def test_graph_launch_at_the_benchmark_shape_matches_the_oracle(kc):
    """Config 2's per-layer shape (B 8, 32 heads, 32768 positions, N 256), two layers, issued
    the way bench.py issues a step: one launch of the captured graph.  Sampled units against
    the oracle with the acceptance rule of the parity tests."""
    wl = ki.config(2)
    c = kc.Context(0, kc.workspace_bytes(wl.B, wl.H, wl.S_cap, wl.N))
    try:
        layers, lens = [], None
        for l in (0, wl.L - 1):
            cache, q, lens, k, v = build_layer(c, wl, l, chunk_T=8192)
            k_tok = k[:, :, wl.S_cap - 1].unsqueeze(1).contiguous()
            v_tok = v[:, :, wl.S_cap - 1].unsqueeze(1).contiguous()
            del k, v
            layers.append(dict(cache=cache, q=q, k_new=k_tok, v_new=v_tok,
                               out=torch.zeros((wl.B, wl.H, wl.d), dtype=torch.float32, device=DEV),
                               idx_out=torch.zeros((wl.B, wl.H, wl.N), dtype=torch.int32, device=DEV),
                               w_out=torch.zeros((wl.B, wl.H, wl.N), dtype=torch.float32, device=DEV)))
        torch.cuda.empty_cache()
        pos = (lens - 1).to(torch.int32)
        wipe_last(layers, lens)
        graph = c.step_graph(layers, wl.H, pos, lens, wl.N)
        for _ in range(2):                      # a replay must give the same again
            clear(layers)
            graph.launch()
            c.synchronize()
            torch.cuda.synchronize()
            for y, l in zip(layers, (0, wl.L - 1)):
                out = y["out"].cpu().numpy()
                idx, w = y["idx_out"].cpu().numpy(), y["w_out"].cpu().numpy()
                for (b, h) in sample_units(wl, 6, seed=l):
                    r = oracle_unit(wl, l, b, h, wl.N)
                    check_unit(r, wl.N, out[b, h], idx[b, h], w[b, h],
                               tag="graph config2 layer %d (%d,%d)" % (l, b, h))
        c.device_check()
        graph.close()
    finally:
        c.close()


@pytest.mark.parametrize("lanes", [0, 1])
def test_ragged_step_graph_follows_changing_lengths(kc, ctx, lanes):
    """A ragged batch large enough for the launch plan (the dense numbering of the chunks that
    exist is rebuilt from the lengths at the start of every step): the captured step is replayed
    after the lengths in device memory have changed - some sequences shrink to one chunk, one
    grows to the full capacity - and every replay is checked against the oracle."""
    wl = ki.config(4, B=40, H=16, Hkv=16, S_cap=8192, N=48, len_range=(600, 8192))
    L = 2
    layers, lens, gen = make_model(kc, ctx, wl, L)
    lens_h0 = lens.cpu().numpy().copy()
    for y, (k, v) in zip(layers, gen):          # the whole capacity holds generated rows
        y["cache"].k.copy_(k)
        y["cache"].v.copy_(v)
        y["k_new"], y["v_new"] = None, None     # nothing is appended: lengths move freely
    pos = (lens - 1).to(torch.int32)
    ctx.set_step_lanes(lanes, split_sequences=True)
    graph = ctx.step_graph(layers, wl.H, pos, lens, wl.N)
    ctx.set_step_lanes(0, split_sequences=True)
    rng = np.random.default_rng(9)
    try:
        for rep in range(3):
            new = lens_h0.copy()
            if rep > 0:
                new = rng.integers(1, wl.S_cap + 1, size=wl.B).astype(np.int32)
                new[0], new[1], new[-1] = wl.S_cap, 1, 513
            lens.copy_(torch.from_numpy(new))
            clear(layers)
            graph.launch()
            ctx.synchronize()
            torch.cuda.synchronize()
            ctx.device_check()
            for l, y in enumerate(layers):
                out, idx, w = (y["out"].cpu().numpy(), y["idx_out"].cpu().numpy(),
                               y["w_out"].cpu().numpy())
                kb, vb = ki.as_bits(gen[l][0]), ki.as_bits(gen[l][1])
                qb = ki.as_bits(y["q"])
                for (b, h) in [(0, 0), (1, 3), (wl.B - 1, wl.H - 1), (7, 2), (20, 15), (33, 9)]:
                    s = int(new[b])
                    r = oracle.decode_unit(qb[b, h], kb[b, h, :s], vb[b, h, :s], oracle.F16, wl.N,
                                           want_scores=True)
                    r["v"] = oracle.decode16(vb[b, h, :s], oracle.F16)
                    check_unit(r, wl.N, out[b, h], idx[b, h], w[b, h],
                               tag="replay %d layer %d (%d,%d) s=%d" % (rep, l, b, h, s))
    finally:
        graph.close()
