"""The seeded input generator: determinism, layout and the stated recipe (CPU only)."""
import numpy as np
import torch

import kcache_inputs as ki


def small(**kw):
    base = dict(L=2, B=3, H=8, Hkv=2, S_cap=256, N=16, dtype="bf16", pivot_frac=0.02, seed=77,
                len_range=(40, 256))
    base.update(kw)
    return ki.Workload("small", **base)


def test_table_is_symmetric_standard_normal():
    t = ki.normal_table()
    assert t.shape == (65536,) and t.dtype == np.float32
    assert np.array_equal(t, -t[::-1])
    assert abs(float(t.astype(np.float64).std()) - 1.0) < 2e-3
    assert (np.diff(t) > 0).all()


def test_generation_is_deterministic_and_units_match_layer_slices():
    wl = small()
    q, k, v, lens = ki.gen_layer(wl, 1)
    q2, k2, v2, lens2 = ki.gen_layer(wl, 1)
    assert torch.equal(q, q2) and torch.equal(k, k2) and torch.equal(v, v2)
    assert np.array_equal(lens, lens2) and lens.min() >= 40 and lens.max() <= 256
    for b, h in [(0, 0), (1, 5), (2, 7)]:
        qb, kb, vb = ki.gen_unit(wl, 1, b, h)
        s = int(lens[b])
        hk = h // wl.G
        assert np.array_equal(qb, ki.as_bits(q[b, h]))
        assert np.array_equal(kb, ki.as_bits(k[b, hk, :s]))
        assert np.array_equal(vb, ki.as_bits(v[b, hk, :s]))


def test_layers_seeds_and_tensors_differ():
    wl = small()
    _, k0, v0, _ = ki.gen_layer(wl, 0)
    _, k1, _, _ = ki.gen_layer(wl, 1)
    _, k2, _, _ = ki.gen_layer(wl.replace(seed=78), 0)
    assert not torch.equal(k0, k1) and not torch.equal(k0, k2) and not torch.equal(k0, v0)


def test_pivots_are_placed_per_query_head_below_the_sequence_length():
    wl = small(dtype="f16")
    lens = wl.seq_lens()
    for b in range(wl.B):
        for h in range(wl.H):
            p = ki.pivot_positions(wl, 0, b, h)
            want = max(1, int(np.floor(wl.pivot_frac * lens[b] + 0.5)))
            assert len(p) == want and len(set(p.tolist())) == want
            assert p.min() >= 0 and p.max() < lens[b]
    # a pivotal K row is the plain row plus 3*sqrt(d)*q/|q| (fp32 add, one rounding)
    _, k, _, _ = ki.gen_layer(wl, 0)
    q = ki.gen_q(wl, 0).float()
    kf = k.float()
    b, h = 1, 3
    hk = h // wl.G
    pos = ki.pivot_positions(wl, 0, b, h)
    others = np.setdiff1d(np.arange(int(lens[b])), np.concatenate(
        [ki.pivot_positions(wl, 0, b, hk * wl.G + g) for g in range(wl.G)]))
    proj = (kf[b, hk] @ q[b, h]) / q[b, h].norm()
    assert proj[torch.from_numpy(pos)].min() > 3 * np.sqrt(wl.d) - 5
    assert proj[torch.from_numpy(others)].abs().max() < 6


def test_named_configs_have_the_stated_shapes():
    c2, c3, c5 = ki.config(2), ki.config(3), ki.config(5)
    assert (c2.L, c2.B, c2.H, c2.Hkv, c2.S_cap, c2.N, c2.dtype) == (32, 8, 32, 32, 32768, 256, "f16")
    assert (c3.H, c3.Hkv, c3.G, c3.dtype, c3.B, c3.S_cap, c3.N) == (32, 8, 4, "bf16", 16, 8192, 128)
    assert (c5.L, c5.H, c5.B, c5.S_cap, c5.N) == (40, 40, 2, 65536, 512)
    # K cache bytes of config 2: 64 GiB
    assert c2.L * c2.B * c2.Hkv * c2.S_cap * c2.d * 2 == 64 * 2 ** 30
    lens = ki.config(4).seq_lens()
    assert lens.shape == (64,) and lens.min() >= 1024 and lens.max() <= 16384
