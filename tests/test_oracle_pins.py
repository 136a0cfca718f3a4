"""Pins of the CPU oracle against things other than itself (CPU only).

Every test names the part of the oracle it pins and the kind of mistake it
would catch.  The paper prints no worked numeric example of the method, so the
pins are closed forms, invariants, brute force and library routines.
"""
import math

import numpy as np
import pytest
import torch

import oracle

F16, BF16 = oracle.F16, oracle.BF16


def bits(a, dtype=F16):
    """fp64/fp32 numpy -> stored 16-bit patterns (round to nearest even via torch)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))
    t = t.to(torch.float16 if dtype == F16 else torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def back(b, dtype=F16):
    """stored patterns -> fp64 via the library conversion (not the oracle's)."""
    t = torch.from_numpy(np.ascontiguousarray(b).view(np.int16))
    t = t.view(torch.float16 if dtype == F16 else torch.bfloat16)
    return t.to(torch.float64).numpy()


def rand_unit(rng, s, d, dtype=F16, scale=1.0):
    q = bits(rng.standard_normal(d) * scale, dtype)
    K = bits(rng.standard_normal((s, d)) * scale, dtype)
    V = bits(rng.standard_normal((s, d)), dtype)
    return q, K, V


# ---------------------------------------------------------------- 16-bit decode
@pytest.mark.parametrize("dtype", [F16, BF16])
def test_decode16_matches_library_conversion_for_every_bit_pattern(dtype):
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.decode16(allbits, dtype)
    want = back(allbits, dtype)
    nan = np.isnan(want)
    assert (np.isnan(got) == nan).all()
    assert (got[~nan] == want[~nan]).all()
    # signed zeros keep their sign
    assert (np.signbit(got[~nan]) == np.signbit(want[~nan])).all()


# ---------------------------------------------------------------- scores + softmax
def test_softmax_sums_to_one_and_is_positive():
    rng = np.random.default_rng(1)
    for s, d in [(1, 8), (7, 16), (300, 128), (2048, 128)]:
        q, K, V = rand_unit(rng, s, d)
        r = oracle.decode_unit(q, K, V, F16, 1, want_scores=True)
        assert abs(r["p"].sum() - 1.0) < 1e-12
        assert (r["p"] > 0).all()


def test_two_score_closed_form_pins_scale_and_sign():
    # d = 4 -> 1/sqrt(d_h) = 1/2.  q.K0 = 4, q.K1 = 0  =>  z = (2, 0),
    # p0 = 1 / (1 + e^-2).  A missing scale gives 1/(1+e^-4), a flipped sign 1/(1+e^2).
    q = bits([4, 0, 0, 0])
    K = bits([[1, 0, 0, 0], [0, 3, -2, 5]])
    V = bits([[1, 2, 3, 4], [-8, 16, 0.5, 0.25]])
    r = oracle.decode_unit(q, K, V, F16, 2, want_scores=True)
    assert r["z"].tolist() == [2.0, 0.0]
    p0 = 1.0 / (1.0 + math.exp(-2.0))
    assert abs(r["p"][0] - p0) < 1e-15 and abs(r["p"][1] - (1 - p0)) < 1e-15
    # out[c] = p0 V[0][c] + p1 V[1][c]: a transposed V operand cannot produce this
    want = p0 * np.array([1, 2, 3, 4.0]) + (1 - p0) * np.array([-8, 16, 0.5, 0.25])
    assert np.allclose(r["out"], want, rtol=0, atol=1e-14)
    # N = 1 keeps only position 0 with its un-renormalised weight
    r1 = oracle.decode_unit(q, K, V, F16, 1)
    assert r1["idx"].tolist() == [0]
    assert np.allclose(r1["out"], p0 * np.array([1, 2, 3, 4.0]), rtol=0, atol=1e-14)


def test_score_uses_every_channel_of_q_and_k():
    # z[t] = (sum_c q[c] K[t][c]) / sqrt(d); with q = e_c only channel c of K matters
    d, s = 16, 5
    rng = np.random.default_rng(2)
    Kf = np.round(rng.standard_normal((s, d)) * 8) / 8
    for c in range(d):
        qf = np.zeros(d)
        qf[c] = 2.0
        r = oracle.decode_unit(bits(qf), bits(Kf), bits(Kf), F16, 1, want_scores=True)
        assert np.array_equal(r["z"], 2.0 * Kf[:, c] / 4.0)


def test_shift_invariance_of_softmax():
    # adding the same vector c to every K row shifts every score by q.c/sqrt(d):
    # the softmax, the selected set and the output do not move.
    rng = np.random.default_rng(3)
    s, d, N = 257, 128, 17
    qf = np.round(rng.standard_normal(d) * 4) / 4
    Kf = np.round(rng.standard_normal((s, d)) * 8) / 8
    cf = np.round(rng.standard_normal(d) * 8) / 8          # K + c stays exact in fp16
    q, K, Kc = bits(qf), bits(Kf), bits(Kf + cf)
    assert np.array_equal(back(Kc), Kf + cf)
    V = bits(rng.standard_normal((s, d)))
    a = oracle.decode_unit(q, K, V, F16, N, want_scores=True)
    b = oracle.decode_unit(q, Kc, V, F16, N, want_scores=True)
    shift = float(qf @ cf) / math.sqrt(d)
    assert np.allclose(b["z"] - a["z"], shift, rtol=0, atol=1e-12)
    assert np.allclose(a["p"], b["p"], rtol=1e-11, atol=0)
    assert np.array_equal(a["idx"], b["idx"])
    assert np.allclose(a["out"], b["out"], rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("s,d", [(1, 64), (33, 128), (500, 128)])
def test_full_n_equals_library_attention(dtype, s, d):
    # N = s is ordinary softmax attention (section 3.1: accuracy approaches the
    # full cache as N grows); compare with torch's scaled_dot_product_attention.
    rng = np.random.default_rng(4 + s)
    q, K, V = rand_unit(rng, s, d, dtype)
    r = oracle.decode_unit(q, K, V, dtype, s)
    tq = torch.from_numpy(back(q, dtype)).reshape(1, 1, 1, d)
    tk = torch.from_numpy(back(K, dtype)).reshape(1, 1, s, d)
    tv = torch.from_numpy(back(V, dtype)).reshape(1, 1, s, d)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).reshape(d).numpy()
    assert np.allclose(r["out"], ref, rtol=1e-11, atol=1e-13)
    assert r["idx"].tolist() == list(range(s))
    assert abs(r["w"].sum() - 1.0) < 1e-12


def test_n_larger_than_s_pads_and_is_full_attention():
    rng = np.random.default_rng(5)
    s, d, N = 9, 32, 16
    q, K, V = rand_unit(rng, s, d)
    full = oracle.decode_unit(q, K, V, F16, s)
    r = oracle.decode_unit(q, K, V, F16, N)
    assert r["idx"].tolist() == list(range(s)) + [-1] * (N - s)
    assert (r["w"][s:] == 0).all()
    assert np.array_equal(r["out"], full["out"])


# ---------------------------------------------------------------- selection
def brute_force_topn(z, N):
    return sorted(sorted(range(len(z)), key=lambda t: (-z[t], t))[:N])


def test_selection_equals_brute_force_sort_on_tiny_inputs_all_n():
    rng = np.random.default_rng(6)
    for s in [1, 2, 3, 5, 16, 37, 64]:
        d = 8
        q, K, V = rand_unit(rng, s, d)
        # duplicate some K rows so that exact ties occur and the tie-break matters
        if s >= 5:
            K[s - 1] = K[0]
            K[s // 2] = K[1]
        z = oracle.decode_unit(q, K, V, F16, 1, want_scores=True)["z"]
        for N in range(1, s + 1):
            r = oracle.decode_unit(q, K, V, F16, N)
            assert r["idx"].tolist() == brute_force_topn(z.tolist(), N), (s, N)


def test_uniform_scores_closed_form_pins_tie_break_and_no_renormalisation():
    # all K rows identical => p uniform = 1/s => lower positions win every tie:
    # I = {0..N-1}, out = (1/s) sum_{t<N} V[t], kept weights sum to N/s (not 1).
    rng = np.random.default_rng(7)
    s, d, N = 40, 16, 7
    q = bits(rng.standard_normal(d))
    K = np.tile(bits(rng.standard_normal(d)), (s, 1))
    Vf = np.round(rng.standard_normal((s, d)) * 16) / 16
    r = oracle.decode_unit(q, K, bits(Vf), F16, N, want_scores=True)
    assert r["idx"].tolist() == list(range(N))
    assert np.allclose(r["p"], 1.0 / s, rtol=1e-14)
    assert abs(r["w"].sum() - N / s) < 1e-14
    assert np.allclose(r["out"], Vf[:N].sum(0) / s, rtol=0, atol=1e-14)


def test_n_equals_one_is_first_argmax():
    rng = np.random.default_rng(8)
    s, d = 50, 16
    q, K, V = rand_unit(rng, s, d)
    z = oracle.decode_unit(q, K, V, F16, 1, want_scores=True)["z"]
    t_max = int(np.argmax(z))
    K[45] = K[t_max]                       # a later exact copy of the best row
    K[t_max + 1 if t_max < 44 else 0] = K[(t_max + 7) % 44]
    z = oracle.decode_unit(q, K, V, F16, 1, want_scores=True)["z"]
    r = oracle.decode_unit(q, K, V, F16, 1)
    assert r["idx"][0] == int(np.argmax(z))        # numpy argmax returns the first maximum


def test_selection_on_scores_equals_selection_on_probabilities():
    # the paper selects on the softmax output; exp is monotone, so ordering by p
    # gives the same set whenever the boundary probabilities differ
    rng = np.random.default_rng(9)
    s, d, N = 400, 64, 33
    q, K, V = rand_unit(rng, s, d, scale=0.5)
    r = oracle.decode_unit(q, K, V, F16, N, want_scores=True)
    order = sorted(range(s), key=lambda t: (-r["p"][t], t))
    assert r["p"][order[N - 1]] != r["p"][order[N]]
    assert sorted(order[:N]) == r["idx"].tolist()


# ---------------------------------------------------------------- combination
def test_dominant_key_returns_its_value_row():
    rng = np.random.default_rng(10)
    s, d = 64, 128
    qf = rng.standard_normal(d)
    Kf = rng.standard_normal((s, d)) * 0.1
    Kf[41] = 6.0 * qf                      # score ~ 6 |q|^2 / sqrt(d) ~ 68 above the rest
    Vf = rng.standard_normal((s, d))
    V = bits(Vf)
    r = oracle.decode_unit(bits(qf), bits(Kf), V, F16, 4)
    assert 41 in r["idx"].tolist()
    assert np.allclose(r["out"], back(V)[41], rtol=0, atol=1e-9)


def test_truncation_error_bound_and_monotone_mass():
    # |out_full - out_N|_inf <= (1 - sum_{t in I} p[t]) * max|V| and the captured
    # mass is non-decreasing in N: both follow from out = sum_{t in I} p[t] V[t].
    rng = np.random.default_rng(11)
    s, d = 300, 32
    q, K, V = rand_unit(rng, s, d)
    full = oracle.decode_unit(q, K, V, F16, s)
    vmax = np.abs(back(V)).max()
    last = 0.0
    for N in [1, 2, 5, 30, 150, 299, 300]:
        r = oracle.decode_unit(q, K, V, F16, N)
        mass = r["w"].sum()
        assert mass >= last - 1e-15
        last = mass
        assert np.abs(full["out"] - r["out"]).max() <= (1 - mass) * vmax + 1e-13
    assert abs(last - 1.0) < 1e-12


def test_weights_are_the_full_softmax_values_at_the_selected_positions():
    rng = np.random.default_rng(12)
    s, d, N = 128, 32, 10
    q, K, V = rand_unit(rng, s, d)
    r = oracle.decode_unit(q, K, V, F16, N, want_scores=True)
    assert np.array_equal(r["w"], r["p"][r["idx"]])
    assert np.allclose(r["out"], r["w"] @ back(V)[r["idx"]], rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- batch layout, GQA, ragged
def make_batch(rng, B, H, Hkv, S_cap, d, dtype):
    q = bits(rng.standard_normal((B, H, d)), dtype)
    K = bits(rng.standard_normal((B, Hkv, S_cap, d)), dtype)
    V = bits(rng.standard_normal((B, Hkv, S_cap, d)), dtype)
    return q, K, V


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_gqa_equals_mha_on_repeated_kv_heads(dtype):
    rng = np.random.default_rng(13)
    B, H, Hkv, S, d, N = 2, 8, 2, 70, 32, 9
    q, K, V = make_batch(rng, B, H, Hkv, S, d, dtype)
    lens = np.array([70, 33], np.int32)
    out, idx, w = oracle.decode_attention(q, K, V, dtype, lens, N)
    Kr = np.repeat(K, H // Hkv, axis=1)           # library repeat: head h <- KV head h // G
    Vr = np.repeat(V, H // Hkv, axis=1)
    out2, idx2, w2 = oracle.decode_attention(q, Kr, Vr, dtype, lens, N)
    assert np.array_equal(out, out2) and np.array_equal(idx, idx2) and np.array_equal(w, w2)


def test_ragged_batch_equals_independent_single_sequence_calls_and_ignores_padding():
    rng = np.random.default_rng(14)
    B, H, Hkv, S, d, N = 4, 4, 4, 90, 16, 12
    q, K, V = make_batch(rng, B, H, Hkv, S, d, F16)
    lens = np.array([90, 1, 5, 47], np.int32)
    out, idx, w = oracle.decode_attention(q, K, V, F16, lens, N, nthreads=3)
    for b in range(B):
        s = int(lens[b])
        for h in range(H):
            r = oracle.decode_unit(q[b, h], K[b, h, :s], V[b, h, :s], F16, N)
            assert np.array_equal(out[b, h], r["out"])
            assert np.array_equal(idx[b, h], r["idx"])
            assert np.array_equal(w[b, h], r["w"])
    # scribbling over the padded rows changes nothing
    K2, V2 = K.copy(), V.copy()
    for b in range(B):
        K2[b, :, lens[b]:] = bits(np.full(d, 30.0))
        V2[b, :, lens[b]:] = bits(np.full(d, -7.0))
    out2, idx2, w2 = oracle.decode_attention(q, K2, V2, F16, lens, N)
    assert np.array_equal(out, out2) and np.array_equal(idx, idx2)


def test_threads_do_not_change_results():
    rng = np.random.default_rng(15)
    q, K, V = make_batch(rng, 3, 6, 3, 64, 16, F16)
    lens = np.array([64, 10, 31], np.int32)
    a = oracle.decode_attention(q, K, V, F16, lens, 8, nthreads=1)
    b = oracle.decode_attention(q, K, V, F16, lens, 8, nthreads=4)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_bad_arguments_are_rejected():
    rng = np.random.default_rng(16)
    q, K, V = make_batch(rng, 1, 2, 2, 8, 8, F16)
    with pytest.raises(ValueError):
        oracle.decode_attention(q, K, V, F16, np.array([0], np.int32), 2)
    with pytest.raises(ValueError):
        oracle.decode_attention(q, K, V, F16, np.array([9], np.int32), 2)
    with pytest.raises(ValueError):
        oracle.decode_attention(q, K, V, F16, np.array([8], np.int32), 0)


# ---------------------------------------------------------------- cache store
def test_store_then_full_attention_equals_library_attention_on_token_major_tensors():
    # store() is pinned through its only observable: after storing token-major
    # K/V at pos, attention over the cache equals library attention over the
    # token-major tensors permuted by torch (a transposed or shifted copy fails).
    rng = np.random.default_rng(17)
    B, T, Hkv, d, S_cap = 2, 11, 3, 16, 32
    k_new = bits(rng.standard_normal((B, T, Hkv, d)))
    v_new = bits(rng.standard_normal((B, T, Hkv, d)))
    kc = np.zeros((B, Hkv, S_cap, d), np.uint16)
    vc = np.zeros((B, Hkv, S_cap, d), np.uint16)
    # a prefix already in the cache, then the new tokens appended behind it
    pre = np.array([4, 0], np.int32)
    k_pre = bits(rng.standard_normal((B, 4, Hkv, d)))
    v_pre = bits(rng.standard_normal((B, 4, Hkv, d)))
    oracle.store(kc, vc, k_pre, v_pre, np.zeros(B, np.int32))
    oracle.store(kc, vc, k_new, v_new, pre)
    q = bits(rng.standard_normal((B, Hkv, d)))
    lens = pre + T
    out, idx, w = oracle.decode_attention(q, kc, vc, F16, lens, S_cap)
    for b in range(B):
        kt = torch.from_numpy(back(k_new[b]))
        vt = torch.from_numpy(back(v_new[b]))
        if pre[b]:
            kt = torch.cat([torch.from_numpy(back(k_pre[b])), kt], 0)
            vt = torch.cat([torch.from_numpy(back(v_pre[b])), vt], 0)
        tq = torch.from_numpy(back(q[b])).reshape(1, Hkv, 1, d)
        ref = torch.nn.functional.scaled_dot_product_attention(
            tq, kt.permute(1, 0, 2).unsqueeze(0), vt.permute(1, 0, 2).unsqueeze(0))
        assert np.allclose(out[b], ref.reshape(Hkv, d).numpy(), rtol=1e-11, atol=1e-13)
    # rows outside [pos, pos+T) are untouched
    assert (kc[1, :, T:] == 0).all() and (vc[0, :, 4 + T:] == 0).all()


def test_store_places_every_row_where_a_slice_assignment_does():
    # Direct pin of the placement (Figure 1, upper half: a layer's new K / V rows are appended
    # to its caches).  Every element of the new rows is a distinct bit pattern, the expected
    # caches are written by numpy slice assignment of the transposed [Hkv][T][d] block at
    # [pos, pos + T), and the comparison is bit for bit: a reversed, shifted or transposed
    # placement inside the range changes at least one element.  Attention over the whole
    # cache cannot see such a permutation when K and V are permuted alike; this test can.
    rng = np.random.default_rng(170)
    B, T, Hkv, d, S_cap = 3, 7, 2, 8, 19
    n = B * T * Hkv * d
    k_new = rng.permutation(n).astype(np.uint16).reshape(B, T, Hkv, d)            # 0 .. n-1
    v_new = (rng.permutation(n) + 20000).astype(np.uint16).reshape(B, T, Hkv, d)  # disjoint from K
    pos = np.array([0, 12, 5], np.int32)            # start, flush with the end, in the middle
    kc = np.full((B, Hkv, S_cap, d), 0xAAAA, np.uint16)
    vc = np.full((B, Hkv, S_cap, d), 0x5555, np.uint16)
    want_k, want_v = kc.copy(), vc.copy()
    for b in range(B):
        want_k[b, :, pos[b]:pos[b] + T, :] = k_new[b].transpose(1, 0, 2)
        want_v[b, :, pos[b]:pos[b] + T, :] = v_new[b].transpose(1, 0, 2)
    oracle.store(kc, vc, k_new, v_new, pos)
    assert np.array_equal(kc, want_k)
    assert np.array_equal(vc, want_v)
    # the 8-bit K variant places rows the same way: V bit for bit, K as the codes of the
    # slice-assigned rows (distinct small values, so that codes differ between neighbours)
    k_vals = bits((rng.permutation(n).reshape(B, T, Hkv, d) % 97 - 48) / 8.0)
    k8 = np.full((B, Hkv, S_cap, d), 0x7F, np.uint8)
    v8 = np.full((B, Hkv, S_cap, d), 0x5555, np.uint16)
    oracle.store_k8(k8, v8, k_vals, v_new, pos, F16, 0)
    want_k8 = np.full((B, Hkv, S_cap, d), 0x7F, np.uint8)
    for b in range(B):
        want_k8[b, :, pos[b]:pos[b] + T, :] = oracle.e4m3_quantise(k_vals[b].transpose(1, 0, 2), F16, 0)
    assert np.array_equal(k8, want_k8)
    assert np.array_equal(v8, want_v)


def test_store_rejects_overflowing_positions():
    kc = np.zeros((1, 1, 4, 8), np.uint16)
    vc = np.zeros((1, 1, 4, 8), np.uint16)
    new = np.zeros((1, 3, 1, 8), np.uint16)
    with pytest.raises(ValueError):
        oracle.store(kc, vc, new, new, np.array([2], np.int32))
    with pytest.raises(ValueError):
        oracle.store(kc, vc, new, new, np.array([-1], np.int32))


# ---------------------------------------------------------------- conventional attention
@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("s,d", [(1, 64), (33, 128), (700, 128)])
def test_conventional_attention_equals_library_attention(dtype, s, d):
    # section 2: softmax(q K^T / sqrt(d_h)) V; library routine: torch SDPA in fp64.
    # Catches a wrong scale, a missing max shift going wrong, K / V swapped, a
    # transposed operand.
    rng = np.random.default_rng(90 + s)
    q, K, V = rand_unit(rng, s, d, dtype, scale=1.5)
    out, p = oracle.full_unit(q, K, V, dtype, want_p=True)
    tq = torch.from_numpy(back(q, dtype)).reshape(1, 1, 1, d)
    tk = torch.from_numpy(back(K, dtype)).reshape(1, 1, s, d)
    tv = torch.from_numpy(back(V, dtype)).reshape(1, 1, s, d)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).reshape(d).numpy()
    assert np.allclose(out, ref, rtol=1e-11, atol=1e-13)
    assert abs(p.sum() - 1.0) < 1e-12 and (p > 0).all()


def test_conventional_attention_uniform_scores_is_the_mean_of_v():
    # identical K rows => p = 1/s => out = mean of the V rows (closed form)
    rng = np.random.default_rng(91)
    s, d = 48, 16
    q = bits(rng.standard_normal(d))
    K = np.tile(bits(rng.standard_normal(d)), (s, 1))
    Vf = np.round(rng.standard_normal((s, d)) * 16) / 16
    out, p = oracle.full_unit(q, K, bits(Vf), F16, want_p=True)
    assert np.allclose(p, 1.0 / s, rtol=1e-14)
    assert np.allclose(out, Vf.mean(0), rtol=0, atol=1e-14)


def test_conventional_attention_two_scores_closed_form():
    # two positions with scores z0, z1: p0 = 1 / (1 + exp(z1 - z0)); pins sign and scale
    d = 4
    q = bits(np.array([2.0, 0.0, 0.0, 0.0]))
    K = bits(np.array([[1.0, 0, 0, 0], [-0.5, 0, 0, 0]]))
    V = bits(np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]]))
    out = oracle.full_unit(q, K, V, F16)
    z0, z1 = 2.0 * 1.0 / 2.0, 2.0 * -0.5 / 2.0
    p0 = 1.0 / (1.0 + math.exp(z1 - z0))
    assert np.allclose(out, [p0, 1.0 - p0, 0, 0], rtol=1e-14, atol=0)


def test_conventional_attention_is_the_n_equals_s_case_of_kcache():
    # section 3.1: with N = s nothing is dropped; two separately written routines agree
    rng = np.random.default_rng(92)
    q, K, V = rand_unit(rng, 257, 128, BF16)
    a = oracle.full_unit(q, K, V, BF16)
    b = oracle.decode_unit(q, K, V, BF16, 257)["out"]
    assert np.allclose(a, b, rtol=1e-12, atol=1e-14)


def test_conventional_attention_batch_gqa_ragged_and_padding():
    # batch routine = per-unit routine on the right KV head and the first s_b rows;
    # rows beyond s_b must not matter
    rng = np.random.default_rng(93)
    B, H, Hkv, S_cap, d = 3, 4, 2, 50, 32
    q = bits(rng.standard_normal((B, H, d)))
    K = bits(rng.standard_normal((B, Hkv, S_cap, d)))
    V = bits(rng.standard_normal((B, Hkv, S_cap, d)))
    lens = np.array([50, 1, 17], np.int32)
    out = oracle.full_attention(q, K, V, F16, lens, nthreads=2)
    K2, V2 = K.copy(), V.copy()
    for b in range(B):
        K2[b, :, lens[b]:] = bits(rng.standard_normal((Hkv, S_cap - lens[b], d)) * 50)
        V2[b, :, lens[b]:] = 0x7C00  # +inf bit pattern beyond the length
    out2 = oracle.full_attention(q, K2, V2, F16, lens)
    assert np.array_equal(out, out2)
    for b in range(B):
        for h in range(H):
            hk = h // (H // Hkv)
            ref = oracle.full_unit(q[b, h], K[b, hk, :lens[b]], V[b, hk, :lens[b]], F16)
            assert np.array_equal(out[b, h], ref)
    with pytest.raises(ValueError):
        oracle.full_attention(q, K, V, F16, np.array([51, 1, 1], np.int32))


# ---------------------------------------------------------------- renormalised variant
def test_renormalised_variant_uniform_scores_closed_form():
    # identical K rows: kept weights become 1/N each, out = mean of the first N V rows
    rng = np.random.default_rng(95)
    s, d, N = 40, 16, 8
    q = bits(rng.standard_normal(d))
    K = np.tile(bits(rng.standard_normal(d)), (s, 1))
    Vf = np.round(rng.standard_normal((s, d)) * 16) / 16
    r = oracle.decode_unit(q, K, bits(Vf), F16, N, renormalise=True)
    assert r["idx"].tolist() == list(range(N))
    assert np.allclose(r["w"], 1.0 / N, rtol=1e-14)
    assert np.allclose(r["out"], Vf[:N].mean(0), rtol=0, atol=1e-14)


def test_renormalised_variant_n_one_returns_the_argmax_row_exactly():
    rng = np.random.default_rng(96)
    q, K, V = rand_unit(rng, 50, 32)
    r = oracle.decode_unit(q, K, V, F16, 1, renormalise=True, want_scores=True)
    t = int(np.argmax(r["z"]))
    assert r["idx"].tolist() == [t] and r["w"][0] == 1.0
    assert np.array_equal(r["out"], back(V[t]))


def test_renormalised_variant_is_the_literal_one_rescaled_and_full_attention_at_n_equal_s():
    rng = np.random.default_rng(97)
    q, K, V = rand_unit(rng, 120, 64, BF16)
    a = oracle.decode_unit(q, K, V, BF16, 17)
    b = oracle.decode_unit(q, K, V, BF16, 17, renormalise=True)
    assert np.array_equal(a["idx"], b["idx"])
    assert abs(b["w"].sum() - 1.0) < 1e-14
    assert np.allclose(b["w"], a["w"] / a["w"].sum(), rtol=1e-14)
    assert np.allclose(b["out"], a["out"] / a["w"].sum(), rtol=1e-12, atol=1e-15)
    full = oracle.full_unit(q, K, V, BF16)
    assert np.allclose(oracle.decode_unit(q, K, V, BF16, 120, renormalise=True)["out"], full,
                       rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- 8-bit K storage (E4M3)
def e4m3_table():
    """Values of the 256 OCP E4M3 codes from the format's definition, written independently
    of the oracle: (-1)^s * 2^(e-7) * (1 + m/8), subnormals 2^-6 * m/8, S.1111.111 = NaN."""
    vals = np.empty(256)
    for c in range(256):
        s_, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            v = np.nan
        elif e == 0:
            v = 2.0 ** -6 * m / 8
        else:
            v = 2.0 ** (e - 7) * (1 + m / 8)
        vals[c] = -v if s_ else v
    return vals


def test_e4m3_decode_matches_the_format_definition_and_torch():
    codes = np.arange(256, dtype=np.uint8)
    got = oracle.e4m3_decode(codes)
    want = e4m3_table()
    nan = np.isnan(want)
    assert (np.isnan(got) == nan).all() and nan.sum() == 2
    assert (got[~nan] == want[~nan]).all()
    assert np.nanmax(got) == 448.0 and got[0x08] == 2.0 ** -6 and got[0x01] == 2.0 ** -9
    if hasattr(torch, "float8_e4m3fn"):      # library decode of the same format
        lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
        assert (lib[~nan] == got[~nan]).all() and np.isnan(lib[nan]).all()


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("k_exp", [0, -3, 2])
def test_e4m3_quantise_is_nearest_ties_to_even_saturating_by_brute_force(dtype, k_exp):
    # every 16-bit input against an exhaustive search over the 254 finite codes
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    x = back(allbits, dtype) * 2.0 ** -k_exp
    got = oracle.e4m3_quantise(allbits, dtype, k_exp)
    table = e4m3_table()
    finite = ~np.isnan(x)
    pos_codes = np.arange(0, 0x7f)                        # non-negative finite codes
    pos_vals = table[pos_codes]
    a = np.abs(x[finite])
    a_sat = np.minimum(a, 448.0)                          # saturation
    dist = np.abs(a_sat[:, None] - pos_vals[None, :])
    best = dist.min(axis=1)
    is_best = dist == best[:, None]
    # ties: the even code (its last fraction bit is 0)
    even = (pos_codes % 2 == 0)[None, :]
    pick = np.where((is_best & even).any(axis=1), (is_best & even).argmax(axis=1),
                    is_best.argmax(axis=1))
    want = pos_codes[pick].astype(np.uint8) | np.where(np.signbit(x[finite]), 0x80, 0).astype(np.uint8)
    assert (got[finite] == want).all()
    assert ((got[~finite] & 0x7f) == 0x7f).all()          # NaN stays NaN
    # representable values are fixed points
    vals = oracle.e4m3_decode(got[finite])
    assert (np.abs(vals) <= 448).all()


def test_k8_unit_is_the_16_bit_unit_on_the_dequantised_rows():
    # when every K value is representable in E4M3 (times 2^e) the two routines must agree
    rng = np.random.default_rng(98)
    s, d, N, e = 90, 32, 11, -2
    codes = rng.integers(0, 0x7f, size=(s, d)).astype(np.uint8) | \
        (rng.integers(0, 2, size=(s, d)).astype(np.uint8) << 7)
    codes[(codes & 0x7f) == 0x7f] = 0x30
    Kf = e4m3_table()[codes] * 2.0 ** e
    Kf = np.clip(Kf, -60000, 60000)
    codes = oracle.e4m3_quantise(bits(Kf), F16, e)        # round trip through fp16 (exact here)
    Kf = oracle.e4m3_decode(codes) * 2.0 ** e
    q = bits(rng.standard_normal(d) * 0.3)
    V = bits(rng.standard_normal((s, d)))
    a = oracle.decode_unit_k8(q, codes, e, V, F16, N, want_scores=True)
    b = oracle.decode_unit(q, bits(Kf), V, F16, N, want_scores=True)
    assert (back(bits(Kf)) == Kf).all()
    assert np.array_equal(a["idx"], b["idx"])
    assert np.allclose(a["z"], b["z"], rtol=1e-13, atol=1e-13)
    assert np.allclose(a["out"], b["out"], rtol=1e-12, atol=1e-14)


def test_store_k8_is_store_followed_by_quantisation():
    rng = np.random.default_rng(99)
    B, T, Hkv, d, S_cap, e = 2, 5, 3, 16, 12, -1
    k_new = bits(rng.standard_normal((B, T, Hkv, d)) * 3)
    v_new = bits(rng.standard_normal((B, T, Hkv, d)))
    pos = np.array([0, 7], np.int32)
    k8 = np.full((B, Hkv, S_cap, d), 0x55, np.uint8)
    v = np.zeros((B, Hkv, S_cap, d), np.uint16)
    oracle.store_k8(k8, v, k_new, v_new, pos, F16, e)
    k16 = np.full((B, Hkv, S_cap, d), 0xFFFF, np.uint16)   # NaN pattern marks untouched rows
    v2 = np.zeros_like(v)
    oracle.store(k16, v2, k_new, v_new, pos)
    touched = k16 != 0xFFFF
    assert np.array_equal(v, v2)
    assert np.array_equal(k8[touched], oracle.e4m3_quantise(k16[touched], F16, e))
    assert (k8[~touched] == 0x55).all()
