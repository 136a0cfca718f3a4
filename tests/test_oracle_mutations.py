"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C
source (on the CPU; the real oracle is untouched), builds it, and requires that at least
one pin of tests/test_oracle_pins.py fails against the mutant."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = open(os.path.join(os.path.dirname(oracle.__file__), "kcache_oracle.c")).read()

# (name, text in the source, replacement)
MUTANTS = [
    ("scale dropped", "const double inv_sqrt_d = 1.0 / sqrt((double)d);\n  for (int32_t t = 0; t < s; ++t) {\n    double acc = 0.0;\n    for (int32_t c = 0; c < d; ++c) {",
     "const double inv_sqrt_d = 1.0;\n  for (int32_t t = 0; t < s; ++t) {\n    double acc = 0.0;\n    for (int32_t c = 0; c < d; ++c) {"),
    ("scale by d instead of sqrt(d)", "const double inv_sqrt_d = 1.0 / sqrt((double)d);\n  for (int32_t t = 0; t < s; ++t) {\n    double acc = 0.0;\n    for (int32_t c = 0; c < d; ++c) {",
     "const double inv_sqrt_d = 1.0 / (double)d;\n  for (int32_t t = 0; t < s; ++t) {\n    double acc = 0.0;\n    for (int32_t c = 0; c < d; ++c) {"),
    ("last channel dropped from the score", "for (int32_t c = 0; c < d; ++c) {\n      const double k = K8", "for (int32_t c = 0; c + 1 < d; ++c) {\n      const double k = K8"),
    ("sign of the score", "z[t] = acc * inv_sqrt_d;\n  }\n\n  /* softmax over all s positions */", "z[t] = -acc * inv_sqrt_d;\n  }\n\n  /* softmax over all s positions */"),
    ("softmax not normalised", "for (int32_t t = 0; t < s; ++t) p[t] /= Z;", ""),
    ("softmax over the first N only", "for (int32_t t = 0; t < s; ++t) {\n    p[t] = exp(z[t] - m);\n    Z += p[t];\n  }",
     "for (int32_t t = 0; t < s; ++t) {\n    p[t] = exp(z[t] - m);\n    if (t < N) Z += p[t];\n  }"),
    ("smallest scores selected", "if (x->z > y->z) return -1;\n  if (x->z < y->z) return 1;", "if (x->z > y->z) return 1;\n  if (x->z < y->z) return -1;"),
    ("ties to the higher position", "return (x->t > y->t) - (x->t < y->t);", "return (x->t < y->t) - (x->t > y->t);"),
    ("one position too few", "int32_t n_eff = N < s ? N : s;\n  for (int32_t j = 0; j < n_eff; ++j) idx[j] = order[j].t;",
     "int32_t n_eff = N < s ? N : s;\n  if (n_eff > 1 && n_eff < s) n_eff -= 1;\n  for (int32_t j = 0; j < n_eff; ++j) idx[j] = order[j].t;"),
    ("weights renormalised by default", "return kco_unit(q, K, NULL, 0, V, dtype, s, d, N, 0, out, idx, w, z_out, p_out);", "return kco_unit(q, K, NULL, 0, V, dtype, s, d, N, 1, out, idx, w, z_out, p_out);"),
    ("variant not renormalised", "return kco_unit(q, K, NULL, 0, V, dtype, s, d, N, 1, out, idx, w, z_out, p_out);", "return kco_unit(q, K, NULL, 0, V, dtype, s, d, N, 0, out, idx, w, z_out, p_out);"),
    ("V channels rotated by one", "out[c] += w[j] * kco_decode(V[(size_t)t * d + c], dtype);", "out[c] += w[j] * kco_decode(V[(size_t)t * d + (c + 1) % d], dtype);"),
    ("q used as V row", "out[c] += w[j] * kco_decode(V[(size_t)t * d + c], dtype);", "out[c] += w[j] * kco_decode(q[c], dtype);"),
    ("V row of the neighbouring position", "int32_t t = idx[j];\n    w[j] = p[t] / divisor;", "int32_t t = idx[j];\n    w[j] = p[t > 0 ? t - 1 : t] / divisor;"),
    ("GQA: query head mapped modulo instead of by division", "int32_t hk = h / G;", "int32_t hk = h % Hkv;"),
    ("batch: every sequence uses the first length", "seq_lens[b], d, N,\n                                out + (size_t)u * d", "seq_lens[0], d, N,\n                                out + (size_t)u * d"),
    ("fp16 subnormals flushed", "v = ldexp((double)frac, -24); /* subnormal", "v = 0.0; /* subnormal"),
    ("bf16 exponent bias off by one", "v = ldexp((double)(frac + 128), expo - 134);", "v = ldexp((double)(frac + 128), expo - 133);"),
    ("e4m3 decode: exponent bias off by one", "v = ldexp((double)(frac + 8), expo - 10);", "v = ldexp((double)(frac + 8), expo - 11);"),
    ("e4m3 decode: subnormals flushed", "v = ldexp((double)frac, -9); /* subnormal: frac/8", "v = 0.0; /* subnormal: frac/8"),
    ("e4m3 quantise: ties away from zero", "double n = nearbyint(ldexp(a, 3 - expo));", "double n = round(ldexp(a, 3 - expo));"),
    ("e4m3 quantise: truncation", "double n = nearbyint(ldexp(a, 3 - expo));", "double n = floor(ldexp(a, 3 - expo));"),
    ("e4m3 quantise: saturates to the NaN code", "if (a >= 448.0) return (uint8_t)(sign | 0x7e);", "if (a >= 448.0) return (uint8_t)(sign | 0x7f);"),
    ("e4m3 quantise: scale applied the wrong way", "out[i] = kco_double_to_e4m3(ldexp(kco_decode(bits[i], dtype), -k_exp));", "out[i] = kco_double_to_e4m3(ldexp(kco_decode(bits[i], dtype), k_exp));"),
    ("k8 unit: exponent ignored", "ldexp(kco_e4m3_to_double(K8[(size_t)t * d + c]), k_exp)", "ldexp(kco_e4m3_to_double(K8[(size_t)t * d + c]), 0)"),
    ("k8 store: V quantised position", "k8_cache[dst] = kco_double_to_e4m3(ldexp(kco_decode(k_new[src], dtype), -k_exp));", "k8_cache[dst] = kco_double_to_e4m3(ldexp(kco_decode(v_new[src], dtype), -k_exp));"),
    ("store: heads and tokens swapped in the source index", "size_t src = (((size_t)b * T + t) * Hkv + hk) * d + c;\n          size_t dst = (((size_t)b * Hkv + hk) * S_cap + (size_t)(pos[b] + t)) * d + c;\n          k_cache[dst] = k_new[src];", "size_t src = (((size_t)b * Hkv + hk) * T + t) * d + c;\n          size_t dst = (((size_t)b * Hkv + hk) * S_cap + (size_t)(pos[b] + t)) * d + c;\n          k_cache[dst] = k_new[src];"),
    ("store: position offset ignored", "(size_t)(pos[b] + t)) * d + c;\n          k_cache[dst] = k_new[src];", "(size_t)(t)) * d + c;\n          k_cache[dst] = k_new[src];"),
    ("store: tokens reversed inside the range", "size_t dst = (((size_t)b * Hkv + hk) * S_cap + (size_t)(pos[b] + t)) * d + c;\n          k_cache[dst] = k_new[src];",
     "size_t dst = (((size_t)b * Hkv + hk) * S_cap + (size_t)(pos[b] + (T - 1 - t))) * d + c;\n          k_cache[dst] = k_new[src];"),
    ("k8 store: tokens reversed inside the range", "size_t dst = (((size_t)b * Hkv + hk) * S_cap + (size_t)(pos[b] + t)) * d + c;\n          k8_cache[dst] =",
     "size_t dst = (((size_t)b * Hkv + hk) * S_cap + (size_t)(pos[b] + (T - 1 - t))) * d + c;\n          k8_cache[dst] ="),
    ("store: V rows written into the K cache's place", "k_cache[dst] = k_new[src];\n          v_cache[dst] = v_new[src];", "k_cache[dst] = v_new[src];\n          v_cache[dst] = k_new[src];"),
    ("conventional attention: scale dropped", "const double inv_sqrt_d = 1.0 / sqrt((double)d);\n  for (int32_t t = 0; t < s; ++t) {\n    double acc = 0.0;\n    for (int32_t c = 0; c < d; ++c)\n      acc += kco_decode(q[c], dtype)",
     "const double inv_sqrt_d = 1.0;\n  for (int32_t t = 0; t < s; ++t) {\n    double acc = 0.0;\n    for (int32_t c = 0; c < d; ++c)\n      acc += kco_decode(q[c], dtype)"),
    ("conventional attention: not normalised", "const double p = exp(z[t] - m) / Z;", "const double p = exp(z[t] - m);"),
    ("conventional attention: K for V", "out[c] += p * kco_decode(V[(size_t)t * d + c], dtype);", "out[c] += p * kco_decode(K[(size_t)t * d + c], dtype);"),
    ("conventional attention: wrong KV head in a group", "size_t kv_off = ((size_t)b * Hkv + h / G) * (size_t)S_cap * d;\n    int rc = kcache_oracle_full_unit", "size_t kv_off = ((size_t)b * Hkv + h % Hkv) * (size_t)S_cap * d;\n    int rc = kcache_oracle_full_unit"),
]

PINS = [getattr(pins, n) for n in dir(pins) if n.startswith("test_")]


def run_pins():
    """Runs every pin (all parameter combinations); returns the names of those that fail."""
    failed = []
    for fn in PINS:
        combos = [{}]
        for mark in getattr(fn, "pytestmark", []):
            if mark.name == "parametrize":
                names = [n.strip() for n in mark.args[0].split(",")]
                vals = [v if isinstance(v, (tuple, list)) else (v,) for v in mark.args[1]]
                combos = [dict(c, **dict(zip(names, v))) for c in combos for v in vals]
        for kw in combos:
            try:
                fn(**kw)
            except Exception:   # a failing assertion, or a mutant that breaks an invariant
                failed.append(fn.__name__)
                break
    return failed


def test_unmutated_oracle_passes_every_pin():
    assert run_pins() == []


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new):
    assert SRC.count(old) == 1, "mutation site not unique / not found: %s" % name
    c_file, so_file = tmp_path / "mutant.c", tmp_path / "mutant.so"
    c_file.write_text(SRC.replace(old, new))
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o",
                           str(so_file), str(c_file), "-lm"])
    real = oracle._load()
    mutant = ctypes.CDLL(str(so_file))
    for sym in ("kcache_oracle_decode16", "kcache_oracle_unit", "kcache_oracle_unit_renormalised",
                "kcache_oracle_decode", "kcache_oracle_full_unit", "kcache_oracle_full_attention",
                "kcache_oracle_store", "kcache_oracle_store_k8", "kcache_oracle_unit_k8",
                "kcache_oracle_e4m3_decode", "kcache_oracle_e4m3_quantise"):
        getattr(mutant, sym).argtypes = getattr(real, sym).argtypes
        getattr(mutant, sym).restype = getattr(real, sym).restype
    oracle._lib = mutant
    try:
        failed = run_pins()
    finally:
        oracle._lib = real
    assert failed, "no pin notices the planted mistake: %s" % name
