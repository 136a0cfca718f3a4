"""ctypes front end of the CPU oracle (oracle/kcache_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the GPU library or its binding.  Inputs
and outputs are numpy arrays; 16-bit tensors travel as their uint16 bit
patterns so that no conversion happens outside the C file.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kcache_oracle.c")
_LIB = os.path.join(_HERE, "libkcache_oracle.so")

F16, BF16 = 0, 1
_lib = None


def build(force=False):
    """Compile the oracle with gcc -O2 (plain C, OpenMP only to split units over threads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_i32, c_i64, c_p = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        lib.kcache_oracle_decode16.argtypes = [c_p, c_i64, ctypes.c_int, c_p]
        lib.kcache_oracle_decode16.restype = None
        lib.kcache_oracle_unit.argtypes = [c_p, c_p, c_p, ctypes.c_int, c_i32, c_i32, c_i32,
                                           c_p, c_p, c_p, c_p, c_p]
        lib.kcache_oracle_unit.restype = ctypes.c_int
        lib.kcache_oracle_unit_renormalised.argtypes = lib.kcache_oracle_unit.argtypes
        lib.kcache_oracle_unit_renormalised.restype = ctypes.c_int
        lib.kcache_oracle_unit_k8.argtypes = [c_p, c_p, ctypes.c_int, c_p, ctypes.c_int, c_i32,
                                              c_i32, c_i32, c_p, c_p, c_p, c_p, c_p]
        lib.kcache_oracle_unit_k8.restype = ctypes.c_int
        lib.kcache_oracle_e4m3_decode.argtypes = [c_p, c_i64, c_p]
        lib.kcache_oracle_e4m3_decode.restype = None
        lib.kcache_oracle_e4m3_quantise.argtypes = [c_p, c_i64, ctypes.c_int, ctypes.c_int, c_p]
        lib.kcache_oracle_e4m3_quantise.restype = None
        lib.kcache_oracle_decode.argtypes = [c_p, c_p, c_p, ctypes.c_int, c_i32, c_i32, c_i32,
                                             c_i32, c_i32, c_p, c_i32, c_p, c_p, c_p, ctypes.c_int]
        lib.kcache_oracle_decode.restype = ctypes.c_int
        lib.kcache_oracle_full_unit.argtypes = [c_p, c_p, c_p, ctypes.c_int, c_i32, c_i32, c_p, c_p]
        lib.kcache_oracle_full_unit.restype = ctypes.c_int
        lib.kcache_oracle_full_attention.argtypes = [c_p, c_p, c_p, ctypes.c_int, c_i32, c_i32,
                                                     c_i32, c_i32, c_i32, c_p, c_p, ctypes.c_int]
        lib.kcache_oracle_full_attention.restype = ctypes.c_int
        lib.kcache_oracle_store.argtypes = [c_p, c_p, c_p, c_p, c_p, c_i32, c_i32, c_i32, c_i32,
                                            c_i32]
        lib.kcache_oracle_store.restype = ctypes.c_int
        lib.kcache_oracle_store_k8.argtypes = [c_p, c_p, c_p, c_p, c_p, c_i32, c_i32, c_i32, c_i32,
                                               c_i32, ctypes.c_int, ctypes.c_int]
        lib.kcache_oracle_store_k8.restype = ctypes.c_int
        _lib = lib
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("16-bit tensors are passed as uint16 bit patterns, got %s" % a.dtype)
    return a


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def decode16(bits, dtype):
    """Exact double values of an array of fp16 (dtype=F16) or bf16 (BF16) bit patterns."""
    bits = _u16(bits)
    out = np.empty(bits.shape, dtype=np.float64)
    _load().kcache_oracle_decode16(_ptr(bits), bits.size, dtype, _ptr(out))
    return out


def e4m3_decode(codes):
    """Exact double values of an array of OCP FP8 E4M3 codes (uint8)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape, np.float64)
    _load().kcache_oracle_e4m3_decode(_ptr(codes), codes.size, _ptr(out))
    return out


def e4m3_quantise(bits, dtype, k_exp):
    """E4M3 codes of the 16-bit values `bits` scaled by 2^-k_exp (nearest, ties to even,
    saturating at 448)."""
    bits = _u16(bits)
    out = np.empty(bits.shape, np.uint8)
    _load().kcache_oracle_e4m3_quantise(_ptr(bits), bits.size, dtype, int(k_exp), _ptr(out))
    return out


def decode_unit_k8(q, K8, k_exp, V, dtype, N, want_scores=False):
    """decode_unit with the K rows given as E4M3 codes K8 [s][d] and the cache exponent."""
    q, V = _u16(q), _u16(V)
    K8 = np.ascontiguousarray(K8, dtype=np.uint8)
    s, d = K8.shape
    assert q.shape == (d,) and V.shape == (s, d)
    out = np.empty(d, np.float64)
    idx = np.empty(N, np.int32)
    w = np.empty(N, np.float64)
    z = np.empty(s, np.float64) if want_scores else None
    p = np.empty(s, np.float64) if want_scores else None
    rc = _load().kcache_oracle_unit_k8(_ptr(q), _ptr(K8), int(k_exp), _ptr(V), dtype, s, d, N,
                                       _ptr(out), _ptr(idx), _ptr(w),
                                       _ptr(z) if want_scores else None,
                                       _ptr(p) if want_scores else None)
    if rc != 0:
        raise ValueError("kcache_oracle_unit_k8 rejected its arguments")
    res = dict(out=out, idx=idx, w=w)
    if want_scores:
        res.update(z=z, p=p)
    return res


def decode_unit(q, K, V, dtype, N, want_scores=False, renormalise=False):
    """One (sequence, head) unit.  q [d], K [s][d], V [s][d] as uint16 bits.

    Returns dict(out [d] f64, idx [N] i32 ascending / -1 padded, w [N] f64,
    and with want_scores: z [s], p [s]).  renormalise selects the variant whose kept
    weights are divided by their sum."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    s, d = K.shape
    assert q.shape == (d,) and V.shape == (s, d)
    out = np.empty(d, np.float64)
    idx = np.empty(N, np.int32)
    w = np.empty(N, np.float64)
    z = np.empty(s, np.float64) if want_scores else None
    p = np.empty(s, np.float64) if want_scores else None
    fn = _load().kcache_oracle_unit_renormalised if renormalise else _load().kcache_oracle_unit
    rc = fn(_ptr(q), _ptr(K), _ptr(V), dtype, s, d, N, _ptr(out), _ptr(idx), _ptr(w),
            _ptr(z) if want_scores else None, _ptr(p) if want_scores else None)
    if rc != 0:
        raise ValueError("kcache_oracle_unit rejected its arguments")
    res = dict(out=out, idx=idx, w=w)
    if want_scores:
        res.update(z=z, p=p)
    return res


def decode_attention(q, K, V, dtype, seq_lens, N, nthreads=1):
    """One layer.  q [B][H][d], K and V [B][Hkv][S_cap][d] (uint16 bits), seq_lens [B].

    Returns (out [B][H][d] f64, idx [B][H][N] i32, w [B][H][N] f64)."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    B, H, d = q.shape
    Bk, Hkv, S_cap, dk = K.shape
    assert (Bk, dk) == (B, d) and V.shape == K.shape
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    assert seq_lens.shape == (B,)
    out = np.empty((B, H, d), np.float64)
    idx = np.empty((B, H, N), np.int32)
    w = np.empty((B, H, N), np.float64)
    rc = _load().kcache_oracle_decode(_ptr(q), _ptr(K), _ptr(V), dtype, B, H, Hkv, S_cap, d,
                                      _ptr(seq_lens), N, _ptr(out), _ptr(idx), _ptr(w),
                                      int(nthreads))
    if rc != 0:
        raise ValueError("kcache_oracle_decode rejected its arguments")
    return out, idx, w


def full_unit(q, K, V, dtype, want_p=False):
    """Conventional attention of one (sequence, head) unit: softmax(q K^T / sqrt(d)) V.

    Returns out [d] f64, or (out, p [s]) with want_p."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    s, d = K.shape
    assert q.shape == (d,) and V.shape == (s, d)
    out = np.empty(d, np.float64)
    p = np.empty(s, np.float64) if want_p else None
    rc = _load().kcache_oracle_full_unit(_ptr(q), _ptr(K), _ptr(V), dtype, s, d, _ptr(out),
                                         _ptr(p) if want_p else None)
    if rc != 0:
        raise ValueError("kcache_oracle_full_unit rejected its arguments")
    return (out, p) if want_p else out


def full_attention(q, K, V, dtype, seq_lens, nthreads=1):
    """Conventional attention, one layer.  Layouts as decode_attention; returns out [B][H][d] f64."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    B, H, d = q.shape
    Bk, Hkv, S_cap, dk = K.shape
    assert (Bk, dk) == (B, d) and V.shape == K.shape
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    assert seq_lens.shape == (B,)
    out = np.empty((B, H, d), np.float64)
    rc = _load().kcache_oracle_full_attention(_ptr(q), _ptr(K), _ptr(V), dtype, B, H, Hkv, S_cap,
                                              d, _ptr(seq_lens), _ptr(out), int(nthreads))
    if rc != 0:
        raise ValueError("kcache_oracle_full_attention rejected its arguments")
    return out


def store(k_cache, v_cache, k_new, v_new, pos):
    """In-place cache store.  k_new, v_new [B][T][Hkv][d] -> caches [B][Hkv][S_cap][d] at pos[b]."""
    for a in (k_cache, v_cache):
        if a.dtype != np.uint16 or not a.flags.c_contiguous or not a.flags.writeable:
            raise TypeError("caches must be writable contiguous uint16 arrays")
    k_new, v_new = _u16(k_new), _u16(v_new)
    B, T, Hkv, d = k_new.shape
    assert v_new.shape == k_new.shape
    assert k_cache.shape == v_cache.shape and k_cache.shape[0] == B and k_cache.shape[1] == Hkv
    S_cap = k_cache.shape[2]
    assert k_cache.shape[3] == d
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    assert pos.shape == (B,)
    rc = _load().kcache_oracle_store(_ptr(k_cache), _ptr(v_cache), _ptr(k_new), _ptr(v_new),
                                     _ptr(pos), B, T, Hkv, S_cap, d)
    if rc != 0:
        raise ValueError("kcache_oracle_store rejected its arguments")


def store_k8(k8_cache, v_cache, k_new, v_new, pos, dtype, k_exp):
    """In-place store into a cache whose K rows are E4M3 codes (uint8) with exponent k_exp."""
    if k8_cache.dtype != np.uint8 or v_cache.dtype != np.uint16:
        raise TypeError("k8_cache must be uint8, v_cache uint16")
    for a in (k8_cache, v_cache):
        if not a.flags.c_contiguous or not a.flags.writeable:
            raise TypeError("caches must be writable contiguous arrays")
    k_new, v_new = _u16(k_new), _u16(v_new)
    B, T, Hkv, d = k_new.shape
    assert v_new.shape == k_new.shape and k8_cache.shape == v_cache.shape
    assert k8_cache.shape[0] == B and k8_cache.shape[1] == Hkv and k8_cache.shape[3] == d
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    rc = _load().kcache_oracle_store_k8(_ptr(k8_cache), _ptr(v_cache), _ptr(k_new), _ptr(v_new),
                                        _ptr(pos), B, T, Hkv, k8_cache.shape[2], d, dtype,
                                        int(k_exp))
    if rc != 0:
        raise ValueError("kcache_oracle_store_k8 rejected its arguments")
