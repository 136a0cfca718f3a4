"""ctypes marshalling for the C ABI declared in include/kcache.h."""
import ctypes
import os
import re

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkcache.so")
_HEADER = os.path.join(os.path.dirname(_HERE), "include", "kcache.h")

KC_F16, KC_BF16 = 0, 1
GATHER_ZEROCOPY, GATHER_STAGED = 0, 1
KERNELS = {"kscan": 0, "select": 1, "gather": 2, "store_k": 3, "store_v": 4, "fused": 5,
           "full": 6}
OPT_PIPELINE_PARTS, OPT_PROFILE, OPT_STAGED_THREADS, OPT_FUSED, OPT_FUSED_ROWS = 0, 1, 2, 3, 4
OPT_STEP_LANES, OPT_RENORMALIZE, OPT_STEP_SPLIT, OPT_GQA_DEDUP, OPT_AUTO_GROW, OPT_XCD_SPREAD = 5, 6, 7, 8, 9, 10
STAT_REALLOCS, STAT_WORKSPACE_BYTES, STAT_TICKETS, STAT_STEP_LANES = 0, 1, 2, 3

_c_i32, _c_i64, _c_p, _c_sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t


class KCacheError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("kcache status %d: %s" % (status, text))
        self.status = status


class _CLayerCache(ctypes.Structure):
    _fields_ = [("k_dev", _c_p), ("v_host", _c_p), ("B", _c_i32), ("Hkv", _c_i32),
                ("S_cap", _c_i32), ("d", _c_i32), ("dtype", _c_i32), ("v_in_hbm", _c_i32),
                ("k_fp8", _c_i32), ("k_exp", _c_i32)]


class _CStepLayer(ctypes.Structure):
    _fields_ = [("cache", _CLayerCache), ("k_new_dev", _c_p), ("v_new_dev", _c_p),
                ("q_dev", _c_p), ("out_dev", _c_p), ("idx_out_dev", _c_p), ("w_out_dev", _c_p)]


_lib = None


def lib_path():
    return _LIB_PATH


def lib():
    """The loaded shared library; built beforehand by paper_2404_18057_amd.build."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                "libkcache.so is missing: build it with `python -m paper_2404_18057_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(_LIB_PATH)
        pp = ctypes.POINTER(_c_p)
        cache_p = ctypes.POINTER(_CLayerCache)
        dbl_p, i64_p = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_c_i64)
        sig = {
            "kcache_version": (ctypes.c_char_p, []),
            "kcache_create": (ctypes.c_int, [pp, ctypes.c_int, _c_sz]),
            "kcache_destroy": (ctypes.c_int, [_c_p]),
            "kcache_workspace_bytes": (_c_sz, [_c_i32, _c_i32, _c_i32, _c_i32]),
            "kcache_last_error": (ctypes.c_char_p, [_c_p]),
            "kcache_set_option": (ctypes.c_int, [_c_p, _c_i32, _c_i64]),
            "kcache_reserve": (ctypes.c_int, [_c_p, cache_p, _c_i32, _c_i32, _c_i32, _c_i32]),
            "kcache_stat": (_c_i64, [_c_p, _c_i32]),
            "kcache_step_lanes_for": (_c_i32, [_c_p, cache_p, _c_i32, _c_i32]),
            "kcache_check_shapes": (ctypes.c_int, [cache_p, _c_i32, _c_i32]),
            "kcache_prefill_store": (ctypes.c_int, [_c_p, cache_p, _c_p, _c_p, _c_p, _c_i32, _c_p,
                                                    _c_p]),
            "kcache_prefill_store_at": (ctypes.c_int, [_c_p, cache_p, _c_p, _c_p, _c_p, _c_i32, _c_p,
                                                       _c_p]),
            "kcache_decode_attention": (ctypes.c_int, [_c_p, cache_p, _c_p, _c_i32, _c_p, _c_i32,
                                                       _c_p, _c_p, _c_p, _c_i32, _c_p]),
            "kcache_decode_attention_static": (ctypes.c_int, [_c_p, cache_p, _c_p, _c_i32, _c_p,
                                                              _c_i32, _c_p, _c_p, _c_p, _c_p]),
            "kcache_static_scratch_bytes": (_c_sz, []),
            "kcache_full_attention": (ctypes.c_int, [_c_p, cache_p, _c_p, _c_i32, _c_p, _c_p, _c_p]),
            "kcache_decode_step": (ctypes.c_int, [_c_p, ctypes.POINTER(_CStepLayer), _c_i32, _c_i32,
                                                  _c_p, _c_p, _c_i32, _c_p]),
            "kcache_step_graph_create": (ctypes.c_int, [_c_p, ctypes.POINTER(_CStepLayer), _c_i32,
                                                        _c_i32, _c_p, _c_p, _c_i32, pp]),
            "kcache_step_graph_launch": (ctypes.c_int, [_c_p, _c_p, _c_p]),
            "kcache_step_graph_destroy": (ctypes.c_int, [_c_p, _c_p]),
            "kcache_synchronize": (ctypes.c_int, [_c_p]),
            "kcache_device_check": (ctypes.c_int, [_c_p]),
            "kcache_profile_read": (ctypes.c_int, [_c_p, _c_i32, dbl_p, i64_p]),
            "kcache_profile_reset": (ctypes.c_int, [_c_p]),
            "kcache_probe_read": (ctypes.c_int, [_c_p, _c_p, _c_sz, _c_i32, _c_p, dbl_p]),
            "kcache_probe_rows": (ctypes.c_int, [_c_p, _c_p, _c_sz, _c_i64, _c_i32, _c_p, dbl_p]),
            "kcache_probe_copy": (ctypes.c_int, [_c_p, _c_p, _c_p, _c_sz, _c_i32, _c_p, dbl_p]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def declared_symbols():
    """Names of the functions include/kcache.h declares (for the export test)."""
    text = open(_HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kcache_[a-z_]+)\s*\(", text)))


def version():
    return lib().kcache_version().decode()


def static_scratch_bytes():
    return int(lib().kcache_static_scratch_bytes())


def workspace_bytes(B, H, S_cap, N):
    return int(lib().kcache_workspace_bytes(B, H, S_cap, N))


class LayerCache:
    """One layer's K cache (device tensor) and V cache, both [B][Hkv][S_cap][d] in
    fp16 or bf16.  The V cache is a pinned host tensor, or a device tensor for a
    layer that keeps V in HBM.  Holds references, owns nothing else."""

    def __init__(self, k_dev, v, k_exp=0):
        """A uint8 k_dev is an 8-bit K cache of E4M3 codes with the scale exponent k_exp."""
        self.k_fp8 = k_dev.dtype == torch.uint8
        if k_dev.shape != v.shape or k_dev.dim() != 4 or \
                (k_dev.dtype != v.dtype and not self.k_fp8):
            raise ValueError("K and V caches must have the same 4-d shape and dtype")
        if not (k_dev.is_contiguous() and v.is_contiguous()):
            raise ValueError("caches must be contiguous")
        if not k_dev.is_cuda:
            raise ValueError("K cache must be a device tensor")
        self.k, self.v = k_dev, v
        self.v_in_hbm = bool(v.is_cuda)
        B, Hkv, S_cap, d = k_dev.shape
        self.c = _CLayerCache(k_dev.data_ptr(), v.data_ptr(), B, Hkv, S_cap, d,
                              _dtype_code(v.dtype), 1 if self.v_in_hbm else 0,
                              1 if self.k_fp8 else 0, int(k_exp) if self.k_fp8 else 0)


class StepGraph:
    """A captured decode step (kcache_step_graph_*).  Keeps its tensors alive."""

    def __init__(self, ctx, handle, keep):
        self._ctx, self._h, self._keep = ctx, handle, keep

    def launch(self, stream=None):
        self._ctx._check(lib().kcache_step_graph_launch(self._ctx._h, self._h,
                                                        _stream_ptr(stream)))

    def close(self):
        if self._h:
            lib().kcache_step_graph_destroy(self._ctx._h, self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _dtype_code(dt):
    if dt == torch.float16:
        return KC_F16
    if dt == torch.bfloat16:
        return KC_BF16
    raise ValueError("dtype must be float16 or bfloat16, got %s" % dt)


def check_shapes(B, Hkv, S_cap, d, dtype_code, H, N):
    """Host-only shape validation (no GPU needed); returns the kc_status."""
    c = _CLayerCache(None, None, B, Hkv, S_cap, d, dtype_code, 0, 0, 0)
    return int(lib().kcache_check_shapes(ctypes.byref(c), H, N))


def _stream_ptr(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


class Context:
    def __init__(self, device=0, workspace_bytes_hint=0, auto_grow=True):
        """auto_grow=True sets KC_OPT_AUTO_GROW: calls size the context on demand (handy for
        tests and scripts; each growth synchronises the device).  With auto_grow=False the
        library's own default applies: size the context with reserve() first."""
        self._h = _c_p()
        rc = lib().kcache_create(ctypes.byref(self._h), int(device), int(workspace_bytes_hint))
        if rc != 0:
            self._h = None
            raise KCacheError(rc, lib().kcache_last_error(None).decode())
        self.device = torch.device("cuda", int(device))
        if auto_grow:
            self.set_option(OPT_AUTO_GROW, 1)

    def reserve(self, cache, H, N, gather_mode=GATHER_ZEROCOPY, step_layers=0):
        """kcache_reserve for the shape of `cache` (a LayerCache; only its shape fields are read)."""
        self._check(lib().kcache_reserve(self._h, ctypes.byref(cache.c), int(H), int(N),
                                         int(gather_mode), int(step_layers)))

    def stat(self, which):
        return int(lib().kcache_stat(self._h, int(which)))

    def step_lanes_for(self, cache, L, H):
        return int(lib().kcache_step_lanes_for(self._h, ctypes.byref(cache.c), int(L), int(H)))

    def close(self):
        if getattr(self, "_h", None):
            lib().kcache_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != 0:
            raise KCacheError(rc, lib().kcache_last_error(self._h).decode())

    def set_option(self, option, value):
        self._check(lib().kcache_set_option(self._h, option, int(value)))

    def set_pipeline_parts(self, parts):
        self.set_option(OPT_PIPELINE_PARTS, parts)

    def set_profile(self, on):
        self.set_option(OPT_PROFILE, 1 if on else 0)

    def set_fused(self, on):
        self.set_option(OPT_FUSED, 1 if on else 0)

    def set_fused_rows(self, rows):
        self.set_option(OPT_FUSED_ROWS, rows)

    def set_staged_threads(self, n):
        self.set_option(OPT_STAGED_THREADS, n)

    def prefill_store(self, cache, k_new, v_new, pos, stream=None, done_event=None):
        """k_new, v_new: device [B][T][Hkv][d]; pos: device int32 [B]."""
        B, T, Hkv, d = k_new.shape
        if v_new.shape != k_new.shape or (B, Hkv, d) != (cache.c.B, cache.c.Hkv, cache.c.d):
            raise ValueError("k_new / v_new shape does not match the cache")
        if k_new.dtype != cache.v.dtype or v_new.dtype != cache.v.dtype:
            raise ValueError("k_new / v_new dtype does not match the cache")
        if not (k_new.is_contiguous() and v_new.is_contiguous() and pos.is_contiguous()):
            raise ValueError("inputs must be contiguous")
        if pos.dtype != torch.int32 or pos.numel() != B or not pos.is_cuda:
            raise ValueError("pos must be a device int32 [B] tensor")
        ev = None
        if done_event is not None:
            if not done_event.cuda_event:
                # torch creates the HIP event lazily at its first record(); without a handle
                # the library would record nothing and a later synchronize() would not wait
                done_event.record(torch.cuda.current_stream() if stream is None else stream)
            ev = ctypes.c_void_p(done_event.cuda_event)
        self._check(lib().kcache_prefill_store(self._h, ctypes.byref(cache.c), _ptr(k_new),
                                               _ptr(v_new), _ptr(pos), T, _stream_ptr(stream), ev))

    def prefill_store_at(self, cache, k_new, v_new, pos_host, stream=None, done_event=None):
        """kcache_prefill_store_at: pos_host is a host int32 sequence / array of B positions."""
        B, T, Hkv, d = k_new.shape
        if v_new.shape != k_new.shape or (B, Hkv, d) != (cache.c.B, cache.c.Hkv, cache.c.d):
            raise ValueError("k_new / v_new shape does not match the cache")
        if k_new.dtype != cache.v.dtype or v_new.dtype != cache.v.dtype:
            raise ValueError("k_new / v_new dtype does not match the cache")
        if not (k_new.is_contiguous() and v_new.is_contiguous()):
            raise ValueError("inputs must be contiguous")
        pos = (ctypes.c_int32 * B)(*[int(p) for p in pos_host])
        ev = None
        if done_event is not None:
            if not done_event.cuda_event:
                done_event.record(torch.cuda.current_stream() if stream is None else stream)
            ev = ctypes.c_void_p(done_event.cuda_event)
        self._check(lib().kcache_prefill_store_at(self._h, ctypes.byref(cache.c), _ptr(k_new),
                                                  _ptr(v_new), pos, T, _stream_ptr(stream), ev))

    def decode_attention(self, cache, q, seq_lens, N, out=None, idx_out=None, w_out=None,
                         gather_mode=GATHER_ZEROCOPY, stream=None):
        """q: device [B][H][d]; seq_lens: device int32 [B].  Returns out fp32 [B][H][d]."""
        B, H, d = q.shape
        if (B, d) != (cache.c.B, cache.c.d) or q.dtype != cache.v.dtype or not q.is_contiguous():
            raise ValueError("q does not match the cache")
        if seq_lens.dtype != torch.int32 or seq_lens.numel() != B or not seq_lens.is_cuda:
            raise ValueError("seq_lens must be a device int32 [B] tensor")
        if out is None:
            out = torch.empty((B, H, d), dtype=torch.float32, device=q.device)
        for t, dt in ((out, torch.float32), (idx_out, torch.int32), (w_out, torch.float32)):
            if t is not None and (t.dtype != dt or not t.is_contiguous() or not t.is_cuda):
                raise ValueError("output tensors must be contiguous device tensors of the ABI type")
        if out.shape != (B, H, d):
            raise ValueError("out must be [B][H][d]")
        for t in (idx_out, w_out):
            if t is not None and tuple(t.shape) != (B, H, N):
                raise ValueError("idx_out / w_out must be [B][H][N]")
        self._check(lib().kcache_decode_attention(
            self._h, ctypes.byref(cache.c), _ptr(q), H, _ptr(seq_lens), int(N), _ptr(out),
            _ptr(idx_out), _ptr(w_out), int(gather_mode), _stream_ptr(stream)))
        return out

    def decode_attention_static(self, cache, q, seq_lens, N, out, idx_out=None, w_out=None,
                                stream=None):
        """kcache_decode_attention_static: the caller passes every output; nothing is allocated."""
        B, H, d = q.shape
        if (B, d) != (cache.c.B, cache.c.d) or q.dtype != cache.v.dtype or not q.is_contiguous():
            raise ValueError("q does not match the cache")
        if seq_lens.dtype != torch.int32 or seq_lens.numel() != B or not seq_lens.is_cuda:
            raise ValueError("seq_lens must be a device int32 [B] tensor")
        for t, dt in ((out, torch.float32), (idx_out, torch.int32), (w_out, torch.float32)):
            if t is not None and (t.dtype != dt or not t.is_contiguous() or not t.is_cuda):
                raise ValueError("output tensors must be contiguous device tensors of the ABI type")
        if out is None or out.shape != (B, H, d):
            raise ValueError("out must be a device fp32 [B][H][d] tensor")
        for t in (idx_out, w_out):
            if t is not None and tuple(t.shape) != (B, H, N):
                raise ValueError("idx_out / w_out must be [B][H][N]")
        self._check(lib().kcache_decode_attention_static(
            self._h, ctypes.byref(cache.c), _ptr(q), H, _ptr(seq_lens), int(N), _ptr(out),
            _ptr(idx_out), _ptr(w_out), _stream_ptr(stream)))
        return out

    def full_attention(self, cache, q, seq_lens, out=None, stream=None):
        """Conventional attention of a layer whose V cache is in HBM.  Returns out fp32 [B][H][d]."""
        B, H, d = q.shape
        if (B, d) != (cache.c.B, cache.c.d) or q.dtype != cache.v.dtype or not q.is_contiguous():
            raise ValueError("q does not match the cache")
        if seq_lens.dtype != torch.int32 or seq_lens.numel() != B or not seq_lens.is_cuda:
            raise ValueError("seq_lens must be a device int32 [B] tensor")
        if out is None:
            out = torch.empty((B, H, d), dtype=torch.float32, device=q.device)
        if out.dtype != torch.float32 or not out.is_contiguous() or not out.is_cuda or \
                out.shape != (B, H, d):
            raise ValueError("out must be a contiguous device fp32 [B][H][d] tensor")
        self._check(lib().kcache_full_attention(self._h, ctypes.byref(cache.c), _ptr(q), H,
                                                _ptr(seq_lens), _ptr(out), _stream_ptr(stream)))
        return out

    def set_gqa_dedup(self, on):
        self.set_option(OPT_GQA_DEDUP, 1 if on else 0)

    def set_xcd_spread(self, on):
        self.set_option(OPT_XCD_SPREAD, 1 if on else 0)

    def set_renormalize(self, on):
        self.set_option(OPT_RENORMALIZE, 1 if on else 0)

    def set_step_lanes(self, lanes, split_sequences=False):
        """Streams a step is spread over (0 = chosen from the shape, the library's default);
        split_sequences: each lane takes a share of the batch through all layers
        (dependency-preserving) instead of whole layers."""
        self.set_option(OPT_STEP_LANES, lanes)
        self.set_option(OPT_STEP_SPLIT, 1 if split_sequences else 0)

    @staticmethod
    def _step_array(layers):
        """layers: sequence of dicts with cache, q, out and optionally k_new, v_new, idx_out,
        w_out (tensors).  Returns the C array; the caller keeps the tensors alive."""
        arr = (_CStepLayer * len(layers))()
        for i, y in enumerate(layers):
            arr[i].cache = y["cache"].c
            for field, key in (("k_new_dev", "k_new"), ("v_new_dev", "v_new"), ("q_dev", "q"),
                               ("out_dev", "out"), ("idx_out_dev", "idx_out"),
                               ("w_out_dev", "w_out")):
                t = y.get(key)
                setattr(arr[i], field, t.data_ptr() if t is not None else None)
        return arr

    def decode_step(self, layers, H, pos, seq_lens, N, stream=None):
        """Append + attention for every layer in one call (see kcache_decode_step)."""
        arr = self._step_array(layers)
        self._check(lib().kcache_decode_step(self._h, arr, len(layers), H, _ptr(pos),
                                             _ptr(seq_lens), int(N), _stream_ptr(stream)))

    def step_graph(self, layers, H, pos, seq_lens, N):
        """The same step captured into a HIP graph; returns a StepGraph to launch per step."""
        arr = self._step_array(layers)
        h = _c_p()
        self._check(lib().kcache_step_graph_create(self._h, arr, len(layers), H, _ptr(pos),
                                                   _ptr(seq_lens), int(N), ctypes.byref(h)))
        return StepGraph(self, h, (list(layers), pos, seq_lens))

    def synchronize(self):
        self._check(lib().kcache_synchronize(self._h))

    def device_check(self):
        self._check(lib().kcache_device_check(self._h))

    def profile_read(self, kernel):
        ms, n = ctypes.c_double(), _c_i64()
        self._check(lib().kcache_profile_read(self._h, KERNELS[kernel], ctypes.byref(ms),
                                              ctypes.byref(n)))
        return ms.value, n.value

    def profile_reset(self):
        self._check(lib().kcache_profile_reset(self._h))

    def probe_read(self, tensor, iters=5, stream=None):
        g = ctypes.c_double()
        nbytes = tensor.numel() * tensor.element_size()
        self._check(lib().kcache_probe_read(self._h, _ptr(tensor), nbytes, iters,
                                            _stream_ptr(stream), ctypes.byref(g)))
        return g.value

    def probe_rows(self, tensor, n_rows, iters=5, stream=None):
        g = ctypes.c_double()
        nbytes = tensor.numel() * tensor.element_size()
        self._check(lib().kcache_probe_rows(self._h, _ptr(tensor), nbytes, int(n_rows), iters,
                                            _stream_ptr(stream), ctypes.byref(g)))
        return g.value

    def probe_copy(self, dst, src, iters=5, stream=None):
        g = ctypes.c_double()
        nbytes = src.numel() * src.element_size()
        if dst.numel() * dst.element_size() < nbytes:
            raise ValueError("dst smaller than src")
        self._check(lib().kcache_probe_copy(self._h, _ptr(dst), _ptr(src), nbytes, iters,
                                            _stream_ptr(stream), ctypes.byref(g)))
        return g.value
