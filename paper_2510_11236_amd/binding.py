"""Thin ctypes binding of the C ABI in include/xq.h.

Argument marshalling only: every step of the path runs in the HIP kernels of
libxq.so.  PyTorch supplies device memory (the arena, the workspace, inputs and
outputs) and the current stream.  There is no fallback: if libxq.so is missing
the import of the library raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libxq.so")
_LIB = None

XQ_DECODE_PAIR_FUSED = 1
XQ_DECODE_VECTOR_ALU = 2
XQ_DECODE_MATRIX_F16 = 4
XQ_DECODE_MERGE_LAUNCH = 8
XQ_DECODE_MERGE_IN_LAUNCH = 16


class XqError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


class XqConfig(C.Structure):
    """Mirror of struct xq_config."""
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "batch", "n_q_heads", "n_kv_heads", "head_dim", "group",
                                         "residual", "max_tokens", "kq", "vq", "km", "vm")] + \
               [("eta1", C.c_float), ("eta2", C.c_float), ("share_group", C.c_int32), ("share_dominant", C.c_int32),
                ("merge_mode", C.c_int32), ("gamma0", C.c_float), ("page_tokens", C.c_int32), ("n_pages", C.c_int32)]


def lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is not built; run `python -m paper_2510_11236_amd.build`")
        L = C.CDLL(_LIB_PATH)
        vp, cfgp = C.c_void_p, C.POINTER(XqConfig)
        L.xq_strerror.restype = C.c_char_p
        L.xq_strerror.argtypes = [C.c_int]
        L.xq_cache_bytes.argtypes = [cfgp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.xq_cache_create.argtypes = [cfgp, vp, C.c_size_t, C.POINTER(vp)]
        L.xq_cache_destroy.restype = None
        L.xq_cache_destroy.argtypes = [vp]
        L.xq_cache_reset.argtypes = [vp]
        L.xq_cache_len.argtypes = [vp, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.xq_cache_layout.argtypes = [vp, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.xq_quantize_pack.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, C.POINTER(C.c_int64), C.c_int32, vp]
        L.xq_quantize_pack_seq.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, vp, C.POINTER(C.c_int64),
                                           C.c_int32, vp]
        L.xq_cache_len_seq.argtypes = [vp, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.xq_cache_reset_seq.argtypes = [vp, C.c_int32]
        L.xq_cache_pages.argtypes = [vp, C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32)]
        L.xq_cache_free_pages.argtypes = [vp, C.POINTER(C.c_int32)]
        L.xq_append_token.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, vp]
        L.xq_prefill_attention_pack.restype = C.c_int
        L.xq_prefill_attention_pack.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, vp, C.POINTER(C.c_int64), vp, C.c_float,
                                                C.c_int32, C.c_int32, vp]
        L.xq_decode_attention.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, C.c_float, vp, C.c_size_t, C.c_int32, vp]
        L.xq_decode_attention_static.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, C.c_float, C.c_int32, vp]
        L.xq_decode_attention_static.restype = C.c_int
        L.xq_unpack_codes.argtypes = [vp, C.c_int32, C.c_int32, vp, vp]
        L.xq_code_delta_histogram.restype = C.c_int
        L.xq_code_delta_histogram.argtypes = [vp, C.c_int32, C.c_int32, vp, vp]
        L.xq_debug_set_tiles_per_split.restype = None
        L.xq_debug_set_tiles_per_split.argtypes = [vp, C.c_int32]
        L.xq_debug_merge_table.restype = C.c_uint32
        L.xq_debug_merge_table.argtypes = [cfgp, C.c_int32]
        L.xq_equivalent_bits.restype = C.c_double
        L.xq_equivalent_bits.argtypes = [cfgp, C.c_int32, C.c_int32]
        for name in ("xq_cache_bytes", "xq_cache_create", "xq_cache_reset", "xq_cache_len", "xq_cache_layout",
                     "xq_quantize_pack", "xq_append_token", "xq_decode_attention", "xq_unpack_codes",
                     "xq_quantize_pack_seq", "xq_cache_len_seq", "xq_cache_reset_seq"):
            getattr(L, name).restype = C.c_int
        _LIB = L
    return _LIB


def strerror(code: int) -> str:
    return lib().xq_strerror(int(code)).decode()


def _check(code, what):
    if code != 0:
        raise XqError(code, what)


def cache_bytes(cfg: XqConfig):
    a, w = C.c_size_t(0), C.c_size_t(0)
    _check(lib().xq_cache_bytes(C.byref(cfg), C.byref(a), C.byref(w)), "xq_cache_bytes")
    return int(a.value), int(w.value)


def equivalent_bits(cfg: XqConfig, include_metadata: bool = False, T: int = 0) -> float:
    return float(lib().xq_equivalent_bits(C.byref(cfg), int(include_metadata), int(T)))


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class XqCache:
    """Owns the device arena and workspace (torch tensors) and the host handle."""

    def __init__(self, cfg: XqConfig, device="cuda:0"):
        self.cfg = cfg
        self.device = torch.device(device)
        arena_bytes, ws_bytes = cache_bytes(cfg)
        self.arena = torch.empty(arena_bytes, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=self.device)
        h = C.c_void_p()
        _check(lib().xq_cache_create(C.byref(cfg), C.c_void_p(self.arena.data_ptr()), arena_bytes, C.byref(h)),
               "xq_cache_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib().xq_cache_destroy(self._h)
            self._h = None

    __del__ = close

    def reset(self):
        _check(lib().xq_cache_reset(self._h), "xq_cache_reset")

    def reset_seq(self, seq):
        _check(lib().xq_cache_reset_seq(self._h, seq), "xq_cache_reset_seq")

    def length(self, layer=0, seq=0):
        t, tq = C.c_int32(0), C.c_int32(0)
        _check(lib().xq_cache_len_seq(self._h, layer, seq, C.byref(t), C.byref(tq)), "xq_cache_len_seq")
        return int(t.value), int(tq.value)

    def layout(self, layer):
        off, sz = (C.c_int64 * 6)(), (C.c_int64 * 6)()
        _check(lib().xq_cache_layout(self._h, layer, off, sz), "xq_cache_layout")
        names = ("k_codes", "v_codes", "k_meta", "v_meta", "k_res", "v_res")
        return {n: (int(off[i]), int(sz[i])) for i, n in enumerate(names)}

    def region(self, layer, name):
        """uint8 view [slices][bytes] of one region of a layer (for tests): one slice per
        (sequence, kv head), or per (page, kv head) for the packed regions of a paged cache."""
        off, sz = self.layout(layer)[name]
        if off < 0:
            return None
        n = self.cfg.batch * self.cfg.n_kv_heads
        if self.cfg.page_tokens and not name.endswith("_res"):
            n = self.cfg.n_pages * self.cfg.n_kv_heads
        return self.arena[off:off + n * sz].view(n, sz)

    def pages(self, seq):
        """Pages held by a sequence of a paged cache, in token order."""
        n = C.c_int32(0)
        _check(lib().xq_cache_pages(self._h, seq, None, 0, C.byref(n)), "xq_cache_pages")
        buf = (C.c_int32 * max(n.value, 1))()
        _check(lib().xq_cache_pages(self._h, seq, buf, n.value, C.byref(n)), "xq_cache_pages")
        return list(buf[:n.value])

    def free_pages(self):
        n = C.c_int32(0)
        _check(lib().xq_cache_free_pages(self._h, C.byref(n)), "xq_cache_free_pages")
        return n.value

    def slice_bytes(self, layer, name, bh):
        """The bytes one (sequence, kv head) holds in a region, in token order (for tests): a row of
        region(), or the sequence's pages one after the other."""
        r = self.region(layer, name)
        if r is None:
            return None
        if not self.cfg.page_tokens or name.endswith("_res"):
            return r[bh]
        bi, h = divmod(bh, self.cfg.n_kv_heads)
        rows = [p * self.cfg.n_kv_heads + h for p in self.pages(bi)]
        if not rows:
            return r[0][:0]
        return r[torch.tensor(rows, device=r.device)].reshape(-1)

    def quantize_pack(self, k: torch.Tensor, v: torch.Tensor, layer0=0):
        """k, v: fp16 [n_layers][b][h_kv][T][D] (any strides with contiguous D)."""
        assert k.dtype == torch.float16 and v.dtype == torch.float16 and k.dim() == 5 and k.shape == v.shape
        assert k.stride() == v.stride() and k.stride(4) == 1 and k.is_cuda
        strides = (C.c_int64 * 4)(*k.stride()[:4])
        _check(lib().xq_quantize_pack(self._h, layer0, k.shape[0], C.c_void_p(k.data_ptr()),
                                      C.c_void_p(v.data_ptr()), strides, k.shape[3], _stream()), "xq_quantize_pack")

    def quantize_pack_seq(self, k: torch.Tensor, v: torch.Tensor, seq0, layer0=0):
        """k, v: fp16 [n_layers][n_seq][h_kv][T][D] for sequences seq0 .. seq0 + n_seq - 1."""
        assert k.dtype == torch.float16 and v.dtype == torch.float16 and k.dim() == 5 and k.shape == v.shape
        assert k.stride() == v.stride() and k.stride(4) == 1 and k.is_cuda
        strides = (C.c_int64 * 4)(*k.stride()[:4])
        _check(lib().xq_quantize_pack_seq(self._h, layer0, k.shape[0], seq0, k.shape[1], C.c_void_p(k.data_ptr()),
                                          C.c_void_p(v.data_ptr()), strides, k.shape[3], _stream()),
               "xq_quantize_pack_seq")

    def prefill_attention_pack(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, sm_scale: float,
                               out: torch.Tensor = None, layer0=0, pack=True):
        """Causal attention of the prompt + quantize/pack of its K/V in one pass.  q: fp16 contiguous
        [n_layers][b][h_q][T][128]; k, v as for quantize_pack -> fp32 [n_layers][b][h_q][T][128]."""
        assert q.is_contiguous() and q.dtype == torch.float16 and q.dim() == 5
        assert k.dtype == torch.float16 and v.dtype == torch.float16 and k.dim() == 5 and k.shape == v.shape
        assert k.stride() == v.stride() and k.stride(4) == 1 and k.is_cuda and q.shape[3] == k.shape[3]
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        assert out.is_contiguous() and out.dtype == torch.float32 and out.shape == q.shape
        strides = (C.c_int64 * 4)(*k.stride()[:4])
        _check(lib().xq_prefill_attention_pack(self._h, layer0, k.shape[0], C.c_void_p(q.data_ptr()), C.c_void_p(k.data_ptr()),
                                               C.c_void_p(v.data_ptr()), strides, C.c_void_p(out.data_ptr()), float(sm_scale),
                                               k.shape[3], 0 if pack else 1, _stream()), "xq_prefill_attention_pack")
        return out

    def append_token(self, k_new: torch.Tensor, v_new: torch.Tensor, layer0=0):
        """k_new, v_new: fp16 contiguous [n_layers][b][h_kv][D]."""
        assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.dtype == torch.float16
        assert k_new.shape == v_new.shape and k_new.dim() == 4
        _check(lib().xq_append_token(self._h, layer0, k_new.shape[0], C.c_void_p(k_new.data_ptr()),
                                     C.c_void_p(v_new.data_ptr()), _stream()), "xq_append_token")

    def decode_attention(self, q: torch.Tensor, sm_scale: float, out: torch.Tensor = None, layer0=0, flags=0):
        """q: fp16 contiguous [n_layers][b][h_q][D] -> fp32 of the same shape."""
        assert q.is_contiguous() and q.dtype == torch.float16 and q.dim() == 4
        if out is None:
            out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
        assert out.is_contiguous() and out.dtype == torch.float32 and out.shape == q.shape
        _check(lib().xq_decode_attention(self._h, layer0, q.shape[0], C.c_void_p(q.data_ptr()),
                                         C.c_void_p(out.data_ptr()), float(sm_scale),
                                         C.c_void_p(self.workspace.data_ptr()), self.workspace.numel(), int(flags),
                                         _stream()), "xq_decode_attention")
        return out

    def decode_attention_static(self, q: torch.Tensor, sm_scale: float, out: torch.Tensor, layer0=0, flags=0):
        """decode_attention with the split partials in the library's static device array; `out`
        must be supplied (this call allocates nothing)."""
        assert q.is_contiguous() and q.dtype == torch.float16 and q.dim() == 4
        assert out.is_contiguous() and out.dtype == torch.float32 and out.shape == q.shape
        _check(lib().xq_decode_attention_static(self._h, layer0, q.shape[0], C.c_void_p(q.data_ptr()),
                                                C.c_void_p(out.data_ptr()), float(sm_scale), int(flags), _stream()),
               "xq_decode_attention_static")
        return out

    def unpack_codes(self, layer, is_v):
        _, tq = self.length(layer)
        c = self.cfg
        out = torch.empty((c.batch, c.n_kv_heads, tq, c.head_dim), dtype=torch.uint8, device=self.device)
        _check(lib().xq_unpack_codes(self._h, layer, int(is_v), C.c_void_p(out.data_ptr()), _stream()),
               "xq_unpack_codes")
        return out

    def code_delta_histogram(self, layer, is_v):
        """Counts of |c_layer - c_layer+1| = 0..3 over all packed elements (int64 tensor of 4)."""
        out = torch.empty(4, dtype=torch.int64, device=self.device)
        _check(lib().xq_code_delta_histogram(self._h, layer, int(is_v), C.c_void_p(out.data_ptr()), _stream()),
               "xq_code_delta_histogram")
        return out

    def set_tiles_per_split(self, n):
        lib().xq_debug_set_tiles_per_split(self._h, int(n))


def config_from_workload(w, max_tokens=None, page_tokens=0, n_pages=0) -> XqConfig:
    """XqConfig for a synth.Workload (marshalling helper)."""
    mt = max_tokens if max_tokens is not None else w.context + w.decode_steps
    return XqConfig(w.n_layers, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.group, w.residual, mt,
                    w.kq, w.vq, w.km, w.vm, w.eta1, w.eta2, w.share_group, w.share_dominant, w.merge_mode, w.gamma0,
                    page_tokens, n_pages)
