"""ctypes front end of the CPU oracle (oracle/xq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  Nothing here imports the product package and the
product never imports this module.

The arithmetic lives in the C file; this module only marshals numpy arrays and
strings the per-layer steps together in the order the paper gives them
(Appendix Alg. 1: quantize or pseudo-quantize each layer, then dequantize each
layer with the codes of the layer that stores them).
"""
import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

_LIB = None


def lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        u16p, u8p, u32p = C.POINTER(C.c_uint16), C.POINTER(C.c_uint8), C.POINTER(C.c_uint32)
        f64p, f32p = C.POINTER(C.c_double), C.POINTER(C.c_float)
        L.xqo_half_to_float.restype = C.c_float
        L.xqo_half_to_float.argtypes = [C.c_uint16]
        L.xqo_float_to_half.restype = C.c_uint16
        L.xqo_float_to_half.argtypes = [C.c_float]
        L.xqo_quantized_len.restype = C.c_int
        L.xqo_quantized_len.argtypes = [C.c_int] * 3
        L.xqo_quantize_group.restype = None
        L.xqo_quantize_group.argtypes = [u16p, C.c_long, C.c_int, C.c_int, C.c_float, u8p, C.c_long, u16p, u16p]
        for f in (L.xqo_quantize_k, L.xqo_quantize_v):
            f.restype = C.c_int
            f.argtypes = [u16p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float, C.c_int, u8p, u16p, u16p]
        for f in (L.xqo_dequant_k, L.xqo_dequant_v):
            f.restype = None
            f.argtypes = [u8p, u16p, u16p, C.c_int, C.c_int, C.c_int, f64p]
        L.xqo_half_rows_to_double.restype = None
        L.xqo_half_rows_to_double.argtypes = [u16p, C.c_long, f64p]
        L.xqo_attention.restype = None
        L.xqo_attention.argtypes = [u16p, f64p, f64p, C.c_int, C.c_int, C.c_double, f32p]
        L.xqo_prefill_attention_row.restype = None
        L.xqo_prefill_attention_row.argtypes = [u16p, u16p, u16p, C.c_int, C.c_int, C.c_double, f32p]
        for f in (L.xqo_pack_k_words, L.xqo_pack_v_words):
            f.restype = None
            f.argtypes = [u8p, C.c_int, C.c_int, C.c_int, u32p]
        L.xqo_merge_codes.restype = None
        L.xqo_merge_codes.argtypes = [u8p, u8p, C.c_long, C.c_int, C.c_int, C.c_float, u8p]
        L.xqo_equivalent_bits.restype = C.c_double
        L.xqo_equivalent_bits.argtypes = [C.c_int] * 5
        L.xqo_equivalent_bits_one.restype = C.c_double
        L.xqo_equivalent_bits_one.argtypes = [C.c_int] * 3
        _LIB = L
    return _LIB


def _p(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


# ------------------------------------------------------------------ scalars
def half_to_float(bits: int) -> float:
    return float(lib().xqo_half_to_float(int(bits)))


def float_to_half(x: float) -> int:
    return int(lib().xqo_float_to_half(float(np.float32(x))))


def quantized_len(T: int, g: int, R: int) -> int:
    return int(lib().xqo_quantized_len(T, g, R))


def equivalent_bits(L, kq, vq, km, vm) -> float:
    return float(lib().xqo_equivalent_bits(L, kq, vq, km, vm))


def equivalent_bits_one(L, q, m) -> float:
    return float(lib().xqo_equivalent_bits_one(L, q, m))


# ------------------------------------------------------------------- groups
def quantize_group(x, B, eta, store_codes=True):
    """One group of fp16 values -> (codes u8 | None, s_hat bits, z_hat bits)."""
    x = _u16(x).reshape(-1)
    g = x.shape[0]
    codes = np.zeros(g, np.uint8) if store_codes else None
    s, z = C.c_uint16(0), C.c_uint16(0)
    lib().xqo_quantize_group(_p(x, C.c_uint16), 1, g, B, float(np.float32(eta)),
                             _p(codes, C.c_uint8) if store_codes else None, 1, C.byref(s), C.byref(z))
    return codes, int(s.value), int(z.value)


def _quantize(fn, x, g, R, B, eta, store_codes, k_layout):
    x = _u16(x)
    T, D = x.shape
    Tq = quantized_len(T, g, R)
    codes = np.zeros((Tq, D), np.uint8) if store_codes else None
    mshape = (Tq // g, D) if k_layout else (Tq, D // g)
    scale = np.zeros(mshape, np.uint16)
    zero = np.zeros(mshape, np.uint16)
    got = fn(_p(x, C.c_uint16), T, D, g, R, B, float(np.float32(eta)), int(bool(store_codes)),
             _p(codes, C.c_uint8) if store_codes else None, _p(scale, C.c_uint16), _p(zero, C.c_uint16))
    assert got == Tq
    return codes, scale, zero


def quantize_k(k, g, R, B, eta, store_codes=True):
    """k: [T][D] fp16 -> (codes [Tq][D] | None, scale [Tq/g][D], zero [Tq/g][D]) (fp16 bits)."""
    return _quantize(lib().xqo_quantize_k, k, g, R, B, eta, store_codes, True)


def quantize_v(v, g, R, B, eta, store_codes=True):
    """v: [T][D] fp16 -> (codes [Tq][D] | None, scale [Tq][D/g], zero [Tq][D/g])."""
    return _quantize(lib().xqo_quantize_v, v, g, R, B, eta, store_codes, False)


def _dequant(fn, codes, scale, zero, g):
    codes = np.ascontiguousarray(codes, np.uint8)
    Tq, D = codes.shape
    out = np.zeros((Tq, D), np.float64)
    if Tq:
        fn(_p(codes, C.c_uint8), _p(_u16(scale), C.c_uint16), _p(_u16(zero), C.c_uint16), Tq, D, g,
           _p(out, C.c_double))
    return out


def dequant_k(codes, scale, zero, g):
    return _dequant(lib().xqo_dequant_k, codes, scale, zero, g)


def dequant_v(codes, scale, zero, g):
    return _dequant(lib().xqo_dequant_v, codes, scale, zero, g)


def half_rows_to_double(x):
    x = _u16(x)
    out = np.zeros(x.shape, np.float64)
    if x.size:
        lib().xqo_half_rows_to_double(_p(x, C.c_uint16), x.size, _p(out, C.c_double))
    return out


def attention(q, Kh, Vh, sigma):
    """q: [D] fp16; Kh, Vh: [T][D] float64 -> [D] float32."""
    q = _u16(q).reshape(-1)
    Kh = np.ascontiguousarray(Kh, np.float64)
    Vh = np.ascontiguousarray(Vh, np.float64)
    T, D = Kh.shape
    out = np.zeros(D, np.float32)
    lib().xqo_attention(_p(q, C.c_uint16), _p(Kh, C.c_double), _p(Vh, C.c_double), T, D, float(sigma),
                        _p(out, C.c_float))
    return out


def prefill_attention(q, K, V, sigma, rows=None):
    """Causal attention of a prompt on its own fp16 K/V: q, K, V [T][D] fp16; query t sees keys
    0..t.  rows: the query positions to compute (default all) -> [len(rows)][D] float32."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    T, D = K.shape
    rows = range(T) if rows is None else rows
    out = np.zeros((len(rows), D), np.float32)
    for i, t in enumerate(rows):
        lib().xqo_prefill_attention_row(_p(q[t], C.c_uint16), _p(K, C.c_uint16), _p(V, C.c_uint16), int(t), D,
                                        float(sigma), _p(out[i], C.c_float))
    return out


def pack_k_words(codes, B):
    codes = np.ascontiguousarray(codes, np.uint8)
    Tq, D = codes.shape
    words = np.zeros(Tq * D * B // 32, np.uint32)
    if Tq:
        lib().xqo_pack_k_words(_p(codes, C.c_uint8), Tq, D, B, _p(words, C.c_uint32))
    return words


def pack_v_words(codes, B):
    codes = np.ascontiguousarray(codes, np.uint8)
    Tq, D = codes.shape
    words = np.zeros(Tq * D * B // 32, np.uint32)
    if Tq:
        lib().xqo_pack_v_words(_p(codes, C.c_uint8), Tq, D, B, _p(words, C.c_uint32))
    return words


def merge_codes(e0, e1, B, mode, gamma0):
    e0 = np.ascontiguousarray(e0, np.uint8)
    e1 = np.ascontiguousarray(e1, np.uint8)
    out = np.zeros(e0.shape, np.uint8)
    if e0.size:
        lib().xqo_merge_codes(_p(e0, C.c_uint8), _p(e1, C.c_uint8), e0.size, B, mode, float(np.float32(gamma0)),
                              _p(out, C.c_uint8))
    return out


# ------------------------------------------------ per-layer schedule (Alg. 1)
@dataclass
class Schedule:
    """kq/vq: layers below hold 2-bit codes, the others 1-bit.  km/vm: from this
    layer on, the second (odd) layer of each pair reuses the codes of the layer
    below it and keeps only its own calibrated scale and zero-point."""
    n_layers: int
    kq: int
    vq: int
    km: int
    vm: int
    eta1: float
    eta2: float
    group: int
    residual: int
    # ablation variants (Sec. 4.3): G consecutive layers share the codes of layer k of the
    # group; merge_mode 1/2/3 forms a pair's stored codes from both layers (Appendix E)
    share_group: int = 2
    share_dominant: int = 0
    merge_mode: int = 0
    gamma0: float = 1.0

    def bits(self, l, is_v):
        return 2 if l < (self.vq if is_v else self.kq) else 1

    def eta(self, B):
        return self.eta2 if B == 2 else self.eta1

    def code_layer(self, l, is_v):
        if l < (self.vm if is_v else self.km):
            return l
        cl = self.share_group * (l // self.share_group) + self.share_dominant
        return cl if cl < self.n_layers else l

    def stores(self, l, is_v):
        return self.code_layer(l, is_v) == l

    def merges_next(self, l, is_v):
        return (self.merge_mode != 0 and l + 1 < self.n_layers and self.stores(l, is_v)
                and self.code_layer(l + 1, is_v) == l)


def cache_slice(sch: Schedule, K, V):
    """Quantization phase for one (batch, kv-head) slice.

    K, V: [L][T][D] fp16 -- the complete history of the slice.  An append is, by
    definition, this function on the history one token longer.
    Returns a list over layers of dicts with the stored items: codes (None for a
    subordinate layer), scale/zero as fp16 bits, and the fp16 residual rows.
    """
    K, V = _u16(K), _u16(V)
    L, T, D = K.shape
    g, R = sch.group, sch.residual
    Tq = quantized_len(T, g, R)
    out = []
    for l in range(L):
        bk, bv = sch.bits(l, False), sch.bits(l, True)
        kc, ks, kz = quantize_k(K[l], g, R, bk, sch.eta(bk), sch.stores(l, False))
        vc, vs, vz = quantize_v(V[l], g, R, bv, sch.eta(bv), sch.stores(l, True))
        # merged pair: the stored codes combine this layer's own codes with the next layer's own
        if sch.merges_next(l, False):
            k1 = quantize_k(K[l + 1], g, R, bk, sch.eta(bk), True)[0]
            kc = merge_codes(kc, k1, bk, sch.merge_mode, sch.gamma0)
        if sch.merges_next(l, True):
            v1 = quantize_v(V[l + 1], g, R, bv, sch.eta(bv), True)[0]
            vc = merge_codes(vc, v1, bv, sch.merge_mode, sch.gamma0)
        out.append(dict(Tq=Tq, T=T, bk=bk, bv=bv, k_codes=kc, k_scale=ks, k_zero=kz,
                        v_codes=vc, v_scale=vs, v_zero=vz,
                        k_res=K[l, Tq:].copy(), v_res=V[l, Tq:].copy()))
    return out


def dequant_slice(sch: Schedule, state, l):
    """Dequantization phase for layer l: codes from the layer that stores them,
    scale and zero-point from layer l itself, residual rows as they are."""
    g = sch.group
    st = state[l]
    kc = state[sch.code_layer(l, False)]["k_codes"]
    vc = state[sch.code_layer(l, True)]["v_codes"]
    Kh = np.concatenate([dequant_k(kc, st["k_scale"], st["k_zero"], g), half_rows_to_double(st["k_res"])], 0)
    Vh = np.concatenate([dequant_v(vc, st["v_scale"], st["v_zero"], g), half_rows_to_double(st["v_res"])], 0)
    return Kh, Vh


def decode_slice(sch: Schedule, state, l, q, sigma):
    """q: [n_rep][D] fp16 (the query heads that map to this kv head) -> [n_rep][D] f32."""
    Kh, Vh = dequant_slice(sch, state, l)
    q = _u16(q)
    return np.stack([attention(q[i], Kh, Vh, sigma) for i in range(q.shape[0])], 0)
