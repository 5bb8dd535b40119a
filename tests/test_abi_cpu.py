"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and its
host logic (config checks, sizes, accounting) behaves -- no GPU needed."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _gold(name):
    rows = []
    for line in open(os.path.join(ROOT, "tests", "golden", name)):
        line = line.split("#")[0].strip()
        if line:
            rows.append(line.split())
    return rows


@pytest.fixture(scope="module")
def xq():
    import paper_2510_11236_amd as xq
    xq.lib()
    return xq


def test_exports_every_declared_symbol(xq):
    hdr = open(os.path.join(ROOT, "include", "xq.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(xq_[a-z_0-9]+)\s*\(", hdr))
    assert {"xq_quantize_pack", "xq_append_token", "xq_decode_attention"} <= names
    L = xq.lib()
    for n in sorted(names):
        assert hasattr(L, n), n


def test_flag_constants_match_header(xq):
    hdr = open(os.path.join(ROOT, "include", "xq.h")).read()
    for name in ("XQ_DECODE_PAIR_FUSED", "XQ_DECODE_VECTOR_ALU", "XQ_DECODE_MATRIX_F16", "XQ_DECODE_MERGE_LAUNCH", "XQ_DECODE_MERGE_IN_LAUNCH"):
        assert int(re.search(r"#define\s+%s\s+(\d+)" % name, hdr).group(1)) == getattr(xq, name)


def _cfg(xq, **kw):
    base = dict(n_layers=32, batch=4, n_q_heads=32, n_kv_heads=32, head_dim=128, group=32, residual=128,
                max_tokens=32768 + 1, kq=32, vq=32, km=0, vm=0, eta1=1 / 6, eta2=0.045)
    base.update(kw)
    return xq.XqConfig(**base)


def test_config_validation(xq):
    assert xq.cache_bytes(_cfg(xq))[0] > 0
    for bad, code in [(dict(head_dim=96), -2), (dict(group=16), -2), (dict(residual=100), -1), (dict(eta1=0.5), -1),
                      (dict(eta2=-0.1), -1), (dict(n_q_heads=48), -1), (dict(n_q_heads=34, n_kv_heads=2), -2),
                      (dict(n_layers=0), -1), (dict(kq=31, km=0), -1), (dict(vq=1, vm=0), -1)]:
        with pytest.raises(xq.XqError) as e:
            xq.cache_bytes(_cfg(xq, **bad))
        assert e.value.code == code, bad
    # an odd boundary below the sharing start is fine: those layers do not share
    assert xq.cache_bytes(_cfg(xq, kq=31, km=32))[0] > 0
    assert xq.strerror(0) == "ok" and "capacity" in xq.strerror(-3)


def test_arena_size_matches_bit_accounting(xq):
    """cfg index 2: codes 1 bit/element (2-bit shared by pairs), metadata 1 bit/element at g=32."""
    cfg = _cfg(xq)
    arena, ws = xq.cache_bytes(cfg)
    Tq, R, D, nbh, L = 32768 - 128 + 32, 128, 128, 4 * 32, 32   # max_tokens 32769 -> one more group
    codes = 2 * (L // 2) * nbh * Tq * D * 2 // 8
    meta = 2 * L * nbh * Tq * D * 4 // 32
    res = 2 * L * nbh * R * D * 2
    assert codes + meta + res <= arena <= codes + meta + res + 8 * L * 256 + 65536
    assert ws > 0


def test_equivalent_bits_golden(xq):
    for L, kq, vq, km, vm, expect, *_ in _gold("equivalent_bits.txt"):
        cfg = _cfg(xq, n_layers=int(L), kq=int(kq), vq=int(vq), km=int(km), vm=int(vm))
        assert xq.equivalent_bits(cfg) == float(expect)


def test_true_bits_include_metadata(xq):
    # 2-bit, g = 32, all pairs shared, T = 32768: 1 (codes) + 1 (fp16 scale+zero per 32) on the
    # packed part, 16 bits on the 128 ring tokens
    cfg = _cfg(xq)
    T, r = 32768, 128
    expect = ((T - r) * (1.0 + 1.0) + r * 16.0) / T
    assert abs(xq.equivalent_bits(cfg, True, T) - expect) < 1e-12
    cfg4 = _cfg(xq, batch=8, n_kv_heads=8, group=64, vq=0)     # K 2-bit, V 1-bit, g = 64, shared
    assert xq.equivalent_bits(cfg4) == 0.75
    expect4 = ((T - r) * (0.75 + 0.5) + r * 16.0) / T
    assert abs(xq.equivalent_bits(cfg4, True, T) - expect4) < 1e-12


def test_group_and_merge_config_checks(xq):
    assert xq.cache_bytes(_cfg(xq, share_group=3, share_dominant=2))[0] > 0
    assert xq.cache_bytes(_cfg(xq, merge_mode=1, gamma0=0.8))[0] > 0
    for bad in (dict(share_group=5), dict(share_group=1), dict(share_group=3, share_dominant=3), dict(merge_mode=4),
                dict(merge_mode=1, gamma0=1.5), dict(merge_mode=2, share_group=3), dict(merge_mode=1, share_dominant=1),
                dict(share_group=4, kq=30, km=0)):      # group {28..31} would mix 2-bit and 1-bit layers
        with pytest.raises(xq.XqError):
            xq.cache_bytes(_cfg(xq, **bad))
    # all key layers and 20 value layers stored at 2 bit -> (2 + 1.25) / 2 = 1.625 for G = 2, 3, 4
    for G, vm in ((2, 8), (3, 14), (4, 16)):
        assert xq.equivalent_bits(_cfg(xq, km=32, vm=vm, share_group=G)) == 1.625


def test_paged_config_checks(xq):
    for kw, code in [(dict(page_tokens=64, n_pages=4), -1), (dict(page_tokens=192, n_pages=4), -1),
                     (dict(page_tokens=128, n_pages=0), -1), (dict(page_tokens=0, n_pages=4), -1)]:
        with pytest.raises(xq.XqError) as e:
            xq.cache_bytes(_cfg(xq, **kw))
        assert e.value.code == code, kw
    # a pool that holds exactly what the contiguous cache holds costs the same, up to the page table
    # and the rounding of each sequence to whole pages
    cfg = _cfg(xq, max_tokens=4096 + 128)              # 4096 packed tokens per sequence
    a0, _ = xq.cache_bytes(cfg)
    a1, _ = xq.cache_bytes(_cfg(xq, max_tokens=4096 + 128, page_tokens=128, n_pages=4 * 32))
    assert abs(a1 - a0) < 0.01 * a0
    # half the pool: half the packed bytes (the fp16 rings are not paged)
    a2, _ = xq.cache_bytes(_cfg(xq, max_tokens=4096 + 128, page_tokens=128, n_pages=2 * 32))
    assert a2 < 0.65 * a0


def _merge_table(xq, bits, mode, gamma0):
    lut = xq.lib().xq_debug_merge_table(C.byref(_cfg(xq, merge_mode=mode, gamma0=gamma0)), bits)
    n = 1 << bits
    return [[(lut >> (bits * (n * e0 + e1))) & (n - 1) for e1 in range(n)] for e0 in range(n)]


def test_merge_table_follows_appendix_e_intervals(xq):
    """The pack kernels' table of merged codes against the interval table of Appendix E
    (tests/golden/gamma_intervals.txt: e_m = e_1 + c for gamma_0 inside the listed interval, and the
    mirrored case with gamma_1), against the oracle's weighted average over a sweep of gamma_0, and
    floor / ceil of the plain mean."""
    from fractions import Fraction
    import numpy as np
    from oracle import xq_oracle as orc
    for delta, c, lo, hi in _gold("gamma_intervals.txt"):
        delta, c, lo, hi = int(delta), int(c), Fraction(lo), Fraction(hi)
        for frac in (Fraction(1, 64), Fraction(1, 2), Fraction(63, 64)):
            g0 = float(lo + (hi - lo) * frac)
            t, tm = _merge_table(xq, 2, 1, g0), _merge_table(xq, 2, 1, 1.0 - g0)
            for e1 in range(0, 4 - delta):
                assert t[e1 + delta][e1] == e1 + c, (delta, c, g0)
                assert tm[e1][e1 + delta] == e1 + c, (delta, c, g0)      # e_1 > e_0: gamma_1 plays gamma_0's part
    e = np.arange(4, dtype=np.uint8)
    e0, e1 = np.repeat(e, 4), np.tile(e, 4)
    for g0 in list(np.linspace(0.0, 1.0, 41)) + [0.166, 0.167, 0.8333, 0.8334, 0.2499, 0.7501]:
        g0 = float(np.float32(g0))
        ref = orc.merge_codes(e0, e1, 2, 1, g0).reshape(4, 4)
        assert np.array_equal(np.array(_merge_table(xq, 2, 1, g0)), ref), g0
        ref1 = orc.merge_codes(np.array([0, 0, 1, 1], np.uint8), np.array([0, 1, 0, 1], np.uint8), 1, 1, g0).reshape(2, 2)
        assert np.array_equal(np.array(_merge_table(xq, 1, 1, g0)), ref1), g0
    for mode, f in ((2, lambda a, b: (a + b) // 2), (3, lambda a, b: (a + b + 1) // 2)):
        assert _merge_table(xq, 2, mode, 0.5) == [[f(a, b) for b in range(4)] for a in range(4)]
    assert xq.lib().xq_debug_merge_table(C.byref(_cfg(xq, merge_mode=1, gamma0=0.5)), 3) == 0
