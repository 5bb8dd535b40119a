"""Helpers shared by the GPU parity tests: run the oracle on slices and compare the
library's stored bytes and attention outputs with it."""
import numpy as np
import torch

from oracle import xq_oracle as orc
from paper_2510_11236_amd import synth
from paper_2510_11236_amd.binding import XqCache, config_from_workload

ATOL = 2e-3   # max-abs tolerance on attention outputs (fp32 accumulation), the stated bar


V_REF = 8.0   # the benchmark's dequantized values stay below this; ATOL is quoted for them


def value_atol(w, state, layers=None):
    """The tolerance for a slice: ATOL * max(1, max |V^| / V_REF) over its dequantized values.
    Every error term of the output is linear in the values (scaling V by a power of two scales
    the kernels' outputs and their errors exactly), so an absolute bar is only meaningful at a
    stated magnitude: ATOL holds for |V^| < V_REF, which covers the benchmark's inputs, and grows
    in proportion beyond.  (The dominant term: the value weights p * s^ travel as fp16, relative
    error 2^-11 each, at worst 2^-11 times the largest group range when all weight sits on one
    token, far less when the softmax averages many.)"""
    sch = schedule_of(w)
    big = 0.0
    for l in (layers if layers is not None else range(w.n_layers)):
        big = max(big, float(np.max(np.abs(orc.dequant_slice(sch, state, l)[1]))))
    return ATOL * max(1.0, big / V_REF)


def schedule_of(w):
    return orc.Schedule(w.n_layers, w.kq, w.vq, w.km, w.vm, w.eta1, w.eta2, w.group, w.residual,
                        w.share_group, w.share_dominant, w.merge_mode, w.gamma0)


def np16(t):
    return t.detach().cpu().contiguous().numpy().view(np.uint16)


def oracle_slice(w, K, V, bi, h):
    """K, V: torch fp16 [L][b][h][T][D] (cpu or gpu) -> oracle state for slice (bi, h)."""
    return orc.cache_slice(schedule_of(w), np16(K[:, bi, h]), np16(V[:, bi, h]))


def check_stored(cache: XqCache, w, state, bi, h, layers=None):
    """Bit-exact comparison of everything the library stored for slice (bi, h)."""
    cfg = cache.cfg
    D, g, R = cfg.head_dim, cfg.group, cfg.residual
    bh = bi * cfg.n_kv_heads + h
    sch = schedule_of(w)
    for l in (layers if layers is not None else range(cfg.n_layers)):
        st = state[l]
        T, Tq = cache.length(l)
        assert (T, Tq) == (st["T"], st["Tq"]), (l, T, Tq, st["T"], st["Tq"])
        for is_v, pre in ((False, "k"), (True, "v")):
            B = st["b" + pre]
            meta = cache.slice_bytes(l, pre + "_meta", bh).cpu().numpy().view(np.uint32)
            n_meta = (Tq // g) * D if not is_v else Tq * (D // g)
            exp_meta = st[pre + "_scale"].astype(np.uint32).reshape(-1) | (st[pre + "_zero"].astype(np.uint32).reshape(-1) << 16)
            assert np.array_equal(meta[:n_meta], exp_meta), f"layer {l} {pre} metadata differs"
            reg = cache.region(l, pre + "_codes")
            if sch.stores(l, is_v):
                assert reg is not None
                words = cache.slice_bytes(l, pre + "_codes", bh).cpu().numpy().view(np.uint32)[:Tq * D * B // 32]
                exp = (orc.pack_v_words if is_v else orc.pack_k_words)(st[pre + "_codes"], B)
                assert np.array_equal(words, exp), f"layer {l} {pre} packed words differ"
            else:
                assert reg is None and st[pre + "_codes"] is None
            ring = cache.region(l, pre + "_res")[bh].cpu().numpy().view(np.uint16).reshape(R, D)
            for i in range(T - Tq):
                assert np.array_equal(ring[(Tq + i) % R], st[pre + "_res"][i]), f"layer {l} {pre} ring token {Tq + i}"


def check_unpack(cache: XqCache, w, state, bi, h):
    sch = schedule_of(w)
    for l in range(cache.cfg.n_layers):
        for is_v, pre in ((False, "k"), (True, "v")):
            if sch.stores(l, is_v) and state[l]["Tq"] > 0:
                got = cache.unpack_codes(l, is_v)[bi, h].cpu().numpy()
                assert np.array_equal(got, state[l][pre + "_codes"]), (l, pre)


def oracle_attention(w, state, q, bi, h, sigma, layers=None):
    """q: torch fp16 [L][b][h_q][D] -> dict layer -> [n_rep][D] float32 for kv head h."""
    rep = w.n_q_heads // w.n_kv_heads
    sch = schedule_of(w)
    out = {}
    for l in (layers if layers is not None else range(w.n_layers)):
        ql = np16(q[l, bi, h * rep:(h + 1) * rep])
        out[l] = orc.decode_slice(sch, state, l, ql, sigma)
    return out


def check_attention(out, w, ref, bi, h, atol=ATOL):
    rep = w.n_q_heads // w.n_kv_heads
    worst = 0.0
    for l, r in ref.items():
        got = out[l, bi, h * rep:(h + 1) * rep].cpu().numpy()
        assert np.all(np.isfinite(got)), f"layer {l} non-finite output"
        err = float(np.max(np.abs(got - r)))
        worst = max(worst, err)
        if err > atol:
            bad = np.argwhere(np.abs(got - r) > atol)
            raise AssertionError(f"layer {l} slice ({bi},{h}): max abs err {err:.3e} > {atol}; {len(bad)} of "
                                 f"{got.size} outputs off, first (head, channel): {bad[:8].tolist()}, "
                                 f"got {got[tuple(bad[0])]:.5f} want {r[tuple(bad[0])]:.5f}")
    return worst


def make_cache(w, max_tokens=None, device="cuda:0", page_tokens=0, n_pages=0):
    return XqCache(config_from_workload(w, max_tokens, page_tokens, n_pages), device)
