"""Parity at the full benchmark sizes, in the launch configuration bench.py times (all layers
in one call, both schedules), on sampled (layer pair, sequence, kv head) slices that the oracle
recomputes from the very fp16 tensors the library consumed."""
import numpy as np
import pytest
import torch

from paper_2510_11236_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tl():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import xq_testlib
    return xq_testlib


def _pair_schedule(tl, w):
    from oracle import xq_oracle as orc
    return orc.Schedule(2, 2 if w.kq >= 2 else 0, 2 if w.vq >= 2 else 0, 0 if w.km < w.n_layers else 2,
                        0 if w.vm < w.n_layers else 2, w.eta1, w.eta2, w.group, w.residual)


def _check_slice(tl, cache, w, pair, bi, h, K2, V2, q, outs, sigma):
    """K2, V2: numpy uint16 [2][T][D] history of the pair for slice (bi, h)."""
    from oracle import xq_oracle as orc
    sch2 = _pair_schedule(tl, w)
    st = orc.cache_slice(sch2, K2, V2)
    cfg = cache.cfg
    D, g, R = cfg.head_dim, cfg.group, cfg.residual
    bh = bi * cfg.n_kv_heads + h
    rep = w.n_q_heads // w.n_kv_heads
    worst = 0.0
    for y in (0, 1):
        l = 2 * pair + y
        T, Tq = cache.length(l)
        assert (T, Tq) == (st[y]["T"], st[y]["Tq"])
        for is_v, pre in ((False, "k"), (True, "v")):
            B = st[y]["b" + pre]
            meta = cache.region(l, pre + "_meta")[bh].cpu().numpy().view(np.uint32)
            exp_meta = st[y][pre + "_scale"].astype(np.uint32).reshape(-1) | (st[y][pre + "_zero"].astype(np.uint32).reshape(-1) << 16)
            assert np.array_equal(meta[:exp_meta.size], exp_meta), (l, pre, "meta")
            if st[y][pre + "_codes"] is not None:
                words = cache.region(l, pre + "_codes")[bh].cpu().numpy().view(np.uint32)[:Tq * D * B // 32]
                exp = (orc.pack_v_words if is_v else orc.pack_k_words)(st[y][pre + "_codes"], B)
                assert np.array_equal(words, exp), (l, pre, "codes")
            else:
                assert cache.region(l, pre + "_codes") is None
            ring = cache.region(l, pre + "_res")[bh].cpu().numpy().view(np.uint16).reshape(R, D)
            for i in range(T - Tq):
                assert np.array_equal(ring[(Tq + i) % R], st[y][pre + "_res"][i]), (l, pre, "ring", i)
        ql = q[l, bi, h * rep:(h + 1) * rep].cpu().numpy().view(np.uint16)
        ref = orc.decode_slice(sch2, st, y, ql, sigma)
        for o in outs:
            got = o[l, bi, h * rep:(h + 1) * rep].cpu().numpy()
            assert np.all(np.isfinite(got))
            err = float(np.max(np.abs(got - ref)))
            worst = max(worst, err)
            assert err <= tl.ATOL, (l, bi, h, err)
    return worst


def _run_full(tl, w, n_append, check_steps, sample_pairs, sample_bh):
    dev = "cuda:0"
    T0 = w.context
    cache = tl.make_cache(w, max_tokens=T0 + n_append)
    sigma = 1.0 / float(np.sqrt(w.head_dim))
    Ttot = T0 + n_append
    new_k = torch.empty((n_append, w.n_layers, w.batch, w.n_kv_heads, w.head_dim), dtype=torch.float16, device=dev)
    new_v = torch.empty_like(new_k)
    hist = {}   # (pair, bi, h) -> ([K_l0, K_l1], [V_l0, V_l1]) numpy uint16 [Ttot][D]
    pend = []
    for l, K, V in synth.kv_layers(w, Ttot, dev):
        new_k[:, l] = K[:, :, T0:].permute(2, 0, 1, 3)
        new_v[:, l] = V[:, :, T0:].permute(2, 0, 1, 3)
        pend.append((K, V))
        if l // 2 in sample_pairs:
            for (bi, h) in sample_bh:
                ks, vs = hist.setdefault((l // 2, bi, h), ([], []))
                ks.append(K[bi, h].cpu().numpy().view(np.uint16))
                vs.append(V[bi, h].cpu().numpy().view(np.uint16))
        if len(pend) == 2:
            Kp = torch.stack([p[0][:, :, :T0] for p in pend], 0)
            Vp = torch.stack([p[1][:, :, :T0] for p in pend], 0)
            cache.quantize_pack(Kp, Vp, layer0=l - 1)
            del Kp, Vp
            pend = []
    del K, V, pend
    torch.cuda.empty_cache()
    worst = 0.0
    for step in range(1, n_append + 1):
        cache.append_token(new_k[step - 1], new_v[step - 1])
        if step in check_steps:
            q = synth.queries(w, step, dev)
            outs = [cache.decode_attention(q, sigma), cache.decode_attention(q, sigma, flags=1)]
            torch.cuda.synchronize()
            T = T0 + step
            for (pair, bi, h), (ks, vs) in hist.items():
                K2 = np.stack([k[:T] for k in ks])
                V2 = np.stack([v[:T] for v in vs])
                worst = max(worst, _check_slice(tl, cache, w, pair, bi, h, K2, V2, q, outs, sigma))
                print(f"  {w.name} step {step} pair {pair} slice ({bi},{h}) ok", flush=True)
    cache.close()
    return worst


def _run_full_mixed(tl, w, sample_layers, sample_bh):
    """Like _run_full but with the oracle run on whole sampled slices (all layers of a slice are
    needed because the schedule differs per layer)."""
    from oracle import xq_oracle as orc
    dev = "cuda:0"
    T0 = w.context
    cache = tl.make_cache(w, max_tokens=T0 + 1)
    sigma = 1.0 / float(np.sqrt(w.head_dim))
    new_k = torch.empty((w.n_layers, w.batch, w.n_kv_heads, w.head_dim), dtype=torch.float16, device=dev)
    new_v = torch.empty_like(new_k)
    layers = sorted({l for pr in sample_layers for l in pr})
    hist = {bh: {} for bh in sample_bh}
    pend = []
    for l, K, V in synth.kv_layers(w, T0 + 1, dev):
        new_k[l] = K[:, :, T0]
        new_v[l] = V[:, :, T0]
        pend.append((K, V))
        if l in layers:
            for (bi, h) in sample_bh:
                hist[(bi, h)][l] = (K[bi, h].cpu().numpy().view(np.uint16), V[bi, h].cpu().numpy().view(np.uint16))
        if len(pend) == 2:
            cache.quantize_pack(torch.stack([p[0][:, :, :T0] for p in pend], 0),
                                torch.stack([p[1][:, :, :T0] for p in pend], 0), layer0=l - 1)
            pend = []
    del K, V, pend
    torch.cuda.empty_cache()
    cache.append_token(new_k, new_v)
    q = synth.queries(w, 1, dev)
    outs = [cache.decode_attention(q, sigma), cache.decode_attention(q, sigma, flags=1)]
    torch.cuda.synchronize()
    sch = tl.schedule_of(w)
    rep = w.n_q_heads // w.n_kv_heads
    worst = 0.0
    for (bi, h), per_layer in hist.items():
        bh = bi * w.n_kv_heads + h
        for (l0, l1) in sample_layers:
            # a two-layer oracle model with the pair's own widths and sharing
            sch2 = orc.Schedule(2, 2 if sch.bits(l0, False) == 2 else 0, 2 if sch.bits(l0, True) == 2 else 0,
                                2 if sch.stores(l1, False) else 0, 2 if sch.stores(l1, True) else 0,
                                w.eta1, w.eta2, w.group, w.residual)
            assert sch.bits(l0, False) == sch.bits(l1, False) and sch.bits(l0, True) == sch.bits(l1, True)
            K2 = np.stack([per_layer[l0][0], per_layer[l1][0]])
            V2 = np.stack([per_layer[l0][1], per_layer[l1][1]])
            st = orc.cache_slice(sch2, K2, V2)
            for y, l in enumerate((l0, l1)):
                T, Tq = cache.length(l)
                for is_v, pre in ((False, "k"), (True, "v")):
                    B = st[y]["b" + pre]
                    meta = cache.region(l, pre + "_meta")[bh].cpu().numpy().view(np.uint32)
                    exp_meta = st[y][pre + "_scale"].astype(np.uint32).reshape(-1) | (st[y][pre + "_zero"].astype(np.uint32).reshape(-1) << 16)
                    assert np.array_equal(meta[:exp_meta.size], exp_meta), (l, pre)
                    if st[y][pre + "_codes"] is not None:
                        words = cache.region(l, pre + "_codes")[bh].cpu().numpy().view(np.uint32)[:Tq * w.head_dim * B // 32]
                        exp = (orc.pack_v_words if is_v else orc.pack_k_words)(st[y][pre + "_codes"], B)
                        assert np.array_equal(words, exp), (l, pre)
                    else:
                        assert cache.region(l, pre + "_codes") is None
                ref = orc.decode_slice(sch2, st, y, q[l, bi, h * rep:(h + 1) * rep].cpu().numpy().view(np.uint16), sigma)
                for o in outs:
                    err = float(np.max(np.abs(o[l, bi, h * rep:(h + 1) * rep].cpu().numpy() - ref)))
                    worst = max(worst, err)
                    assert err <= tl.ATOL, (l, bi, h, err)
            print(f"  {w.name} layers {l0},{l1} slice ({bi},{h}) ok", flush=True)
    cache.close()
    return worst


def test_cfg2_full_size(tl):
    w = synth.workloads()[2]
    worst = _run_full(tl, w, n_append=1, check_steps={1}, sample_pairs={0, 15},
                      sample_bh=[(0, 0), (3, 31), (1, 17)])
    print("cfg2 full size worst attention error", worst)


def test_cfg3_full_size_gqa(tl):
    w = synth.workloads()[3]
    worst = _run_full(tl, w, n_append=1, check_steps={1}, sample_pairs={0, 15},
                      sample_bh=[(0, 0), (7, 7), (4, 3)])
    print("cfg3 full size worst attention error", worst)


def test_gqa_group32_full_size(tl):
    """The GQA shape at the paper's group size 32 with 2-bit keys and values (four query heads per
    kv head in one workgroup, four key groups per tile)."""
    w = synth.workloads()[8]
    worst = _run_full(tl, w, n_append=1, check_steps={1}, sample_pairs={0, 15},
                      sample_bh=[(0, 0), (7, 7), (3, 5)])
    print("GQA g=32 full size worst attention error", worst)


def test_cfg1_full_size_unshared(tl):
    w = synth.workloads()[1]
    worst = _run_full(tl, w, n_append=1, check_steps={1}, sample_pairs={0, 7, 15},
                      sample_bh=[(0, 0), (0, 31), (0, 13)])
    print("cfg1 full size worst attention error", worst)


def test_cfg4_prefill_pack_then_64_decode_steps(tl):
    """13B shape: pack the 16k prompt, then 64 append+decode steps; the ring flushes at steps
    1 and 33.  Checked on sampled slices right at and after the flush steps and at the end."""
    w = synth.workloads()[4]
    worst = _run_full(tl, w, n_append=64, check_steps={1, 2, 33, 64}, sample_pairs={0, 19},
                      sample_bh=[(0, 0), (15, 39)])
    print("cfg4 full size worst attention error", worst)


def test_paper_main_schedule_full_size(tl):
    """kq=30, vq=2, km=32, vm=16 (the paper's main configuration, 1.375 equivalent bits): keys
    never shared, values 1-bit and shared from layer 16 on; mixed bit widths inside one call, and
    a fused-schedule request that must fall back to one layer per workgroup (values-only sharing)."""
    w = synth.workloads()[5]

    worst = _run_full_mixed(tl, w, sample_layers=[(0, 1), (14, 15), (16, 17), (30, 31)], sample_bh=[(0, 0), (3, 31)])
    print("paper main schedule worst attention error", worst)


def test_llama_row_schedule(tl):
    """kq=28, vq=0, km=32, vm=28 (the Llama2-7b row of the paper's configuration table, 1.40625
    equivalent bits) at that model's 8192-token limit, and the Mistral GQA shape (32 query heads
    over 8 kv heads) with the main schedule kq=30, vq=2, km=32, vm=16 at its 30000-token limit."""
    base = synth.workloads()[5]
    w = synth.scaled(base, name="llama_row_8k_b4", context=8192, kq=28, vq=0, km=32, vm=28, seed=28)
    worst = _run_full_mixed(tl, w, sample_layers=[(0, 1), (26, 27), (28, 29), (30, 31)], sample_bh=[(1, 5), (3, 30)])
    w = synth.scaled(base, name="mistral_gqa_30k_b4", context=30000, n_kv_heads=8, seed=30)
    worst = max(worst, _run_full_mixed(tl, w, sample_layers=[(0, 1), (16, 17), (30, 31)], sample_bh=[(0, 7), (2, 3)]))
    print("configuration-table schedules worst attention error", worst)


def test_long_context_256k(tl):
    """One sequence of 262 221 tokens (ragged last tile, ring not full): the longest single
    sequence the split plan sees here (2048 tiles over 64 splits); offsets inside a slice pass
    2^25 bytes and the per-layer regions 2^28."""
    base = synth.workloads()[2]
    w = synth.scaled(base, name="long_256k", n_layers=2, batch=1, n_q_heads=8, n_kv_heads=8, context=262144 + 77 - 3,
                     seed=77)
    worst = _run_full(tl, w, n_append=3, check_steps={3}, sample_pairs={0}, sample_bh=[(0, 0), (0, 7)])
    print("256k context worst attention error", worst)
