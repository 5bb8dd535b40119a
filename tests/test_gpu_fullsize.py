"""Parity at the full benchmark sizes, in the launch configuration bench.py times (all layers
in one call, both schedules), on a seeded sample of at least 64 (layer pair, sequence, kv head)
slices per configuration -- every slice when there are fewer -- that the oracle recomputes, on a
pool of host threads, from the very fp16 tensors the library consumed.  The sample always holds
the first and last pair, sequence and kv head."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from paper_2510_11236_amd import synth

pytestmark = pytest.mark.gpu

N_SAMPLE = 64
N_THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module")
def tl():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import xq_testlib
    return xq_testlib


def _sample_slices(w, n=N_SAMPLE, n_pairs=6):
    """Seeded sample of n distinct (pair, sequence, kv head) triples over n_pairs layer pairs
    (first, last and seeded middle ones); the corners of the index space are always in it."""
    rng = np.random.default_rng(9000 + w.seed)
    P = w.n_layers // 2
    pairs = sorted({0, P - 1} | set(rng.choice(P, size=min(n_pairs, P), replace=False).tolist()))
    lb, lh = w.batch - 1, w.n_kv_heads - 1
    picked = {(0, 0, 0), (P - 1, lb, lh), (0, lb, 0), (P - 1, 0, lh), (0, 0, lh), (P - 1, lb, 0)}
    space = [(p, bi, h) for p in pairs for bi in range(w.batch) for h in range(w.n_kv_heads)]
    for i in rng.permutation(len(space)):
        if len(picked) >= min(n, len(space)):
            break
        picked.add(space[i])
    return sorted(picked)


def _pair_schedule(tl, w):
    from oracle import xq_oracle as orc
    return orc.Schedule(2, 2 if w.kq >= 2 else 0, 2 if w.vq >= 2 else 0, 0 if w.km < w.n_layers else 2,
                        0 if w.vm < w.n_layers else 2, w.eta1, w.eta2, w.group, w.residual)


def _oracle_pair(sch2, K2, V2, q2, sigma):
    """Host-thread job: the oracle's stored items and attention outputs of one pair slice.
    K2, V2: uint16 [2][T][D]; q2: uint16 [2][rep][D]."""
    from oracle import xq_oracle as orc
    st = orc.cache_slice(sch2, K2, V2)
    exp = []
    for y in (0, 1):
        e = {"T": st[y]["T"], "Tq": st[y]["Tq"]}
        for is_v, pre in ((False, "k"), (True, "v")):
            e[pre + "_meta"] = (st[y][pre + "_scale"].astype(np.uint32).reshape(-1) |
                                (st[y][pre + "_zero"].astype(np.uint32).reshape(-1) << 16))
            c = st[y][pre + "_codes"]
            e[pre + "_words"] = None if c is None else (orc.pack_v_words if is_v else orc.pack_k_words)(c, st[y]["b" + pre])
            e[pre + "_res"] = st[y][pre + "_res"]
        e["ref"] = orc.decode_slice(sch2, st, y, q2[y], sigma)
        exp.append(e)
    return exp


def _compare_pair(tl, cache, w, layers, bi, h, exp, outs):
    """Main-thread half of a slice check: stored bytes bit for bit, attention to the stated bar."""
    cfg = cache.cfg
    D, R = cfg.head_dim, cfg.residual
    bh = bi * cfg.n_kv_heads + h
    rep = w.n_q_heads // w.n_kv_heads
    worst = 0.0
    for y, l in enumerate(layers):
        e = exp[y]
        T, Tq = cache.length(l, bi)
        assert (T, Tq) == (e["T"], e["Tq"])
        for pre in ("k", "v"):
            meta = cache.region(l, pre + "_meta")[bh].cpu().numpy().view(np.uint32)
            assert np.array_equal(meta[:e[pre + "_meta"].size], e[pre + "_meta"]), (l, bi, h, pre, "meta")
            if e[pre + "_words"] is not None:
                words = cache.region(l, pre + "_codes")[bh].cpu().numpy().view(np.uint32)[:e[pre + "_words"].size]
                assert np.array_equal(words, e[pre + "_words"]), (l, bi, h, pre, "codes")
            else:
                assert cache.layout(l)[pre + "_codes"][0] < 0
            ring = cache.region(l, pre + "_res")[bh].cpu().numpy().view(np.uint16).reshape(R, D)
            idx = (Tq + np.arange(T - Tq)) % R
            assert np.array_equal(ring[idx], e[pre + "_res"]), (l, bi, h, pre, "ring")
        for o in outs:
            got = o[l, bi, h * rep:(h + 1) * rep].cpu().numpy()
            assert np.all(np.isfinite(got))
            err = float(np.max(np.abs(got - e["ref"])))
            worst = max(worst, err)
            assert err <= tl.ATOL, (l, bi, h, err)
    return worst


def _check_sample(tl, cache, w, jobs, q, outs, sigma, what):
    """jobs: list of ((l0, l1), bi, h, sch2, K2, V2).  Oracle on the thread pool, comparison here."""
    rep = w.n_q_heads // w.n_kv_heads
    q_host = q.cpu().numpy().view(np.uint16)

    def work(j):
        (l0, l1), bi, h, sch2, K2, V2 = j
        q2 = np.stack([q_host[l0, bi, h * rep:(h + 1) * rep], q_host[l1, bi, h * rep:(h + 1) * rep]])
        return _oracle_pair(sch2, K2, V2, q2, sigma)

    worst = 0.0
    with ThreadPoolExecutor(max_workers=N_THREADS) as ex:
        for j, exp in zip(jobs, ex.map(work, jobs)):
            worst = max(worst, _compare_pair(tl, cache, w, j[0], j[1], j[2], exp, outs))
    print(f"  {what}: {len(jobs)} (pair, sequence, kv head) slices x 2 layers x {len(outs)} schedules ok, "
          f"worst attention error {worst:.2e}", flush=True)
    return worst


def _run_full(tl, w, n_append, check_steps, sample=None):
    dev = "cuda:0"
    T0 = w.context
    sample = _sample_slices(w) if sample is None else sample
    by_pair = {}
    for (p, bi, h) in sample:
        by_pair.setdefault(p, []).append((bi, h))
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
        for (bi, h) in by_pair.get(l // 2, ()):
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
    sch2 = _pair_schedule(tl, w)
    worst = 0.0
    for step in range(1, n_append + 1):
        cache.append_token(new_k[step - 1], new_v[step - 1])
        if step in check_steps:
            q = synth.queries(w, step, dev)
            outs = [cache.decode_attention(q, sigma), cache.decode_attention(q, sigma, flags=1)]
            torch.cuda.synchronize()
            T = T0 + step
            jobs = [((2 * p, 2 * p + 1), bi, h, sch2, np.stack([k[:T] for k in ks]), np.stack([v[:T] for v in vs]))
                    for (p, bi, h), (ks, vs) in sorted(hist.items())]
            worst = max(worst, _check_sample(tl, cache, w, jobs, q, outs, sigma, f"{w.name} step {step} (T = {T})"))
    cache.close()
    return worst, len(hist)


def _run_full_mixed(tl, w, sample_layers, n_bh=None):
    """Like _run_full for schedules that differ per layer: the sampled layer pairs are given (one
    per kind of layer the schedule has), each checked on n_bh seeded (sequence, kv head) slices
    with a two-layer oracle model of the pair's own widths and sharing."""
    from oracle import xq_oracle as orc
    dev = "cuda:0"
    T0 = w.context
    nbh = w.batch * w.n_kv_heads
    n_bh = n_bh or -(-N_SAMPLE // len(sample_layers))
    rng = np.random.default_rng(9100 + w.seed)
    by_layer = {}
    for (l0, l1) in sample_layers:
        picks = {0, nbh - 1}
        for x in rng.permutation(nbh).tolist():
            if len(picks) >= min(n_bh, nbh):
                break
            picks.add(x)
        for l in (l0, l1):
            by_layer[l] = sorted(divmod(x, w.n_kv_heads) for x in picks)
    cache = tl.make_cache(w, max_tokens=T0 + 1)
    sigma = 1.0 / float(np.sqrt(w.head_dim))
    new_k = torch.empty((w.n_layers, w.batch, w.n_kv_heads, w.head_dim), dtype=torch.float16, device=dev)
    new_v = torch.empty_like(new_k)
    hist = {}
    pend = []
    for l, K, V in synth.kv_layers(w, T0 + 1, dev):
        new_k[l] = K[:, :, T0]
        new_v[l] = V[:, :, T0]
        pend.append((K, V))
        for (bi, h) in by_layer.get(l, ()):
            hist[(l, bi, h)] = (K[bi, h].cpu().numpy().view(np.uint16), V[bi, h].cpu().numpy().view(np.uint16))
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
    jobs = []
    for (l0, l1) in sample_layers:
        # a two-layer oracle model with the pair's own widths and sharing
        sch2 = orc.Schedule(2, 2 if sch.bits(l0, False) == 2 else 0, 2 if sch.bits(l0, True) == 2 else 0,
                            2 if sch.stores(l1, False) else 0, 2 if sch.stores(l1, True) else 0,
                            w.eta1, w.eta2, w.group, w.residual)
        assert sch.bits(l0, False) == sch.bits(l1, False) and sch.bits(l0, True) == sch.bits(l1, True)
        for (bi, h) in by_layer[l0]:
            jobs.append(((l0, l1), bi, h, sch2, np.stack([hist[(l0, bi, h)][0], hist[(l1, bi, h)][0]]),
                         np.stack([hist[(l0, bi, h)][1], hist[(l1, bi, h)][1]])))
    worst = _check_sample(tl, cache, w, jobs, q, outs, sigma, f"{w.name} (T = {T0 + 1})")
    cache.close()
    return worst, len(jobs)


def test_cfg2_full_size(tl):
    w = synth.workloads()[2]
    worst, n = _run_full(tl, w, n_append=1, check_steps={1})
    assert n >= N_SAMPLE
    print("cfg2 full size worst attention error", worst)


def test_cfg3_full_size_gqa(tl):
    w = synth.workloads()[3]
    worst, n = _run_full(tl, w, n_append=1, check_steps={1})
    assert n >= N_SAMPLE
    print("cfg3 full size worst attention error", worst)


def test_gqa_group32_full_size(tl):
    """The GQA shape at the paper's group size 32 with 2-bit keys and values (four query heads per
    kv head in one workgroup, four key groups per tile)."""
    w = synth.workloads()[8]
    worst, n = _run_full(tl, w, n_append=1, check_steps={1})
    assert n >= N_SAMPLE
    print("GQA g=32 full size worst attention error", worst)


def test_cfg1_full_size_unshared(tl):
    w = synth.workloads()[1]
    worst, n = _run_full(tl, w, n_append=1, check_steps={1})
    assert n >= N_SAMPLE
    print("cfg1 full size worst attention error", worst)


def test_cfg4_prefill_pack_then_64_decode_steps(tl):
    """13B shape: pack the 16k prompt, then 64 append+decode steps; the ring flushes at steps
    1 and 33.  Checked on the sampled slices at each flush step, the step after it, and the end."""
    w = synth.workloads()[4]
    worst, n = _run_full(tl, w, n_append=64, check_steps={1, 2, 33, 34, 64})
    assert n >= N_SAMPLE
    print("cfg4 full size worst attention error", worst)


def test_paper_main_schedule_full_size(tl):
    """kq=30, vq=2, km=32, vm=16 (the paper's main configuration, 1.375 equivalent bits): keys
    never shared, values 1-bit and shared from layer 16 on; mixed bit widths inside one call, and
    a fused-schedule request that must fall back to one layer per workgroup (values-only sharing)."""
    w = synth.workloads()[5]
    worst, n = _run_full_mixed(tl, w, sample_layers=[(0, 1), (14, 15), (16, 17), (30, 31)])
    assert n >= N_SAMPLE
    print("paper main schedule worst attention error", worst)


def test_llama_row_schedule(tl):
    """kq=28, vq=0, km=32, vm=28 (the Llama2-7b row of the paper's configuration table, 1.40625
    equivalent bits) at that model's 8192-token limit, and the Mistral GQA shape (32 query heads
    over 8 kv heads) with the main schedule kq=30, vq=2, km=32, vm=16 at its 30000-token limit."""
    base = synth.workloads()[5]
    w = synth.scaled(base, name="llama_row_8k_b4", context=8192, kq=28, vq=0, km=32, vm=28, seed=28)
    worst, n = _run_full_mixed(tl, w, sample_layers=[(0, 1), (26, 27), (28, 29), (30, 31)])
    assert n >= N_SAMPLE
    w = synth.scaled(base, name="mistral_gqa_30k_b4", context=30000, n_kv_heads=8, seed=30)
    worst2, n = _run_full_mixed(tl, w, sample_layers=[(0, 1), (16, 17), (30, 31)])
    assert n >= N_SAMPLE
    print("configuration-table schedules worst attention error", max(worst, worst2))


def test_long_context_256k(tl):
    """One sequence of 262 221 tokens (ragged last tile, ring not full): the longest single
    sequence the split plan sees here (2048 tiles over 64 splits); offsets inside a slice pass
    2^25 bytes and the per-layer regions 2^28.  All 8 slices of the one pair are checked."""
    base = synth.workloads()[2]
    w = synth.scaled(base, name="long_256k", n_layers=2, batch=1, n_q_heads=8, n_kv_heads=8, context=262144 + 77 - 3,
                     seed=77)
    worst, n = _run_full(tl, w, n_append=3, check_steps={3}, sample=[(0, 0, h) for h in range(8)])
    assert n == 8
    print("256k context worst attention error", worst)
