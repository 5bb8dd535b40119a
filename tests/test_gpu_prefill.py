"""xq_prefill_attention_pack: the prompt's causal attention with the quantize + pack of its K/V in
the same kernel.  Stored bytes must equal the oracle's (and therefore xq_quantize_pack's) bit for bit;
the attention outputs are compared with the oracle's causal attention on the fp16 K/V.

Tolerance of the attention output: max-abs 2e-3 for values of order one (scaled like the decode
bar, see xq_testlib.value_atol): the softmax weights enter the second matrix product as fp16
(relative error 2^-11 each), scores and sums are fp32."""
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


def _queries(w, T, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(7000 + seed)
    return torch.randn((w.n_layers, w.batch, w.n_q_heads, T, w.head_dim), generator=g).to(torch.float16)


def _check_rows(tl, out, w, Q, K, V, sigma, rows, slices):
    from oracle import xq_oracle as orc
    rep = w.n_q_heads // w.n_kv_heads
    worst = 0.0
    for (l, bi, hq) in slices:
        h = hq // rep
        ref = orc.prefill_attention(tl.np16(Q[l, bi, hq]), tl.np16(K[l, bi, h]), tl.np16(V[l, bi, h]), sigma, rows=rows)
        got = out[l, bi, hq].cpu().numpy()[list(rows)]
        assert np.all(np.isfinite(got))
        err = float(np.max(np.abs(got - ref)))
        worst = max(worst, err)
        assert err <= tl.ATOL, (l, bi, hq, err)
    return worst


@pytest.mark.parametrize("g,rep,kq,vq,km,T", [(32, 1, 4, 4, 0, 700), (64, 4, 4, 0, 0, 1000), (32, 2, 2, 2, 4, 333),
                                               (64, 1, 0, 4, 2, 129), (32, 4, 4, 4, 0, 64), (32, 1, 4, 4, 0, 1)])
def test_prefill_attention_pack_small(tl, g, rep, kq, vq, km, T):
    """Every output row and every stored byte on small prompts: ragged lengths around the 64-token
    tiles and 128-query blocks, both group sizes, GQA, 1- and 2-bit layers, shared and unshared."""
    w = synth.scaled(synth.workloads()[1], n_layers=4, batch=2, n_q_heads=2 * rep, n_kv_heads=2, group=g,
                     kq=kq, vq=vq, km=km, vm=km, eta1=1 / 6, eta2=0.045, seed=80 + g + rep)
    K1, V1 = synth.kv_all(w, T + 1)        # the prompt and one more token for the append below
    K, V = K1[:, :, :, :T].contiguous(), V1[:, :, :, :T].contiguous()
    Q = _queries(w, T, w.seed)
    sigma = 1.0 / float(np.sqrt(w.head_dim))
    cache = tl.make_cache(w, max_tokens=T + 2)
    out = cache.prefill_attention_pack(Q.cuda(), K.cuda(), V.cuda(), sigma)
    out_only = tl.make_cache(w, max_tokens=T + 2)
    out2 = out_only.prefill_attention_pack(Q.cuda(), K.cuda(), V.cuda(), sigma, pack=False)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)                      # the pack does not touch the attention
    assert out_only.length(0) == (0, 0)
    slices = [(l, bi, hq) for l in (0, 3) for bi in range(w.batch) for hq in range(w.n_q_heads)]
    worst = _check_rows(tl, out, w, Q, K, V, sigma, range(T), slices)
    for bi in range(w.batch):
        for h in range(w.n_kv_heads):
            st = tl.oracle_slice(w, K, V, bi, h)
            tl.check_stored(cache, w, st, bi, h)
    # the cache is in the state xq_quantize_pack leaves: append + decode work on it
    cache.append_token(K1[:, :, :, T].contiguous().cuda(), V1[:, :, :, T].contiguous().cuda())
    q = synth.queries(w).cuda()
    dec = cache.decode_attention(q, sigma)
    st = tl.oracle_slice(w, K1, V1, 0, 0)
    tl.check_attention(dec, w, tl.oracle_attention(w, st, q, 0, 0, sigma), 0, 0)
    print(f"prefill g={g} rep={rep} T={T}: worst attention error {worst:.2e}")
    cache.close()
    out_only.close()


def test_prefill_attention_pack_paged_and_errors(tl):
    from paper_2510_11236_amd import XqError
    w = synth.scaled(synth.workloads()[2], n_layers=2, batch=2, n_q_heads=2, n_kv_heads=2, seed=85)
    T = 600
    K, V = synth.kv_all(w, T)
    Q = _queries(w, T, 85)
    sigma = 0.09
    cache = tl.make_cache(w, max_tokens=T + 2, page_tokens=128, n_pages=12)
    out = cache.prefill_attention_pack(Q.cuda(), K.cuda(), V.cuda(), sigma)
    for bi in range(2):
        for h in range(2):
            tl.check_stored(cache, w, tl.oracle_slice(w, K, V, bi, h), bi, h)
    _check_rows(tl, out, w, Q, K, V, sigma, [0, 63, 64, 127, 128, 599], [(1, 1, 1)])
    with pytest.raises(XqError) as e:        # the layers are no longer empty
        cache.prefill_attention_pack(Q.cuda(), K.cuda(), V.cuda(), sigma)
    assert e.value.code == -4
    with pytest.raises(XqError) as e:        # the scale must be positive
        cache.prefill_attention_pack(Q.cuda(), K.cuda(), V.cuda(), -sigma, pack=False)
    assert e.value.code == -1
    cache.close()
    w64 = synth.scaled(synth.workloads()[0], n_layers=2)
    c64 = tl.make_cache(w64, max_tokens=64)
    q64 = torch.zeros((2, 1, 4, 40, 64), dtype=torch.float16, device="cuda")
    k64 = torch.zeros((2, 1, 4, 40, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(XqError) as e:        # head_dim 64 is not built
        c64.prefill_attention_pack(q64, k64, k64, 0.1)
    assert e.value.code == -2
    c64.close()


def test_prefill_attention_pack_full_size_and_saving(tl):
    """The cfg2 shape (batch 4, 32 heads, 32768 tokens), one layer pair: sampled output rows and
    stored slices against the oracle, and the measured saving of the fused pass over attention
    followed by xq_quantize_pack."""
    w = synth.scaled(synth.workloads()[2], n_layers=2, seed=86)
    T = w.context
    dev = "cuda:0"
    Ks, Vs = [], []
    for l, K, V in synth.kv_layers(w, T, dev):
        Ks.append(K)
        Vs.append(V)
    Kd, Vd = torch.stack(Ks), torch.stack(Vs)
    del Ks, Vs, K, V
    g = torch.Generator(device=dev)
    g.manual_seed(7086)
    Q = torch.randn((2, w.batch, w.n_q_heads, T, 128), generator=g, device=dev, dtype=torch.float32).to(torch.float16)
    sigma = 1.0 / float(np.sqrt(128))
    out = torch.empty(Q.shape, dtype=torch.float32, device=dev)

    def timed(fn):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    fused = tl.make_cache(w, max_tokens=T + 2)
    split = tl.make_cache(w, max_tokens=T + 2)
    out_split = torch.empty_like(out)
    fused.prefill_attention_pack(Q, Kd, Vd, sigma, out=out)          # warm-up (clocks, code load)
    tf, ta, tp = [], [], []
    for r in range(4):                                   # the two routes in turn, in alternating order; medians
        fused.reset()
        split.reset()

        def run_fused():
            tf.append(timed(lambda: fused.prefill_attention_pack(Q, Kd, Vd, sigma, out=out)))

        def run_split():
            ta.append(timed(lambda: split.prefill_attention_pack(Q, Kd, Vd, sigma, out=out_split, pack=False)))
            tp.append(timed(lambda: split.quantize_pack(Kd, Vd)))

        for f in ((run_fused, run_split) if r % 2 == 0 else (run_split, run_fused)):
            f()
    med = lambda x: float(np.median(x))
    t_fused, t_attn, t_pack = med(tf), med(ta), med(tp)
    print("fused runs " + ", ".join(f"{x:.1f}" for x in tf) + "; attention-only runs " + ", ".join(f"{x:.1f}" for x in ta))
    assert torch.equal(out, out_split)
    Tq = fused.length(0)[1]
    used = {"k_codes": Tq * 128 * 2 // 8, "v_codes": Tq * 128 * 2 // 8, "k_meta": Tq // w.group * 128 * 4,
            "v_meta": Tq * (128 // w.group) * 4}
    for name, n in used.items():
        for l in range(2):
            a, b = fused.region(l, name), split.region(l, name)
            if a is not None:
                assert torch.equal(a[:, :n], b[:, :n]), (name, l)     # the two routes store the same bytes
    saving = (t_attn + t_pack - t_fused) / (t_attn + t_pack)
    flops = 2 * w.batch * w.n_q_heads * (T * (T + 1) / 2) * 128 * 2 * 2
    print(f"prefill cfg2 shape, one layer pair: fused {t_fused:.1f} ms; attention alone {t_attn:.1f} ms + pack {t_pack:.2f} ms; "
          f"saving {100 * saving:.2f} %; attention at {flops / (t_attn * 1e-3) / 1e12:.0f} TFLOP/s")
    rng = np.random.default_rng(86)
    rows = sorted({0, 1, 63, 64, 127, 128, T - 1, T - 129} | set(rng.integers(0, T, size=24).tolist()))
    slices = [(0, 0, 0), (1, w.batch - 1, w.n_q_heads - 1)] + [(int(rng.integers(2)), int(rng.integers(w.batch)), int(rng.integers(w.n_q_heads))) for _ in range(6)]
    Kc, Vc, Qc = Kd.cpu(), Vd.cpu(), None
    worst = 0.0
    from oracle import xq_oracle as orc
    for (l, bi, hq) in slices:
        ref = orc.prefill_attention(tl.np16(Q[l, bi, hq]), tl.np16(Kc[l, bi, hq]), tl.np16(Vc[l, bi, hq]), sigma, rows=rows)
        got = out[l, bi, hq].cpu().numpy()[rows]
        err = float(np.max(np.abs(got - ref)))
        worst = max(worst, err)
        assert err <= tl.ATOL, (l, bi, hq, err)
    for (bi, h) in [(0, 0), (3, 31), (1, 17), (2, 5)]:
        tl.check_stored(fused, w, tl.oracle_slice(w, Kc, Vc, bi, h), bi, h)
    print(f"prefill cfg2 shape: {len(slices)} slices x {len(rows)} rows ok, worst attention error {worst:.2e}")
    fused.close()
    split.close()
