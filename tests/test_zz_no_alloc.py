"""xq_decode_attention_static (split partials in the library's static device array, for callers
that cannot allocate) against xq_decode_attention on the same cache: same kernels, same plan, so
the outputs must be equal bit for bit (which is inside the 2e-3 parity bar).  Two calls in a row
on one GPU, the second on a smaller input, so that the array still holds the first call's
partials when the second runs."""
import numpy as np
import pytest
import torch

from paper_2510_11236_amd import synth
from paper_2510_11236_amd.binding import XqError

pytestmark = pytest.mark.gpu


def _case(tl, w, T):
    K, V = synth.kv_all(w, T)
    cache = tl.make_cache(w, max_tokens=T + 1)
    cache.quantize_pack(K.cuda(), V.cuda())
    return cache, synth.queries(w).cuda(), K, V


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import xq_testlib as tl
    base = synth.workloads()[2]
    # first: 4 layers (two sharing pairs), GQA 2:1, 2900 tokens -> several splits per slice
    w_big = synth.scaled(base, n_layers=4, batch=2, n_q_heads=8, n_kv_heads=4, seed=71)
    # second, smaller in every respect: 2 layers, 1 sequence, 700 tokens, fewer splits
    w_small = synth.scaled(base, n_layers=2, batch=1, n_q_heads=2, n_kv_heads=2, seed=72)
    big = _case(tl, w_big, 2900)
    small = _case(tl, w_small, 700)
    sigma = 1.0 / float(np.sqrt(base.head_dim))
    for flags in (0, 1, 2, 3):
        want, got = [], []
        for cache, q, _, _ in (big, small):
            want.append(cache.decode_attention(q, sigma, flags=flags))
        torch.cuda.synchronize()
        # the two static calls back to back, nothing in between
        for cache, q, _, _ in (big, small):
            got.append(cache.decode_attention_static(q, sigma, torch.full(q.shape, float("nan"), dtype=torch.float32,
                                                                          device=q.device), flags=flags))
        torch.cuda.synchronize()
        for name, a, b in zip(("first (large)", "second (small)"), want, got):
            assert torch.isfinite(b).all(), (name, flags)
            assert torch.equal(a, b), f"{name} call, flags {flags}: max abs diff {(a - b).abs().max().item():.3e}"
    # and the small result is the oracle's, within the stated bar
    cache, q, K, V = small
    out = cache.decode_attention_static(q, sigma, torch.empty(q.shape, dtype=torch.float32, device=q.device), flags=1)
    torch.cuda.synchronize()
    for h in range(w_small.n_kv_heads):
        st = tl.oracle_slice(w_small, K, V, 0, h)
        tl.check_attention(out, w_small, tl.oracle_attention(w_small, st, q, 0, h, sigma), 0, h)
    # one layer at a time (the per-layer calling mode) through the same array
    cache, q, _, _ = big
    ref = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    out = torch.empty_like(ref)
    for l in range(w_big.n_layers):     # (a one-layer call plans its own splits: compare like with like)
        cache.decode_attention(q[l:l + 1], sigma, out=ref[l:l + 1], layer0=l)
    for l in range(w_big.n_layers):
        cache.decode_attention_static(q[l:l + 1], sigma, out[l:l + 1], layer0=l)
    torch.cuda.synchronize()
    assert torch.equal(ref, out)
    big[0].close()
    small[0].close()


def test_static_scratch_rejects_oversized_call():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import xq_testlib as tl
    # 16 layers x 8 x 32 heads, 4096 packed tokens forced to one tile per split: 33 partials of
    # 520 bytes for each of 4096 heads = 70.3 MB > the 64 MiB array
    w = synth.scaled(synth.workloads()[1], n_layers=16, batch=8, seed=73)
    T = 4096 + 128
    cache = tl.make_cache(w, max_tokens=T)
    z = torch.zeros((1, 1, 1, T, w.head_dim), dtype=torch.float16, device="cuda:0")
    z = z.expand(w.n_layers, w.batch, w.n_kv_heads, T, w.head_dim)
    cache.quantize_pack(z, z)
    q = synth.queries(w).cuda()
    out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    cache.set_tiles_per_split(1)
    with pytest.raises(XqError) as e:
        cache.decode_attention_static(q, 0.1, out)
    assert e.value.code == -3
    cache.set_tiles_per_split(0)           # the automatic plan fits
    cache.decode_attention_static(q, 0.1, out)
    ref = cache.decode_attention(q, 0.1)
    torch.cuda.synchronize()
    assert torch.equal(ref, out)
    cache.close()
