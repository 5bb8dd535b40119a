"""GPU parity over a seeded sample of the configuration space: head size, group size, ring
length, bit widths, sharing thresholds, layer groups, query heads per kv head, batch, prompt
length, number of appended tokens and contiguous or paged storage are drawn at random (fixed
seeds) within the documented limits; stored bytes are compared bit for bit and attention to 2e-3 against the oracle."""
import os

import numpy as np
import pytest
import torch

from paper_2510_11236_amd import synth

pytestmark = pytest.mark.gpu


def _draw(seed):
    r = np.random.default_rng(1000 + seed)
    D = int(r.choice([64, 128]))
    g = int(r.choice([32, 64]))
    R = g * int(r.integers(1, 5))
    L = int(r.integers(1, 7))
    G = int(r.choice([2, 2, 2, 3, 4]))
    k = int(r.integers(0, G))
    # thresholds on group boundaries so that every sharing group has one bit width
    def thr():
        return int(r.choice([0, L] + [G * i for i in range(1, L // G + 1)]))
    kq, vq = thr(), thr()
    km, vm = int(r.integers(0, L + 1)), int(r.integers(0, L + 1))
    merge = int(r.choice([0, 0, 0, 1, 2, 3])) if (G == 2 and k == 0) else 0
    rep = int(r.choice([1, 1, 2, 3, 4, 5, 8]))
    h_kv = int(r.integers(1, 4))
    batch = int(r.integers(1, 4))
    T0 = int(r.choice([int(r.integers(1, 2 * R + 2)), int(r.integers(1, 1200))]))
    n_app = int(r.choice([0, int(r.integers(1, g + 3)), int(r.integers(1, 3 * g))]))
    page = int(r.choice([0, 0, 128, 256, 1024]))
    spare = int(r.integers(0, 3))
    kw = dict(head_dim=D, group=g, residual=R, n_layers=L, share_group=G, share_dominant=k, kq=kq, vq=vq,
                km=km, vm=vm, merge_mode=merge, gamma0=float(r.choice([0.7, 0.3, 0.5])) if merge == 1 else (0.5 if merge else 1.0),
                n_q_heads=rep * h_kv, n_kv_heads=h_kv, batch=batch, eta1=float(r.choice([0.0, 1 / 6, 0.2])),
                eta2=float(r.choice([0.0, 0.045, 0.09])))
    return kw, T0, n_app, page, spare


def _valid(tl, kw):
    """The library's own config check decides (bit widths must agree inside a sharing group,
    merging needs whole pairs, ...); a rejected draw is skipped, not bent into shape."""
    from paper_2510_11236_amd import XqError, cache_bytes
    from paper_2510_11236_amd.binding import config_from_workload
    w = synth.scaled(synth.workloads()[1], name="random", **kw)
    try:
        cache_bytes(config_from_workload(w, max_tokens=64))
    except XqError:
        return None
    return w


# XQ_RANDOM_SEEDS=first:last widens (or moves) the sample, e.g. for a long run after a kernel change
_SEEDS = range(*[int(x) for x in os.environ.get("XQ_RANDOM_SEEDS", "0:120").split(":")])


@pytest.mark.parametrize("seed", _SEEDS)
def test_random_config(seed):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import xq_testlib as tl
    kw, T0, n_app, page, spare = _draw(seed)
    w = _valid(tl, kw)
    if w is None:
        pytest.skip(f"draw {seed} is not a valid configuration: {kw}")
    w = synth.scaled(w, seed=500 + seed)
    print(f"seed {seed}: T0={T0} appends={n_app} page={page} {kw}", flush=True)
    T = T0 + n_app
    K, V = synth.kv_all(w, T)
    Kd, Vd = K.cuda(), V.cuda()
    if page:
        # a pool just large enough (plus 0..2 pages); prefill the sequences last to first so that
        # page numbers do not follow the sequence order
        tq = 0 if T <= w.residual else w.group * ((T - w.residual + w.group - 1) // w.group)
        cache = tl.make_cache(w, max_tokens=T + 1, page_tokens=page, n_pages=max(1, w.batch * ((tq + page - 1) // page)) + spare)
        for i in reversed(range(w.batch)):
            cache.quantize_pack_seq(Kd[:, i:i + 1, :, :T0], Vd[:, i:i + 1, :, :T0], seq0=i)
    else:
        cache = tl.make_cache(w, max_tokens=T + 1)
        cache.quantize_pack(Kd[:, :, :, :T0], Vd[:, :, :, :T0])
    for t in range(T0, T):
        cache.append_token(Kd[:, :, :, t].contiguous(), Vd[:, :, :, t].contiguous())
    q = synth.queries(w).cuda()
    sigma = 1.0 / np.sqrt(w.head_dim)
    # flag 1: pairs share a workgroup; flag 2: the vector-ALU kernels instead of the matrix-instruction ones
    outs = [cache.decode_attention(q, sigma), cache.decode_attention(q, sigma, flags=1),
            cache.decode_attention(q, sigma, flags=2 + (seed // 2) % 2)]
    # flags 8 / 16: the split partials merged by a launch of its own / by the last decode workgroup to arrive
    cache.set_tiles_per_split(1 + seed % 3)
    outs.append(cache.decode_attention(q, sigma, flags=seed % 6 | (16, 8, 0)[seed % 3]))
    cache.set_tiles_per_split(4096)       # one split
    outs.append(cache.decode_attention(q, sigma, flags=(seed // 3) % 6 | (0, 16, 8)[seed % 3]))
    torch.cuda.synchronize()
    worst = 0.0
    for bi in range(w.batch):
        for h in range(w.n_kv_heads):
            st = tl.oracle_slice(w, K, V, bi, h)
            tl.check_stored(cache, w, st, bi, h)
            if st[0]["Tq"] > 0:
                tl.check_unpack(cache, w, st, bi, h)
            ref = tl.oracle_attention(w, st, q, bi, h, sigma)
            for o in outs:
                worst = max(worst, tl.check_attention(o, w, ref, bi, h))
    cache.close()
    print(f"seed {seed}: worst attention error {worst:.2e}", flush=True)
