"""GPU parity, one small case per built instantiation of the decode kernel: head size, group size,
key and value bit width, query heads per kv head, and the three ways a layer is served (own codes,
a sharing pair with one layer per workgroup, a sharing pair in one workgroup), in both kernel
families.  Attention is compared with the oracle to 2e-3."""
import numpy as np
import pytest
import torch

from paper_2510_11236_amd import synth

pytestmark = pytest.mark.gpu

CASES = [(128, g, bk, bv, rep) for g in (32, 64) for bk in (1, 2) for bv in (1, 2) for rep in (1, 2, 4)] + \
        [(64, g, bk, bv, 1) for g in (32, 64) for bk in (1, 2) for bv in (1, 2)]


@pytest.mark.parametrize("D,g,bk,bv,rep", CASES)
def test_every_instantiation(D, g, bk, bv, rep):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import xq_testlib as tl
    L, T = 2, 300
    sigma = 1.0 / np.sqrt(D)
    for shared in (False, True):
        w = synth.scaled(synth.workloads()[1 if D == 128 else 0], n_layers=L, batch=1, n_q_heads=rep, n_kv_heads=1,
                         group=g, residual=64, kq=L if bk == 2 else 0, vq=L if bv == 2 else 0,
                         km=0 if shared else L, vm=0 if shared else L, eta1=1 / 6, eta2=0.045, seed=40 + bk + 2 * bv)
        K, V = synth.kv_all(w, T)
        cache = tl.make_cache(w, max_tokens=T)
        cache.quantize_pack(K.cuda(), V.cuda())
        q = synth.queries(w).cuda()
        # flag 1: the pair in one workgroup (where the shape allows); flag 2: vector-ALU kernels
        outs = [cache.decode_attention(q, sigma, flags=f) for f in (0, 1, 2, 3, 4, 5)]
        torch.cuda.synchronize()
        st = tl.oracle_slice(w, K, V, 0, 0)
        tl.check_stored(cache, w, st, 0, 0)
        ref = tl.oracle_attention(w, st, q, 0, 0, sigma)
        for o in outs:
            tl.check_attention(o, w, ref, 0, 0)
        cache.close()
