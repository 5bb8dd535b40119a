"""Seeded synthetic KV/query generators shared by the tests, bench.py and smoke().

This module holds no arithmetic of the method (no quantization, no attention):
it only draws the inputs.  The shapes and statistics follow the five workload
descriptions this build is measured on: keys ~ N(0,1) with a few outlier
channels scaled up in layer 0, adjacent layers correlated as
x_l = 0.9 * x_{l-1} + 0.3 * N(0,1), values likewise (with or without the
outlier channels), queries ~ N(0,1); everything cast to fp16 per layer.
They stand in for the LongBench / TruthfulQA activations of 7B-13B models that
the paper measures on, which are not available offline.
"""
from dataclasses import dataclass, field
from typing import Iterator, Optional, Tuple

import torch


@dataclass
class Workload:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int            # tokens in the cache after prefill
    group: int
    residual: int
    kq: int                 # layers below kq hold 2-bit key codes, others 1-bit
    vq: int
    km: int                 # cross-layer sharing for key layers >= km
    vm: int
    eta1: float
    eta2: float
    seed: int
    decode_steps: int = 1   # tokens appended (one per sequence per step)
    outlier_scale: float = 10.0
    outlier_channels: Optional[Tuple[int, ...]] = None   # None: 4 per kv head drawn from the seed
    v_outliers: bool = False
    share_group: int = 2    # G layers share one code tensor ...
    share_dominant: int = 0  # ... stored by layer k of the group
    merge_mode: int = 0     # 0 dominant only, 1 weighted round, 2 floor, 3 ceil (pairs only)
    gamma0: float = 1.0


def workloads():
    """The five configurations (index 0 is the CPU-seconds case)."""
    return [
        Workload("cfg0_tiny_pair", 2, 1, 4, 4, 64, 512, 32, 32, 2, 2, 0, 0, 1.0 / 6.0, 0.045, 0,
                 outlier_scale=8.0, outlier_channels=(3, 17), v_outliers=True),
        Workload("cfg1_7b_4k_unshared", 32, 1, 32, 32, 128, 4096, 32, 128, 32, 32, 32, 32, 0.0, 0.0, 1),
        Workload("cfg2_7b_32k_b4_shared", 32, 4, 32, 32, 128, 32768, 32, 128, 32, 32, 0, 0, 1.0 / 6.0, 0.045, 2),
        Workload("cfg3_gqa8b_32k_b8_k2v1_g64", 32, 8, 32, 8, 128, 32768, 64, 128, 32, 0, 0, 0, 1.0 / 6.0, 0.045, 3),
        Workload("cfg4_13b_16k_b16_prefill_decode64", 40, 16, 40, 40, 128, 16384, 32, 128, 40, 40, 0, 0,
                 1.0 / 6.0, 0.045, 4, decode_steps=64),
        # not one of the five measured configurations: the schedule of the paper's main experiments
        # (configuration table: kq=30, vq=2, km=32, vm=16 -> 1.375 equivalent bits) on the 7B shape
        Workload("paper_main_schedule_7b_32k_b4", 32, 4, 32, 32, 128, 32768, 32, 128, 30, 2, 32, 16,
                 1.0 / 6.0, 0.045, 5),
        # scaling checks on the 7B shape with all pairs shared: one very long sequence; a large batch
        Workload("long_7b_256k_b1_shared", 32, 1, 32, 32, 128, 262144, 32, 128, 32, 32, 0, 0, 1.0 / 6.0, 0.045, 6),
        Workload("wide_7b_32k_b16_shared", 32, 16, 32, 32, 128, 32768, 32, 128, 32, 32, 0, 0, 1.0 / 6.0, 0.045, 7),
        # the GQA shape of cfg3 at the paper's group size 32, 2-bit keys and values, all pairs shared
        Workload("gqa8b_32k_b8_k2v2_g32_shared", 32, 8, 32, 8, 128, 32768, 32, 128, 32, 32, 0, 0, 1.0 / 6.0, 0.045, 8),
    ]


def scaled(w: Workload, **kw) -> Workload:
    """Copy of a workload with some fields replaced (reduced shapes for tests)."""
    d = dict(w.__dict__)
    d.update(kw)
    return Workload(**d)


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def outlier_mask(w: Workload, device="cpu") -> torch.Tensor:
    """[h_kv][D] multiplier applied to layer-0 keys."""
    m = torch.ones(w.n_kv_heads, w.head_dim, dtype=torch.float32)
    if w.outlier_channels is not None:
        for c in w.outlier_channels:
            m[:, c] = w.outlier_scale
    else:
        g = _gen("cpu", 7919 * (w.seed + 1))
        for h in range(w.n_kv_heads):
            idx = torch.randperm(w.head_dim, generator=g)[:4]
            m[h, idx] = w.outlier_scale
    return m.to(device)


def kv_layers(w: Workload, n_tokens: int, device="cpu",
              batch_slice: Optional[slice] = None) -> Iterator[Tuple[int, torch.Tensor, torch.Tensor]]:
    """Yield (layer, K_l, V_l), each [b][h_kv][n_tokens][D] fp16 on `device`.

    Layers come in order because each is 0.9 * previous + 0.3 * noise (in fp32,
    before the fp16 cast).  batch_slice restricts the batch range that is kept
    (the stream drawn is the same, so slices agree with the full tensor only
    when the same device and the full batch are used; tests use one or the other).
    """
    b = w.batch
    shape = (b, w.n_kv_heads, n_tokens, w.head_dim)
    gk, gv = _gen(device, 1000 + w.seed), _gen(device, 2000 + w.seed)
    mask = outlier_mask(w, device)[None, :, None, :]
    k = torch.randn(shape, generator=gk, device=device, dtype=torch.float32) * mask
    v = torch.randn(shape, generator=gv, device=device, dtype=torch.float32)
    if w.v_outliers:
        v = v * mask
    for l in range(w.n_layers):
        if l > 0:
            k = 0.9 * k + 0.3 * torch.randn(shape, generator=gk, device=device, dtype=torch.float32)
            v = 0.9 * v + 0.3 * torch.randn(shape, generator=gv, device=device, dtype=torch.float32)
        kk, vv = k.to(torch.float16), v.to(torch.float16)
        if batch_slice is not None:
            kk, vv = kk[batch_slice], vv[batch_slice]
        yield l, kk, vv


def kv_all(w: Workload, n_tokens: int, device="cpu"):
    """K, V: [L][b][h_kv][n_tokens][D] fp16 (small workloads only)."""
    ks, vs = [], []
    for _, k, v in kv_layers(w, n_tokens, device):
        ks.append(k)
        vs.append(v)
    return torch.stack(ks, 0), torch.stack(vs, 0)


def queries(w: Workload, step: int = 0, device="cpu") -> torch.Tensor:
    """[L][b][h_q][D] fp16 queries for decode step `step`."""
    g = _gen(device, 3000 + 131 * w.seed + step)
    return torch.randn((w.n_layers, w.batch, w.n_q_heads, w.head_dim), generator=g, device=device,
                       dtype=torch.float32).to(torch.float16)
