#!/usr/bin/env python3
"""Benchmark of the quantized-KV decode hot path on one MI355X.

A step = one decode step of the whole hot path for every layer: append one new token per
sequence (with the ring flush when it falls due) and decode attention of one query per head
over the packed cache + fp16 ring.  Inputs are synthetic, seeded, resident in HBM before the
timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2] [--schedule auto|sequential|fused]
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
HBM_TARGET_FRAC = 0.70            # the stated target on the 32k-context configurations
FAMILY_FLAGS = {"matrix": 0, "matrix_f16": 4, "vector_alu": 2}


def kernel_sources_hash():
    """sha256 over the library's kernel sources: counter figures stored in profiles/traffic.json are
    only attached to a run whose kernels are the ones they were measured on."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2510_11236_amd", "csrc")
    for name in sorted(os.listdir(d)):
        h.update(name.encode())
        h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def algorithmic_bytes(w, T, fused):
    """HBM bytes one decode-attention pass over all layers must read: every packed code and
    its fp16 scale/zero once per layer that uses it (once per pair when fused), the fp16 ring,
    queries; plus the fp32 outputs written.  Split partials are workspace, not counted."""
    g, R, D = w.group, w.residual, w.head_dim
    over = T - R
    Tq = 0 if over <= 0 else g * ((over + g - 1) // g)
    r = T - Tq
    nbh = w.batch * w.n_kv_heads
    total = 0
    for l in range(w.n_layers):
        bk = 2 if l < w.kq else 1
        bv = 2 if l < w.vq else 1
        k_shared = not (l < w.km or l % 2 == 0)
        v_shared = not (l < w.vm or l % 2 == 0)
        k_codes = Tq * D * bk // 8
        v_codes = Tq * D * bv // 8
        if fused and k_shared and v_shared:   # the library fuses a pair only when it shares both code sets
            k_codes = v_codes = 0
        meta = Tq * D * 4 // g * 2
        ring = r * D * 2 * 2
        total += nbh * (k_codes + v_codes + meta + ring)
        total += w.batch * w.n_q_heads * D * (2 + 4)
    return total


def cpu_baseline(w, slices, q_cpu, sigma, T):
    """Oracle decode (dequantize + attention) timed on host threads over a bounded sample."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import xq_oracle as orc
    sch = orc.Schedule(w.n_layers, w.kq, w.vq, w.km, w.vm, w.eta1, w.eta2, w.group, w.residual)
    rep = w.n_q_heads // w.n_kv_heads
    jobs = []
    # a pair on its own is a 2-layer model with the pair's schedule
    sch2 = orc.Schedule(2, 2 if w.kq > 0 else 0, 2 if w.vq > 0 else 0, 0 if w.km < w.n_layers else 2,
                        0 if w.vm < w.n_layers else 2, w.eta1, w.eta2, w.group, w.residual)
    keys = list(slices)
    threads = min(2 * len(keys), os.cpu_count() or 1, 16)
    orc.lib()
    tp = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:       # quantization phase (the pack leg)
        states = list(ex.map(lambda k: orc.cache_slice(sch2, slices[k][0], slices[k][1]), keys))
    pack_s = time.perf_counter() - tp
    pack_bytes = sum(slices[k][0].nbytes + slices[k][1].nbytes for k in keys)
    for (bi, h), st in zip(keys, states):
        for l in (0, 1):
            jobs.append((sch2, st, l, q_cpu[l, bi, h * rep:(h + 1) * rep].numpy().view(np.uint16)))

    def run(j):
        return orc.decode_slice(j[0], j[1], j[2], j[3], sigma)

    run(jobs[0])
    t1 = time.perf_counter()
    for j in jobs[:4]:
        run(j)
    one_core = 4 / (time.perf_counter() - t1)        # slice-layers per second on one thread
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(run, jobs))
    dt = time.perf_counter() - t0
    slice_layers_per_s = len(jobs) / dt
    t_step = w.n_layers * w.batch * w.n_kv_heads / slice_layers_per_s
    return {"value": w.batch * T / t_step, "unit": "KV tokens/s", "cores": threads, "kind": "oracle",
            "pack_GBps_fp16_read": pack_bytes / pack_s / 1e9,
            "one_core_value": w.batch * T / (w.n_layers * w.batch * w.n_kv_heads / one_core),
            "sample": f"{len(jobs)} (layer, sequence, kv-head) slices of the first layer pair at T={T}, "
                      f"dequantize+attention in fp64, {dt:.1f} s wall, scaled linearly to all "
                      f"{w.n_layers * w.batch * w.n_kv_heads} slices"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=2)
    ap.add_argument("--schedule", default="auto", choices=["auto", "sequential", "fused", "per_layer"],
                    help="auto: times sequential and pair-fused and takes the faster (all layers in one call); per_layer: the "
                         "timed step makes one decode call per layer, as a decoder must (for profiles of that mode)")
    ap.add_argument("--page-tokens", type=int, default=0,
                    help="keep the packed tokens in pool pages of this many tokens (0: one region per sequence)")
    ap.add_argument("--family", default="matrix", choices=sorted(FAMILY_FLAGS),
                    help="decode kernels of the timed steps: matrix (default: 4x4x4 fp16 matrix instruction, 2-bit keys "
                         "of GQA shapes on the 16x16x128 fp8 x fp4 one), matrix_f16 (everything on the 4x4x4 fp16 one), "
                         "vector_alu (no matrix instructions)")
    ap.add_argument("--vector-alu", action="store_true", help="same as --family vector_alu")
    ap.add_argument("--print-kernel-hash", action="store_true", help="print the hash of the kernel sources and exit")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-slices", type=int, default=96)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.print_kernel_hash:
        print(kernel_sources_hash())
        return
    if args.vector_alu:
        args.family = "vector_alu"
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (every (sequence, kv head) slice is independent, "
              "so more GPUs would each take a share of the heads with no exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(2)

    if args.calibrate_copy:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda:0")     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "calibrate_copy_bytes_written": src.numel() * 4}))
        return

    from paper_2510_11236_amd import synth
    from paper_2510_11236_amd.binding import XqCache, config_from_workload, equivalent_bits

    w = synth.workloads()[args.workload]
    if w.head_dim != 128:
        args.family = "vector_alu"          # the only kernels at head_dim 64
    dev = "cuda:0"
    torch.cuda.set_device(0)
    n_extra = args.warmup + args.steps
    T0 = w.context
    if args.page_tokens:
        P = args.page_tokens
        tq_max = w.group * ((T0 + n_extra + 1 - w.residual + w.group - 1) // w.group)
        per_seq = (tq_max + P - 1) // P
        cfg = config_from_workload(w, max_tokens=T0 + n_extra + 1, page_tokens=P, n_pages=w.batch * per_seq)
        cache = XqCache(cfg, dev)
        # hand the pages out in a scrambled order: fill the pool through layer 0 sequence by sequence,
        # release the sequences in another order (the pool is a stack), then prefill for real
        dummy = torch.zeros((1, 1, w.n_kv_heads, T0 + n_extra, w.head_dim), dtype=torch.float16, device=dev)
        for i in range(w.batch):
            cache.quantize_pack_seq(dummy, dummy, seq0=i)
        for i in sorted(range(w.batch), key=lambda i: (i * 7 + 3) % w.batch):
            cache.reset_seq(i)
        del dummy
    else:
        cfg = config_from_workload(w, max_tokens=T0 + n_extra + 1)
        cache = XqCache(cfg, dev)
    sigma = 1.0 / float(np.sqrt(w.head_dim))

    # ---- synthetic KV, packed layer pair by layer pair (also the pack measurement)
    Ttot = T0 + n_extra
    new_k = torch.empty((n_extra, w.n_layers, w.batch, w.n_kv_heads, w.head_dim), dtype=torch.float16, device=dev)
    new_v = torch.empty_like(new_k)
    # distinct (sequence, kv head) slices for the oracle baseline, spread over the batch and the heads
    nbh = w.batch * w.n_kv_heads
    stride = next(s for s in (37, 41, 43, 47, 53, 1) if np.gcd(s, nbh) == 1)
    sample = [divmod((3 + stride * i) % nbh, w.n_kv_heads) for i in range(min(args.cpu_slices, nbh))]
    slices = {}
    pack_ms, pack_bytes, pack_written = 0.0, 0, 0
    pend = []
    for l, K, V in synth.kv_layers(w, Ttot, dev):
        new_k[:, l] = K[:, :, T0:].permute(2, 0, 1, 3)
        new_v[:, l] = V[:, :, T0:].permute(2, 0, 1, 3)
        pend.append((K, V))
        if l < 2 and not args.no_cpu_baseline:
            for (bi, h) in sample:
                kk, vv = K[bi, h, :T0].cpu().numpy().view(np.uint16), V[bi, h, :T0].cpu().numpy().view(np.uint16)
                if l == 0:
                    slices[(bi, h)] = ([kk], [vv])
                else:
                    slices[(bi, h)][0].append(kk)
                    slices[(bi, h)][1].append(vv)
        if len(pend) == 2 or l == w.n_layers - 1:
            Kp = torch.stack([p[0][:, :, :T0] for p in pend], 0)
            Vp = torch.stack([p[1][:, :, :T0] for p in pend], 0)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            cache.quantize_pack(Kp, Vp, layer0=l + 1 - len(pend))
            e1.record()
            torch.cuda.synchronize()
            pack_ms += e0.elapsed_time(e1)
            pack_bytes += Kp.numel() * 2 * 2
            for ll in range(l + 1 - len(pend), l + 1):     # bytes the pack writes: codes (storing layers) + metadata
                for is_v in (False, True):
                    bits = 2 if ll < (w.vq if is_v else w.kq) else 1
                    stores = ll < (w.vm if is_v else w.km) or ll % 2 == 0
                    tq = 0 if T0 <= w.residual else w.group * ((T0 - w.residual + w.group - 1) // w.group)
                    elems = w.batch * w.n_kv_heads * tq * w.head_dim
                    pack_written += elems * (bits if stores else 0) // 8 + elems * 4 // w.group
            del Kp, Vp
            pend = []
    del K, V
    torch.cuda.empty_cache()
    slices = {k: (np.stack(v[0]), np.stack(v[1])) for k, v in slices.items()}

    # ---- choose the schedule
    qs = [synth.queries(w, step, dev) for step in range(4)]
    out = torch.empty(qs[0].shape, dtype=torch.float32, device=dev)

    def time_decode(flags, n=5):
        for i in range(12):     # the clock settles over the first launches after a change of load
            cache.decode_attention(qs[i % 4], sigma, out=out, flags=flags)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            cache.decode_attention(qs[i % 4], sigma, out=out, flags=flags)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    # --schedule auto times both schedules (untimed probes) and takes the faster; an explicit
    # schedule runs no probes, so that a profile of the run holds only warmup + timed launches
    alu = FAMILY_FLAGS[args.family]
    # a pair shares a workgroup only when some odd layer shares both code sets and the kernel's weight
    # tables hold two layers of every query-head part (4, 2, 1) of a kv head: 2 * part * 128 / g <= 16
    rep = w.n_q_heads // w.n_kv_heads
    parts = [4] * (rep // 4) + [2] * (rep % 4 // 2) + [1] * (rep % 2) if w.head_dim == 128 else [1]
    can_fuse = (any(l % 2 == 1 and l >= w.km and l >= w.vm for l in range(w.n_layers)) and
                all(2 * p * (128 // w.group) <= 16 for p in parts))
    probe = {}
    if args.schedule == "auto":
        probe["sequential"] = time_decode(alu, 20)
        if can_fuse:
            probe["fused"] = time_decode(1 | alu, 20)
        # the pair-fused schedule has to win by 2 % to be taken (for GQA pairs the two are on a par)
        schedule = "fused" if probe.get("fused", float("inf")) < 0.98 * probe["sequential"] else "sequential"
    else:
        schedule = args.schedule if (args.schedule != "fused" or can_fuse) else "sequential"
    per_layer_steps = schedule == "per_layer"
    flags = (1 if schedule == "fused" else 0) | alu
    # counter figures of earlier rocprofv3 runs, only if they were taken on these very kernel sources
    prof = {}
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file) and not args.page_tokens:
        try:
            prof = json.load(open(traffic_file))
            if prof.get("_kernel_sources_hash") != kernel_sources_hash():
                prof = {}
        except Exception:
            prof = {}
    fam_key = "" if args.family == "matrix" else ":" + args.family

    def sched_entry(name, ms, fam=""):
        """algorithmic_frac: the bytes the schedule's layers consume (shared codes counted once per layer
        that reads them unless a pair is fused) over the time, as a fraction of the HBM peak -- for the
        sequential schedule on sharing pairs that is NOT HBM traffic (the second layer's codes come from
        L2); traffic_frac is the measured HBM traffic of the launch over the time."""
        ab = algorithmic_bytes(w, T0, fused=(name == "fused"))
        e = {"decode_ms": ms, "kv_tokens_per_s": w.batch * T0 / (ms * 1e-3), "algorithmic_GBps": ab / (ms * 1e-3) / 1e9,
             "algorithmic_frac": ab / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        tb = prof.get(f"{w.name}:{name}{fam}")
        e["traffic_frac"] = tb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS if tb else None
        # the 70 % target of the 32k configurations, for this family and schedule (same rule as roofline.target_met)
        consumed = algorithmic_bytes(w, T0, fused=False) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS
        e["consumed_frac"] = consumed
        e["target_met"] = (e["algorithmic_frac"] >= HBM_TARGET_FRAC) if T0 >= 32768 else None
        e["target_met_on_consumed_bytes"] = (consumed >= HBM_TARGET_FRAC) if T0 >= 32768 else None
        return e

    by_schedule = {name: sched_entry(name, ms, fam_key) for name, ms in probe.items()}
    # every kernel family on both schedules (decode only, all layers in one call)
    by_family = {}
    if args.schedule == "auto":
        for fam, fl in FAMILY_FLAGS.items():
            if w.head_dim != 128 and fam != "vector_alu":
                continue
            by_family[fam] = {}
            for name, sf in (("sequential", 0), ("fused", 1)):
                if sf and not can_fuse:
                    continue
                ms = probe[name] if fl == alu else time_decode(sf | fl, 10)
                by_family[fam][name] = sched_entry(name, ms, "" if fam == "matrix" else ":" + fam)

    # how a real decoder must call it: one call per layer (layer l+1's query needs layer l's output)
    # eagerly, and as one HIP graph of the same calls replayed (the library only enqueues kernels, so a
    # capture records them; a replay takes the host's launch cost out of the figure)
    def time_per_layer_calls(n=10):
        def once():
            for l in range(w.n_layers):
                cache.decode_attention(qs[0][l:l + 1], sigma, out=out[l:l + 1], layer0=l, flags=alu)

        def timed(fn):
            for _ in range(6):       # (the first replays of a fresh graph are slow: its upload, the clock)
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n

        eager = timed(once)
        side = torch.cuda.Stream()
        graph_ms = None
        try:
            with torch.cuda.stream(side):
                once()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    once()
            torch.cuda.synchronize()
            graph_ms = timed(g.replay)
        except Exception as ex:      # a capture failure must not take the benchmark line with it
            print(f"bench.py: graph capture of the per-layer calls failed: {ex}", file=sys.stderr)
            torch.cuda.synchronize()
        ab = algorithmic_bytes(w, T0, fused=False)   # a call per layer reads the shared codes once per layer
        best = min(x for x in (eager, graph_ms) if x)
        return {"eager_ms": eager, "graph_replay_ms": graph_ms, "calls": w.n_layers,
                "algorithmic_frac": ab / (best * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                "kv_tokens_per_s": w.batch * T0 / (best * 1e-3)}

    per_layer = time_per_layer_calls() if args.schedule == "auto" else None

    # ---- warmup + timed steps
    def step(i, ev=None):
        cache.append_token(new_k[i], new_v[i])
        if ev is not None:
            ev[0].record()
        if per_layer_steps:
            for l in range(w.n_layers):
                cache.decode_attention(qs[i % 4][l:l + 1], sigma, out=out[l:l + 1], layer0=l, flags=flags)
        else:
            cache.decode_attention(qs[i % 4], sigma, out=out, flags=flags)
        if ev is not None:
            ev[1].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t_begin, t_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_begin.record()
    for i in range(args.steps):
        step(args.warmup + i, evs[i])
    t_end.record()
    torch.cuda.synchronize()
    total_ms = t_begin.elapsed_time(t_end)
    ms_per_step = total_ms / args.steps
    decode_ms = float(np.mean([a.elapsed_time(b) for a, b in evs]))
    T_mid = T0 + args.warmup + (args.steps + 1) // 2
    kv_tok_s = w.batch * T_mid / (ms_per_step * 1e-3)

    alg = algorithmic_bytes(w, T_mid, fused=bool(flags & 1))
    achieved = alg / (decode_ms * 1e-3) / 1e9
    # the bytes the layers consume: shared codes counted once per layer that reads them, whatever the
    # schedule does about fetching them once (what a layer-by-layer implementation has to fetch)
    consumed = algorithmic_bytes(w, T_mid, fused=False)
    consumed_frac = consumed / (decode_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS
    res = {
        "metric": "decode_attention_kv_tokens_per_s", "value": kv_tok_s, "unit": "KV tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "layers": w.n_layers, "batch": w.batch, "q_heads": w.n_q_heads,
                   "kv_heads": w.n_kv_heads, "head_dim": w.head_dim, "context": T0, "group": w.group,
                   "residual": w.residual, "kq": w.kq, "vq": w.vq, "km": w.km, "vm": w.vm,
                   "schedule": schedule,
                   "decode_kernels": args.family,
                   "page_tokens": args.page_tokens,
                   "step": "append 1 token/sequence + decode attention, " + ("one call per layer" if per_layer_steps else "all layers in one call")},
        "roofline": {"bound": "hbm", "kernel": "xq_decode_kernel", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": None,
                     "algorithmic_bytes_per_launch": alg, "decode_ms": decode_ms,
                     "consumed_bytes_per_launch": consumed, "consumed_frac": consumed_frac,
                     "target_frac": HBM_TARGET_FRAC if T0 >= 32768 else None,
                     "target_met": (achieved / HBM_PEAK_GBPS >= HBM_TARGET_FRAC) if T0 >= 32768 else None,
                     "target_met_on_consumed_bytes": (consumed_frac >= HBM_TARGET_FRAC) if T0 >= 32768 else None,
                     "target_basis": "target_met: frac >= 0.70, frac pricing the HBM bytes the timed schedule must fetch (shared codes "
                                     "once per fused pair). target_met_on_consumed_bytes: the looser reading, consumed_frac >= 0.70, "
                                     "pricing the bytes the layers consume (shared codes once per layer that reads them), i.e. "
                                     "step time <= those bytes / 0.70 / 8 TB/s; it can exceed 1 for a fused schedule"},
        "token_head_layers_per_s": w.n_layers * w.batch * w.n_kv_heads * T_mid / (ms_per_step * 1e-3),
        "decode_only_by_schedule": by_schedule,
        "decode_only_by_family": by_family,
        "decode_one_call_per_layer": per_layer,
        "append_ms": ms_per_step - decode_ms,
        "pack_GBps_fp16_read": pack_bytes / (pack_ms * 1e-3) / 1e9,
        "pack_roofline": {"bound": "hbm", "kernel": "xq_pack_wave_kernel",
                          "achieved": (pack_bytes + pack_written) / (pack_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS,
                          "unit": "GB/s", "frac": (pack_bytes + pack_written) / (pack_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                          "bytes_read": pack_bytes, "bytes_written": pack_written},
        "equivalent_bits": {"paper_definition": equivalent_bits(cfg), "with_metadata_and_ring": equivalent_bits(cfg, True, T0)},
    }
    # HBM traffic and issue counters: NOT measured by this run.  They are the figures of the committed
    # rocprofv3 counter runs of this same command (profiles/), attached only when the kernel sources
    # still hash to what those runs were taken on; otherwise left null.
    tb = prof.get(f"{w.name}:{schedule}{fam_key}")
    res["roofline"]["traffic"] = tb
    res["roofline"]["traffic_source"] = (f"profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs on kernel sources "
                                         f"{prof.get('_kernel_sources_hash')})") if tb else None
    insts = prof.get(f"{w.name}:{schedule}{fam_key}:valu_wave_instructions")
    if insts:
        # second roof: vector-ALU issue.  Peak = 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions/s;
        # achieved = the launch's counted VALU instructions (SQ_INSTS_VALU, 64 lanes each; the matrix
        # instructions are among them) over the measured duration.
        peak = 256 * 4 * 16 * 2.4e9
        ach = insts * 64 / (decode_ms * 1e-3)
        res["alu_issue"] = {"achieved": ach, "peak": peak, "unit": "lane-instructions/s", "frac": ach / peak,
                            "valu_wave_instructions_per_launch": insts,
                            "of_which_matrix_instructions": prof.get(f"{w.name}:{schedule}{fam_key}:mfma_wave_instructions"),
                            "source": "profiles/traffic.json"}
    if not args.no_cpu_baseline:
        q_cpu = qs[0].cpu()
        res["cpu_baseline"] = cpu_baseline(w, slices, q_cpu, sigma, T0)
    else:
        res["cpu_baseline"] = None
    print(json.dumps(res))


if __name__ == "__main__":
    main()
