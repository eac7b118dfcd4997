#!/usr/bin/env python3
"""Benchmark of the parallel-drafting attention hot path on one MI355X.

A step is one pass of the whole path over one synthetic sequence: for every query-row segment,
forward (O, LSE) then backward (dQ, dK, dV) with dK/dV accumulated across segments in fp32
(peagle_attn_step_partitioned).  The tile map is built once before the timed region (amortized
mask construction) and its build time is reported separately.  Inputs are resident in HBM when
the timed region starts.

Prints ONE JSON line: effective (useful, unmasked-pair) TFLOP/s of forward+backward, the
roofline of the dominant kernel from HIP-event launch durations measured in this run, and the
fp64 CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA


def _kernel_source_hash() -> str:
    """sha256 of the attention kernel sources: names the code a counter run measured."""
    import hashlib
    h = hashlib.sha256()
    for name in ("attn_kernels.hip", "mfma_util.h", "attn_kernels.h"):
        with open(os.path.join(ROOT, "paper_2602_01469_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def _read_traffic(workload: str):
    """HBM bytes per dK/dV-kernel launch from the committed rocprofv3 --pmc summary of this workload - only if that
    summary was taken on the kernel sources as they are now (it records their hash); otherwise None: a counter
    figure of other code is not reported."""
    path = os.path.join(ROOT, "profiles", f"dkdv_kernel_{workload}_traffic.txt")
    if not os.path.exists(path):
        return None
    fields = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.strip().split("=", 1)
            fields[k] = v
    if fields.get("kernel_source_sha256_16") != _kernel_source_hash() or "traffic_bytes_per_launch" not in fields:
        return None
    return float(fields["traffic_bytes_per_launch"])


def cpu_baseline(cfg, bits, sample_anchors: int):
    """The oracle as it stands on a bounded sample of the workload's own inputs: the rows and keys of the first
    `sample_anchors` anchors (all depths) of one KV group, dense fp64 forward+backward (by position invariance
    that is the complete problem of a sequence cut after those anchors).  Returns useful TFLOP/s on the host cores;
    `all_heads_s_extrapolated` scales the measured time to every KV group of the full workload by useful pairs."""
    import numpy as np
    from oracle import peagle_oracle as orc
    from peagle_inputs import bf16_bits_to_f64, useful_pairs
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    qb, kb, vb, dob = bits
    Ls, K, D = min(sample_anchors, cfg.L), cfg.K, cfg.D
    grp = cfg.Hq // cfg.Hkv
    g = cfg.Hkv - 1
    idx = np.concatenate([d * cfg.L + np.arange(Ls) for d in range(K)])
    hs = slice(g * grp, (g + 1) * grp)
    q, do = bf16_bits_to_f64(qb[idx][:, hs]), bf16_bits_to_f64(dob[idx][:, hs])
    k, v = bf16_bits_to_f64(kb[idx][:, g:g + 1]), bf16_bits_to_f64(vb[idx][:, g:g + 1])
    t0 = time.perf_counter()
    orc.attn_backward(q, k, v, do, Ls, K, cfg.scale)
    dt = time.perf_counter() - t0
    flops = 14 * D * grp * useful_pairs(Ls, K)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"the workload's own inputs cut after {Ls} anchors x K={K} depths (T={Ls * K} rows), KV head {g} "
                      f"with its {grp} query heads, dense fp64 forward+backward, {dt:.1f} s",
            "all_heads_s_extrapolated": dt * cfg.Hkv * useful_pairs(cfg.L, K) / useful_pairs(Ls, K)}


def trace_lengths(quantiles):
    """Sequence lengths at the given quantiles of the paper's training-length distribution (its Fig. 1
    caption: median 3,891, P90 10,800, P99 20,000 tokens), log-linear between and beyond the three
    published points, rounded up to 16 anchors and capped at 20480."""
    import math
    pts = [(0.5, 3891.0), (0.9, 10800.0), (0.99, 20000.0)]
    out = []
    for q in quantiles:
        (q0, l0), (q1, l1) = (pts[0], pts[1]) if q <= pts[1][0] else (pts[1], pts[2])
        t = (q - q0) / (q1 - q0)
        L = math.exp(math.log(l0) + t * (math.log(l1) - math.log(l0)))
        out.append(min(20480, max(16, int(math.ceil(L / 16.0)) * 16)))
    return out


def sweep(args) -> int:
    """Throughput over sequence length with ONE tile map built for the maximum length: every shorter
    sequence uses its prefix (the per-example crop of the amortized mask).  K=8, 64/8 heads, D=64,
    segments of 2048 anchors; inputs are seeded N(0,1) bf16 drawn on the device (throughput only)."""
    import torch

    import paper_2602_01469_amd as pe
    from peagle_inputs import useful_flops
    pe.load_library()
    torch.cuda.set_device(0)
    K, Hq, Hkv, D, L_max = 8, 64, 8, 64, 20480
    bounds = list(range(0, L_max, 2048)) + [L_max]
    torch.zeros(1, device="cuda")  # (the first HIP call of a process takes tens of milliseconds of its own)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tm = pe.peagle_build_tilemap(L_max, K, bounds, device=0)
    build_ms = (time.perf_counter() - t0) * 1e3
    stream = torch.cuda.current_stream()
    qs = [0.1, 0.25, 0.5, 0.75, 0.9, 0.95, 0.99]
    rows = []
    gen = torch.Generator(device="cuda").manual_seed(7)
    for q, L in zip(qs, trace_lengths(qs)):
        T = L * K
        mk = lambda h: torch.randn((T, h, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        qt, kt, vt, dot = mk(Hq), mk(Hkv), mk(Hkv), mk(Hq)
        shape = pe.Shape(L, K, Hq, Hkv, D)
        o, dq = torch.empty_like(qt), torch.empty_like(qt)
        lse = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
        dk = torch.empty((T, Hkv, D), dtype=torch.float32, device="cuda")
        dv = torch.empty_like(dk)
        ws = torch.empty(pe.peagle_workspace_bytes(tm, shape), dtype=torch.uint8, device="cuda")
        S = len(bounds) - 1
        step = lambda: pe.peagle_attn_step_partitioned(tm, shape, 0, S, qt, kt, vt, dot, o, lse, dq, dk, dv, None, None,
                                                       ws, stream)
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        n = 5
        t0 = time.perf_counter()
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / n
        fl = useful_flops(L, K, Hq, D)
        rows.append({"quantile": q, "L": L, "T": T, "ms_per_step": ms, "tflops": fl / (ms * 1e-3) / 1e12,
                     "finite": bool(torch.isfinite(dk).all().item())})
        del qt, kt, vt, dot, o, dq, lse, dk, dv, ws
    print(json.dumps({"metric": "effective masked-attn TFLOP/s fwd+bwd over sequence length (one tile map, prefix views)",
                      "unit": "TFLOP/s", "n_gpus": 1, "data": "synthetic", "dtype": "bf16",
                      "config": {"workload": f"length sweep at the trace quantiles, K={K} Hq={Hq} Hkv={Hkv} D={D}, "
                                             f"tile map for L_max={L_max}, segments of 2048 anchors"},
                      "tilemap_build_ms": build_ms, "sweep": rows}))
    return 0


def sampled(args) -> int:
    """The named workload under Conditional Drop-token sampling with the given retention rate
    (a sampled tile map, built per sequence and timed separately): same segments, T = kept positions
    only.  Useful FLOPs count the pairs of kept positions."""
    import numpy as np
    import torch

    import paper_2602_01469_amd as pe
    from peagle_inputs import CONFIGS, cod_depth_counts, make_inputs_tokens, useful_pairs, useful_pairs_sampled
    pe.load_library()
    torch.cuda.set_device(0)
    cfg = CONFIGS[args.workload]
    bounds = cfg.seg_bounds()
    S = len(bounds) - 1
    count = cod_depth_counts(cfg.L, cfg.K, args.cod_retention, cfg.seed)
    t0 = time.perf_counter()
    tm = pe.peagle_build_tilemap_sampled(count, cfg.K, bounds, device=0)
    build_ms = (time.perf_counter() - t0) * 1e3
    info = tm.info()
    T = tm.tokens(cfg.L)
    dev = lambda x: torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    q, k, v, do = (dev(x) for x in make_inputs_tokens(cfg, T))
    shape = pe.Shape(cfg.L, cfg.K, cfg.Hq, cfg.Hkv, cfg.D, cfg.scale)
    o, dq = torch.empty_like(q), torch.empty_like(q)
    lse = torch.empty((cfg.Hq, T), dtype=torch.float32, device="cuda")
    dk = torch.empty((T, cfg.Hkv, cfg.D), dtype=torch.float32, device="cuda")
    dv = torch.empty_like(dk)
    ws = torch.empty(pe.peagle_workspace_bytes(tm, shape), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    step = lambda: pe.peagle_attn_step_partitioned(tm, shape, 0, S, q, k, v, do, o, lse, dq, dk, dv, None, None, ws,
                                                   stream)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)
    pairs = useful_pairs_sampled(count)
    flops = 14 * cfg.D * cfg.Hq * pairs
    print(json.dumps({
        "metric": "effective masked-attn TFLOP/s fwd+bwd (useful FLOPs of kept positions), drop-token sampled sequence",
        "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} with retention {args.cod_retention}: L={cfg.L} K={cfg.K} kept positions "
                               f"T={T} of {cfg.T}, Hq={cfg.Hq} Hkv={cfg.Hkv} D={cfg.D}, {S} segments, seed {cfg.seed}"},
        "kept_positions": T, "useful_pairs": pairs, "useful_pairs_dense": useful_pairs(cfg.L, cfg.K),
        "useful_over_computed_pairs": pairs / ((info["n_full"] + info["n_partial"]) * 128 * 64),
        "tilemap_build_ms": build_ms,
        "tilemap": {"device_bytes": info["device_bytes"], "n_masks": info["n_masks"], "n_row_tiles": info["n_row_tiles"],
                    "n_full": info["n_full"], "n_partial": info["n_partial"]},
        "finite": bool(torch.isfinite(dk).all().item() and torch.isfinite(dv).all().item())}))
    return 0


def packed(args) -> int:
    """A batch of sequences packed before the expansion and run as one problem (one launch per kernel for the
    whole batch): lengths at evenly spaced quantiles of the paper's trace-length distribution up to the
    median, K=8, 64/8 heads, D=64, dense.  Compared with running the same sequences one after another."""
    import numpy as np
    import torch

    import paper_2602_01469_amd as pe
    from peagle_inputs import useful_pairs
    pe.load_library()
    torch.cuda.set_device(0)
    K, Hq, Hkv, D = 8, 64, 8, 64
    n = args.packed
    lens = trace_lengths([0.05 + 0.45 * i / max(n - 1, 1) for i in range(n)])
    L = sum(lens)
    T = L * K
    gen = torch.Generator(device="cuda").manual_seed(11)
    mk = lambda h: torch.randn((T, h, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    q, k, v, do = mk(Hq), mk(Hkv), mk(Hkv), mk(Hq)
    o, dq = torch.empty_like(q), torch.empty_like(q)
    lse = torch.empty((Hq, T), dtype=torch.float32, device="cuda")
    dk = torch.empty((T, Hkv, D), dtype=torch.float32, device="cuda")
    dv = torch.empty_like(dk)
    stream = torch.cuda.current_stream()
    t0 = time.perf_counter()
    tm = pe.peagle_build_tilemap_packed(lens, K, None, None, device=0)
    build_ms = (time.perf_counter() - t0) * 1e3
    shape = pe.Shape(L, K, Hq, Hkv, D)
    ws = torch.empty(pe.peagle_workspace_bytes(tm, shape), dtype=torch.uint8, device="cuda")
    step = lambda: pe.peagle_attn_step_partitioned(tm, shape, 0, 1, q, k, v, do, o, lse, dq, dk, dv, None, None, ws, stream)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)

    ms_packed = timed(step)
    finite = bool(torch.isfinite(dk).all().item() and torch.isfinite(dv).all().item() and torch.isfinite(o.float()).all().item())
    # the same sequences one after another, each with its own dense map and tensors
    singles = []
    for Lq in lens:
        Tq = Lq * K
        mkq = lambda h: torch.randn((Tq, h, D), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        tq, tk, tv, tdo = mkq(Hq), mkq(Hkv), mkq(Hkv), mkq(Hq)
        one = {"tm": pe.peagle_build_tilemap(Lq, K, None, device=0), "shape": pe.Shape(Lq, K, Hq, Hkv, D),
               "t": (tq, tk, tv, tdo, torch.empty_like(tq), torch.empty((Hq, Tq), dtype=torch.float32, device="cuda"),
                     torch.empty_like(tq), torch.empty((Tq, Hkv, D), dtype=torch.float32, device="cuda"),
                     torch.empty((Tq, Hkv, D), dtype=torch.float32, device="cuda"))}
        one["ws"] = torch.empty(pe.peagle_workspace_bytes(one["tm"], one["shape"]), dtype=torch.uint8, device="cuda")
        singles.append(one)

    def run_singles():
        for one in singles:
            tq, tk, tv, tdo, to, tl, tdq, tdk, tdv = one["t"]
            pe.peagle_attn_step_partitioned(one["tm"], one["shape"], 0, 1, tq, tk, tv, tdo, to, tl, tdq, tdk, tdv, None,
                                            None, one["ws"], stream)
    ms_singles = timed(run_singles)
    prof = pe.peagle_attn_step_profiled(tm, shape, 0, 1, q, k, v, do, o, lse, dq, dk, dv, ws, stream)
    prof_singles = {}
    for one in singles:
        tq, tk, tv, tdo, to, tl, tdq, tdk, tdv = one["t"]
        pr = pe.peagle_attn_step_profiled(one["tm"], one["shape"], 0, 1, tq, tk, tv, tdo, to, tl, tdq, tdk, tdv, one["ws"],
                                          stream)
        for name, (ms, _) in pr.items():
            prof_singles[name] = prof_singles.get(name, 0.0) + ms
    flops = 14 * D * Hq * sum(useful_pairs(Lq, K) for Lq in lens)
    info = tm.info()
    print(json.dumps({
        "metric": "effective masked-attn TFLOP/s fwd+bwd (useful FLOPs), packed variable-length batch",
        "value": flops / (ms_packed * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_packed, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{n} sequences of {lens} anchors packed into one problem, K={K} Hq={Hq} Hkv={Hkv} D={D}"},
        "one_by_one_ms": ms_singles, "one_by_one_tflops": flops / (ms_singles * 1e-3) / 1e12,
        "kernels_ms": {name: v[0] for name, v in prof.items()}, "one_by_one_kernels_ms": prof_singles,
        "tilemap_build_ms": build_ms, "tilemap": {"n_row_tiles": info["n_row_tiles"], "n_full": info["n_full"],
                                                  "n_partial": info["n_partial"], "device_bytes": info["device_bytes"]},
        "finite": finite}))
    return 0


def rope(args) -> int:
    """The named workload with rotary embedding around the step (unrotated Q and K in, gradients in the
    unrotated frame out): whole-step time beside the plain step on the same inputs, per-kernel times from
    HIP events, and the rotation kernel against the HBM roofline (it streams Q and K once each way)."""
    import numpy as np
    import torch

    import paper_2602_01469_amd as pe
    from peagle_inputs import CONFIGS, make_inputs, useful_flops
    pe.load_library()
    torch.cuda.set_device(0)
    cfg = CONFIGS[args.workload]
    bounds = cfg.seg_bounds()
    S = len(bounds) - 1
    tm = pe.peagle_build_tilemap(cfg.L, cfg.K, bounds, device=0)
    T = cfg.T
    dev = lambda x: torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    q, k, v, do = (dev(x) for x in make_inputs(cfg))
    shape = pe.Shape(cfg.L, cfg.K, cfg.Hq, cfg.Hkv, cfg.D, cfg.scale)
    o, dq = torch.empty_like(q), torch.empty_like(q)
    lse = torch.empty((cfg.Hq, T), dtype=torch.float32, device="cuda")
    dk = torch.empty((T, cfg.Hkv, cfg.D), dtype=torch.float32, device="cuda")
    dv = torch.empty_like(dk)
    ws = torch.empty(pe.peagle_rope_workspace_bytes(tm, shape), dtype=torch.uint8, device="cuda")
    n_pos = pe.peagle_rope_positions(tm, cfg.L)
    table = torch.empty((n_pos, 2, cfg.D // 2), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pe.peagle_rope_table(args.rope, cfg.D, n_pos, table, stream)
    torch.cuda.synchronize()
    table_ms = (time.perf_counter() - t0) * 1e3
    plain = lambda: pe.peagle_attn_step_partitioned(tm, shape, 0, S, q, k, v, do, o, lse, dq, dk, dv, None, None, ws,
                                                    stream)
    roped = lambda: pe.peagle_attn_step_partitioned_rope(tm, shape, 0, S, q, k, v, do, table, o, lse, dq, dk, dv, None,
                                                         None, ws, stream)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)

    ms_plain = timed(plain) if not args.partitioned_only else None
    ms = timed(roped)
    # the first-layer form: depth-0 keys / values of their own, one shared vector for every other position
    ms_shared = None
    if not args.partitioned_only:
        k0, v0 = k[:cfg.L].contiguous(), v[:cfg.L].contiguous()
        ks, vs = k[cfg.L].contiguous(), v[cfg.L].contiguous()
        dk0, dv0 = torch.empty((cfg.L, cfg.Hkv, cfg.D), dtype=torch.float32, device="cuda"), None
        dv0 = torch.empty_like(dk0)
        dks = torch.empty((cfg.Hkv, cfg.D), dtype=torch.float32, device="cuda")
        dvs = torch.empty_like(dks)
        ws2 = torch.empty(pe.peagle_rope_shared_workspace_bytes(tm, shape), dtype=torch.uint8, device="cuda")
        ms_shared = timed(lambda: pe.peagle_attn_step_rope_shared(tm, shape, q, k0, ks, v0, vs, do, table, o, lse, dq, dk0,
                                                                  dv0, dks, dvs, ws2, stream))
        del ws2
    flops = useful_flops(cfg.L, cfg.K, cfg.Hq, cfg.D)
    out = {
        "metric": "effective masked-attn TFLOP/s fwd+bwd (useful FLOPs), rotary embedding of Q and K inside the step",
        "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} with rotary embedding (base {args.rope:g}): L={cfg.L} K={cfg.K} Hq={cfg.Hq} "
                               f"Hkv={cfg.Hkv} D={cfg.D}, {S} segments, seed {cfg.seed}"},
        "plain_ms_per_step": ms_plain, "rope_overhead": None if ms_plain is None else ms / ms_plain,
        "shared_chain_vectors_ms_per_step": ms_shared,
        "rope_table_ms": table_ms, "rope_positions": n_pos,
        "finite": bool(torch.isfinite(dk).all().item() and torch.isfinite(dv).all().item())}
    if not args.partitioned_only:
        reps, prof = 5, {}
        for rep in range(reps + 1):     # the first profiled step (event creation, cold) is not counted
            pr = pe.peagle_attn_step_rope_profiled(tm, shape, 0, S, q, k, v, do, table, o, lse, dq, dk, dv, ws, stream)
            if rep:
                for name, (kms, n) in pr.items():
                    a = prof.setdefault(name, [0.0, 0])
                    a[0] += kms / reps
                    a[1] = n
        out["kernel_ms_per_step"] = {name: prof[name][0] for name in prof}
        out["kernel_launches_per_step"] = {name: prof[name][1] for name in prof}
        # rotation: two launches per step (Q, then K), each element read once and written once
        moved = 2 * 2 * T * (cfg.Hq + cfg.Hkv) * cfg.D
        rope_ms = prof["rope"][0]
        out["roofline"] = {"bound": "hbm", "kernel": "rope_rotate_kernel", "achieved": moved / (rope_ms * 1e-3) / 1e9,
                           "peak": 8000.0, "unit": "GB/s", "frac": moved / (rope_ms * 1e-3) / 1e9 / 8000.0,
                           "traffic": None, "bytes_per_step": moved, "ms_per_step": rope_ms}
    print(json.dumps(out))
    return 0


def decode(args) -> int:
    """Inference-side drafting step (all K draft positions of C requests against their paged KV caches):
    time per call from HIP events on the launch stream and the cache bytes it reads against the HBM peak.
    Shapes: the serving setting of the paper (C = 4, K = 7, GPT-OSS heads) at the training-trace median
    context, and a batch large enough to occupy the memory system (C = 64, 8192-token contexts)."""
    import numpy as np
    import torch

    import paper_2602_01469_amd as pe
    pe.load_library()
    torch.cuda.set_device(0)
    results = []
    for name, C_, K, Hq, Hkv, D, ctx in (("serving C=4 K=7 ctx=4096", 4, 7, 64, 8, 64, 4096),
                                         ("serving C=2 K=5 ctx=20000", 2, 5, 64, 8, 64, 20000),
                                         ("batch C=64 K=7 ctx=8192", 64, 7, 64, 8, 64, 8192),
                                         ("batch C=64 K=7 ctx=8192 D=128", 64, 7, 32, 4, 128, 8192)):
        pages_per = (ctx + 63) // 64
        n_pages = C_ * pages_per
        shape = pe.DecodeShape(C_, K, Hq, Hkv, D, n_pages, pages_per)
        g = torch.Generator(device="cuda").manual_seed(7)
        rnd = lambda *sh: torch.randn(*sh, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        q, kn, vn = rnd(C_, K, Hq, D), rnd(C_, K, Hkv, D), rnd(C_, K, Hkv, D)
        kp, vp = rnd(n_pages, Hkv, 64, D), rnd(n_pages, Hkv, 64, D)
        bt = torch.randperm(n_pages, generator=g, device="cuda").to(torch.int32).view(C_, pages_per).contiguous()
        cl = torch.full((C_,), ctx, dtype=torch.int32, device="cuda")
        o = torch.empty_like(q)
        lse = torch.empty((C_, Hq, K), dtype=torch.float32, device="cuda")
        status = torch.zeros((C_,), dtype=torch.int32, device="cuda")
        ws = torch.empty(pe.peagle_draft_decode_workspace_bytes(shape), dtype=torch.uint8, device="cuda")
        call = lambda: pe.peagle_draft_decode(shape, q, kn, vn, kp, vp, bt, cl, o, lse, status, ws,
                                              torch.cuda.current_stream())
        for _ in range(max(args.warmup, 3)):
            call()
        torch.cuda.synchronize()
        # The calls are recorded into a HIP graph and replayed: a serving loop drives the C ABI directly, and
        # the argument checks of the Python binding (tens of microseconds per call) are not part of the path.
        reps = max(args.steps, 20)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(reps):
                call()
        graph.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        cache_bytes = 2 * C_ * ctx * Hkv * D * 2
        results.append({"workload": name, "us_per_call": us, "cache_bytes": cache_bytes,
                        "GBps": cache_bytes / (us * 1e-6) / 1e9, "frac_of_hbm_peak": cache_bytes / (us * 1e-6) / 8e12,
                        "splits": pe.peagle_draft_decode_splits(shape), "workspace_bytes": ws.numel(),
                        "status_ok": bool((status == 0).all().item()),
                        "finite": bool(torch.isfinite(o.float()).all().item())})
    big = results[2]
    print(json.dumps({
        "metric": "KV-cache read rate of the inference-side drafting attention (cache bytes / time per call)",
        "value": big["GBps"], "unit": "GB/s", "n_gpus": 1, "steps": max(args.steps, 20), "warmup": max(args.warmup, 3),
        "ms_per_step": big["us_per_call"] * 1e-3, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": big["workload"] + ", Hq=64 Hkv=8 D=64, 64-token pages, shuffled block table"},
        "roofline": {"bound": "hbm", "kernel": "draft_decode_kernel + draft_decode_combine_kernel",
                     "achieved": big["GBps"], "peak": 8000.0, "unit": "GB/s", "frac": big["frac_of_hbm_peak"],
                     "traffic": None},
        "shapes": results}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3_median")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-anchors", type=int, default=2048)
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the headline workload, time a sweep of sequence lengths on one tile map")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one 256 MiB device-to-device copy (reference dispatch for HBM byte counters)")
    ap.add_argument("--cod-retention", type=float, default=None,
                    help="instead of the headline (dense) workload, time the same shape under drop-token sampling "
                         "with this retention rate")
    ap.add_argument("--partitioned-only", action="store_true",
                    help="skip the unpartitioned comparison pass (keeps a profiler trace to the partitioned launches)")
    ap.add_argument("--packed", type=int, default=None,
                    help="instead of the headline workload, time a packed batch of this many short sequences")
    ap.add_argument("--rope", type=float, default=None, metavar="BASE",
                    help="run the workload with rotary embedding of Q and K inside the step (e.g. 500000)")
    ap.add_argument("--decode", action="store_true",
                    help="time the inference-side drafting attention (paged KV cache) instead of the training step")
    ap.add_argument("--seg-anchors", type=int, default=None,
                    help="override the anchors per query-row segment (diagnostic; the default is the workload's)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    if args.sweep:
        return sweep(args)
    if args.cod_retention is not None:
        return sampled(args)
    if args.packed is not None:
        return packed(args)
    if args.rope is not None:
        return rope(args)
    if args.decode:
        return decode(args)

    import torch

    import paper_2602_01469_amd as pe
    from peagle_inputs import CONFIGS, make_inputs, useful_flops, useful_pairs

    pe.load_library()  # fails loudly if the HIP extension is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    cfg = CONFIGS[args.workload]
    if args.seg_anchors is not None:
        import dataclasses
        cfg = dataclasses.replace(cfg, seg_anchors=args.seg_anchors)
    bounds = cfg.seg_bounds()
    S = len(bounds) - 1

    # Amortized mask construction: the host part (classification, lists, mask pool) and the part that needs the
    # device (allocation and upload), each timed after the HIP runtime is up (one small allocation first:
    # the first HIP call of a process takes tens of milliseconds of its own).
    torch.zeros(1, device="cuda")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pe.peagle_build_tilemap(cfg.L, cfg.K, bounds, device=-1)
    tilemap_host_ms = (time.perf_counter() - t0) * 1e3
    t0 = time.perf_counter()
    tm = pe.peagle_build_tilemap(cfg.L, cfg.K, bounds, device=0)
    tilemap_ms = (time.perf_counter() - t0) * 1e3
    info = tm.info()

    import numpy as np
    qb, kb, vb, dob = make_inputs(cfg)
    dev = lambda x: torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    q, k, v, do = dev(qb), dev(kb), dev(vb), dev(dob)
    cpu = None if args.no_cpu_baseline else (qb, kb, vb, dob)
    del qb, kb, vb, dob
    shape = pe.Shape(cfg.L, cfg.K, cfg.Hq, cfg.Hkv, cfg.D, cfg.scale)
    T = cfg.T
    o = torch.empty((T, cfg.Hq, cfg.D), dtype=torch.bfloat16, device="cuda")
    dq = torch.empty_like(o)
    lse = torch.empty((cfg.Hq, T), dtype=torch.float32, device="cuda")
    dk = torch.empty((T, cfg.Hkv, cfg.D), dtype=torch.float32, device="cuda")
    dv = torch.empty_like(dk)
    ws = torch.empty(pe.peagle_workspace_bytes(tm, shape), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        pe.peagle_attn_step_partitioned(tm, shape, 0, S, q, k, v, do, o, lse, dq, dk, dv, None, None, ws, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)

    # the same steps once more with an event pair around each (median and minimum), and the
    # unpartitioned pass over the same inputs (what within-sequence partitioning costs)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(max(args.steps, 1))]
    for a, b in evs:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in evs)

    def whole():
        pe.peagle_attn_fwd(tm, shape, -1, q, k, v, o, lse, stream)
        pe.peagle_attn_bwd(tm, shape, -1, q, k, v, o, do, lse, dq, dk, dv, 0, ws, stream)
    ms_whole = None
    if not args.partitioned_only:
        for _ in range(2):
            whole()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(max(args.steps // 2, 1)):
            whole()
        torch.cuda.synchronize()
        ms_whole = (time.perf_counter() - t0) * 1e3 / max(args.steps // 2, 1)

    # per-kernel launch durations: HIP events on the launch stream, same workload, same launches
    prof_reps = 5
    acc = {}
    for _ in range(prof_reps):
        pr = pe.peagle_attn_step_profiled(tm, shape, 0, S, q, k, v, do, o, lse, dq, dk, dv, ws, stream)
        for name, (ms, n) in pr.items():
            a = acc.setdefault(name, [0.0, 0])
            a[0] += ms
            a[1] += n
    kernels = {name: {"ms_per_step": a[0] / prof_reps, "launches_per_step": a[1] // prof_reps,
                      "avg_launch_ms": a[0] / max(a[1], 1)} for name, a in acc.items() if a[1] > 0}
    mfma_ceiling = pe.peagle_measure_mfma_ceiling(stream)
    # the same issue loop on changing pseudo-random operands: the chip holds a lower clock under that load
    mfma_ceiling_random = pe.peagle_measure_mfma_ceiling(stream, random_operands=True)
    torch.cuda.synchronize()
    # The same step on all-zero operands: identical instruction stream and launches, almost no switching
    # activity in the matrix cores, so the chip keeps its full clock - the difference to ms_per_step is what the
    # power limit costs on real data (context only: zeros are not a workload).
    ms_zero = None
    if not args.partitioned_only:
        qz, kz, vz, doz = (torch.zeros_like(x) for x in (q, k, v, do))
        zstep = lambda: pe.peagle_attn_step_partitioned(tm, shape, 0, S, qz, kz, vz, doz, o, lse, dq, dk, dv, None,
                                                        None, ws, stream)
        for _ in range(3):
            zstep()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(max(args.steps // 2, 1)):
            zstep()
        torch.cuda.synchronize()
        ms_zero = (time.perf_counter() - t0) * 1e3 / max(args.steps // 2, 1)
        del qz, kz, vz, doz
    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")   # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    flops = useful_flops(cfg.L, cfg.K, cfg.Hq, cfg.D)
    pairs = useful_pairs(cfg.L, cfg.K)
    value = flops / (ms_per_step * 1e-3) / 1e12
    # dominant kernel: dK/dV.  Algorithmic flops per unmasked pair per query head: S and dP
    # recompute (2D each) + dV (2D) + dK (2D) = 8D; the dQ kernel carries 2D, the forward 4D.
    dkdv = kernels["dkdv"]
    dkdv_flops_per_launch = 8 * cfg.D * cfg.Hq * pairs / max(dkdv["launches_per_step"], 1)
    achieved = dkdv_flops_per_launch / (dkdv["avg_launch_ms"] * 1e-3) / 1e12
    props = torch.cuda.get_device_properties(0)
    dinfo = pe.peagle_device_info()
    # tile pairs actually computed (128 rows x 64 keys each) vs useful pairs
    computed_pairs = (info["n_full"] + info["n_partial"]) * 128 * 64
    out = {
        "metric": "effective masked-attn TFLOP/s fwd+bwd (useful FLOPs) & % of bf16 MFMA peak",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_median": per_step[len(per_step) // 2],
        "ms_per_step_min": per_step[0],
        "unpartitioned_ms_per_step": ms_whole,
        "partition_overhead": ms_per_step / ms_whole if ms_whole else None,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: L={cfg.L} K={cfg.K} T={cfg.T} Hq={cfg.Hq} Hkv={cfg.Hkv} D={cfg.D}, "
                               f"{S} query-row segments of {cfg.seg_anchors or cfg.L} anchors, fwd+bwd, seed {cfg.seed}",
                   "L": cfg.L, "K": cfg.K, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "D": cfg.D, "segments": S},
        "pct_of_bf16_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "pct_of_measured_mfma_ceiling": 100.0 * value / mfma_ceiling if mfma_ceiling > 0 else None,
        "measured_mfma_ceiling_tflops": mfma_ceiling,
        "measured_mfma_ceiling_random_operands_tflops": mfma_ceiling_random,
        "pct_of_measured_mfma_ceiling_random_operands": 100.0 * value / mfma_ceiling_random if mfma_ceiling_random > 0 else None,
        "ms_per_step_on_zero_operands": ms_zero,
        "useful_flops_per_step": flops,
        "useful_over_computed_pairs": pairs / computed_pairs,
        "tilemap_build_ms": tilemap_ms,
        "tilemap_build_host_part_ms": tilemap_host_ms,
        "tilemap_upload_part_ms": max(tilemap_ms - tilemap_host_ms, 0.0),
        "tilemap": {"device_bytes": info["device_bytes"], "n_masks": info["n_masks"], "n_full": info["n_full"],
                    "n_partial": info["n_partial"]},
        "kernels": kernels,
        "device": {"name": props.name, "arch": getattr(props, "gcnArchName", ""), "cus": dinfo["compute_units"],
                   "clock_mhz": dinfo["clock_khz"] / 1e3},
        "roofline": {"bound": "mfma", "kernel": "dkdv_kernel", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": _read_traffic(cfg.name)},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, cpu, args.cpu_sample_anchors)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
