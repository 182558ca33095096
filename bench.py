#!/usr/bin/env python3
"""Benchmark of the CentroidKV hot path on one MI355X.

A step = one pass of the whole path over one batch of synthetic input that is already resident
in HBM: ckv_compress of a full-model KV cache (all layers folded into the batch dimension, one
launch per kernel per round) followed by one decode step of attention over the compressed cache
(one ckv_decode_attn call per layer, as a model would issue them).

Prints ONE JSON line.  `value` = context tokens pushed through the whole step per second.
`roofline` describes the kernel with the largest share of GPU time; its launch durations come from
HIP events the library records on the launch stream during the timed steps.  Only that kernel is
bracketed there: events around every launch slow the 32 short attention layers of a step by about
a quarter.  `kernels` lists the same figures for every hot kernel; the other kernels' come from a
few untimed profile steps (each entry says which).  `cpu_baseline` is the numpy oracle timed on a
bounded sample.
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

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published

# HBM bytes per launch of a kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (one counter per
# run), each scaled by what the same counter reads for the library's plain row-copy kernel of known
# size; see profiles/bench_config3_hbm_traffic.txt for the runs and the factors.  Filled in by hand
# from those runs: {(workload, kernel): bytes per launch averaged over the launches of one step}.
MEASURED_TRAFFIC = {
    ("config3", "merge_keys_bf16"): int((4227434.2 * 2.0 + 4489327.4) * 1024),
    ("config3", "merge_origin_bf16"): int((6423693.0 * 2.0 + 4292654.6) * 1024),
    ("config3", "match_bf16"): int((3172452.1 * 2.0 + 98304.0) * 1024),
    ("config3", "attn_partial_bf16"): int((66165.0 * 2.0 + 1040.0) * 1024),
}

WORKLOADS = {
    # the headline configuration: full-model prefill compression, Llama-3-8B KV shape, 128k tokens
    "config3": dict(layers=32, kv_heads=8, q_heads=32, dim=128, seq=131072, chunk=1024, retain=0.25,
                    alpha=0.9, n_outlier=4, desc="llama3-8b 32Lx8KVx128 bf16, seq 131072, chunk 1024, "
                    "retain 25% (rounds [1,1]) + 1 GQA decode step (32 q heads) over the compressed cache"),
    # one layer, 32k tokens (small: one launch is a few microseconds)
    "config2": dict(layers=1, kv_heads=8, q_heads=32, dim=128, seq=32768, chunk=1024, retain=0.25,
                    alpha=0.9, n_outlier=4, desc="llama3-8b single layer 8KVx128 bf16, seq 32768, chunk 1024, "
                    "retain 25% + 1 GQA decode step"),
}


def algorithmic_work(cfg, plan, fused=True, deferred=False):
    """Algorithmic bytes / flops of one step, per kernel (whole launch set of that kernel).

    deferred: a round with r = 1 that is followed by another round writes keys and degrees only
    (kernel merge_keys_bf16, which also exports 3 bytes of member lists per token) and the next
    round (merge_origin_bf16) reads its keys and degrees, and every ORIGINAL value row once.

    Mirrors the library's schedule: two consecutive rounds whose first merges every edge (r = 1)
    run as ONE pass (kernel fused2_bf16: reads K, V once, writes the final rows) when chunk = 1024,
    bf16, dim 128 and the length is a multiple of 2048; other rounds run as match + merge."""
    n_bh = cfg["layers"] * cfg["kv_heads"]
    d, e, c = cfg["dim"], 2, cfg["chunk"]
    work = {"match_bf16": 0.0, "merge_bf16": 0.0, "merge_keys_bf16": 0.0, "merge_origin_bf16": 0.0,
            "fused2_bf16": 0.0, "attn_partial_bf16": 0.0}
    origin_len = None       # length of the cache whose values the current round rebuilds from
    flops = {"fused2_bf16": 0.0}
    j, J = 0, len(plan.round_r)

    def match_flops(s_in):
        full, tail = divmod(s_in, c)
        return full * 2 * (c // 2) * (c // 2) * d + 2 * ((tail + 1) // 2) * (tail // 2) * d

    while j < J:
        s_in = plan.round_len[j]
        deg_in = 0 if j == 0 else 4
        if fused and j + 1 < J and plan.round_r[j] == 1.0 and c == 1024 and d == 128 and s_in % 2048 == 0:
            s_out = plan.round_len[j + 2]
            work["fused2_bf16"] += n_bh * (s_in * (2 * d * e + deg_in + 4) + s_out * (2 * d * e + 4))
            flops["fused2_bf16"] += n_bh * (match_flops(s_in) + match_flops(plan.round_len[j + 1]))
            j += 2
            continue
        s_out = plan.round_len[j + 1]
        full, tail = divmod(s_in, c)
        work["match_bf16"] += n_bh * match_flops(s_in)                       # 2*|A|*|B|*d per chunk
        n_src = full * (c // 2) + (tail + 1) // 2
        if origin_len is not None:      # second round of a deferred pair
            org_deg = 0 if j == 1 else 4
            work["merge_origin_bf16"] += n_bh * (s_in * (d * e + 4 + 4) + n_src * 8 + origin_len * (d * e + org_deg + 3)
                                                 + s_out * (2 * d * e + 4))
            origin_len = None
        elif deferred and j + 1 < J and plan.round_r[j] == 1.0:
            work["merge_keys_bf16"] += n_bh * (s_in * (d * e + deg_in + 4 + 3) + n_src * 8 + s_out * (d * e + 4))
            origin_len = s_in
        else:
            work["merge_bf16"] += n_bh * (s_in * (2 * d * e + deg_in + 4) + n_src * 8 + s_out * (2 * d * e + 4))
        j += 1
    work["attn_partial_bf16"] = n_bh * plan.out_seq * (2 * d * e + 4)        # K', V' rows + degree
    work["_fused2_flops"] = flops["fused2_bf16"]
    return work


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config3", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stage", default="all", choices=["all", "match", "compress", "decode", "copy"],
                    help="time only one stage of the path (kernel tuning / profiling); the JSON line is "
                         "the full contract only for 'all'")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the serving-shape context figures (profiling runs: only the step's own launches)")
    ap.add_argument("--seed", type=int, default=2024)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists).",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2506_11418_amd as ckv
    from synth import kv_device

    cfg = WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    Ly, H, Hq, D, S = cfg["layers"], cfg["kv_heads"], cfg["q_heads"], cfg["dim"], cfg["seq"]

    # ---- inputs, resident in HBM --------------------------------------------------------------
    n_sets = 1 if Ly >= 8 else 8          # small workloads rotate over distinct buffers (MALL is 256 MB)
    sets = []
    for i in range(n_sets):
        K = torch.empty((Ly, H, S, D), dtype=torch.bfloat16, device=dev)
        V = torch.empty_like(K)
        for l in range(Ly):
            kv_device(args.seed + i, H, S, D, "bf16", cfg["alpha"], cfg["n_outlier"], layer=l, device=dev,
                      out_k=K[l], out_v=V[l])
        sets.append((K, V))
    gen = torch.Generator(device=dev).manual_seed(args.seed + 99)
    q = torch.randn((Ly, 1, Hq, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)

    lay = ckv.layout_of(sets[0][0])
    params = ckv.make_params(cfg["chunk"], cfg["retain"])
    plan = ckv.plan(lay, params)
    L2 = plan.out_seq
    K_out = torch.empty((Ly, H, L2, D), dtype=torch.bfloat16, device=dev)
    V_out = torch.empty_like(K_out)
    deg_out = torch.empty((Ly, H, L2), dtype=torch.int32, device=dev)
    assign = torch.empty((Ly, H, S), dtype=torch.int32, device=dev)
    ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device=dev)
    attn_lay = ckv.layout_of(K_out[0:1])
    attn_ws = torch.empty(ckv.decode_attn_workspace(attn_lay, Hq), dtype=torch.uint8, device=dev)
    o = torch.empty((Ly, 1, Hq, D), dtype=torch.bfloat16, device=dev)
    if args.stage == "copy":
        K_copy, V_copy = torch.empty_like(sets[0][0]), torch.empty_like(sets[0][1])
        deg_copy = torch.empty((Ly, H, S), dtype=torch.int32, device=dev)
    torch.cuda.synchronize()

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * args.steps)]

    def step(i, timed):
        K, V = sets[i % n_sets]
        if timed:
            ev[3 * i].record()
        if args.stage == "match":
            ckv.match(K, cfg["chunk"])
        elif args.stage == "copy":      # zero rounds: a plain row copy of known size (counter calibration)
            ckv.compress(K, V, cfg["chunk"], retain_ratio=1.0, out=(K_copy, V_copy, deg_copy, assign), workspace=ws)
        elif args.stage != "decode" or i == 0:
            ckv.compress(K, V, cfg["chunk"], retain_ratio=cfg["retain"], out=(K_out, V_out, deg_out, assign),
                         workspace=ws)
        if timed:
            ev[3 * i + 1].record()
        if args.stage in ("all", "decode"):
            for l in range(Ly):
                ckv.decode_attn(q[l], K_out[l:l + 1], V_out[l:l + 1], deg=deg_out[l:l + 1], out=o[l],
                                workspace=attn_ws)
        if timed:
            ev[3 * i + 2].record()

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()

    def kernel_table(ktimes, n_steps):
        """Per-kernel time, achieved rate and roofline fraction from the library's launch events."""
        work = algorithmic_work(cfg, plan, fused="fused2_bf16" in ktimes, deferred="merge_keys_bf16" in ktimes)
        kernels = {}
        for name, (tot_ms, launches) in ktimes.items():
            per_step_ms = tot_ms / n_steps
            ent = {"ms_per_step": round(per_step_ms, 4), "launches_per_step": launches / n_steps,
                   "avg_launch_us": round(tot_ms * 1e3 / max(launches, 1), 2)}
            if name == "match_bf16":
                ach = work[name] / (per_step_ms * 1e-3) / 1e12
                ent.update(bound="mfma", achieved=round(ach, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                           frac=round(ach / PEAK_BF16_TFLOPS, 4))
            elif name in work and work[name] > 0:
                ach = work[name] / (per_step_ms * 1e-3) / 1e9
                ent.update(bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                           frac=round(ach / PEAK_HBM_GBS, 4))
                if name == "fused2_bf16":   # its similarity contractions, as a second reading
                    tf = work["_fused2_flops"] / (per_step_ms * 1e-3) / 1e12
                    ent.update(mfma_TFLOPs=round(tf, 1), mfma_frac=round(tf / PEAK_BF16_TFLOPS, 4))
            kernels[name] = ent
        if args.stage == "match" and "match_bf16" in kernels:      # ckv_match runs the first round only
            one = algorithmic_work(cfg, type(plan)(plan.round_len[1], plan.round_len[:2], plan.round_r[:1], 0), False)
            ach = one["match_bf16"] / (kernels["match_bf16"]["ms_per_step"] * 1e-3) / 1e12
            kernels["match_bf16"].update(achieved=round(ach, 1), frac=round(ach / PEAK_BF16_TFLOPS, 4))
        return kernels, work

    def group_of(k):
        # launches of one kernel function are taken together: the merge kernel's modes (full, keys-only,
        # origin: one template, named apart in the timing only) count as one kernel
        return "merge_kernel (all modes)" if k.startswith("merge_") else k

    # ---- profile pass (untimed): every kernel bracketed by events -> the per-kernel table and the
    # dominant kernel.  Bracketing every launch costs the 32 short attention layers about a quarter of
    # their speed, so the timed region below brackets the dominant kernel only.
    n_profile = 3
    ckv.timing_select(None)
    ckv.timing_reset()
    ckv.timing_enable(True)
    for i in range(n_profile):
        step(i, False)
    torch.cuda.synchronize()
    ckv.timing_enable(False)
    kernels, work = kernel_table(ckv.timing_read(), n_profile)
    groups = {}
    for k in kernels:
        if k in work and "bound" in kernels[k]:
            groups.setdefault(group_of(k), []).append(k)
    dom = max(groups, key=lambda gname: sum(kernels[k]["ms_per_step"] for k in groups[gname])) if groups else None

    # ---- timed region ---------------------------------------------------------------------------
    if dom is not None:
        ckv.timing_select("merge_" if dom.startswith("merge_kernel") else dom)
    ckv.timing_reset()
    ckv.timing_enable(dom is not None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ckv.timing_enable(False)
    ktimes = ckv.timing_read()
    ckv.timing_select(None)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    comp_ms = float(np.mean([ev[3 * i].elapsed_time(ev[3 * i + 1]) for i in range(args.steps)]))
    dec_ms = float(np.mean([ev[3 * i + 1].elapsed_time(ev[3 * i + 2]) for i in range(args.steps)]))

    # ---- roofline of the dominant kernel, from the events of the timed steps ---------------------
    roofline = None
    if dom is not None:
        timed, _ = kernel_table(ktimes, args.steps)
        members = [k for k in groups[dom] if k in timed]
        for k in members:
            kernels[k] = dict(timed[k], measured="timed steps")
        for k in kernels:
            kernels[k].setdefault("measured", f"{n_profile} untimed profile steps")
        t_ms = sum(timed[k]["ms_per_step"] for k in members)
        n_launch = sum(timed[k]["launches_per_step"] for k in members)
        first = timed[members[0]]
        scale = 1e12 if first["bound"] == "mfma" else 1e9
        ach = sum(work[k] for k in members) / (t_ms * 1e-3) / scale
        traffic = [MEASURED_TRAFFIC.get((args.workload, k)) for k in members]
        roofline = {"kernel": dom, "bound": first["bound"], "achieved": round(ach, 1), "peak": first["peak"],
                    "unit": first["unit"], "frac": round(ach / first["peak"], 4),
                    "avg_launch_us": round(t_ms * 1e3 / n_launch, 2),
                    "traffic": None if any(t is None for t in traffic) else int(
                        sum(t * timed[k]["launches_per_step"] for t, k in zip(traffic, members)) / n_launch)}

    # ---- CPU baseline: the oracle as it stands, on a bounded sample ---------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        n_heads = 16
        n_heads = min(n_heads, Ly * H)
        Kh = sets[0][0].reshape(Ly * H, S, D)[:n_heads].to("cpu").to(torch.float64).numpy()
        Vh = sets[0][1].reshape(Ly * H, S, D)[:n_heads].to("cpu").to(torch.float64).numpy()
        qh = torch.randn((n_heads * (Hq // H), D), generator=torch.Generator().manual_seed(args.seed)).to(
            torch.bfloat16).to(torch.float64).numpy()
        c0 = time.perf_counter()
        outs = [oracle.compress(Kh[h], Vh[h], cfg["chunk"], plan.round_r, "bf16") for h in range(n_heads)]
        oracle.app_attn(qh, np.stack([x["K"] for x in outs]), np.stack([x["V"] for x in outs]),
                        np.stack([x["deg"] for x in outs]))
        c1 = time.perf_counter()
        frac_of_model = n_heads / (Ly * H)
        cpu = {"value": round(S * frac_of_model / (c1 - c0), 2), "unit": "tokens/s", "cores": int(cores),
               "kind": "oracle",
               "sample": f"{n_heads} of {Ly * H} (layer, KV head) sequences of {S} tokens: oracle.compress "
                         f"(rounds {plan.round_r}) + oracle.app_attn, {c1 - c0:.1f} s; scaled to whole-model tokens"}

    # ---- context figure: one layer of the batch-16 serving shape ---------------------------------
    # 16 sequences x 8 KV heads x 8192 centroids (32768 tokens at 25%), 32 query heads; kernel time
    # from the library's events.  Not part of `value`.
    serving = None
    if args.stage == "all" and not args.no_context:
        Bs, Ls = 16, 8192
        gK = torch.randn((Bs, H, Ls, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        gV = torch.randn((Bs, H, Ls, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        gq = torch.randn((Bs, Hq, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        gdeg = torch.randint(1, 9, (Bs, H, Ls), generator=gen, device=dev, dtype=torch.int32)
        go = torch.empty_like(gq)
        gws = torch.empty(ckv.decode_attn_workspace(ckv.layout_of(gK), Hq), dtype=torch.uint8, device=dev)
        for _ in range(3):
            ckv.decode_attn(gq, gK, gV, deg=gdeg, out=go, workspace=gws)
        torch.cuda.synchronize()
        ckv.timing_reset()
        ckv.timing_enable(True)
        for _ in range(20):
            ckv.decode_attn(gq, gK, gV, deg=gdeg, out=go, workspace=gws)
        torch.cuda.synchronize()
        ckv.timing_enable(False)
        tt = ckv.timing_read()
        us = tt["attn_partial_bf16"][0] / tt["attn_partial_bf16"][1] * 1e3
        byts = Bs * H * Ls * (2 * D * 2 + 4)
        serving = {"shape": f"batch {Bs} x {H} KV heads x {Ls} centroids x {D}, {Hq} q heads, bf16, one layer",
                   "attn_partial_us": round(us, 2), "GBps": round(byts / us / 1e3, 1),
                   "frac_of_hbm_peak": round(byts / us / 1e3 / PEAK_HBM_GBS, 4),
                   "attn_combine_us": round(tt["attn_combine"][0] / tt["attn_combine"][1] * 1e3, 2)}
        # the same batch attending over UNCOMPRESSED caches of 32768 tokens (degrees NULL): what the
        # compression buys a decode step.  Attention only, one layer; the rest of a model is not here.
        uK = torch.randn((Bs, H, 4 * Ls, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        uV = torch.randn((Bs, H, 4 * Ls, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        uws = torch.empty(ckv.decode_attn_workspace(ckv.layout_of(uK), Hq), dtype=torch.uint8, device=dev)
        for _ in range(2):
            ckv.decode_attn(gq, uK, uV, out=go, workspace=uws)
        torch.cuda.synchronize()
        ckv.timing_reset()
        ckv.timing_enable(True)
        for _ in range(10):
            ckv.decode_attn(gq, uK, uV, out=go, workspace=uws)
        torch.cuda.synchronize()
        ckv.timing_enable(False)
        tu = ckv.timing_read()
        uus = (tu["attn_partial_bf16"][0] / tu["attn_partial_bf16"][1] + tu["attn_combine"][0] / tu["attn_combine"][1]) * 1e3
        cus = us + serving["attn_combine_us"]
        serving["uncompressed_32768_attn_us"] = round(uus, 2)
        serving["attention_only_tokens_per_s_32_layers"] = {"compressed": round(Bs / (32 * cus * 1e-6), 1),
                                                            "uncompressed": round(Bs / (32 * uus * 1e-6), 1)}
        del uK, uV, uws
        ckv.decode_attn(gq, gK, gV, deg=gdeg, out=go, workspace=gws)     # `go` again holds the compressed result
        # the same tokens in a block-paged pool (blocks of 16 tokens, shuffled), read in place
        bs = 16
        nblk = Bs * Ls // bs
        perm = torch.randperm(nblk, generator=gen, device=dev).to(torch.int32)
        table = perm.reshape(Bs, Ls // bs).contiguous()
        idx = table.to(torch.int64)
        K_pool = torch.empty((nblk, H, bs, D), dtype=torch.bfloat16, device=dev)
        V_pool = torch.empty_like(K_pool)
        deg_pool = torch.empty((nblk, H, bs), dtype=torch.int32, device=dev)
        K_pool[idx.flatten()] = gK.reshape(Bs, H, Ls // bs, bs, D).permute(0, 2, 1, 3, 4).reshape(nblk, H, bs, D)
        V_pool[idx.flatten()] = gV.reshape(Bs, H, Ls // bs, bs, D).permute(0, 2, 1, 3, 4).reshape(nblk, H, bs, D)
        deg_pool[idx.flatten()] = gdeg.reshape(Bs, H, Ls // bs, bs).permute(0, 2, 1, 3).reshape(nblk, H, bs)
        plens = torch.full((Bs,), Ls, dtype=torch.int32, device=dev)
        po = torch.empty_like(gq)
        for _ in range(3):
            ckv.paged_decode_attn(gq, K_pool, V_pool, deg_pool, table, plens, Ls, out=po, workspace=gws)
        torch.cuda.synchronize()
        if not torch.equal(po, go):
            raise RuntimeError("paged attention differs from strided attention on the same tokens")
        ckv.timing_reset()
        ckv.timing_enable(True)
        for _ in range(20):
            ckv.paged_decode_attn(gq, K_pool, V_pool, deg_pool, table, plens, Ls, out=po, workspace=gws)
        torch.cuda.synchronize()
        ckv.timing_enable(False)
        tp = ckv.timing_read()
        pus = tp["attn_partial_paged_bf16"][0] / tp["attn_partial_paged_bf16"][1] * 1e3
        serving["paged_block16_attn_partial_us"] = round(pus, 2)
        serving["paged_block16_GBps"] = round(byts / pus / 1e3, 1)
        del K_pool, V_pool, deg_pool
        # in-place compression of a paged cache (gather -> compress -> scatter) against the strided call on
        # the same tokens: 16 sequences x 8 KV heads x 32768 tokens, blocks of 16, retain 25%
        Sp = 32768
        nblk = Bs * Sp // bs
        ptable0 = torch.randperm(nblk, generator=gen, device=dev).to(torch.int32).reshape(Bs, Sp // bs).contiguous()
        K_pool = torch.randn((nblk, H, bs, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        V_pool = torch.randn((nblk, H, bs, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        deg_pool = torch.ones((nblk, H, bs), dtype=torch.int32, device=dev)
        pl = ckv.paged_layout_of(K_pool, ptable0)
        _, _, pbytes = ckv.paged_compress_plan(pl, Sp, ckv.make_params(cfg["chunk"], cfg["retain"]))
        pws = torch.empty(pbytes, dtype=torch.uint8, device=dev)
        sK, sV, _ = ckv.paged_gather(K_pool, V_pool, deg_pool, ptable0, Sp)          # the same tokens, strided
        s_out = ckv.compress(sK, sV, cfg["chunk"], retain_ratio=cfg["retain"], want_assign=False)
        sws = torch.empty(ckv.plan(ckv.layout_of(sK), ckv.make_params(cfg["chunk"], cfg["retain"])).workspace_bytes,
                          dtype=torch.uint8, device=dev)
        times = {}
        for kind in ("paged", "strided"):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            tot = 0.0
            for it in range(4):
                ptable = ptable0.clone()
                deg_pool.fill_(1)
                torch.cuda.synchronize()
                e0.record()
                if kind == "paged":      # the cache is compacted in place: every repetition starts from a fresh table
                    ckv.paged_compress(K_pool, V_pool, deg_pool, ptable, Sp, cfg["chunk"], retain_ratio=cfg["retain"],
                                       workspace=pws)
                else:
                    ckv.compress(sK, sV, cfg["chunk"], retain_ratio=cfg["retain"], want_assign=False,
                                 out=(s_out[0], s_out[1], s_out[2], None), workspace=sws)
                e1.record()
                torch.cuda.synchronize()
                if it > 0:
                    tot += e0.elapsed_time(e1)
            times[kind] = tot / 3
        serving["paged_compress_16x8x32768_ms"] = round(times["paged"], 3)
        serving["strided_compress_16x8x32768_ms"] = round(times["strided"], 3)
        del K_pool, V_pool, deg_pool, sK, sV, s_out, pws, sws
        # What this part's memory system gives a plain read + write stream: the library's row-copy kernel
        # (ckv_compress with no round to run) over the whole input cache, timed the same way.  The merge
        # kernels move the same kind of traffic and are to be read against this, not only against 8 TB/s.
        if Ly * H * S * D * 2 >= (1 << 32):
            Kc, Vc = torch.empty_like(sets[0][0]), torch.empty_like(sets[0][1])
            degc = torch.empty((Ly, H, S), dtype=torch.int32, device=dev)
            for _ in range(2):
                ckv.compress(sets[0][0], sets[0][1], cfg["chunk"], retain_ratio=1.0, out=(Kc, Vc, degc, assign), workspace=ws)
            torch.cuda.synchronize()
            ckv.timing_reset()
            ckv.timing_enable(True)
            for _ in range(5):
                ckv.compress(sets[0][0], sets[0][1], cfg["chunk"], retain_ratio=1.0, out=(Kc, Vc, degc, assign), workspace=ws)
            torch.cuda.synchronize()
            ckv.timing_enable(False)
            tc = ckv.timing_read()
            cp_us = tc["copy_rows"][0] / tc["copy_rows"][1] * 1e3
            cp_bytes = 2 * Ly * H * S * D * 2          # one launch copies K (or V): read + written
            serving["plain_copy_kernel"] = {"GBps": round(cp_bytes / cp_us / 1e3, 1), "us": round(cp_us, 1),
                                            "what": "the library's row-copy kernel, one launch = 8 GiB read + 8 GiB written"}
            del Kc, Vc, degc

    dec_bytes = work["attn_partial_bf16"]
    out = {
        "metric": "KV tokens compressed/sec + decode-attn HBM GB/s (fraction of MI355X peak)",
        "value": round(S / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {cfg['desc']}", "layers": Ly, "kv_heads": H, "q_heads": Hq,
                   "head_dim": D, "seq_len": S, "chunk": cfg["chunk"], "retain_ratio": cfg["retain"],
                   "rounds": plan.round_r, "compressed_len": L2, "parallelism": "1 GPU"},
        "compress_ms": round(comp_ms, 4), "decode_ms": round(dec_ms, 4),
        "compress_tokens_per_s": round(S / (comp_ms * 1e-3), 1),
        "compress_head_tokens_per_s": round(S * Ly * H / (comp_ms * 1e-3), 1),
        "decode_attn_GBps_wall": round(dec_bytes / (dec_ms * 1e-3) / 1e9, 1),
        "roofline": roofline, "kernels": kernels, "decode_serving_layer": serving, "cpu_baseline": cpu,
    }
    if args.stage != "all":
        out["stage"] = args.stage
    print(json.dumps(out))


if __name__ == "__main__":
    main()
