#!/usr/bin/env python3
"""Benchmark of the CentroidKV hot path on one MI355X.

Workloads (--workload), all on synthetic sequence-correlated caches already resident in HBM:
  config3 (default, the headline): full-model prefill compression, 32 layers x 8 KV heads x 128,
      131072 tokens, chunk 1024, retain 25%.  A step = ckv_compress of the whole cache (layers
      folded into the batch dimension) + one GQA decode step over the compressed cache (one
      ckv_decode_attn call per layer, as a model would issue them).  value = context tokens / step time.
  config2: the same on one layer of 32768 tokens (small: launches of a few microseconds).
  config4: serving decode.  16 sequences x 32 layers, each cache compressed beforehand from 32768
      tokens to 8192 centroids; a step = one decoded token per sequence: per layer ckv_append of the
      new (k, v, 1) and ckv_decode_attn over the grown cache; the same loop over the uncompressed
      caches (degrees NULL) is timed beside it.  value = decoded tokens / s, attention path only
      (the rest of a model - projections, MLP, sampling - is not part of this library).
  config5: extreme context.  1 048 576 tokens x 32 layers (128 GiB of K and V), chunk 2048, retain
      25%.  A step = ckv_compress layer by layer (one call per layer; the compressed layers, 32 GiB,
      are kept) + 64 decode steps of 32 ckv_decode_attn calls each.  value = context tokens / step time.

Prints ONE JSON line.  `roofline` describes the kernel with the largest share of GPU time; its launch
durations come from HIP events the library records on the launch stream during the timed steps.
Only that kernel is bracketed there (events around every launch slow short kernels down); `kernels`
lists the same figures for every hot kernel, the others' from a few untimed profile steps (each
entry says which).  `cpu_baseline` is the numpy oracle timed on a bounded sample.
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
METRIC = "KV tokens compressed/sec + decode-attn HBM GB/s (fraction of MI355X peak)"

# HBM bytes per launch of a kernel as rocprofv3 counted them: RECORDED constants, not measured by this
# run.  They come from --pmc FETCH_SIZE / WRITE_SIZE runs (one counter per run), each scaled by what the
# same counter reads for the library's plain row-copy kernel of known size; the runs and the factors are
# in profiles/bench_config3_hbm_traffic.txt.  {(workload, kernel): bytes per launch averaged over the
# launches of one step}.  A kernel without an entry reports null.
RECORDED_TRAFFIC = {
    ("config3", "merge_keys_bf16"): int((4227475.6 * 2.0 + 4489354.7) * 1024),
    ("config3", "merge_origin_bf16"): int((6426238.5 * 2.0 + 4292656.4) * 1024),
    ("config3", "match_bf16"): int((3172450.7 * 2.0 + 98304.0) * 1024),
    ("config3", "attn_bf16"): int((66704.0 * 2.0 + 1080.3) * 1024),
}
TRAFFIC_SOURCE = "profiles/bench_config3_hbm_traffic.txt"

WORKLOADS = {
    "config3": dict(layers=32, kv_heads=8, q_heads=32, dim=128, seq=131072, chunk=1024, retain=0.25,
                    alpha=0.9, n_outlier=4, steps=10, warmup=3,
                    desc="llama3-8b 32Lx8KVx128 bf16, seq 131072, chunk 1024, retain 25% (rounds [1,1]) "
                         "+ 1 GQA decode step (32 q heads) over the compressed cache"),
    "config2": dict(layers=1, kv_heads=8, q_heads=32, dim=128, seq=32768, chunk=1024, retain=0.25,
                    alpha=0.9, n_outlier=4, steps=10, warmup=3,
                    desc="llama3-8b single layer 8KVx128 bf16, seq 32768, chunk 1024, retain 25% + 1 GQA decode step"),
    "config4": dict(layers=32, kv_heads=8, q_heads=32, dim=128, seq=32768, chunk=1024, retain=0.25, batch=16,
                    alpha=0.9, n_outlier=4, steps=128, warmup=8,
                    desc="serving decode: batch 16 x 32 layers x 8KVx128 bf16, caches compressed 32768 -> 8192 "
                         "beforehand, 128 decode steps (append + GQA attention, 32 q heads); uncompressed baseline beside it"),
    "config5": dict(layers=32, kv_heads=8, q_heads=32, dim=128, seq=1048576, chunk=2048, retain=0.25,
                    alpha=0.95, n_outlier=4, steps=2, warmup=1, decode_steps=64,
                    desc="extreme context: 32Lx8KVx128 bf16, seq 1048576 (128 GiB of K and V), chunk 2048, retain 25% "
                         "(rounds [1,1]), compressed layer by layer, + 64 GQA decode steps over the 32 compressed layers"),
}


def match_flops(s_in, c, d):
    """2*|A|*|B|*d per chunk (Table 1's quarter-n-c-d term)."""
    full, tail = divmod(s_in, c)
    return full * 2 * (c // 2) * (c // 2) * d + 2 * ((tail + 1) // 2) * (tail // 2) * d


def algorithmic_work(n_bh, d, c, round_len, round_r, out_seq, deferred):
    """Algorithmic bytes / flops of one compression + one decode step, per kernel (the whole launch
    set of that kernel), for bf16 caches.

    deferred: a round with r = 1 that is followed by another round writes keys and degrees only
    (kernel merge_keys_bf16, which also exports 3 bytes of member lists per token) and the next
    round (merge_origin_bf16) reads its keys and degrees, and every ORIGINAL value row once."""
    e = 2
    work = {"match_bf16": 0.0, "merge_bf16": 0.0, "merge_keys_bf16": 0.0, "merge_origin_bf16": 0.0, "attn_bf16": 0.0}
    origin_len = None       # length of the cache whose values the current round rebuilds from
    J = len(round_r)
    for j in range(J):
        s_in, s_out = round_len[j], round_len[j + 1]
        deg_in = 0 if j == 0 else 4
        full, tail = divmod(s_in, c)
        work["match_bf16"] += n_bh * match_flops(s_in, c, d)
        n_src = full * (c // 2) + (tail + 1) // 2
        if origin_len is not None:      # second round of a deferred pair
            org_deg = 0 if j == 1 else 4
            work["merge_origin_bf16"] += n_bh * (s_in * (d * e + 4 + 4) + n_src * 8 + origin_len * (d * e + org_deg + 3)
                                                 + s_out * (2 * d * e + 4))
            origin_len = None
        elif deferred and j + 1 < J and round_r[j] == 1.0:
            work["merge_keys_bf16"] += n_bh * (s_in * (d * e + deg_in + 4 + 3) + n_src * 8 + s_out * (d * e + 4))
            origin_len = s_in
        else:
            work["merge_bf16"] += n_bh * (s_in * (2 * d * e + deg_in + 4) + n_src * 8 + s_out * (2 * d * e + 4))
    work["attn_bf16"] = n_bh * out_seq * (2 * d * e + 4)        # K', V' rows + degree
    return work


def kernel_table(ktimes, work, n_steps):
    """Per-kernel time, achieved rate and roofline fraction from the library's launch events.
    work: algorithmic flops (match) or bytes (the others) per step for each kernel name."""
    kernels = {}
    for name, (tot_ms, launches) in ktimes.items():
        per_step_ms = tot_ms / n_steps
        ent = {"ms_per_step": round(per_step_ms, 4), "launches_per_step": launches / n_steps,
               "avg_launch_us": round(tot_ms * 1e3 / max(launches, 1), 2)}
        if name == "match_bf16" and work.get(name, 0) > 0:
            ach = work[name] / (per_step_ms * 1e-3) / 1e12
            ent.update(bound="mfma", achieved=round(ach, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                       frac=round(ach / PEAK_BF16_TFLOPS, 4))
        elif work.get(name, 0) > 0:
            ach = work[name] / (per_step_ms * 1e-3) / 1e9
            ent.update(bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                       frac=round(ach / PEAK_HBM_GBS, 4))
        kernels[name] = ent
    return kernels


def group_of(k):
    # launches of one kernel function are taken together: the merge kernel's modes (full, keys-only,
    # origin: one template, named apart in the timing only) count as one kernel
    return "merge_kernel (all modes)" if k.startswith("merge_") else k


def roofline_of(ckv, workload, run_steps, n_steps, work, n_profile=2):
    """Profile pass (every kernel bracketed, untimed), then the timed pass with only the dominant
    kernel bracketed.  run_steps(n, timed) runs n steps and returns their wall time in seconds.
    Returns (seconds of the timed pass, roofline dict, kernels dict)."""
    import torch
    ckv.timing_select(None)
    ckv.timing_reset()
    ckv.timing_enable(True)
    run_steps(n_profile, False)
    torch.cuda.synchronize()
    ckv.timing_enable(False)
    kernels = kernel_table(ckv.timing_read(), work, n_profile)
    groups = {}
    for k in kernels:
        if "bound" in kernels[k]:
            groups.setdefault(group_of(k), []).append(k)
    dom = max(groups, key=lambda gname: sum(kernels[k]["ms_per_step"] for k in groups[gname])) if groups else None
    if dom is not None:
        ckv.timing_select("merge_" if dom.startswith("merge_kernel") else dom)
    ckv.timing_reset()
    ckv.timing_enable(dom is not None)
    secs = run_steps(n_steps, True)
    ckv.timing_enable(False)
    ktimes = ckv.timing_read()
    ckv.timing_select(None)
    roofline = None
    if dom is not None:
        timed = kernel_table(ktimes, work, n_steps)
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
        traffic = [RECORDED_TRAFFIC.get((workload, k)) for k in members]
        have = not any(t is None for t in traffic)
        roofline = {"kernel": dom, "bound": first["bound"], "achieved": round(ach, 1), "peak": first["peak"],
                    "unit": first["unit"], "frac": round(ach / first["peak"], 4),
                    "avg_launch_us": round(t_ms * 1e3 / n_launch, 2),
                    "traffic": int(sum(t * timed[k]["launches_per_step"] for t, k in zip(traffic, members)) / n_launch)
                    if have else None,
                    "traffic_source": f"recorded constant from {TRAFFIC_SOURCE}, not measured by this run" if have else None}
    return secs, roofline, kernels


def mfma_ceiling(ckv):
    """The bf16 MFMA rate this chip sustains when nothing but MFMA instructions run (the library's
    measurement kernel: pseudo-random operands, one workgroup per CU), in TFLOP/s.  Context for the
    similarity kernel's fraction of the nominal peak; not part of any step."""
    out = {}
    for name, mode, waves in (("registers_8_waves", 0, 8), ("registers_4_waves", 0, 4), ("lds_operand_per_2_mfma_8_waves", 1, 8),
                              ("lds_operand_per_4_mfma_4_waves", 2, 4)):
        tf = ckv.mfma_ceiling(mode, waves, 10000) / 1e12
        out[name] = {"TFLOPs": round(tf, 1), "frac_of_nominal_peak": round(tf / PEAK_BF16_TFLOPS, 4)}
    out["what"] = ("bf16 MFMA 32x32x16 only, every CU busy, operands in registers or one fragment read from LDS per 2 / 4 "
                   "MFMAs; the chip lowers its clock under this load, so the nominal 2500 TFLOP/s is not reached by any kernel")
    return out


def blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        return len(os.sched_getaffinity(0))


def base_line(args, cfg, value, ms_per_step, extra_config):
    return {"metric": METRIC, "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": dict({"workload": f"{args.workload}: {cfg['desc']}", "layers": cfg["layers"],
                            "kv_heads": cfg["kv_heads"], "q_heads": cfg["q_heads"], "head_dim": cfg["dim"],
                            "seq_len": cfg["seq"], "chunk": cfg["chunk"], "retain_ratio": cfg["retain"],
                            "parallelism": "1 GPU"}, **extra_config)}


# ---------------------------------------------------------------------------------------------------
# config3 / config2: prefill compression + one decode step
# ---------------------------------------------------------------------------------------------------
def run_prefill(args, cfg):
    import numpy as np
    import torch

    import paper_2506_11418_amd as ckv
    from synth import kv_device

    dev = torch.device("cuda:0")
    Ly, H, Hq, D, S = cfg["layers"], cfg["kv_heads"], cfg["q_heads"], cfg["dim"], cfg["seq"]
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
    params = ckv.make_params(cfg["chunk"], cfg["retain"], route=args.route)
    plan = ckv.plan(lay, params)
    L2 = plan.out_seq
    K_out = torch.empty((Ly, H, L2, D), dtype=torch.bfloat16, device=dev)
    V_out = torch.empty_like(K_out)
    deg_out = torch.empty((Ly, H, L2), dtype=torch.int32, device=dev)
    assign = torch.empty((Ly, H, S), dtype=torch.int32, device=dev)
    ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device=dev)
    attn_lay = ckv.layout_of(K_out[0:1])
    attn_ws = torch.zeros(ckv.decode_attn_workspace(attn_lay, Hq), dtype=torch.uint8, device=dev)
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
                         workspace=ws, route=args.route)
        if timed:
            ev[3 * i + 1].record()
        if args.stage in ("all", "decode"):
            for l in range(Ly):
                ckv.decode_attn(q[l], K_out[l:l + 1], V_out[l:l + 1], deg=deg_out[l:l + 1], out=o[l],
                                workspace=attn_ws)
        if timed:
            ev[3 * i + 2].record()

    def run_steps(n, timed):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            step(i, timed)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    run_steps(args.warmup, False)
    ckv.timing_reset()
    ckv.timing_enable(True)
    step(0, False)
    torch.cuda.synchronize()
    ckv.timing_enable(False)
    deferred = "merge_keys_bf16" in ckv.timing_read()
    work = algorithmic_work(Ly * H, D, cfg["chunk"], plan.round_len, plan.round_r, plan.out_seq, deferred)
    if args.stage == "match":       # ckv_match runs the first round only
        work["match_bf16"] = Ly * H * match_flops(S, cfg["chunk"], D)
    secs, roofline, kernels = roofline_of(ckv, args.workload, run_steps, args.steps, work, n_profile=3)
    ms_per_step = secs * 1e3 / args.steps
    comp_ms = float(np.mean([ev[3 * i].elapsed_time(ev[3 * i + 1]) for i in range(args.steps)]))
    dec_ms = float(np.mean([ev[3 * i + 1].elapsed_time(ev[3 * i + 2]) for i in range(args.steps)]))

    # ---- CPU baseline: the oracle as it stands, on a bounded sample ---------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_heads = min(16, Ly * H)
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
        cpu = {"value": round(S * frac_of_model / (c1 - c0), 2), "unit": "tokens/s", "cores": int(blas_threads()),
               "kind": "oracle",
               "sample": f"{n_heads} of {Ly * H} (layer, KV head) sequences of {S} tokens: oracle.compress "
                         f"(rounds {plan.round_r}) + oracle.app_attn, {c1 - c0:.1f} s; scaled to whole-model tokens"}

    context = None
    if args.stage == "all" and not args.no_context:
        context = context_figures(ckv, cfg, sets, assign, ws, gen, dev)
    if args.stage in ("all", "match") and not args.no_context:
        context = dict(context or {}, mfma_ceiling_measured=mfma_ceiling(ckv))
        best = max(v["TFLOPs"] for v in context["mfma_ceiling_measured"].values() if isinstance(v, dict))
        if "match_bf16" in kernels and "achieved" in kernels["match_bf16"]:
            kernels["match_bf16"]["frac_of_measured_mfma_ceiling"] = round(kernels["match_bf16"]["achieved"] / best, 4)

    out = base_line(args, cfg, S / (ms_per_step * 1e-3), ms_per_step,
                    {"rounds": plan.round_r, "compressed_len": L2})
    out.update({"compress_ms": round(comp_ms, 4), "decode_ms": round(dec_ms, 4),
                "compress_tokens_per_s": round(S / (comp_ms * 1e-3), 1) if comp_ms > 0 else None,
                "compress_head_tokens_per_s": round(S * Ly * H / (comp_ms * 1e-3), 1) if comp_ms > 0 else None,
                "decode_attn_GBps_wall": round(work["attn_bf16"] / (dec_ms * 1e-3) / 1e9, 1) if dec_ms > 0 else None,
                "roofline": roofline, "kernels": kernels, "context": context, "cpu_baseline": cpu})
    if args.stage != "all":
        out["stage"] = args.stage
    return out


def context_figures(ckv, cfg, sets, assign, ws, gen, dev):
    """Figures beside the headline, not part of `value`: the same tokens in a block-paged pool read in
    place, in-place compression of a paged cache against the strided call, and what the memory system
    gives a plain read + write stream of the same size (the library's row-copy kernel)."""
    import torch
    H, Hq, D, Ly, S = cfg["kv_heads"], cfg["q_heads"], cfg["dim"], cfg["layers"], cfg["seq"]
    ctx = {}
    Bs, Ls, bs = 16, 8192, 16
    gK = torch.randn((Bs, H, Ls, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    gV = torch.randn((Bs, H, Ls, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    gq = torch.randn((Bs, Hq, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    gdeg = torch.randint(1, 9, (Bs, H, Ls), generator=gen, device=dev, dtype=torch.int32)
    go, po = torch.empty_like(gq), torch.empty_like(gq)
    gws = torch.zeros(ckv.decode_attn_workspace(ckv.layout_of(gK), Hq), dtype=torch.uint8, device=dev)
    nblk = Bs * Ls // bs
    table = torch.randperm(nblk, generator=gen, device=dev).to(torch.int32).reshape(Bs, Ls // bs).contiguous()
    idx = table.to(torch.int64).flatten()
    K_pool = torch.empty((nblk, H, bs, D), dtype=torch.bfloat16, device=dev)
    V_pool = torch.empty_like(K_pool)
    deg_pool = torch.empty((nblk, H, bs), dtype=torch.int32, device=dev)
    K_pool[idx] = gK.reshape(Bs, H, Ls // bs, bs, D).permute(0, 2, 1, 3, 4).reshape(nblk, H, bs, D)
    V_pool[idx] = gV.reshape(Bs, H, Ls // bs, bs, D).permute(0, 2, 1, 3, 4).reshape(nblk, H, bs, D)
    deg_pool[idx] = gdeg.reshape(Bs, H, Ls // bs, bs).permute(0, 2, 1, 3).reshape(nblk, H, bs)
    plens = torch.full((Bs,), Ls, dtype=torch.int32, device=dev)
    byts = Bs * H * Ls * (2 * D * 2 + 4)
    res = {}
    for kind in ("strided", "paged"):
        call = (lambda: ckv.decode_attn(gq, gK, gV, deg=gdeg, out=go, workspace=gws)) if kind == "strided" else \
               (lambda: ckv.paged_decode_attn(gq, K_pool, V_pool, deg_pool, table, plens, Ls, out=po, workspace=gws))
        for _ in range(3):
            call()
        torch.cuda.synchronize()
        ckv.timing_reset()
        ckv.timing_enable(True)
        for _ in range(20):
            call()
        torch.cuda.synchronize()
        ckv.timing_enable(False)
        tt = ckv.timing_read()
        name = "attn_bf16" if kind == "strided" else "attn_paged_bf16"
        us = tt[name][0] / tt[name][1] * 1e3
        res[kind] = {"us": round(us, 2), "GBps": round(byts / us / 1e3, 1),
                     "frac_of_hbm_peak": round(byts / us / 1e3 / PEAK_HBM_GBS, 4)}
    if not torch.equal(po, go):
        raise RuntimeError("paged attention differs from strided attention on the same tokens")
    ctx["decode_layer_batch16"] = {"shape": f"batch {Bs} x {H} KV heads x {Ls} centroids x {D}, {Hq} q heads, bf16, one layer",
                                   "strided": res["strided"], "paged_block16": res["paged"]}
    del K_pool, V_pool, deg_pool, gK, gV
    # in-place compression of a paged cache against the strided call on the same tokens:
    # 16 sequences x 8 KV heads x 32768 tokens, blocks of 16, retain 25%
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
    ctx["paged_compress_16x8x32768_ms"] = round(times["paged"], 3)
    ctx["strided_compress_16x8x32768_ms"] = round(times["strided"], 3)
    del K_pool, V_pool, deg_pool, sK, sV, s_out, pws, sws
    # the paper's own hyper-parameters (Sec. 6.1: chunk 256, 16 sinks, 64 recents, fractions annealed from
    # 0.8 by 0.2; the floor of the schedule, which the paper leaves open, at 0.2) on 8 of the workload's layers
    if Ly >= 8:
        pK, pV = sets[0][0][:8], sets[0][1][:8]
        sched = ckv.schedule_annealed(S, 256, int(cfg["retain"] * S), 0.8, 0.2, 0.2, 16, 64)
        kwp = dict(rounds=sched, n_sink=16, n_recent=64)
        pplan = ckv.plan(ckv.layout_of(pK), ckv.make_params(256, **kwp))
        pout = (torch.empty((8, H, pplan.out_seq, D), dtype=torch.bfloat16, device=dev),
                torch.empty((8, H, pplan.out_seq, D), dtype=torch.bfloat16, device=dev),
                torch.empty((8, H, pplan.out_seq), dtype=torch.int32, device=dev), None)
        pws2 = torch.empty(max(pplan.workspace_bytes, 256), dtype=torch.uint8, device=dev)
        for _ in range(2):
            ckv.compress(pK, pV, 256, out=pout, workspace=pws2, want_assign=False, **kwp)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            ckv.compress(pK, pV, 256, out=pout, workspace=pws2, want_assign=False, **kwp)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        ctx["paper_default_setup"] = {"what": f"8 layers x {H} KV heads x {S} tokens, chunk 256, 16 sinks, 64 recents, "
                                              f"annealed fractions {[round(float(r), 2) for r in sched]} -> {pplan.out_seq} tokens",
                                      "ms": round(ms, 3), "model_tokens_per_s": round(S / (ms * 4) * 1e3, 1)}
        del pout, pws2
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
        ctx["plain_copy_kernel"] = {"GBps": round(cp_bytes / cp_us / 1e3, 1), "us": round(cp_us, 1),
                                    "what": "the library's row-copy kernel, one launch = 8 GiB read + 8 GiB written"}
    return ctx


# ---------------------------------------------------------------------------------------------------
# config4: serving decode over pre-compressed caches, uncompressed baseline beside it
# ---------------------------------------------------------------------------------------------------
def run_serving(args, cfg):
    import torch

    import paper_2506_11418_amd as ckv
    from synth import kv_device

    dev = torch.device("cuda:0")
    Ly, H, Hq, D, S, B = cfg["layers"], cfg["kv_heads"], cfg["q_heads"], cfg["dim"], cfg["seq"], cfg["batch"]
    n_new = args.steps + args.warmup + 2                 # room for every appended token of a pass
    params = ckv.make_params(cfg["chunk"], cfg["retain"])
    L2 = ckv.plan(ckv.Layout(B, H, S, D, H * S * D, S * D, D, ckv.BF16, 0), params).out_seq
    cap_c, cap_u = L2 + n_new, S + n_new
    cK = torch.empty((Ly, B, H, cap_c, D), dtype=torch.bfloat16, device=dev)
    cV = torch.empty_like(cK)
    cdeg = torch.ones((Ly, B, H, cap_c), dtype=torch.int32, device=dev)
    uK = torch.empty((Ly, B, H, cap_u, D), dtype=torch.bfloat16, device=dev)       # the uncompressed baseline's caches
    uV = torch.empty_like(uK)
    for l in range(Ly):
        for b in range(B):      # 16 distinct sequences per layer
            kv_device(args.seed + 1000 * b, H, S, D, "bf16", cfg["alpha"], cfg["n_outlier"], layer=l, device=dev,
                      out_k=uK[l, b, :, :S], out_v=uV[l, b, :, :S])
        ckv.compress(uK[l, :, :, :S], uV[l, :, :, :S], cfg["chunk"], retain_ratio=cfg["retain"], want_assign=False,
                     out=(cK[l], cV[l], cdeg[l], None))
    gen = torch.Generator(device=dev).manual_seed(args.seed + 99)
    n_rot = 8                                             # fresh queries / new tokens per step, rotating over 8 sets
    q = torch.randn((n_rot, Ly, B, Hq, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k_new = torch.randn((n_rot, Ly, B, H, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v_new = torch.randn((n_rot, Ly, B, H, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    o = torch.empty((Ly, B, Hq, D), dtype=torch.bfloat16, device=dev)
    lens_c = torch.empty((Ly, B), dtype=torch.int32, device=dev)
    lens_u = torch.empty((Ly, B), dtype=torch.int32, device=dev)
    ws_c = torch.zeros(ckv.decode_attn_workspace(ckv.layout_of(cK[0], cdeg[0]), Hq), dtype=torch.uint8, device=dev)
    ws_u = torch.zeros(ckv.decode_attn_workspace(ckv.layout_of(uK[0]), Hq), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()

    def decode_step(i, compressed):
        r = i % n_rot
        for l in range(Ly):
            if compressed:
                ckv.append(k_new[r, l], v_new[r, l], cK[l], cV[l], cdeg[l], lens=lens_c[l])
                ckv.decode_attn(q[r, l], cK[l], cV[l], lens=lens_c[l], deg=cdeg[l], out=o[l], workspace=ws_c)
            else:
                ckv.append(k_new[r, l], v_new[r, l], uK[l], uV[l], None, lens=lens_u[l])
                ckv.decode_attn(q[r, l], uK[l], uV[l], lens=lens_u[l], out=o[l], workspace=ws_u)

    def make_runner(compressed):
        def run_steps(n, timed):
            (lens_c if compressed else lens_u).fill_(L2 if compressed else S)     # every pass starts from the prefill state
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(n):
                decode_step(i, compressed)
            torch.cuda.synchronize()
            return time.perf_counter() - t0
        return run_steps

    # bytes one decode step must read at the middle of a pass (the caches grow by one row per step)
    work_c = {"attn_bf16": Ly * B * H * (L2 + (args.steps + 1) / 2) * (2 * D * 2 + 4)}
    run_c, run_u = make_runner(True), make_runner(False)
    run_c(args.warmup, False)
    secs, roofline, kernels = roofline_of(ckv, args.workload, run_c, args.steps, work_c)
    ms_per_step = secs * 1e3 / args.steps
    run_u(min(args.warmup, 2), False)
    n_u = max(args.steps // 4, 1)                         # the baseline moves 4x the bytes: a quarter of the steps
    work_u = {"attn_bf16": Ly * B * H * (S + (n_u + 1) / 2) * (2 * D * 2)}
    secs_u, roof_u, kern_u = roofline_of(ckv, args.workload, run_u, n_u, work_u)
    ms_u = secs_u * 1e3 / n_u

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        nb = 2      # sequences of one layer
        Kh = cK[0, :nb, :, :L2].to("cpu").to(torch.float64).numpy()
        Vh = cV[0, :nb, :, :L2].to("cpu").to(torch.float64).numpy()
        dh = cdeg[0, :nb, :, :L2].to("cpu").to(torch.int64).numpy()
        qh = q[0, 0, :nb].to("cpu").to(torch.float64).numpy()
        reps = 8
        c0 = time.perf_counter()
        for _ in range(reps):
            for b in range(nb):
                oracle.app_attn(qh[b], Kh[b], Vh[b], dh[b])
        c1 = time.perf_counter()
        per_seq_layer = (c1 - c0) / (reps * nb)
        cpu = {"value": round(1.0 / (per_seq_layer * Ly), 3), "unit": "tokens/s", "cores": int(blas_threads()),
               "kind": "oracle",
               "sample": f"oracle.app_attn over {nb} of {B} sequences of one layer ({H} KV heads x {L2} centroids, {Hq} q "
                         f"heads), {reps} repetitions, {c1 - c0:.1f} s; scaled to {Ly} layers per decoded token"}

    out = base_line(args, cfg, B / (ms_per_step * 1e-3), ms_per_step,
                    {"batch": B, "compressed_len": L2, "value_is": "decoded tokens per second, attention path only "
                     "(per layer: cache append + GQA attention); the rest of a model is not part of this library"})
    out.update({"decode_ms": round(ms_per_step, 4),
                "decode_attn_GBps_wall": round(work_c["attn_bf16"] / (ms_per_step * 1e-3) / 1e9, 1),
                "uncompressed_baseline": {"ms_per_step": round(ms_u, 4), "tokens_per_s": round(B / (ms_u * 1e-3), 1),
                                          "steps": n_u,
                                          "decode_attn_GBps_wall": round(work_u["attn_bf16"] / (ms_u * 1e-3) / 1e9, 1),
                                          "roofline": roof_u, "kernels": kern_u},
                "speedup_vs_uncompressed": round(ms_u / ms_per_step, 3),
                "roofline": roofline, "kernels": kernels, "cpu_baseline": cpu})
    return out


# ---------------------------------------------------------------------------------------------------
# config5: 1M-token context, compressed layer by layer, then 64 decode steps
# ---------------------------------------------------------------------------------------------------
def run_extreme(args, cfg):
    import numpy as np
    import torch

    import paper_2506_11418_amd as ckv
    from synth import kv_device

    dev = torch.device("cuda:0")
    Ly, H, Hq, D, S = cfg["layers"], cfg["kv_heads"], cfg["q_heads"], cfg["dim"], cfg["seq"]
    n_dec = cfg["decode_steps"]
    K = torch.empty((Ly, H, S, D), dtype=torch.bfloat16, device=dev)       # 64 GiB
    V = torch.empty_like(K)
    for l in range(Ly):
        kv_device(args.seed, H, S, D, "bf16", cfg["alpha"], cfg["n_outlier"], layer=l, device=dev, out_k=K[l], out_v=V[l])
    params = ckv.make_params(cfg["chunk"], cfg["retain"])
    plan = ckv.plan(ckv.layout_of(K[0:1]), params)
    L2 = plan.out_seq
    cK = torch.empty((Ly, H, L2, D), dtype=torch.bfloat16, device=dev)     # the compressed layers are kept: 16 GiB + 16 GiB
    cV = torch.empty_like(cK)
    cdeg = torch.empty((Ly, H, L2), dtype=torch.int32, device=dev)
    assign = torch.empty((1, H, S), dtype=torch.int32, device=dev)          # one layer's map, reused
    ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device=dev)
    gen = torch.Generator(device=dev).manual_seed(args.seed + 99)
    q = torch.randn((8, Ly, 1, Hq, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    o = torch.empty((Ly, 1, Hq, D), dtype=torch.bfloat16, device=dev)
    attn_ws = torch.zeros(ckv.decode_attn_workspace(ckv.layout_of(cK[0:1]), Hq), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3 * args.steps)]

    def step(i, timed):
        if timed:
            ev[3 * i].record()
        for l in range(Ly):       # one call per layer, as a layer-streamed prefill would issue them
            ckv.compress(K[l:l + 1], V[l:l + 1], cfg["chunk"], retain_ratio=cfg["retain"],
                         out=(cK[l:l + 1], cV[l:l + 1], cdeg[l:l + 1], assign), workspace=ws)
        if timed:
            ev[3 * i + 1].record()
        for t in range(n_dec):
            for l in range(Ly):
                ckv.decode_attn(q[t % 8, l], cK[l:l + 1], cV[l:l + 1], deg=cdeg[l:l + 1], out=o[l], workspace=attn_ws)
        if timed:
            ev[3 * i + 2].record()

    def run_steps(n, timed):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            step(i, timed)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    run_steps(args.warmup, False)
    work = algorithmic_work(Ly * H, D, cfg["chunk"], plan.round_len, plan.round_r, plan.out_seq, deferred=True)
    work["attn_bf16"] *= n_dec
    secs, roofline, kernels = roofline_of(ckv, args.workload, run_steps, args.steps, work, n_profile=1)
    ms_per_step = secs * 1e3 / args.steps
    comp_ms = float(np.mean([ev[3 * i].elapsed_time(ev[3 * i + 1]) for i in range(args.steps)]))
    dec_ms = float(np.mean([ev[3 * i + 1].elapsed_time(ev[3 * i + 2]) for i in range(args.steps)]))

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        Ss = 131072                       # a 64-chunk prefix of one (layer, head) sequence
        Kh = K[0, 0, :Ss].to("cpu").to(torch.float64).numpy()
        Vh = V[0, 0, :Ss].to("cpu").to(torch.float64).numpy()
        qh = q[0, 0, 0, :Hq // H].to("cpu").to(torch.float64).numpy()
        c0 = time.perf_counter()
        res = oracle.compress(Kh, Vh, cfg["chunk"], plan.round_r, "bf16")
        c1 = time.perf_counter()
        for _ in range(4):
            oracle.app_attn(qh, res["K"][None], res["V"][None], res["deg"][None])
        c2 = time.perf_counter()
        # one step of the workload = every (layer, head) sequence compressed once + n_dec decode steps over it
        per_seq = (c1 - c0) * (S / Ss) + (c2 - c1) / 4 * (S / Ss) * n_dec
        cpu = {"value": round(S / (per_seq * Ly * H), 3), "unit": "tokens/s", "cores": int(blas_threads()),
               "kind": "oracle",
               "sample": f"a {Ss}-token prefix of 1 of {Ly * H} (layer, KV head) sequences: oracle.compress (chunk "
                         f"{cfg['chunk']}, rounds {plan.round_r}) {c1 - c0:.1f} s + 4 x oracle.app_attn {c2 - c1:.1f} s; "
                         f"scaled to {S} tokens, {Ly * H} sequences and {n_dec} decode steps"}

    out = base_line(args, cfg, S / (ms_per_step * 1e-3), ms_per_step,
                    {"rounds": plan.round_r, "compressed_len": L2, "decode_steps_per_step": n_dec,
                     "compress_calls": "one ckv_compress per layer (layer-streamed)"})
    out.update({"compress_ms": round(comp_ms, 4), "decode_ms": round(dec_ms, 4),
                "decode_ms_per_token": round(dec_ms / n_dec, 4),
                "compress_tokens_per_s": round(S / (comp_ms * 1e-3), 1),
                "compress_head_tokens_per_s": round(S * Ly * H / (comp_ms * 1e-3), 1),
                "decode_attn_GBps_wall": round(work["attn_bf16"] / (dec_ms * 1e-3) / 1e9, 1),
                "decode_tokens_per_s_attention_only": round(n_dec / (dec_ms * 1e-3), 2),
                "roofline": roofline, "kernels": kernels, "cpu_baseline": cpu})
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="default: the workload's own (config4: its 128 decode steps)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="config3", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stage", default="all", choices=["all", "match", "compress", "decode", "copy"],
                    help="config2/config3 only: time one stage of the path (kernel tuning / profiling); the JSON "
                         "line is the full contract only for 'all'")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the context figures (profiling runs: only the step's own launches)")
    ap.add_argument("--seed", type=int, default=2024)
    ap.add_argument("--route", default=None, choices=["full_rounds", "defer_always"],
                    help="config3 only: force one of the library's bit-identical kernel routes (default: the library chooses)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists).",
              file=sys.stderr)
        sys.exit(2)
    cfg = WORKLOADS[args.workload]
    if args.steps is None:
        args.steps = cfg["steps"]
    if args.warmup is None:
        args.warmup = cfg["warmup"]
    import torch
    torch.cuda.set_device(torch.device("cuda:0"))
    if args.workload == "config4":
        out = run_serving(args, cfg)
    elif args.workload == "config5":
        out = run_extreme(args, cfg)
    else:
        out = run_prefill(args, cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
