#!/usr/bin/env python3
"""Benchmark of the ESS decode-step hot path on one MI355X.

One "step" = one layer-step: index score -> top-k -> Sparse Memory Pool
look-up / LRU update -> miss fetch from pinned host memory -> sparse MLA decode
(Attn0 / Attn1 / merge), for the whole batch of one layer, through
`ess_decode_step`.  Inputs are synthetic (seeded), resident in HBM / pinned
host memory before the timed region starts; the slot pool is brought to its
steady state by admitting the 32 access-trace sets that precede the decode
steps (LRU-Warmup, Sec. 3.2), whatever --warmup is.

Prints ONE JSON line (see the keys below).  `roofline` is for the dominant
kernel, the index-score key stream; its duration is measured with HIP events
recorded by the library on the launch stream during the timed steps.
`cpu_baseline` times the CPU oracle on a bounded sample of the same workload.
Ratios are formed from one set of steps each: `value`, the roofline and
`misses_per_step` from the timed steps, the stage table and the host-link
rate from the stage pass that follows them.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
HOST_LINK_PEAK_GBS = 64.0    # PCIe Gen5 x16, one direction

# indexer 64 heads x 128 fp8, top-2048, 128 attention heads x 576 bf16 (all workloads)
COMMON = dict(Hi=64, Di=128, k=2048, H=128, qk_max=8, w_levels=8, w_den=16)
WORKLOADS = {
    # name: batch, query tokens, context, per-sequence lengths, slot ratio (None = resident), step-to-step overlap
    "cfg2": dict(cfg=2, B=32, T=1, L=32768, lens=None, ratio=None, rho=None,
                 desc="B32 ctx32768 T1, Latent-Cache resident in HBM"),
    "cfg3": dict(cfg=3, B=64, T=1, L=32768, lens=None, ratio=0.25, rho=0.8,
                 desc="B64 ctx32768 T1, Latent-Cache in pinned host memory, 25% GPU slots, 80% top-k overlap"),
    "cfg4": dict(cfg=4, B=64, T=1, L=131072, lens=(98304, 131072), ratio=0.10, rho=0.7,
                 desc="B64 ctx in [98304,131072] T1, Latent-Cache in pinned host memory, 10% GPU slots, 70% top-k overlap"),
    # multi-token decode over 61 layers run back to back: one step = 61 layer-steps; per layer its own
    # Indexer-Cache, slot pool and cache state; ONE host pool aliased by all layers (61 x 11 GB of pinned
    # memory cannot exist) and one access trace replayed by every layer
    "cfg5": dict(cfg=5, B=128, T=2, L=131072, lens=None, ratio=0.10, rho=0.7, layers=61, fmt="fp8",
                 desc="B128 ctx131072 T2 (causal offset), fp8 e4m3 Latent-Cache entries (656 B) in pinned host memory, "
                      "10% GPU slots, 70% top-k overlap, 61 layers back to back"),
}
# HBM bytes per launch of the index-score kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, keyed by the
# exact workload and flags they were measured on: (workload, overlap, paged, append) -> (bytes per step, source)
MEASURED_TRAFFIC = {
    # (475,444 + 482,774) KiB: FETCH_SIZE x 2.00 + WRITE_SIZE of the two half-batch launches of a split-batch step
    ("cfg4", "auto", False, False): ((475444 + 482774) * 1024, "profiles/pmc_traffic_cfg4.md"),
}
SELECT_FLAGS = 0             # --dense-scores / --fused-select: force one form of stages 1-2 (ESS_FLAG_DENSE_SCORES / _FUSED_SELECT)
ADMIT_SETS = 32              # access-trace sets admitted (untimed) before any decode step: LRU-Warmup, Sec. 3.2


def build_workload(name, steps_needed, overlap="auto", layers=None, rho=None, ratio=None):
    import torch
    from paper_2512_10576_amd import binding as bnd, synth
    wl = dict(WORKLOADS[name]); wl.update(COMMON)
    if rho is not None:
        wl["rho"] = rho
    if ratio is not None:
        wl["ratio"] = ratio
    B, T, L, k, H = wl["B"], wl["T"], wl["L"], wl["k"], wl["H"]
    n_layers = layers if layers is not None else wl.get("layers", 1)
    wl["layers"] = n_layers
    fp8 = wl.get("fmt") == "fp8"
    stride = 656 if fp8 else 1152
    seed = 1000 * wl["cfg"]
    dev = "cuda"
    q_attn = synth.attn_query(seed, B, T, H, device=dev)
    if wl["lens"] is None:
        ctx_len = torch.full((B,), L, dtype=torch.int32, device=dev)
    else:
        ctx_len = synth.ctx_lengths(seed, B, wl["lens"][0], wl["lens"][1], device=dev)
    S = L if wl["ratio"] is None else int(math.ceil(wl["ratio"] * L - 1e-9))
    flags = {"da": 0, "serial": bnd.ESS_FLAG_SERIAL, "dba": bnd.ESS_FLAG_DBA, "auto": bnd.ESS_FLAG_AUTO}[overlap]
    flags |= SELECT_FLAGS
    cfg = bnd.make_config(B, T, L, wl["Hi"], wl["Di"], k, H, latent_fmt=bnd.ESS_FMT_FP8 if fp8 else bnd.ESS_FMT_BF16,
                          row_stride=stride, slots_per_seq=S, flags=flags)
    ctx = bnd.Context(cfg)
    rows = synth.latent_rows_fp8 if fp8 else synth.latent_rows_bf16
    host_pool = None
    if wl["ratio"] is not None:
        host_pool = torch.empty((B, L, stride), dtype=torch.uint8, pin_memory=True)
        for b in range(B):
            host_pool[b].copy_(rows(seed + b, L, device=dev))
        torch.cuda.synchronize()
    q_idx, w, keys, caches = None, None, [], []
    for layer in range(n_layers):                    # seed = 1000 * cfg + layer
        q_idx, w, key = synth.indexer_inputs(seed + layer, B, T, wl["Hi"], wl["Di"], L, wl["qk_max"], wl["w_levels"],
                                             wl["w_den"], device=dev)
        keys.append(key)
        if wl["ratio"] is None:
            pool = torch.empty((B, L, stride), dtype=torch.uint8, device=dev)
            for b in range(B):
                pool[b].copy_(rows(seed + b, L, device=dev))
            cache = bnd.Cache.allocate(cfg, B, slot_pool=pool)
        else:
            cache = bnd.Cache.allocate(cfg, B, host_pool=host_pool)
        ctx.cache_reset(cache, B)
        caches.append(cache)
    trace = None
    if wl["rho"] is not None:
        tr = synth.TopkTrace(seed, ctx_len, T, k, wl["rho"], device=dev)
        trace = [tr.next() for _ in range(steps_needed)]      # set s-1 drives LRU step s (admission or decode step)
    torch.cuda.synchronize()
    return dict(wl=wl, name=name, overlap=overlap, ctx=ctx, cfg=cfg, cache=caches[0], caches=caches, q_idx=q_idx, w=w,
                key=keys[0], keys=keys, q_attn=q_attn, ctx_len=ctx_len, host_pool=host_pool, trace=trace, S=S,
                stride=stride, fmt=1 if fp8 else 0,
                idx_out=torch.empty((B, T, k), dtype=torch.int32, device=dev),
                out=torch.empty((B, T, H, 512), dtype=torch.bfloat16, device=dev),
                lse=torch.empty((B, T, H), dtype=torch.float32, device=dev),
                miss=torch.empty((B,), dtype=torch.int32, device=dev))


def run_steps(W, first_step, n):
    """n steps; a step runs every layer once (one layer-step each), each layer on its own cache and keys"""
    ctx = W["ctx"]
    for i in range(n):
        s = first_step + i
        ov = W["trace"][s - 1] if W["trace"] is not None else None
        for cache, key in zip(W["caches"], W["keys"]):
            ctx.decode_step(cache, W["q_idx"], W["w"], key, W["ctx_len"], W["q_attn"], s, W["idx_out"],
                            W["out"], W["lse"], W["miss"], ov, W.get("block_table"))
            if W.get("append"):                      # the step's new entries enter the caches; the context grows
                ctx.append(cache, W["new_key"], W["new_rows"], key, W["ctx_len"], s)


def algorithmic_bytes(W, misses_per_step):
    """Bytes the method must move per layer-step, by stage."""
    wl = W["wl"]
    lens = W["ctx_len"].cpu().numpy().astype("int64")
    B, T, k, H = wl["B"], wl["T"], wl["k"], wl["H"]
    key_bytes = wl["Di"] + (4 if W.get("paged") else 0)           # paged Indexer-Cache: one float32 scale per key
    a1 = int(lens.sum()) * (key_bytes + 4 * T) + B * T * wl["Hi"] * (wl["Di"] + 4)
    # the emitting form of the kernel (--fused-select) writes no score array: keys and queries only
    a1_emit = int(lens.sum()) * key_bytes + B * T * wl["Hi"] * (wl["Di"] + 4)
    a2 = int(lens.sum()) * 4 * T + B * T * k * 4
    a4 = B * T * k * W["stride"] + B * T * H * (576 * 2 + 512 * 2 + 4)
    fill = int(misses_per_step * W["stride"])
    fused = bool(SELECT_FLAGS & 16) and not (SELECT_FLAGS & 8)
    return dict(index_score=a1, index_in_step=a1_emit if fused else a1, topk=a2, attention_rows=a4, fill=fill)


def warm_slot_pool(W):
    """LRU-Warmup (Sec. 3.2): the ADMIT_SETS access-trace sets that precede the decode steps are admitted to every
    layer's slot pool as LRU steps 1..ADMIT_SETS, so that the pool is in its steady state whatever --warmup is.
    Returns (first decode step number, GB/s of the first admission: every entry a miss, scattered over the pool --
    the rate the fetch kernel reaches on the host link with nothing beside it)."""
    import torch
    if W["trace"] is None:
        return 1, None
    ctx, wl = W["ctx"], W["wl"]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    link = None
    for li, cache in enumerate(W["caches"]):
        for s in range(ADMIT_SETS):
            tok = W["trace"][s].reshape(wl["B"], wl["T"] * wl["k"])
            if li == 0 and s == 0:
                torch.cuda.synchronize()
                e0.record()
            ctx.cache_admit(cache, tok, s + 1)
            if li == 0 and s == 0:
                e1.record()
                torch.cuda.synchronize()
                first = ctx.get_stats()["misses"]
                link = first * W["stride"] / (e0.elapsed_time(e1) * 1e-3) / 1e9
    torch.cuda.synchronize()
    return ADMIT_SETS + 1, link


def _median(xs):
    ys = sorted(xs)
    n = len(ys)
    return ys[n // 2] if n % 2 else 0.5 * (ys[n // 2 - 1] + ys[n // 2])


def measure(name, steps, warmup, overlap="auto", layers=None, rho=None, ratio=None, append=False, paged=False,
            stage_steps=None, alone=True):
    """Timed region: `steps` steps after the slot-pool warm-up and `warmup` untimed steps.  Inside it the index-score
    kernel carries its own start / stop events on at least 16 steps (all of them below 32 steps) and one event per
    step marks the step boundaries (median / min).  A second, untimed pass over the following `stage_steps` steps
    records every stage and reads its own miss count, so that each ratio is formed from one set of steps."""
    import torch
    if stage_steps is None:
        stage_steps = max(16, min(steps, 64))
    n_trace = ADMIT_SETS + warmup + steps + stage_steps
    W = build_workload(name, n_trace, overlap, layers, rho, ratio)
    if append:
        from paper_2512_10576_amd import synth
        assert W["wl"]["layers"] == 1, "--append: one layer (the layers of a workload share ctx_len)"
        wl = W["wl"]
        _, _, nk = synth.indexer_inputs(77, wl["B"], 1, wl["Hi"], wl["Di"], wl["T"], wl["qk_max"], wl["w_levels"],
                                        wl["w_den"], device="cuda")
        rows = synth.latent_rows_fp8 if W["fmt"] == 1 else synth.latent_rows_bf16
        W["new_key"] = nk.contiguous()
        W["new_rows"] = rows(78, wl["B"] * wl["T"], device="cuda").reshape(wl["B"], wl["T"], W["stride"]).contiguous()
        W["append"] = True
    if paged:
        # the same keys in a paged pool (pages of 64 keys + 64 scales in random order, every page of max_ctx mapped)
        assert W["wl"]["layers"] == 1 and not append, "--paged: one layer, fixed context"
        wl = W["wl"]
        B, L, Di = wl["B"], wl["L"], wl["Di"]
        npp = L // 64
        g = torch.Generator(device="cuda").manual_seed(123)
        perm = torch.randperm(B * npp, generator=g, device="cuda")
        pages = torch.empty((B * npp, 64 * (Di + 4)), dtype=torch.uint8, device="cuda")
        pages[perm, : 64 * Di] = W["key"].view(B * npp, 64 * Di)
        scales = (0.5 + torch.rand((B * npp, 64), generator=g, device="cuda")).to(torch.float32)
        pages[perm, 64 * Di:] = scales.view(torch.uint8)
        W["block_table"] = perm.to(torch.int32).view(B, npp).contiguous()
        W["keys"] = [pages]
        W["key"] = pages
        W["paged"] = True
        del scales
    nl = W["wl"]["layers"]
    ctx = W["ctx"]
    first, link_alone = warm_slot_pool(W)
    run_steps(W, first, warmup)
    torch.cuda.synchronize()
    ctx.reset_stats()
    # ---- timed region
    every = max(1, (steps * nl) // 16)
    ctx.profile_enable(steps * nl, stage_mask=0x01, every=every)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    dba_steps = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        run_steps(W, first + warmup + i, 1)
        marks[i + 1].record()
        dba_steps += 1 if ctx.last_overlap() == 1 else 0
    t_enq = time.perf_counter() - t0                 # host time to enqueue the timed steps (no waiting)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the index-score launches of a sampled step one by one (a split-batch step has two: the first with the chip to
    # itself, the second beside the first half's fetch)
    per_launch = {}
    for srec in range(min(steps * nl // every, steps * nl)):
        try:
            iv = [ms for ms, stage in ctx.profile_intervals(srec) if stage == 0]
        except Exception:
            break
        per_launch.setdefault(len(iv), []).append(iv)
    prof_idx = ctx.profile_read()
    stats = ctx.get_stats()
    step_ms = [marks[i].elapsed_time(marks[i + 1]) / nl for i in range(steps)]       # per layer-step
    index_ms = sum(p[0] for p in prof_idx) / len(prof_idx)        # all index-score launches of a sampled layer-step
    launches = 1.0 + dba_steps / steps                            # a split-batch step launches the kernel twice
    misses_timed = stats["misses"] / max(steps * nl, 1)
    # ---- stage pass (untimed for `value`): every stage recorded, its own miss count
    ctx.reset_stats()
    ctx.profile_enable(stage_steps * nl, stage_mask=0x3F)
    run_steps(W, first + warmup + steps, stage_steps)
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    misses_stage = ctx.get_stats()["misses"] / max(stage_steps * nl, 1)
    ctx.profile_enable(0)
    stage = [sum(p[i] for p in prof) / len(prof) for i in range(6)]
    # ---- the index-score kernel by itself on the same inputs (whole batch, nothing running beside it)
    wl = W["wl"]
    index_alone_ms = None
    if alone:
        score = torch.empty((wl["B"], wl["T"], wl["L"]), dtype=torch.float32, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n_alone = 16
        for i in range(3 + n_alone):
            if i == 3:
                e0.record()
            if W.get("paged"):
                ctx.index_score_paged(W["q_idx"], W["w"], W["key"], W["block_table"], W["ctx_len"], score)
            else:
                ctx.index_score(W["q_idx"], W["w"], W["key"], W["ctx_len"], score)
        e1.record()
        torch.cuda.synchronize()
        index_alone_ms = e0.elapsed_time(e1) / n_alone
        del score
    ab = algorithmic_bytes(W, misses_timed)
    ab_stage = algorithmic_bytes(W, misses_stage)
    ms_step = dt / (steps * nl) * 1e3                            # per layer-step
    hbm_stream_bytes = ab["index_in_step"] + ab["topk"] + ab["attention_rows"]
    hbm_stream_ms = stage[0] + stage[1] + stage[3] + stage[4]
    res = dict(
        layer_steps_per_s=steps * nl / dt, ms_per_step=dt / steps * 1e3, ms_per_layer_step=ms_step, layers=nl,
        ms_per_layer_step_median=_median(step_ms), ms_per_layer_step_min=min(step_ms),
        stage_ms=dict(index_score=stage[0], topk=stage[1], bookkeeping=stage[2], attn0=stage[3], attn1_merge=stage[4],
                      fetch=stage[5]),
        stage_steps=stage_steps, misses_per_step_stage_pass=misses_stage,
        index_score_GBs=ab["index_in_step"] / (index_ms * 1e-3) / 1e9, index_ms_timed=index_ms, index_samples=len(prof_idx),
        index_alone_ms=index_alone_ms,
        index_alone_GBs=(ab["index_score"] / (index_alone_ms * 1e-3) / 1e9) if index_alone_ms else None,
        index_launches_per_step=launches,
        index_launch_ms=[sum(x[i] for x in v) / len(v) for n, v in sorted(per_launch.items()) if len(v) * 2 >= sum(len(w) for w in per_launch.values()) for i in range(n)],
        hbm_stream_GBs=hbm_stream_bytes / (hbm_stream_ms * 1e-3) / 1e9,
        hbm_stream_frac_of_peak=hbm_stream_bytes / (hbm_stream_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        whole_step_hbm_frac=(hbm_stream_bytes / (ms_step * 1e-3) / 1e9) / HBM_PEAK_GBS,
        host_enqueue_ms_per_layer_step=t_enq / (steps * nl) * 1e3,
        misses_per_step=misses_timed, overlap_used=("da", "dba", "serial")[ctx.last_overlap()],
        # fetch rate: bytes and time of the same (stage-pass) steps
        host_link_GBs=(ab_stage["fill"] / (stage[5] * 1e-3) / 1e9) if stage[5] > 0 else None,
        host_link_frac_of_peak=(ab_stage["fill"] / (stage[5] * 1e-3) / 1e9 / HOST_LINK_PEAK_GBS) if stage[5] > 0 else None,
        host_link_alone_GBs=link_alone,
        algorithmic_bytes=ab,
    )
    return W, res


def measured_peaks(W):
    """What a plain kernel reaches on this GPU, beside the nominal peaks: a pure read stream and a copy (over the
    workload's index keys, at most 1 GiB)."""
    import torch
    from paper_2512_10576_amd import binding as bnd
    src = W["key"].view(-1)
    n = min(src.numel(), 1 << 30) // 16 * 16
    src = src[:n]
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(bnd.CALIB_READ_WGS, dtype=torch.int32, device="cuda")
    out = {}
    for what in ("read", "copy"):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(2 + 8):
            if i == 2:
                e0.record()
            if what == "read":
                bnd.calib_read(src, sink)
            else:
                bnd.calib_copy(dst, src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 8
        out[what] = n * (1 if what == "read" else 2) / (ms * 1e-3) / 1e9
    del dst
    return out


CPU_BASELINE_STEPS = 4       # about 10-15 s of CPU time for the whole cfg4 batch on 16 cores


def cpu_baseline(W, budget_seqs):
    """The CPU oracle, as it stands, on the first `budget_seqs` sequences of the workload (one step)."""
    import numpy as np
    from oracle import ess_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    wl = W["wl"]
    n = min(budget_seqs, wl["B"])
    q_idx = W["q_idx"][:n].cpu().numpy(); w = W["w"][:n].cpu().numpy(); key = W["key"][:n].cpu().numpy()
    ctx_len = W["ctx_len"][:n].cpu().numpy()
    q_bits = W["q_attn"][:n].view(__import__("torch").int16).cpu().numpy().view(np.uint16)
    L, S = wl["L"], W["S"]
    if W["host_pool"] is not None:
        host = W["host_pool"][:n].numpy()
        cache = O.SlotCache(n, L, S)
        pool = np.zeros((n, S, W["stride"]), np.uint8)
        ovs = [W["trace"][s][:n].cpu().numpy() for s in range(min(CPU_BASELINE_STEPS, len(W["trace"])))]
    else:
        host = None
        cache = O.SlotCache(n, L, L); cache.make_resident_identity()
        pool = W["cache"].slot_pool[:n].cpu().numpy()
        ovs = [None] * CPU_BASELINE_STEPS
    t0 = time.perf_counter()
    for s, ov in enumerate(ovs):                                 # the access trace's first steps, from an empty pool
        O.decode_step(q_idx, w, key, ctx_len, wl["k"], cache, pool, host, q_bits, W["fmt"], 576 ** -0.5, s + 1, ov)
    dt = time.perf_counter() - t0
    return dict(value=len(ovs) / (dt * wl["B"] / n), unit="layer-steps/s", cores=int(threads), kind="oracle",
                sample="%d of %d sequences of %s, the first %d layer-steps of the access trace (the first from an empty "
                       "pool), scaled linearly to the batch; %.1f s of CPU time" % (n, wl["B"], W["name"], len(ovs), dt))


def sweep_overlap(name, steps, warmup):
    """Fetch overlap modes against the miss count (paper Sec. 3.3, the DA / DBA comparison): the step-to-step
    overlap rho of the top-k sets sets the misses per sequence; every mode runs the same traces."""
    import torch
    rows = []
    for rho in (0.98, 0.95, 0.9, 0.8, 0.7, 0.5, 0.3):
        row = {"rho": rho}
        for ov in ("serial", "da", "dba", "auto"):
            W, r = measure(name, steps, warmup, ov, rho=rho)
            row["misses_per_seq"] = r["misses_per_step"] / W["wl"]["B"]
            row[ov + "_ms"] = r["ms_per_layer_step"]
            if ov == "auto":
                row["auto_used"] = r["overlap_used"]
            W["ctx"].close(); del W
            torch.cuda.empty_cache()
        rows.append(row)
        print("rho %.2f misses/seq %.0f serial %.3f da %.3f dba %.3f auto %.3f (%s) ms" % (
            rho, row["misses_per_seq"], row["serial_ms"], row["da_ms"], row["dba_ms"], row["auto_ms"], row["auto_used"]),
            file=sys.stderr, flush=True)
    return rows


def sweep_ratio(name, steps, warmup):
    """Misses and step time against the Sparse Memory Ratio (paper Sec. 3.2 / 4), with the pool warmed by
    `warmup` steps, and the misses of the first steps after a reset with and without LRU-Warmup (the sets of
    32 earlier steps admitted through ess_cache_admit, oldest first)."""
    import torch
    rows = []
    for ratio in (0.05, 0.1, 0.2, 0.3, 0.5, 1.0):
        W, r = measure(name, steps, warmup, "da", ratio=ratio)
        ctx, cache, B = W["ctx"], W["cache"], W["wl"]["B"]
        first = {}
        for mode in ("cold", "lru_warmup"):
            ctx.cache_reset(cache, B)
            if mode == "lru_warmup":
                for s in range(32):
                    ctx.cache_admit(cache, W["trace"][s][:, -1].contiguous(), s + 1)
            torch.cuda.synchronize()
            per_step = []
            for s in range(4):
                ctx.reset_stats()
                run_steps(W, 33 + s, 1)
                per_step.append(ctx.get_stats()["misses"] / B)
            first[mode] = per_step
        rows.append({"ratio": ratio, "slots_per_seq": W["S"], "misses_per_seq": r["misses_per_step"] / B,
                     "ms_per_layer_step": r["ms_per_layer_step"], "fetch_ms": r["stage_ms"]["fetch"],
                     "host_link_GBs": r["host_link_GBs"], "first_steps_cold": first["cold"],
                     "first_steps_lru_warmup": first["lru_warmup"]})
        print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
        ctx.close(); del W
        torch.cuda.empty_cache()
    return rows


def sweep_granularity():
    """Host-to-device rate of scattered Latent-Cache entries (paper Sec. 3.1): one memcpy call per entry
    against the fetch kernel that reads the pinned pool through its device mapping, at both entry sizes."""
    import torch
    from paper_2512_10576_amd import binding as bnd
    rows = []
    B, L, k = 8, 131072, 2048
    g = torch.Generator().manual_seed(7)
    for stride, fmt in ((656, bnd.ESS_FMT_FP8), (1152, bnd.ESS_FMT_BF16)):
        n = B * k
        host = torch.empty((B, L, stride), dtype=torch.uint8, pin_memory=True)
        host.random_(0, 255, generator=g)
        dst = torch.empty((n, stride), dtype=torch.uint8, device="cuda")
        pos = torch.stack([torch.randperm(L, generator=g)[:k] for _ in range(B)])             # [B,k] distinct per sequence
        flat = (pos + torch.arange(B).unsqueeze(1) * L).reshape(-1).to(torch.int64).contiguous()
        for rep in range(2):                                                                   # second pass timed
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            bnd.calib_memcpy_rows(dst, host, flat, stride, stride)
            torch.cuda.synchronize()
            dt_memcpy = time.perf_counter() - t0
        ok = bool((dst.cpu() == host.view(-1, stride)[flat]).all())
        # the fetch kernel on the same entries: an empty slot cache makes every selected entry a miss
        cfg = bnd.make_config(B, 1, L, 64, 128, k, 128, latent_fmt=fmt, row_stride=stride, slots_per_seq=2 * k)
        ctx = bnd.Context(cfg)
        cache = bnd.Cache.allocate(cfg, B, host_pool=host)
        ctx_len = torch.full((B,), L, dtype=torch.int32, device="cuda")
        slot_idx = torch.empty((B, 1, k), dtype=torch.int32, device="cuda")
        idx = pos.to(torch.int32).reshape(B, 1, k).cuda()
        times = []
        for rep in range(3):
            ctx.cache_reset(cache, B)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ctx.gather_latent(cache, idx, ctx_len, 1, slot_idx, None, None)
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t0)
        got = torch.gather(cache.slot_pool.view(B, 2 * k, stride), 1,
                           slot_idx.view(B, k, 1).long().expand(B, k, stride)).reshape(n, stride)
        ok = ok and bool((got.cpu() == host.view(-1, stride)[flat]).all())
        # write-back direction: ess_append of 2 new entries for each of 4096 sequences (stores through the
        # device mapping of the pinned pool), timed over the whole call
        Ba, Ta, La = 4096, 2, 64
        cfg_a = bnd.make_config(Ba, Ta, La, 4, 32, 8, 8, latent_fmt=fmt, row_stride=stride, slots_per_seq=16)
        ctx_a = bnd.Context(cfg_a)
        host_a = torch.zeros((Ba, La, stride), dtype=torch.uint8, pin_memory=True)
        cache_a = bnd.Cache.allocate(cfg_a, Ba, host_pool=host_a)
        ctx_a.cache_reset(cache_a, Ba)
        key_a = torch.zeros((Ba, La, 32), dtype=torch.uint8, device="cuda")
        nk_a = torch.ones((Ba, Ta, 32), dtype=torch.uint8, device="cuda")
        nr_a = torch.empty((Ba, Ta, stride), dtype=torch.uint8, device="cuda").random_(0, 255)
        len_a = torch.zeros((Ba,), dtype=torch.int32, device="cuda")
        t_app = []
        for rep in range(4):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ctx_a.append(cache_a, nk_a, nr_a, key_a, len_a, rep + 1)
            torch.cuda.synchronize()
            t_app.append(time.perf_counter() - t0)
        ok = ok and bool((host_a[:, 6:8] == nr_a.cpu()).all()) and int(len_a.min()) == 8
        d2h = Ba * Ta * stride / min(t_app) / 1e9
        ctx_a.close()
        del host_a, cache_a
        rows.append({"entry_bytes": stride, "entries": n, "memcpy_per_entry_GBs": n * stride / dt_memcpy / 1e9,
                     "append_writeback_GBs": d2h, "append_entries": Ba * Ta,
                     "memcpy_us_per_entry": dt_memcpy / n * 1e6, "fetch_kernel_GBs": n * stride / min(times) / 1e9,
                     "fetch_includes": "bookkeeping kernel + fetch kernel, wall clock", "bytes_verified": ok})
        print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
        ctx.close()
        del host, dst, cache
        torch.cuda.empty_cache()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="cfg4", choices=sorted(WORKLOADS))
    ap.add_argument("--overlap", default="auto", choices=["auto", "da", "dba", "serial"],
                    help="overlap of the miss fetch (paper Sec. 3.3): da = fetch beside Attn0, dba = split batch, auto = the\n"
                         "library picks one of the two per step from the previous step's miss count")
    ap.add_argument("--layers", type=int, default=None, help="layers run back to back per step (default: the workload's)")
    ap.add_argument("--dense-scores", action="store_true",
                    help="index score and top-k always through the full score array (for comparison)")
    ap.add_argument("--fused-select", action="store_true",
                    help="index score and top-k always in the fused form, without a score array (for comparison)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-32k", action="store_true", help="skip the extra 32K-context measurement (cfg2)")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the measurements of the other offloaded configurations (cfg3, cfg5 on 8 layers)")
    ap.add_argument("--cpu-seqs", type=int, default=64, help="sequences of the batch the CPU oracle is timed on")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) so that rocprofv3 --pmc counters can be scaled")
    ap.add_argument("--append", action="store_true",
                    help="after every layer-step write the step's new entries into the caches (ess_append): the context "
                         "grows by T per step (default: context held fixed, as the baseline workload states)")
    ap.add_argument("--paged", action="store_true",
                    help="index keys in a paged pool with one scale per key (pages of 64 keys in random order, 132 bytes "
                         "per key) instead of the flat array")
    ap.add_argument("--sweep", default=None, choices=["overlap", "ratio", "granularity"],
                    help="instead of the benchmark line: overlap = serial / DA / DBA step time against the miss count; "
                         "ratio = misses and step time against the Sparse Memory Ratio, with and without LRU-Warmup; "
                         "granularity = per-entry memcpy against the fetch kernel (prints one JSON object)")
    a = ap.parse_args()
    global SELECT_FLAGS
    SELECT_FLAGS = (8 if a.dense_scores else 0) | (16 if a.fused_select else 0)
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path shards by sequence with no collective); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2512_10576_amd import binding
    binding.load()                                   # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    if a.sweep:
        rows = {"overlap": lambda: sweep_overlap(a.workload, a.steps, a.warmup),
                "ratio": lambda: sweep_ratio(a.workload, a.steps, a.warmup),
                "granularity": sweep_granularity}[a.sweep]()
        print(json.dumps({"sweep": a.sweep, "workload": a.workload, "steps": a.steps, "warmup": a.warmup, "rows": rows}))
        return

    if a.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            binding.calib_copy(dst, src)             # k_calib_copy: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    W, res = measure(a.workload, a.steps, a.warmup, a.overlap, a.layers, append=a.append, paged=a.paged)
    ab = res["algorithmic_bytes"]
    # In the timed region a split-batch (DBA) step launches the kernel twice, once per half of the batch, the second
    # beside the first half's fetch; achieved = bytes of a step / time of its launches, which is also
    # bytes per launch / average launch time.  `alone` is the same kernel on the whole batch with the GPU to itself.
    nlaunch = res["index_launches_per_step"]
    traffic = MEASURED_TRAFFIC.get((a.workload, a.overlap, a.paged, a.append)) if (a.layers is None and SELECT_FLAGS == 0) else None
    roof = dict(bound="hbm", kernel="k_index_score", achieved=res["index_score_GBs"], peak=HBM_PEAK_GBS, unit="GB/s",
                frac=res["index_score_GBs"] / HBM_PEAK_GBS,
                traffic=(traffic[0] / nlaunch) if traffic else None, traffic_source=traffic[1] if traffic else None,
                algorithmic_bytes_per_launch=ab["index_in_step"] / nlaunch, avg_launch_ms=res["index_ms_timed"] / nlaunch,
                launches_per_step=nlaunch, sampled_steps=res["index_samples"],
                per_launch_ms=res["index_launch_ms"],
                per_launch_frac=[ab["index_in_step"] / max(len(res["index_launch_ms"]), 1) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS
                                 for ms in res["index_launch_ms"]],
                alone=dict(achieved=res["index_alone_GBs"], frac=res["index_alone_GBs"] / HBM_PEAK_GBS,
                           algorithmic_bytes_per_launch=ab["index_score"], avg_launch_ms=res["index_alone_ms"]))
    peaks = measured_peaks(W)
    out = {
        "metric": "decode-step sparse-attn layer-steps/sec", "value": res["layer_steps_per_s"], "unit": "layer-steps/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": res["ms_per_step"], "ms_per_layer_step": res["ms_per_layer_step"],
        "ms_per_layer_step_median": res["ms_per_layer_step_median"], "ms_per_layer_step_min": res["ms_per_layer_step_min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp8 indexer / bf16 attention",
        "data": "synthetic",
        "config": {"workload": "%s: %s" % (a.workload, W["wl"]["desc"]), "indexer": "64 heads x 128 fp8 e4m3",
                   "topk": 2048, "attention": "128 heads x 576 bf16 absorbed MLA", "slots_per_seq": W["S"],
                   "overlap": W["overlap"] + (" (ran %s)" % res["overlap_used"] if W["overlap"] == "auto" else ""),
                   "layers_per_step": res["layers"], "q_tokens": W["wl"]["T"],
                   "context": "grows by T per step (ess_append after every step)" if a.append else "fixed",
                   "indexer_cache": "paged, 64 keys + 64 scales per page" if a.paged else "flat",
                   "slot_pool_warmup": ("%d access-trace sets admitted through ess_cache_admit before the %d warm-up steps"
                                        % (ADMIT_SETS, a.warmup)) if W["trace"] is not None else "none (resident)"},
        "roofline": roof,
        "peaks": {"hbm_nominal_GBs": HBM_PEAK_GBS, "hbm_read_measured_GBs": peaks["read"], "hbm_copy_measured_GBs": peaks["copy"],
                  "host_link_nominal_GBs": HOST_LINK_PEAK_GBS, "host_link_measured_GBs": res["host_link_alone_GBs"],
                  "note": "measured = a plain read / copy kernel over the index keys, and the first admission (every entry a "
                          "miss: bookkeeping kernel + fetch kernel, nothing beside them)"},
        "stages": {k: res[k] for k in ("stage_ms", "stage_steps", "misses_per_step_stage_pass", "host_enqueue_ms_per_layer_step",
                                       "hbm_stream_GBs", "hbm_stream_frac_of_peak", "whole_step_hbm_frac",
                                       "misses_per_step", "host_link_GBs", "host_link_frac_of_peak")},
        "paper_context": "simulated whole-model gains of the paper: +69.4% at 32K, +123% at 128K (not comparable)",
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(W, a.cpu_seqs)
    W["ctx"].close()
    del W
    torch.cuda.empty_cache()

    def leg(name, steps, warmup, **kw):
        W2, r2 = measure(name, steps, warmup, alone=False, **kw)
        d = {"workload": "%s: %s" % (name, W2["wl"]["desc"]), "steps": steps, "warmup": warmup, "layers_per_step": r2["layers"],
             "layer_steps_per_s": r2["layer_steps_per_s"], "ms_per_layer_step": r2["ms_per_layer_step"],
             "ms_per_layer_step_median": r2["ms_per_layer_step_median"], "ms_per_layer_step_min": r2["ms_per_layer_step_min"],
             "stage_ms": r2["stage_ms"], "host_enqueue_ms_per_layer_step": r2["host_enqueue_ms_per_layer_step"],
             "index_score_GBs": r2["index_score_GBs"], "hbm_stream_frac_of_peak": r2["hbm_stream_frac_of_peak"],
             "misses_per_step": r2["misses_per_step"], "host_link_GBs": r2["host_link_GBs"],
             "overlap_used": r2["overlap_used"]}
        W2["ctx"].close()
        del W2
        torch.cuda.empty_cache()
        return d

    if not a.no_32k and a.workload != "cfg2":
        # resident workload: nothing to warm in the caches, but a 0.1 ms step needs a few hundred untimed
        # steps before the GPU runs at its steady rate (+2.5 % against 32 of them)
        out["ctx32k"] = leg("cfg2", a.steps, max(a.warmup, 256))
    if not a.no_extra and a.workload == "cfg4" and not (a.append or a.paged):
        # the other named configurations, so that each has a number from this run: 32K context with the
        # Latent-Cache offloaded, and the multi-token configuration on a reduced number of layers (8 of 61, each
        # with its own index keys, slot pool and cache state: 16 GiB of keys, far beyond the Infinity Cache)
        out["ctx32k_offload"] = leg("cfg3", a.steps, a.warmup)
        out["cfg5_8_layers"] = leg("cfg5", max(2, a.steps // 8), 2, layers=8, stage_steps=2)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
