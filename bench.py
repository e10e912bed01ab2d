#!/usr/bin/env python3
"""Benchmark of the visual-token-reduction path (score + select + gather) on one MI355X.

A step is one covspec_reduce call over one batch of a synthetic workload whose inputs are
already resident in HBM.  Prints ONE JSON line: images/sec, the roofline position of the
dominant kernel (stage times measured live with HIP events recorded by the library on the
work stream), the CPU oracle timed on a bounded sample of the same workload, and images/sec of
every workload in both pipelines.
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

# MI355X published peaks
PEAK = {"hbm_GBps": 8000.0, "mfma_bf16_TFLOPs": 2500.0, "mfma_fp64_TFLOPs": 78.6, "valu_fp64_TFLOPs": 78.6}

PROFILES = os.path.join(ROOT, "profiles")
COUNTER_FILES = {"reduce5": "reduce_workload5_paper_hbm_counters.txt", "vocab": "verify_draft_s64_l8_v151936_hbm_counters.txt"}


def counter_traffic(which, kernels):
    """Bytes per launch that crossed the L2 <-> memory-fabric boundary for the kernels named (summed), read from the
    tracked rocprofv3 --pmc summary under profiles/ (FETCH_SIZE and WRITE_SIZE in KiB per launch, each scaled by the
    factor the summary's calibration line states for a plain copy of known size).  `kernels` are the names as the
    profiler prints them (matched as prefixes of a table row).  None when the file, the calibration or one of the
    kernels is missing: a summary that no longer covers the kernel that runs gives no figure rather than a stale one."""
    import re
    try:
        text = open(os.path.join(PROFILES, COUNTER_FILES[which])).read()
    except OSError:
        return None
    cal = re.search(r"FETCH_SIZE\[KiB\] \* 1024 \* (\d+\.\d+).*?WRITE_SIZE\[KiB\] \* 1024 \* (\d+\.\d+)", text, re.S)
    if not cal:
        return None
    f_fetch, f_write = float(cal.group(1)), float(cal.group(2))
    total = 0.0
    for k in kernels:
        row = re.search(r"^" + re.escape(k) + r"[^\n]*?\s{2,}(\d+)\s+(\d+)\s+(\d+)\s", text, re.M)
        if not row:
            return None
        total += int(row.group(2)) * 1024 * f_fetch + int(row.group(3)) * 1024 * f_write
    return total


def _params(C, w, rel, lr):
    return C.Params(batch=w.batch, n_tokens=w.n_tokens, d_model=w.d_model, n_query=w.n_query, n_heads=w.n_heads,
                    n_act_layers=w.n_act_layers, dtype=w.dtype, rel_mode=rel, lr_mode=lr, preselect_m=w.preselect_m,
                    rank_r=w.rank_r, keep_k=w.keep_k, lam=w.lam)


def _upload(batch, dtype):
    import numpy as np
    import torch
    import covspec_inputs as I
    out = {}
    for k, v in batch.items():
        if dtype == I.BF16:
            out[k] = torch.from_numpy(np.ascontiguousarray(v).view(np.int16)).cuda().view(torch.bfloat16)
        else:
            out[k] = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).cuda()
    return out


def _gen(w, workers=16):
    from concurrent.futures import ThreadPoolExecutor
    import numpy as np
    import covspec_inputs as I
    with ThreadPoolExecutor(max_workers=min(workers, w.batch)) as ex:
        per = list(ex.map(lambda b: I.make_image(w, b), range(w.batch)))
    out = {k: np.stack([p[k] for p in per]) for k in ("X", "Q", "hidden")}
    out.update(I.make_weights(w))
    return out


def _wname(w):
    return "%d:%s B=%d N=%d d=%d T=%d H=%d K=%d k=%d M=%d r=%d" % (
        w.cid, w.name, w.batch, w.n_tokens, w.d_model, w.n_query, w.n_heads, w.n_act_layers, w.keep_k, w.preselect_m, w.rank_r)


def time_reduce(C, p, dev, ws, steps, warmup, both=False):
    """ms per step of covspec_reduce over K steps bracketed by synchronisation: the median of the per-call times
    between HIP events recorded on the work stream before every call and after the last.  With `both`, also the
    wall-clock mean over the same K steps (returned second)."""
    import statistics
    import torch
    k, _, _ = C.resolve(p)
    idx = torch.empty(p.batch, k, dtype=torch.int32, device="cuda")
    tok = torch.empty(p.batch, k, p.d_model, dtype=dev["X"].dtype, device="cuda")
    args = (p, dev["X"], dev["hidden"], dev["Q"], dev["Wq"], dev["Wk"])
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    for _ in range(warmup):
        C.reduce(*args, workspace=ws, idx_out=idx, tokens_out=tok)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        ev[i].record()
        C.reduce(*args, workspace=ws, idx_out=idx, tokens_out=tok)
    ev[steps].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    med = statistics.median(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    return (med, wall) if both else med


def stage_times(C, p, dev, ws, steps):
    """Mean ms per stage over `steps` calls, from events the library records on the work stream."""
    import torch
    k, _, _ = C.resolve(p)
    idx = torch.empty(p.batch, k, dtype=torch.int32, device="cuda")
    tok = torch.empty(p.batch, k, p.d_model, dtype=dev["X"].dtype, device="cuda")
    sets = []
    for _ in range(steps):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(C.NUM_STAGE_EVENTS)]
        for e in evs:
            e.record()           # creates the underlying hipEvent_t
        sets.append(evs)
    torch.cuda.synchronize()
    for evs in sets:
        C.reduce(p, dev["X"], dev["hidden"], dev["Q"], dev["Wq"], dev["Wk"], workspace=ws, idx_out=idx,
                 tokens_out=tok, stage_events=evs)
    torch.cuda.synchronize()
    out = {}
    for i, name in enumerate(C.STAGES):
        out[name] = sum(evs[i].elapsed_time(evs[i + 1]) for evs in sets) / steps
    probe = sum(evs[C.PROBE_BEGIN].elapsed_time(evs[C.PROBE_END]) for evs in sets) / steps
    return out, probe


def gram_flops(B, M, d, tile):
    """Flops the Gram kernel executes: square tiles on and below the diagonal only (the rest is mirrored)."""
    t = (M + tile - 1) // tile
    return 2.0 * B * (t * (t + 1) // 2) * tile * tile * d


def contraction_fractions(w, modes, stages):
    """Fraction of the MFMA peak of the stages that are contractions, from the stage times of the same run: executed
    flops (the three bf16 planes of the folded query matrix counted three times, Gram tiles on and below the diagonal
    only) over the stage's time, which also holds that stage's small non-MFMA kernels."""
    import covspec_inputs as I
    B, N, d, T = w.batch, w.n_tokens, w.d_model, w.n_query
    if w.dtype != I.BF16 or modes != (0, 0):
        return None
    peak = PEAK["mfma_bf16_TFLOPs"] * 1e12
    planes = 3
    work = {"token_projection": 2.0 * B * N * d * d,
            "query_side (e(q), folded query matrix in 3 planes)": 2.0 * B * T * d * d * (1 + planes),
            "relevance (token x folded query products in 3 planes)": 2.0 * B * N * d * T * planes,
            "gram (tiles on and below the diagonal)": gram_flops(B, w.preselect_m, d, 128)}
    key = {"token_projection": "token_projection", "query_side (e(q), folded query matrix in 3 planes)": "query_side",
           "relevance (token x folded query products in 3 planes)": "relevance", "gram (tiles on and below the diagonal)": "gram"}
    return {k: round(v / (stages[key[k]] * 1e-3) / peak, 4) for k, v in work.items() if stages[key[k]] > 0}


def roofline_for(w, p, p_modes, stages, probe_ms, C):
    """Roofline object of the kernel the step spends most of its time in.

    Candidates are the kernels that make up (nearly) all of a stage by themselves, with the stage time as the
    launch duration, and the fp64 product of the subspace iteration, timed by the library's probe events
    around one of its equal launches.  achieved = algorithmic work of one launch / its measured duration.
    """
    import covspec_inputs as I
    B, N, d, T, K = w.batch, w.n_tokens, w.d_model, w.n_query, w.n_act_layers
    M, k = w.preselect_m, w.keep_k
    e = 2 if w.dtype == I.BF16 else 4
    bf = e == 2
    # name -> (kernel, bound, peak, unit, algorithmic work per launch, launches per step, ms per launch)
    cand = {
        "token_projection": ("gemm_nt_ring_kernel<rownorm2>" if (bf and p_modes[0] == 0) else
                             "gemm_nt_ring_kernel<store>" if bf else "gemm64_kernel<f32>",
                             "mfma", PEAK["mfma_bf16_TFLOPs"] if bf else PEAK["mfma_fp64_TFLOPs"], "TFLOP/s",
                             2.0 * B * N * d * d / 1e12, 1, stages["token_projection"]),
        "activity": ("activity_kernel", "hbm", PEAK["hbm_GBps"], "GB/s", (K + 1) * B * N * d * e / 1e9, 1,
                     stages["activity"]),
        "gather": ("gather_rows_kernel", "hbm", PEAK["hbm_GBps"], "GB/s", 2.0 * B * k * d * e / 1e9, 1,
                   stages["gather"]),
        # the Gram matrix is symmetric: only the tiles on and below the diagonal are computed, and only those are counted
        "gram": ("gemm_gram_dma_kernel (tiles on and below the diagonal)" if (bf and p_modes[1] == 0) else "gemm64_kernel<gather> (tiles on and below the diagonal)",
                 "mfma", PEAK["mfma_bf16_TFLOPs"] if (bf and p_modes[1] == 0) else PEAK["mfma_fp64_TFLOPs"],
                 "TFLOP/s", gram_flops(B, M, d, 128 if (bf and p_modes[1] == 0) else 64) / 1e12, 1, stages["gram"]),
    }
    n_probe, pr, pc, pk = C.probe_launches(p)
    if n_probe > 0 and probe_ms > 0:
        cand["lowrank_product"] = ("gemm64_kernel<f64,f64,store>", "mfma", PEAK["mfma_fp64_TFLOPs"], "TFLOP/s",
                                   2.0 * B * pr * pc * pk / 1e12, n_probe, probe_ms)
    elif p_modes[1] == 1:
        cand["lowrank"] = ("greedy_kernel", "alu", PEAK["valu_fp64_TFLOPs"], "TFLOP/s", 1.0 * B * M * k * k / 1e12, 1,
                           stages["lowrank"])
    dom = max(cand, key=lambda s: cand[s][5] * cand[s][6])
    kern, bound, peak, unit, work, launches, ms = cand[dom]
    achieved = work / (ms / 1e3)
    # the counter summary covers workload 5 in the paper pipeline; names as the profiler prints them
    prof_name = {"gemm_nt_ring_kernel<rownorm2>": "gemm_nt_ring_kernel<1>", "activity_kernel": "activity_kernel<"}.get(kern)
    traffic = counter_traffic("reduce5", [prof_name]) if (w.cid == 5 and p_modes == (0, 0) and prof_name) else None
    return {"bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
            "frac": round(achieved / peak, 5), "traffic": traffic, "kernel": kern,
            "launches_per_step": launches, "avg_launch_ms": round(ms, 5),
            "ms_per_step_in_kernel": round(ms * launches, 4)}


def cpu_baseline(w, batch, rel, lr, budget_s=20.0):
    """The oracle, as it stands, on a bounded sample of the workload's images."""
    import covspec_inputs as I
    from oracle import covspec_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([t.get("num_threads", 1) for t in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    op = O.Params(n_heads=w.n_heads, rel_mode=rel, lr_mode=lr, preselect_m=w.preselect_m, rank_r=w.rank_r,
                  keep_k=w.keep_k, lam=w.lam)
    Wq, Wk = I.as_f64(batch["Wq"], w.dtype), I.as_f64(batch["Wk"], w.dtype)
    done, t0 = 0, time.perf_counter()
    while done < w.batch and (done == 0 or (time.perf_counter() - t0) * (done + 1) / done < budget_s):
        b = done
        O.reduce(I.as_f64(batch["X"][b], w.dtype), I.as_f64(batch["hidden"][b], w.dtype),
                 I.as_f64(batch["Q"][b], w.dtype), Wq, Wk, op)
        done += 1
    dt = time.perf_counter() - t0
    return {"value": round(done / dt, 4), "unit": "images/s", "cores": int(cores), "kind": "oracle",
            "sample": "first %d of %d images of the workload, %.1f s (fp64 NumPy incl. conversion of the stored inputs)"
                      % (done, w.batch, dt)}


def verify_bench(a):
    """--verify: the speculative verification step (paper Sec. II-A) over a full vocabulary, its own JSON line.

    A step is one covspec_verify call: 64 sequences x 8 drafted positions x 151,936 words, bf16 logits resident in
    HBM.  Algorithmic bytes per call = both logit tensors read once (2 S L V e) plus the small per-position
    inputs and outputs; `achieved` is that figure over the WHOLE call's time (five kernels), so it understates
    the streaming kernel's own rate.
    """
    import numpy as np
    import torch
    import covspec_inputs as I
    import paper_2605_02218_amd as C
    C.load_library()
    torch.cuda.set_device(0)
    S, L, V, dtype = 64, 8, I.VERIFY_VOCAB, I.BF16
    d = I.make_verify_batch(S, L, V, dtype, seed=2024, copy_rows=2)
    zt = torch.from_numpy(d["zt"].view(np.int16)).cuda().view(torch.bfloat16)
    zd = torch.from_numpy(d["zd"].view(np.int16)).cuda().view(torch.bfloat16)
    tok, ua, ur = (torch.from_numpy(d[k]).cuda() for k in ("tok", "u_acc", "u_res"))
    p = C.VerifyParams(S, L, V, dtype)
    ws = torch.empty(C.verify_workspace_size(p) + 256, dtype=torch.uint8, device="cuda")
    for _ in range(a.warmup):
        C.verify(p, zt, zd, tok, ua, ur, workspace=ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(a.steps):
        C.verify(p, zt, zd, tok, ua, ur, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / a.steps
    ms = e0.elapsed_time(e1) / a.steps
    alg = 2.0 * S * L * V * 2 + S * L * 12 + S * 12
    line = {"metric": "drafted positions verified/sec (softmax, acceptance, residual draw over the vocabulary)",
            "value": round(S * L / max(ms, wall_ms) * 1e3, 1), "unit": "positions/s", "n_gpus": 1, "steps": a.steps,
            "warmup": a.warmup, "ms_per_step": round(max(ms, wall_ms), 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "verify S=%d L=%d V=%d" % (S, L, V), "entry_point": "covspec_verify"},
            "roofline": {"bound": "hbm", "achieved": round(alg / (ms * 1e-3) / 1e9, 1), "peak": PEAK["hbm_GBps"], "unit": "GB/s",
                         "frac": round(alg / (ms * 1e-3) / 1e9 / PEAK["hbm_GBps"], 4), "traffic": counter_traffic("vocab", ["verify_stats_kernel", "verify_accept_kernel", "verify_rowpass64_kernel", "verify_sample_kernel"]),
                         "kernel": "whole call (verify_stats_kernel streams the logits)", "device_ms": round(ms, 4)}}
    if not a.no_cpu_baseline:
        from oracle import verify_oracle as VO
        t0 = time.perf_counter()
        n = 0
        while n < S and time.perf_counter() - t0 < 10.0:
            VO.verify(I.as_f64(d["zt"][n], dtype), I.as_f64(d["zd"][n], dtype), d["tok"][n], d["u_acc"][n], d["u_res"][n])
            n += 1
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": round(n * L / dt, 2), "unit": "positions/s", "cores": 1, "kind": "oracle",
                                "sample": "%d of the %d sequences of the same batch" % (n, S)}
    print(json.dumps(line), flush=True)


def draft_bench(a):
    """--draft: the draft-side vocabulary pass (paper Sec. III-B margin gate, Sec. III-C candidates), own JSON line.

    A step is one covspec_draft_gate call: 64 sequences x 8 positions x 151,936 words of bf16 draft logits resident
    in HBM, F_0 = 8, rho = 1/2.  Algorithmic bytes per call = the logits read once (S L V e) plus the small outputs;
    `achieved` is that figure over the whole call's time (two kernels).
    """
    import numpy as np
    import torch
    import covspec_inputs as I
    import paper_2605_02218_amd as C
    C.load_library()
    torch.cuda.set_device(0)
    S, L, V, dtype, F0, rho, gamma = 64, 8, I.VERIFY_VOCAB, I.BF16, 8, 0.5, 0.5
    d = I.make_verify_batch(S, L, V, dtype, seed=2024, copy_rows=2)
    zd = torch.from_numpy(d["zd"].view(np.int16)).cuda().view(torch.bfloat16)
    tok = torch.from_numpy(d["tok"]).cuda()
    p = C.DraftParams(S, L, V, dtype, F0, rho, gamma)
    ws = torch.empty(C.draft_workspace_size(p) + 256, dtype=torch.uint8, device="cuda")
    for _ in range(a.warmup):
        C.draft_gate(p, zd, tok, workspace=ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(a.steps):
        C.draft_gate(p, zd, tok, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / a.steps
    ms = e0.elapsed_time(e1) / a.steps
    alg = 1.0 * S * L * V * 2 + S * L * (4 + 4 + 4 + 4 * F0)
    line = {"metric": "drafted positions gated/sec (margin gate and bonus-token candidates over the vocabulary)",
            "value": round(S * L / max(ms, wall_ms) * 1e3, 1), "unit": "positions/s", "n_gpus": 1, "steps": a.steps,
            "warmup": a.warmup, "ms_per_step": round(max(ms, wall_ms), 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "draft gate S=%d L=%d V=%d F0=%d rho=%g gamma=%g" % (S, L, V, F0, rho, gamma),
                       "entry_point": "covspec_draft_gate"},
            "roofline": {"bound": "hbm", "achieved": round(alg / (ms * 1e-3) / 1e9, 1), "peak": PEAK["hbm_GBps"], "unit": "GB/s",
                         "frac": round(alg / (ms * 1e-3) / 1e9 / PEAK["hbm_GBps"], 4), "traffic": counter_traffic("vocab", ["draft_scan_kernel", "draft_merge_kernel"]),
                         "kernel": "whole call (draft_scan_kernel streams the logits)", "device_ms": round(ms, 4)}}
    if not a.no_cpu_baseline:
        from oracle import draft_oracle as DO
        t0 = time.perf_counter()
        n = 0
        while n < S and time.perf_counter() - t0 < 10.0:
            DO.draft_pass(I.as_f64(d["zd"][n], dtype), d["tok"][n], F0, float(np.float32(rho)), float(np.float32(gamma)))
            n += 1
        dt = time.perf_counter() - t0
        line["cpu_baseline"] = {"value": round(n * L / dt, 2), "unit": "positions/s", "cores": 1, "kind": "oracle",
                                "sample": "%d of the %d sequences of the same batch" % (n, S)}
    print(json.dumps(line), flush=True)


def ragged_bench(a):
    """--ragged: covspec_reduce_ragged on a dynamic-resolution batch, own JSON line.

    64 images of workload 5's width and structure (d = 4096, 128 keywords, bf16, keep ratio 1/9) whose token counts
    are 256 per tile with 4..12 tiles (the tile grids of a dynamic-resolution vision encoder), sorted by size so
    that equal sizes form runs.  A step is one call over the packed batch; images/sec with the runs on one stream
    and dealt to two and to five.
    """
    from concurrent.futures import ThreadPoolExecutor
    from dataclasses import replace
    import numpy as np
    import torch
    import covspec_inputs as I
    import paper_2605_02218_amd as C
    C.load_library()
    torch.cuda.set_device(0)
    base = I.WORKLOADS[5]
    tiles = sorted([4, 6, 6, 8, 9, 12, 12, 12] * 8)
    ws_ = [replace(base, batch=1, n_tokens=256 * t, keep_k=0, preselect_m=0, rank_r=0) for t in tiles]
    with ThreadPoolExecutor(max_workers=16) as ex:
        per = list(ex.map(lambda bw: I.make_image(bw[1], bw[0]), enumerate(ws_)))
    wts = I.make_weights(base)
    d = base.d_model

    def up(x):
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda().view(torch.bfloat16)

    X = up(np.concatenate([p["X"] for p in per]))
    Q = up(np.concatenate([p["Q"] for p in per]))
    Hd = up(np.concatenate([p["hidden"].reshape(-1, d) for p in per]))
    Wq, Wk = up(wts["Wq"]), up(wts["Wk"])
    del per
    nt, nq = [w.n_tokens for w in ws_], [w.n_query for w in ws_]
    p = C.Params(batch=1, n_tokens=1, d_model=d, n_query=1, n_heads=base.n_heads, n_act_layers=base.n_act_layers, dtype=C.BF16,
                 keep_ratio=1.0 / 9.0, lam=base.lam)
    ks, runs = C.ragged_resolve(p, nt, nq)
    idx = torch.empty(sum(ks), dtype=torch.int32, device="cuda")
    tok = torch.empty(sum(ks), d, dtype=torch.bfloat16, device="cuda")
    res = {}
    for ns in (1, 2, 5):
        streams = [torch.cuda.Stream() for _ in range(ns)]
        wsb = torch.empty(C.ragged_workspace_size(p, nt, nq, ns) + 256, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()

        def step():
            C.reduce_ragged(p, nt, nq, X, Hd, Q, Wq, Wk, streams=streams, workspace=wsb, idx_out=idx, tokens_out=tok, sync=False)

        for _ in range(max(1, a.warmup // 2)):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            step()
        torch.cuda.synchronize()
        res[ns] = (time.perf_counter() - t0) * 1e3 / a.steps
        del wsb
    best = min(res.values())
    line = {"metric": "images/sec for visual-token reduction (score+select+gather), ragged batch", "value": round(len(tiles) / best * 1e3, 2),
            "unit": "images/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(best, 4),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "ragged: 64 images, d=%d T=%d, N = 256 x tiles, tiles 4..12 (%d tokens in all, %d runs), keep 1/9"
                       % (d, base.n_query, sum(nt), runs), "entry_point": "covspec_reduce_ragged"},
            "ms_per_step_by_streams": {str(k): round(v, 3) for k, v in res.items()},
            "tokens_per_s": round(sum(nt) / best * 1e3, 1)}
    print(json.dumps(line), flush=True)


def ablation_bench(a):
    """--ablations: what each term of the selector costs, own JSON line.

    covspec_reduce on the chosen workload (default 5) with the selector variants of Table II and Sec. III-A.3:
    the paper's selector; the M -> k cut on the fused score alone (no low-rank stage); random tokens (no scores at
    all); full-token (k = M = N: scores are computed, everything is kept and gathered); query-only (lambda = 1) and
    activity-only (lambda = 0) scores in front of the paper's low-rank stage.
    """
    from dataclasses import replace
    import torch
    import covspec_inputs as I
    import paper_2605_02218_amd as C
    C.load_library()
    torch.cuda.set_device(0)
    w = I.WORKLOADS[a.workload]
    dev = _upload(_gen(w), w.dtype)
    base = _params(C, w, 0, 0)
    cases = {
        "paper selector": base,
        "fused-score top-k (no low-rank stage)": replace(base, lr_mode=C.LR_SCORE_TOPK),
        "random tokens (no scores)": replace(base, lr_mode=C.LR_RANDOM, seed=1),
        "full-token (k = M = N, score-only cut)": replace(base, lr_mode=C.LR_SCORE_TOPK, keep_k=w.n_tokens, preselect_m=w.n_tokens),
        "query-only scores (lambda = 1)": replace(base, lam=1.0),
        "activity-only scores (lambda = 0)": replace(base, lam=0.0),
    }
    res = {}
    for name, p in cases.items():
        ws = C.alloc_workspace(p)
        res[name] = round(time_reduce(C, p, dev, ws, a.steps, a.warmup), 4)
        del ws
    ms = res["paper selector"]
    line = {"metric": "images/sec for visual-token reduction (score+select+gather)", "value": round(w.batch / ms * 1e3, 3), "unit": "images/s",
            "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16" if w.dtype == I.BF16 else "f64", "data": "synthetic",
            "config": {"workload": _wname(w), "entry_point": "covspec_reduce", "pipeline": "selector ablations"},
            "ms_per_step_by_selector": res}
    print(json.dumps(line), flush=True)


def stream_bench(a):
    """--stream: covspec_stream_step in its steady state, own JSON line.

    Four videos of workload 4's kind (frames of 1024 tokens, d = 1536, bf16, slowly drifting content) advance one
    frame per step: 256 tokens pre-selected per frame, 1024 kept across frames, r = 128, so every step decides
    among 1280 candidates.  Scores are inputs (a score pass over the frame precedes the step in a pipeline).
    Beside it: the same decision without the carried Gram matrix (covspec_select over the 1280 stacked candidate
    rows, which recomputes all of it), and the oracle on the host.
    """
    import numpy as np
    import torch
    import covspec_inputs as I
    import paper_2605_02218_amd as C
    C.load_library()
    torch.cuda.set_device(0)
    B, n_frame, d, m, k, r = 4, 1024, 1536, 256, 1024, 128
    n_frames = 6
    vids = [I.make_video_stream(n_frames, n_frame, d, dtype=I.BF16, seed=b) for b in range(B)]

    def up(x):
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda().view(torch.bfloat16)

    Xf = [up(np.stack([v[0][f] for v in vids])) for f in range(n_frames)]
    sf = [torch.from_numpy(np.stack([v[1][f] for v in vids])).cuda() for f in range(n_frames)]
    p = C.StreamParams(batch=B, n_frame=n_frame, d_model=d, frame_m=m, keep_k=k, rank_r=r, dtype=C.BF16)
    ws = torch.empty(C.stream_workspace_size(p) + 256, dtype=torch.uint8, device="cuda")
    states = [C.stream_alloc_state(p), C.stream_alloc_state(p)]
    n_keep, f = 0, 0
    while n_keep < k:                                    # fill the memory
        n_keep, _ = C.stream_step(p, n_keep, f * n_frame, Xf[f % n_frames], sf[f % n_frames], states[f & 1] if n_keep else None,
                                  states[(f + 1) & 1], workspace=ws)
        f += 1

    def step():
        nonlocal f
        C.stream_step(p, k, f * n_frame, Xf[f % n_frames], sf[f % n_frames], states[f & 1], states[(f + 1) & 1], workspace=ws)
        f += 1

    def timed(fn):
        for _ in range(a.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / a.steps

    ms = timed(step)
    # the same decision from scratch: stack the candidates and let covspec_select recompute their Gram matrix
    ps = C.Params(batch=B, n_tokens=k + m, d_model=d, n_query=1, dtype=C.BF16, keep_k=k, preselect_m=k + m, rank_r=r)
    wss = C.alloc_workspace(ps)
    Zc = torch.cat([states[f & 1][0], Xf[0][:, :m]], dim=1).contiguous()
    flat = torch.zeros(B, k + m, dtype=torch.float32, device="cuda")
    ms_scratch = None if a.no_comparison else timed(lambda: C.select(ps, Zc, flat, wss))

    cpu = None
    if not a.no_cpu_baseline:
        from oracle import stream_oracle as S
        st = S.empty_state(d)
        X0 = [I.as_f64(vids[0][0][g], I.BF16) for g in range(n_frames)]
        g, n0 = 0, 0
        while st.rows.shape[0] < k:
            S.stream_step(st, X0[g % n_frames], vids[0][1][g % n_frames], g * n_frame, m, k, r)
            g += 1
        t0 = time.perf_counter()
        done = 0
        while done < 2 or time.perf_counter() - t0 < 10.0:
            S.stream_step(st, X0[g % n_frames], vids[0][1][g % n_frames], g * n_frame, m, k, r)
            g += 1
            done += 1
        dt = time.perf_counter() - t0
        cpu = {"value": round(done / dt, 3), "unit": "frames/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
               "kind": "oracle", "sample": "%d steady-state frames of one video (%.1f s)" % (done, dt)}
    line = {"metric": "frames/sec for the streaming low-rank selection (steady state)", "value": round(B / ms * 1e3, 2), "unit": "frames/s",
            "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "stream: %d videos, frames of %d tokens x %d, %d pre-selected per frame, %d kept, r=%d (%d candidates per step)"
                       % (B, n_frame, d, m, k, r, k + m), "entry_point": "covspec_stream_step"},
            "from_scratch_ms_per_step": None if ms_scratch is None else round(ms_scratch, 4), "tokens_per_s": round(B * n_frame / ms * 1e3, 1), "cpu_baseline": cpu}
    print(json.dumps(line), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=5, help="1..5 (default 5: the largest single-GPU workload)")
    ap.add_argument("--pipeline", choices=["paper", "variant"], default="paper")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--all", action="store_true", help="(default behaviour now) time every workload in both pipelines")
    ap.add_argument("--headline-only", action="store_true",
                    help="time only the chosen workload and pipeline (short runs under a profiler)")
    ap.add_argument("--verify", action="store_true", help="time the speculative verification step instead (own JSON line)")
    ap.add_argument("--draft", action="store_true", help="time the draft-side margin gate / candidate pass instead (own JSON line)")
    ap.add_argument("--ragged", action="store_true", help="time covspec_reduce_ragged on a dynamic-resolution batch (own JSON line)")
    ap.add_argument("--ablations", action="store_true", help="time the selector ablations on the chosen workload (own JSON line)")
    ap.add_argument("--stream", action="store_true", help="time covspec_stream_step in its steady state (own JSON line)")
    ap.add_argument("--no-comparison", action="store_true", help="with --stream: leave out the from-scratch comparison (clean kernel profiles)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run three plain 1 GiB device copies and exit (reference reading for the HBM byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (images shard trivially across GPUs; no multi-GPU path "
                 "exists or is measured) -- rerun with --gpus 1")

    import torch
    if a.copy_calibration:
        # a copy of known size: 2^30 bytes read, 2^30 bytes written per launch
        torch.cuda.set_device(0)
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "launches": 3}), flush=True)
        return
    if a.verify:
        verify_bench(a)
        return
    if a.draft:
        draft_bench(a)
        return
    if a.ragged:
        ragged_bench(a)
        return
    if a.stream:
        stream_bench(a)
        return
    if a.ablations:
        ablation_bench(a)
        return
    import covspec_inputs as I
    import paper_2605_02218_amd as C
    C.load_library()
    torch.cuda.set_device(0)
    modes = (0, 0) if a.pipeline == "paper" else (1, 1)
    w = I.WORKLOADS[a.workload]

    batch = _gen(w)
    dev = _upload(batch, w.dtype)
    p = _params(C, w, *modes)
    ws = C.alloc_workspace(p)
    ms, wall_ms = time_reduce(C, p, dev, ws, a.steps, a.warmup, both=True)
    stages, probe_ms = stage_times(C, p, dev, ws, min(a.steps, 10))
    line = {
        "metric": "images/sec for visual-token reduction (score+select+gather)",
        "value": round(w.batch / ms * 1e3, 3), "unit": "images/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms, 4), "ms_per_step_wall_mean": round(wall_ms, 4), "timing": "median of per-call HIP event times",
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == I.BF16 else "f64", "data": "synthetic",
        "config": {"workload": "%d:%s B=%d N=%d d=%d T=%d H=%d K=%d k=%d M=%d r=%d" % (
            w.cid, w.name, w.batch, w.n_tokens, w.d_model, w.n_query, w.n_heads, w.n_act_layers, w.keep_k,
            w.preselect_m, w.rank_r), "pipeline": "paper: cosine-max relevance + rank-r SVD energy" if modes == (0, 0)
            else "variant: attention-softmax relevance + greedy residual picks", "entry_point": "covspec_reduce"},
        "roofline": roofline_for(w, p, modes, stages, probe_ms, C),
        "stages_ms": {k: round(v, 4) for k, v in stages.items()},
        "mfma_peak_fraction_by_stage": contraction_fractions(w, modes, stages),
        # the stages grouped by the entry point that runs them on its own
        "entry_points_ms": {"covspec_score": round(sum(stages[k] for k in ("query_side", "token_projection", "relevance", "activity", "fuse")), 4),
                            "covspec_select": round(sum(stages[k] for k in ("preselect", "gram", "lowrank", "keep")), 4),
                            "gather": round(stages["gather"], 4)},
    }
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, batch, *modes)
    if not a.headline_only:
        # every workload in both pipelines (images/s of covspec_reduce, whole batch per call, inputs generated once
        # per workload): the other nine figures beside the headline one
        table = {"%d:%s" % (w.cid, a.pipeline): round(w.batch / ms * 1e3, 2)}
        other = (1, 1) if modes == (0, 0) else (0, 0)
        p2 = _params(C, w, *other)
        ws2 = C.alloc_workspace(p2)
        table["%d:%s" % (w.cid, "variant" if other == (1, 1) else "paper")] = round(
            w.batch / time_reduce(C, p2, dev, ws2, max(5, a.steps // 2), 2) * 1e3, 2)
        del ws2, dev, ws, batch
        for cid in sorted(I.WORKLOADS):
            if cid == w.cid:
                continue
            wo = I.WORKLOADS[cid]
            devo = _upload(_gen(wo), wo.dtype)
            for name, m in (("paper", (0, 0)), ("variant", (1, 1))):
                po = _params(C, wo, *m)
                wso = C.alloc_workspace(po)
                # small batches are latency-bound and their first calls see the clocks ramp up: more warm-up and steps
                table["%d:%s" % (cid, name)] = round(wo.batch / time_reduce(C, po, devo, wso, 20 if wo.batch <= 8 else 10, 5) * 1e3, 2)
                del wso
            del devo
            torch.cuda.empty_cache()
        line["images_per_s_by_workload_and_pipeline"] = dict(sorted(table.items()))
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
