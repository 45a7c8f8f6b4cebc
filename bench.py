#!/usr/bin/env python3
"""Benchmark of the SentenceKV decode hot path on one MI355X.

A "step" is one decode step of the whole model: for every layer, one skv_decode_step call
(scores of all buckets -> budgeted selection -> attention over the retrieved tokens read straight
from the HBM pool).  The prefill side (segmentation + mean key vectors) runs once before the timed
region and is timed separately.  Inputs are synthetic and resident in HBM before timing starts.

Prints ONE JSON line:  metric / value = achieved HBM GB/s of the decode step (algorithmic bytes of
the fused path over wall time) for cfg1 (32K context, one sequence), us_per_layer, live timings of the
four stand-alone kernels, the roofline of the kernel the timed step runs (one launch per layer), the CPU
oracle timed on a bounded sample of the same workload (one thread, and all cores), and under "extras" the
same measurement for cfg2 (128K context; host-pool gather separately) and cfg4 (ragged batch), under
"batched" for 16 and 64 sequences of cfg1's shape.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2504_00970_amd as skv          # noqa: E402
from workload import gen                    # noqa: E402

HBM_PEAK_GBPS = 8000.0                      # MI355X datasheet HBM3E bandwidth
N_QUERY_SETS = 16                           # distinct query sets rotated across steps


SV_TABLE = {"f32": (4, torch.float32, skv.SKV_F32), "bf16": (2, torch.bfloat16, skv.SKV_BF16),
            "fp8": (1, torch.uint8, skv.SKV_FP8_E4M3)}       # bytes per element, torch storage, library code


def i32(a, dev):
    return torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32)).to(dev)


class Timer:
    """HIP events on the stream the kernels are launched on (torch's current stream)."""

    def __init__(self):
        self.a = torch.cuda.Event(enable_timing=True)
        self.b = torch.cuda.Event(enable_timing=True)

    def __enter__(self):
        self.a.record()
        return self

    def __exit__(self, *exc):
        self.b.record()
        self.b.synchronize()
        self.ms = self.a.elapsed_time(self.b)


def capture(ctx, fn):
    """Record fn()'s launches into a HIP graph (the library launches on the capturing stream)."""
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        ctx.set_stream(torch.cuda.current_stream().cuda_stream)
        fn()
    ctx.set_stream(torch.cuda.current_stream().cuda_stream)
    return g


def step_spread(run_step, set_query, steps, layers_per_step):
    """Per-step times of `steps` further steps (an event after every step): median, 10th and 90th percentile in us per
    layer.  Run after the timed region, which is measured as a whole."""
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    evs[0].record()
    for i in range(steps):
        set_query(i)
        run_step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    us = np.array([evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]) * 1e3 / layers_per_step
    if len(us) == 0:
        return None
    return {"median": round(float(np.median(us)), 3), "p10": round(float(np.percentile(us, 10)), 3),
            "p90": round(float(np.percentile(us, 90)), 3), "steps": steps}


def measured_traffic(workload, kernel):
    """HBM bytes per launch from the committed rocprofv3 counter runs (profiles/), or None."""
    try:
        t = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))[workload][kernel]
        return int(t["fetch_bytes"] + t["write_bytes"])
    except (OSError, KeyError, ValueError):
        return None


def decode_bytes(wl, S, n_tok_sum, n_sel_sum, fused=True, sv_bytes=4):
    """Algorithmic bytes of one layer's decode step (what the method itself has to move)."""
    H, D, e = wl.n_kv_heads, wl.head_dim, wl.elt_bytes
    q_bytes = wl.n_q_heads * D * e
    score = S * H * D * sv_bytes + S * H * 4 + q_bytes
    select = S * H * 4 + S * 8 + (n_tok_sum + 2 * n_sel_sum) * 4
    kv = 2 * n_tok_sum * D * e
    attend = kv + n_tok_sum * 4 + q_bytes + wl.n_q_heads * D * 4
    gather = 2 * kv + n_tok_sum * 4
    total = score + select + attend + (0 if fused else gather)
    return dict(score=score, select=select, gather=gather, attend=attend, total=total)


def run_single_sequence(args, wl, budget):
    dev = "cuda:0"
    L, H, Hq, D, T = wl.n_layers, wl.n_kv_heads, wl.n_q_heads, wl.head_dim, wl.n_tokens
    t0 = time.time()
    lengths = gen.sentence_lengths(wl.len_dist, T, args.seed)
    tok = gen.token_stream(lengths, wl.vocab, wl.term_mod, args.seed)
    bitmap = gen.terminator_bitmap(wl.vocab, wl.term_mod)
    inp = gen.decode_inputs(wl, seed=args.seed, device=dev)
    qsets = gen.queries(N_QUERY_SETS * L, Hq, D, wl.torch_dtype, args.seed + 1, dev).view(N_QUERY_SETS, L, Hq, D)
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    S_cap = len(lengths) + 8
    sv_bytes, sv_torch, sv_code = SV_TABLE[args.semvec_dtype]
    sv16 = args.semvec_dtype != "f32"                        # a reduced table: no committed traffic counters
    ctx = skv.Context(skv.Desc(n_layers=L, n_q_heads=Hq, n_kv_heads=H, kv_dtype=skv.dtype_code(wl.torch_dtype),
                               max_tokens=T, max_sentences=S_cap, max_budget=budget, max_batch=1,
                               semvec_dtype=sv_code))

    # ---- prefill: segmentation + semantic vectors (HIP path), timed once -----------------------------
    d_tok, d_bm = i32(tok, dev), torch.as_tensor(bitmap.view(np.int32)).to(dev)
    seg_id = torch.empty(T, dtype=torch.int32, device=dev)
    sent_off = torch.empty(S_cap + 1, dtype=torch.int32, device=dev)
    sent_len = torch.empty(S_cap, dtype=torch.int32, device=dev)
    n_sent = torch.empty(4, dtype=torch.int32, device=dev)
    S = ctx.segment(d_tok, d_bm, wl.vocab, seg_id, sent_off, sent_len, n_sent)
    assert S == len(lengths), (S, len(lengths))
    semvec = torch.empty(L, H, S, D, dtype=sv_torch, device=dev)
    ctx.build_semvec(inp.K, sent_off, S, semvec)
    torch.cuda.synchronize()
    with Timer() as t_seg:
        ctx.segment(d_tok, d_bm, wl.vocab, seg_id, sent_off, sent_len, n_sent, sync=False)
    with Timer() as t_sv:
        ctx.build_semvec(inp.K, sent_off, S, semvec)
    semvec_bytes = L * H * T * D * wl.elt_bytes + L * H * S * D * sv_bytes

    # ---- decode ---------------------------------------------------------------------------------------
    cu_tok, cu_sent = i32([0, T], dev), i32([0, S], dev)
    d_budget = i32([budget], dev)
    out = torch.empty(L, Hq, D, dtype=torch.float32, device=dev)
    n_tok_rec = torch.zeros(N_QUERY_SETS, L, H, dtype=torch.int32, device=dev)

    q_cur = torch.empty(L, Hq, D, dtype=wl.torch_dtype, device=dev)     # the step's queries (graph input)

    # a model with few layers (cfg0 has one) is walked several times per step, so that a step is not all launch overhead
    passes = max(1, 32 // L)

    def layers(record_into=None):
        for _ in range(1 if record_into is not None else passes):
            for l in range(L):
                ctx.decode_step(l, 1, q_cur[l], q_cur[l], inp.K, inp.V, T, semvec, S, cu_tok, cu_sent, sent_off, sent_len,
                                d_budget, out[l], None, None, None if record_into is None else record_into[l])

    for i in range(N_QUERY_SETS):            # records n_tok of every (query set, layer)
        q_cur.copy_(qsets[i])
        layers(record_into=n_tok_rec[i])
    torch.cuda.synchronize()

    def timed(run_step):
        for i in range(args.warmup):
            q_cur.copy_(qsets[i % N_QUERY_SETS])
            run_step()
        torch.cuda.synchronize()
        wall0 = time.perf_counter()
        with Timer() as t:
            for i in range(args.steps):
                q_cur.copy_(qsets[i % N_QUERY_SETS])
                run_step()
        torch.cuda.synchronize()
        wall = time.perf_counter() - wall0
        return max(t.ms, wall * 1e3) / max(args.steps, 1)

    ms_direct = timed(layers)                # one host call per layer
    graph = capture(ctx, layers)             # the same launches replayed as one HIP graph per decode step
    ms_graph = timed(graph.replay)
    ms_per_step = ms_graph if args.launch == "graph" else ms_direct
    spread = step_spread(graph.replay if args.launch == "graph" else layers,
                         lambda i: q_cur.copy_(qsets[i % N_QUERY_SETS]), args.steps, L * passes)

    n_tok_all = n_tok_rec.cpu().numpy().astype(np.int64)
    used = [i % N_QUERY_SETS for i in range(args.steps)]
    n_tok_layer = float(n_tok_all[used].sum(axis=2).mean()) if used else 0.0     # sum over heads, mean over layer-steps
    n_sel_layer = n_tok_layer / float(lengths.mean())
    bytes_layer = decode_bytes(wl, S, n_tok_layer, n_sel_layer, fused=True, sv_bytes=sv_bytes)
    us_per_layer = ms_per_step * 1e3 / (L * passes)
    gbps = bytes_layer["total"] / (us_per_layer * 1e-6) / 1e9

    # ---- per-kernel live timing: each stage launched back-to-back over all layers ------------------------
    score = torch.empty(L, H, S, dtype=torch.float32, device=dev)
    sel = torch.empty(L, H, ctx.desc.max_sel, dtype=torch.int32, device=dev)
    n_sel = torch.empty(L, 8 if H < 8 else H, dtype=torch.int32, device=dev)
    n_tok = torch.empty(L, 8 if H < 8 else H, dtype=torch.int32, device=dev)
    tok_idx = torch.empty(L, H, budget, dtype=torch.int32, device=dev)
    K_sel = torch.empty(L, H, budget, D, dtype=wl.torch_dtype, device=dev)
    V_sel = torch.empty_like(K_sel)
    lse = torch.empty(L, Hq, dtype=torch.float32, device=dev)
    qs = qsets[0]
    stages = {
        "score": lambda l: ctx.score(l, qs[l], semvec, S, score[l]),
        "select": lambda l: ctx.select(score[l], sent_off, sent_len, S, budget, sel[l], n_sel[l], tok_idx[l], n_tok[l]),
        "gather": lambda l: ctx.gather(l, inp.K, inp.V, T, tok_idx[l], n_tok[l], budget, K_sel[l], V_sel[l]),
        "attend": lambda l: ctx.attend(qs[l], K_sel[l], V_sel[l], n_tok[l], budget, out[l], lse[l]),
    }
    kern = {}
    reps = max(2, min(20, args.steps))
    for name, fn in stages.items():
        def all_layers(fn=fn):
            for _ in range(passes):
                for l in range(L):
                    fn(l)
        all_layers()
        g = capture(ctx, all_layers)
        g.replay()
        torch.cuda.synchronize()
        with Timer() as t:
            for _ in range(reps):
                g.replay()
        kern[name] = t.ms * 1e3 / (reps * L * passes)
    nt_chain = float(n_tok[:, :H].sum().item()) / L
    b_unf = decode_bytes(wl, S, nt_chain, nt_chain / float(lengths.mean()), fused=False, sv_bytes=sv_bytes)
    kernels = {k: dict(us=round(v, 3), bytes=int(b_unf[k]), GBps=round(b_unf[k] / (v * 1e-6) / 1e9, 1))
               for k, v in kern.items()}
    # The timed step is ONE kernel per layer (attend_kernel in its single-launch form: scores, selection and attention
    # of the layer), so the dominant kernel's launch is the layer: its algorithmic bytes are the step's, its duration
    # the per-layer time of the timed region (launch to launch, HIP events on the launching stream).
    copy_peak = measured_copy_peak(dev)
    roofline = dict(bound="hbm", kernel="attend_kernel<bf16, G, single-launch step, 128-token blocks>" if wl.dtype == "bf16"
                    else "attend_kernel<fp32, G, single-launch step, 128-token blocks>",
                    achieved=round(gbps, 1), peak=HBM_PEAK_GBPS, unit="GB/s", frac=round(gbps / HBM_PEAK_GBPS, 4),
                    traffic=None if sv16 else measured_traffic(wl.name, "decode_step_kernel"),
                    bytes_per_launch=int(bytes_layer["total"]), us_per_launch=round(us_per_layer, 3),
                    launches_per_layer=1, measured_copy_peak_GBps=round(copy_peak, 1),
                    frac_of_measured_copy_peak=round(gbps / copy_peak, 4))

    cpu = cpu_baseline(args, wl, inp, semvec, lengths, qsets, budget) if not args.no_cpu_baseline else None
    host_pool = host_pool_gather(args, wl, ctx, inp, tok_idx, n_tok, budget, K_sel) if args.host_pool_layers > 0 else None

    return {
        "metric": "decode-step achieved HBM GB/s (score+select+gather+attn) at %s ctx" % _ctx_name(T),
        "value": round(gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "layers": L, "layer_passes_per_step": passes, "q_heads": Hq, "kv_heads": H, "head_dim": D, "context": T,
                   "sentences": S, "budget": budget, "batch": 1, "path": "skv_decode_step (score+select+attend from pool, one launch per layer)",
                   "kv_pool": "hbm", "launch": args.launch, "semvec_dtype": args.semvec_dtype},
        "us_per_layer": round(us_per_layer, 3),
        "us_per_layer_direct_launch": round(ms_direct * 1e3 / (L * passes), 3),
        "us_per_layer_hip_graph": round(ms_graph * 1e3 / (L * passes), 3),
        "us_per_layer_per_step": spread,
        "bytes_per_layer": int(bytes_layer["total"]),
        "hbm_frac": round(gbps / HBM_PEAK_GBPS, 4),
        "mean_tokens_selected_per_head": round(n_tok_layer / H, 1),
        "kernels_unfused": kernels,
        "unfused_us_per_layer": round(sum(kern.values()), 3),
        "unfused_GBps": round(b_unf["total"] / (sum(kern.values()) * 1e-6) / 1e9, 1),
        "prefill": {"segment_us": round(t_seg.ms * 1e3, 1), "semvec_ms": round(t_sv.ms, 3),
                    "semvec_GBps": round(semvec_bytes / (t_sv.ms * 1e-3) / 1e9, 1)},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "host_pool_gather": host_pool,
        "input_gen_s": round(gen_s, 1),
    }


def host_pool_gather(args, wl, ctx, inp, tok_idx, n_tok, budget, ref_K_sel):
    """skv_gather with the K/V pool in pinned, device-mapped host memory (the paper's CPU-offloaded store):
    the kernel's 16-byte loads cross PCIe.  Reported next to the pinned host-to-device copy rate."""
    dev = "cuda:0"
    n = min(args.host_pool_layers, wl.n_layers)
    H, D, T = wl.n_kv_heads, wl.head_dim, wl.n_tokens
    # the host pool keeps the [L][Hkv][T][D] layout; only the first n layers are filled and used
    Kh = torch.empty(n, H, T, D, dtype=wl.torch_dtype, pin_memory=True).copy_(inp.K[:n])
    Vh = torch.empty(n, H, T, D, dtype=wl.torch_dtype, pin_memory=True).copy_(inp.V[:n])
    K_sel = torch.zeros(n, H, budget, D, dtype=wl.torch_dtype, device=dev)
    V_sel = torch.zeros_like(K_sel)
    torch.cuda.synchronize()

    def run():
        for l in range(n):
            ctx.gather(l, Kh, Vh, T, tok_idx[l], n_tok[l], budget, K_sel[l], V_sel[l], pool_in_host=True)

    run()
    torch.cuda.synchronize()
    reps = 5
    with Timer() as t:
        for _ in range(reps):
            run()
    us = t.ms * 1e3 / (reps * n)
    rows = float(n_tok[:n, :H].sum().item()) / n
    pcie_bytes = 2 * rows * D * wl.elt_bytes
    valid = torch.arange(budget, device=dev)[None, :] < n_tok[0, :H, None]                   # rows the gather wrote
    same = bool(torch.equal(K_sel[0].view(torch.int16)[valid], ref_K_sel[0].view(torch.int16)[valid]))
    big = torch.empty(256 << 20, dtype=torch.uint8, pin_memory=True)
    dst = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    dst.copy_(big, non_blocking=True)
    torch.cuda.synchronize()
    with Timer() as tc:
        for _ in range(4):
            dst.copy_(big, non_blocking=True)
    h2d = 4 * (256 << 20) / (tc.ms * 1e-3) / 1e9
    return {"layers": n, "us_per_layer": round(us, 2), "bytes_over_pcie_per_layer": int(pcie_bytes),
            "GBps": round(pcie_bytes / (us * 1e-6) / 1e9, 2), "pinned_h2d_copy_GBps": round(h2d, 2),
            "frac_of_h2d_copy": round(pcie_bytes / (us * 1e-6) / 1e9 / h2d, 3), "rows_match_hbm_pool": same}


def run_ragged(args, wl):
    """cfg4: a ragged batch of B sequences, one skv_decode_step call per layer.  Only `resident` layers of
    the 80-layer pool are kept in HBM (the full pool would be ~190 GB); a step cycles through them."""
    dev = "cuda:0"
    R = args.resident_layers
    L, H, Hq, D, B = wl.n_layers, wl.n_kv_heads, wl.n_q_heads, wl.head_dim, wl.batch
    t0 = time.time()
    inp = gen.ragged_inputs(wl, seed=args.seed, device=dev, resident_layers=R)
    T_total, S_total = int(inp.cu_tok[-1]), int(inp.cu_sent[-1])
    budget = int(inp.budget.max())
    qsets = gen.queries(N_QUERY_SETS * R * B, Hq, D, wl.torch_dtype, args.seed + 1, dev).view(N_QUERY_SETS, R, B, Hq, D)
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    sv_bytes, sv_torch, sv_code = SV_TABLE[args.semvec_dtype]
    sv16 = args.semvec_dtype != "f32"                        # a reduced table: no committed traffic counters
    ctx = skv.Context(skv.Desc(n_layers=R, n_q_heads=Hq, n_kv_heads=H, kv_dtype=skv.dtype_code(wl.torch_dtype),
                               max_tokens=T_total, max_sentences=S_total, max_budget=budget, max_batch=B,
                               semvec_dtype=sv_code))
    glob_off = i32(gen.offsets_of(inp.sent_len), dev)
    semvec = torch.empty(R, H, S_total, D, dtype=sv_torch, device=dev)
    ctx.build_semvec(inp.K, glob_off, S_total, semvec)
    torch.cuda.synchronize()
    with Timer() as t_sv:
        ctx.build_semvec(inp.K, glob_off, S_total, semvec)
    d = [i32(x, dev) for x in (inp.cu_tok, inp.cu_sent, inp.sent_off, inp.sent_len, inp.budget)]
    out = torch.empty(R, B, Hq, D, dtype=torch.float32, device=dev)
    n_tok_rec = torch.zeros(R, B, H, dtype=torch.int32, device=dev)
    q_cur = torch.empty(R, B, Hq, D, dtype=wl.torch_dtype, device=dev)

    def layers(record=False):
        for l in range(L):
            r = l % R
            ctx.decode_step(r, B, q_cur[r], q_cur[r], inp.K, inp.V, T_total, semvec, S_total, *d, out[r], None, None,
                            n_tok_rec[r] if record else None)

    q_cur.copy_(qsets[0])
    layers(record=True)
    torch.cuda.synchronize()

    def timed(run_step):
        for i in range(args.warmup):
            q_cur.copy_(qsets[i % N_QUERY_SETS])
            run_step()
        torch.cuda.synchronize()
        wall0 = time.perf_counter()
        with Timer() as t:
            for i in range(args.steps):
                q_cur.copy_(qsets[i % N_QUERY_SETS])
                run_step()
        torch.cuda.synchronize()
        return max(t.ms, (time.perf_counter() - wall0) * 1e3) / max(args.steps, 1)

    ms_direct = timed(layers)
    graph = capture(ctx, layers)
    ms_graph = timed(graph.replay)
    ms_per_step = ms_graph if args.launch == "graph" else ms_direct
    spread = step_spread(graph.replay if args.launch == "graph" else layers,
                         lambda i: q_cur.copy_(qsets[i % N_QUERY_SETS]), args.steps, L)
    n_tok_layer = float(n_tok_rec.sum().item()) / R
    mean_len = float(inp.sent_len.mean())
    bl = decode_bytes(wl, S_total, n_tok_layer, n_tok_layer / mean_len, fused=True, sv_bytes=sv_bytes)
    bl["total"] += (B - 1) * wl.n_q_heads * D * (wl.elt_bytes * 2 + 4)          # q and out of the other sequences
    us_per_layer = ms_per_step * 1e3 / L
    gbps = bl["total"] / (us_per_layer * 1e-6) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        orc = oracle.get("f32")
        K0, V0, sv0, q0 = gen.to_numpy(inp.K[0]), gen.to_numpy(inp.V[0]), gen.to_numpy(semvec[0]), gen.to_numpy(qsets[0, 0])
        done, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < args.cpu_seconds:
            b = done % B
            a0, a1, s0, s1 = int(inp.cu_tok[b]), int(inp.cu_tok[b + 1]), int(inp.cu_sent[b]), int(inp.cu_sent[b + 1])
            orc.decode_step(q0[b], q0[b], np.ascontiguousarray(K0[:, a0:a1]), np.ascontiguousarray(V0[:, a0:a1]),
                            np.ascontiguousarray(sv0[:, s0:s1]), inp.sent_off[s0 + b: s1 + b + 1], inp.sent_len[s0:s1],
                            int(inp.budget[b]))
            done += 1
        dt = time.perf_counter() - t0
        cpu = {"value": round(bl["total"] / B * done / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "us_per_layer": round(dt / done * B * 1e6, 1),
               "sample": "%d sequence-steps of layer 0 (sequences in turn), score+select+gather+attend, single thread, fp32" % done}
    return {
        "metric": "decode-step achieved HBM GB/s (score+select+gather+attn), ragged batch",
        "value": round(gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "layers": L, "resident_layers": R, "q_heads": Hq, "kv_heads": H, "head_dim": D,
                   "batch": B, "tokens_total": T_total, "sentences_total": S_total, "budget": budget,
                   "path": "skv_decode_step (one call per layer for the whole batch)", "kv_pool": "hbm",
                   "launch": args.launch, "semvec_dtype": args.semvec_dtype},
        "us_per_layer": round(us_per_layer, 3),
        "us_per_layer_direct_launch": round(ms_direct * 1e3 / L, 3),
        "us_per_layer_hip_graph": round(ms_graph * 1e3 / L, 3),
        "us_per_layer_per_step": spread,
        "bytes_per_layer": int(bl["total"]), "hbm_frac": round(gbps / HBM_PEAK_GBPS, 4),
        "mean_tokens_selected_per_head": round(n_tok_layer / (B * H), 1),
        "prefill": {"semvec_ms": round(t_sv.ms, 3),
                    "semvec_GBps": round((R * H * T_total * D * wl.elt_bytes + R * H * S_total * D * sv_bytes) / (t_sv.ms * 1e-3) / 1e9, 1)},
        "roofline": dict(bound="hbm", kernel="score_kernel + select_attend_stream_kernel (batch step)", achieved=round(gbps, 1),
                         peak=HBM_PEAK_GBPS, unit="GB/s", frac=round(gbps / HBM_PEAK_GBPS, 4),
                         traffic=None if sv16 else measured_traffic(wl.name, "decode_step"), bytes_per_launch=int(bl["total"]),
                         us_per_launch=round(us_per_layer, 3)),
        "cpu_baseline": cpu, "input_gen_s": round(gen_s, 1),
    }


def run_prefill(args, wl):
    """cfg3: sentence segmentation of a token stream and the mean-key table of every layer and KV head."""
    dev = "cuda:0"
    L, H, D, T = wl.n_layers, wl.n_kv_heads, wl.head_dim, wl.n_tokens
    p = gen.prefill_inputs(wl, seed=args.seed, device=dev)
    S_cap = len(p.lengths) + 64
    ctx = skv.Context(skv.Desc(n_layers=L, n_q_heads=wl.n_q_heads, n_kv_heads=H, kv_dtype=skv.dtype_code(wl.torch_dtype),
                               max_tokens=T, max_sentences=S_cap, max_budget=16, max_batch=1))
    d_tok, d_bm = i32(p.tok, dev), torch.as_tensor(p.bitmap.view(np.int32)).to(dev)
    seg_id = torch.empty(T, dtype=torch.int32, device=dev)
    sent_off = torch.empty(S_cap + 1, dtype=torch.int32, device=dev)
    sent_len = torch.empty(S_cap, dtype=torch.int32, device=dev)
    n_sent = torch.empty(4, dtype=torch.int32, device=dev)
    S = ctx.segment(d_tok, d_bm, wl.vocab, seg_id, sent_off, sent_len, n_sent)
    assert S == len(p.lengths)
    semvec = torch.empty(L, H, S, D, dtype=torch.float32, device=dev)

    def step():
        ctx.segment(d_tok, d_bm, wl.vocab, seg_id, sent_off, sent_len, n_sent, sync=False)
        ctx.build_semvec(p.K, sent_off, S, semvec)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    with Timer() as t:
        for _ in range(args.steps):
            step()
    ms = t.ms / max(args.steps, 1)
    with Timer() as t_seg:
        for _ in range(10):
            ctx.segment(d_tok, d_bm, wl.vocab, seg_id, sent_off, sent_len, n_sent, sync=False)
    with Timer() as t_sv:
        for _ in range(10):
            ctx.build_semvec(p.K, sent_off, S, semvec)
    sv_bytes = L * H * T * D * wl.elt_bytes + L * H * S * D * 4
    seg_bytes = 2 * 4 * T + 4 * T + 8 * S
    gbps = (sv_bytes + seg_bytes) / (ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        orc = oracle.get("f32")
        K0 = gen.to_numpy(p.K[:1])
        t0 = time.perf_counter()
        _, off, _, _ = orc.segment(p.tok, p.bitmap, wl.vocab)
        n = 0
        while True:
            orc.semvec(K0, off)
            n += 1
            if time.perf_counter() - t0 > args.cpu_seconds:
                break
        dt = time.perf_counter() - t0
        cpu = {"value": round(n * (sv_bytes / L) / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "segmentation once + mean keys of layer 0 (%d of %d layers) %d times, single thread, fp32" % (1, L, n)}
    sv_gbps = sv_bytes / (t_sv.ms / 10 * 1e-3) / 1e9
    return {
        "metric": "prefill segmentation + semantic-vector build, achieved HBM GB/s at %s tokens" % _ctx_name(T),
        "value": round(gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "layers": L, "kv_heads": H, "head_dim": D, "tokens": T, "sentences": S,
                   "path": "skv_segment + skv_build_semvec"},
        "segment_us": round(t_seg.ms * 100, 2), "semvec_ms": round(t_sv.ms / 10, 4), "bytes_per_step": int(sv_bytes + seg_bytes),
        "roofline": dict(bound="hbm", kernel="semvec_kernel", achieved=round(sv_gbps, 1), peak=HBM_PEAK_GBPS, unit="GB/s",
                         frac=round(sv_gbps / HBM_PEAK_GBPS, 4), traffic=measured_traffic(wl.name, "semvec_kernel"),
                         bytes_per_launch=int(sv_bytes)),
        "cpu_baseline": cpu,
    }


def run_retention(args, wl):
    """Prefill-side token retention on cfg3's prompt: observation-window importance (N = 32 window tokens), global
    top-k with k = 2 x 2048 (r = 2, budget 2048), pool compaction and the mean keys of the retained buckets."""
    dev = "cuda:0"
    L, H, Hq, D, T = wl.n_layers, wl.n_kv_heads, wl.n_q_heads, wl.head_dim, wl.n_tokens
    N, k = args.window, args.keep
    Tp = T - N
    p = gen.prefill_inputs(wl, seed=args.seed, device=dev)
    V = torch.empty_like(p.K)
    for l in range(L):
        V[l].copy_(gen.kv_layer(p.lengths, H, D, wl.torch_dtype, args.seed, l, dev)[1])
    q_obs = gen.queries(L * Hq, N, D, wl.torch_dtype, args.seed + 2, dev).view(L, Hq, N, D)
    S_cap = len(p.lengths) + 64
    ctx = skv.Context(skv.Desc(n_layers=L, n_q_heads=Hq, n_kv_heads=H, kv_dtype=skv.dtype_code(wl.torch_dtype),
                               max_tokens=T, max_sentences=S_cap, max_budget=16, max_batch=1))
    d_tok, d_bm = i32(p.tok, dev), torch.as_tensor(p.bitmap.view(np.int32)).to(dev)
    seg_id = torch.empty(T, dtype=torch.int32, device=dev)
    sent_off = torch.empty(S_cap + 1, dtype=torch.int32, device=dev)
    sent_len = torch.empty(S_cap, dtype=torch.int32, device=dev)
    n_sent = torch.empty(4, dtype=torch.int32, device=dev)
    S = ctx.segment(d_tok, d_bm, wl.vocab, seg_id, sent_off, sent_len, n_sent)
    alpha = torch.empty(L, Tp, dtype=torch.float32, device=dev)
    work = torch.empty(ctx.token_importance_work_bytes(T, N), dtype=torch.uint8, device=dev)
    keep = torch.empty(L, k, dtype=torch.int32, device=dev)
    n_keep = torch.empty(max(L, 4), dtype=torch.int32, device=dev)
    r_off = torch.empty(L, S + 1, dtype=torch.int32, device=dev)
    r_len = torch.empty(L, S, dtype=torch.int32, device=dev)
    K_ret = torch.empty(L, H, k, D, dtype=wl.torch_dtype, device=dev)
    V_ret = torch.empty_like(K_ret)
    semvec = torch.empty(L, H, S, D, dtype=torch.float32, device=dev)

    stages = {
        "importance": lambda: ctx.token_importance(q_obs, p.K, T, N, alpha, work),
        "retain": lambda: ctx.retain(alpha, Tp, k, seg_id, S, keep, n_keep, r_off, r_len),
        "compact": lambda: ctx.compact_pool(p.K, V, T, keep, k, n_keep, K_ret, V_ret),
        "semvec": lambda: ctx.build_semvec_layers(K_ret, r_off, S, semvec),
    }

    def step():
        for fn in stages.values():
            fn()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    with Timer() as t:
        for _ in range(args.steps):
            step()
    ms = t.ms / max(args.steps, 1)
    stage_ms = {}
    for name, fn in stages.items():
        with Timer() as ts:
            for _ in range(5):
                fn()
        stage_ms[name] = round(ts.ms / 5, 4)
    e = wl.elt_bytes
    flops = 2.0 * 2 * L * Hq * N * T * D                      # two sweeps (row statistics, column sums) of Q K^T
    imp_bytes = L * H * T * D * e + L * Hq * N * D * e + L * Tp * 4      # keys once, window queries, alpha
    step_bytes = imp_bytes + L * Tp * 4 + L * k * 4 + 2 * 2 * L * H * k * D * e + L * H * k * D * e + L * H * S * D * 4
    imp_s = stage_ms["importance"] * 1e-3
    tflops = flops / imp_s / 1e12
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        orc = oracle.get("f32")
        q0, K0 = gen.to_numpy(q_obs[0]), gen.to_numpy(p.K[0])
        t0 = time.perf_counter()
        a0 = orc.token_importance(q0, K0)
        orc.retain(a0, k, seg_id.cpu().numpy(), S)
        dt = time.perf_counter() - t0
        cpu = {"value": round(flops / 2 / L / dt / 1e12, 6), "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
               "ms_per_layer": round(dt * 1e3, 1),
               "sample": "importance + retention of layer 0 (1 of %d layers), one sweep of Q K^T, single thread, fp32" % L}
    return {
        "metric": "prefill token retention (importance + top-k + compaction + mean keys), ms per prompt at %s tokens" % _ctx_name(T),
        "value": round(ms, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name + "_retention", "layers": L, "q_heads": Hq, "kv_heads": H, "head_dim": D, "tokens": T,
                   "window": N, "keep": k, "sentences": S,
                   "path": "skv_token_importance + skv_retain + skv_compact_pool + skv_build_semvec_layers"},
        "stage_ms": stage_ms, "bytes_per_step": int(step_bytes), "GBps": round(step_bytes / (ms * 1e-3) / 1e9, 1),
        # The importance is a dense contraction (MFMA) but sweeps the keys twice with ~256 flop per key byte: HBM time
        # dominates, so it is priced against HBM on its algorithmic bytes (keys ONCE); the MFMA figures are given too.
        "roofline": dict(bound="hbm", kernel="importance_stats_kernel + importance_colsum_kernel",
                         achieved=round(imp_bytes / imp_s / 1e9, 1), peak=HBM_PEAK_GBPS, unit="GB/s",
                         frac=round(imp_bytes / imp_s / 1e9 / HBM_PEAK_GBPS, 4), traffic=measured_traffic(wl.name, "importance"),
                         bytes_per_launch=int(imp_bytes), ms_per_launch=stage_ms["importance"],
                         mfma_TFLOPs=round(tflops, 1), mfma_peak_TFLOPs=2500.0, mfma_frac=round(tflops / 2500.0, 4),
                         flops_per_launch=int(flops)),
        "cpu_baseline": cpu,
    }


STAMP_LABELS = {0: "kernel start", 12: "own share of the scores stored", 13: "all scores of the pair published",
                1: "buckets in registers", 2: "cut known", 3: "selection compacted", 4: "pool rows of the block's positions",
                5: "K/V loads issued", 6: "logits and value tile done", 7: "partial written", 8: "arrived at the pair's counter",
                10: "partials loaded (merging block)", 11: "merged in LDS (merging block)", 9: "output written (merging block)"}


def run_phase_stamps(args, wl, budget):
    """Phase stamps of skv_decode_step's last kernel (profiling build, csrc/skv_stamps.h): one launch at a time, the
    100 MHz clock of thread 0 of every block at the marked places, relative to the launch's first block start."""
    import ctypes
    from paper_2504_00970_amd import binding
    lib = binding._lib()
    lib.skv_stamps_read.argtypes, lib.skv_stamps_read.restype = [ctypes.c_void_p, ctypes.c_int], ctypes.c_int
    dev = "cuda:0"
    H, Hq, D = wl.n_kv_heads, wl.n_q_heads, wl.head_dim
    B = max(wl.batch, 1)
    R = min(wl.n_layers, args.resident_layers)
    if wl.batch > 1:
        inp = gen.ragged_inputs(wl, seed=args.seed, device=dev, resident_layers=R)
    else:
        w1 = wl.scaled(batch=1, t_range=(wl.n_tokens, wl.n_tokens), budgets=(budget,))
        inp = gen.ragged_inputs(w1, seed=args.seed, device=dev, resident_layers=R)
    T_total, S_total = int(inp.cu_tok[-1]), int(inp.cu_sent[-1])
    budget = int(inp.budget.max())
    sv_bytes, sv_torch, sv_code = SV_TABLE[args.semvec_dtype]
    ctx = skv.Context(skv.Desc(n_layers=R, n_q_heads=Hq, n_kv_heads=H, kv_dtype=skv.dtype_code(wl.torch_dtype),
                               max_tokens=T_total, max_sentences=S_total, max_budget=budget, max_batch=B, semvec_dtype=sv_code))
    semvec = torch.empty(R, H, S_total, D, dtype=sv_torch, device=dev)
    ctx.build_semvec(inp.K, i32(gen.offsets_of(inp.sent_len), dev), S_total, semvec)
    d = [i32(x, dev) for x in (inp.cu_tok, inp.cu_sent, inp.sent_off, inp.sent_len, inp.budget)]
    qsets = gen.queries(N_QUERY_SETS * R * B, Hq, D, wl.torch_dtype, args.seed + 1, dev).view(N_QUERY_SETS, R, B, Hq, D)
    out = torch.empty(B, Hq, D, dtype=torch.float32, device=dev)
    n_words = 4096 * 16
    buf = np.zeros(n_words, dtype=np.uint64)

    def read():
        assert lib.skv_stamps_read(buf.ctypes.data, n_words) == 0
        return buf.reshape(4096, 16).astype(np.int64)

    def step(i):
        r = i % R
        q = qsets[i % N_QUERY_SETS, r]
        ctx.decode_step(r, B, q, q, inp.K, inp.V, T_total, semvec, S_total, *d, out, None, None, None)

    for i in range(args.warmup * R):
        step(i)
    read()
    rel = {k: [] for k in STAMP_LABELS}
    launches = max(args.steps, 1)
    per_block = []                         # [launch][block][slot], us since the launch's first block start (< 0: not stamped)
    for i in range(launches):
        for j in range(3):                 # the stamped launch follows two others back to back, as in a decode step
            step(i * 3 + j)
        st = read()                        # the table holds the last writer of every slot: with identical grids, the last launch
        t0 = st[:, 0][st[:, 0] > 0].min()
        for k in STAMP_LABELS:
            col = st[:, k]
            rel[k].append((col[col >= t0] - t0) / 100.0)
        per_block.append((st - t0) / 100.0)
    rows = []
    for k, name in STAMP_LABELS.items():
        x = np.concatenate(rel[k]) if rel[k] else np.zeros(0)
        if len(x) == 0:
            continue
        rows.append({"slot": k, "phase": name, "blocks_per_launch": round(len(x) / launches, 1),
                     "median_us": round(float(np.median(x)), 2), "p10_us": round(float(np.percentile(x, 10)), 2),
                     "p90_us": round(float(np.percentile(x, 90)), 2), "max_us": round(float(x.max()), 2)})
    rows.sort(key=lambda r: r["median_us"])
    # The same stamps block by block (blocks are numbered x + gridDim.x * y; the hardware deals consecutive blocks to the
    # XCDs in turn): where the "logits and value tile done" stamp (slot 6: the block's streaming is over) falls by block
    # number modulo 8, how much one block's time varies from launch to launch, and how much the blocks' means differ.
    pb = np.stack(per_block)
    n_blocks = int((pb[0, :, 6] >= 0).sum())
    spread = None
    if n_blocks >= 8 and all(int((x[:, 6] >= 0).sum()) == n_blocks for x in pb):
        done, issued = pb[:, :n_blocks, 6], pb[:, :n_blocks, 5]
        mean_b = done.mean(axis=0)
        spread = {"blocks": n_blocks, "slot": 6,
                  "mean_done_us_by_block_mod_8": [round(float(done[:, k::8].mean()), 2) for k in range(8)],
                  "std_over_launches_of_one_block_us": round(float(done.std(axis=0).mean()), 2),
                  "std_over_blocks_of_their_means_us": round(float(mean_b.std()), 2),
                  "block_means_min_max_us": [round(float(mean_b.min()), 2), round(float(mean_b.max()), 2)]}
        if B > 1 and n_blocks % B == 0:    # blocks of a sequence are contiguous: (pairs of the sequence) x (blocks per pair)
            per = n_blocks // B
            spread["by_sequence"] = [{"buckets": int(inp.cu_sent[s + 1] - inp.cu_sent[s]),
                                      "kv_issued_us": round(float(issued[:, s * per:(s + 1) * per].mean()), 2),
                                      "done_us": round(float(done[:, s * per:(s + 1) * per].mean()), 2)} for s in range(B)]
    return {"phase_stamps": rows, "per_block": spread, "workload": wl.name, "batch": B, "budget": budget, "tokens_total": T_total,
            "sentences_total": S_total, "launches": launches, "semvec_dtype": args.semvec_dtype,
            "note": "us since the first block start of the launch; thread 0 of every block; kernel = the last launch of skv_decode_step"}


def run_launch_floor(args):
    """What a dependent chain of near-empty kernels costs on this GPU: 32 "layers" of 1, 2 or 3 launches of the library's
    smallest kernel (skv_merge_lse on one head: 64 threads, 1 KB) replayed as a HIP graph, and launched directly.  The
    decode step of one sequence cannot be faster per layer than the chain with as many launches per layer."""
    dev = "cuda:0"
    ctx = skv.Context(skv.Desc(n_layers=1, n_q_heads=8, n_kv_heads=8, kv_dtype=skv.SKV_BF16, max_tokens=64, max_sentences=8,
                               max_budget=16, max_batch=1))
    a, b, o = (torch.zeros(8, 128, device=dev) for _ in range(3))
    la, lb, lo = (torch.zeros(8, device=dev) for _ in range(3))
    L, rows = 32, []
    for per_layer in (1, 2, 3):
        def chain():
            for _ in range(L * per_layer):
                ctx.merge_lse(1, a, la, b, lb, o, lo)
        chain()
        g = capture(ctx, chain)
        res = {}
        for name, fn in (("graph", g.replay), ("direct", chain)):
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            reps = max(args.steps, 20)
            with Timer() as t:
                for _ in range(reps):
                    fn()
            res[name] = t.ms * 1e3 / (reps * L)
        rows.append({"launches_per_layer": per_layer, "us_per_layer_hip_graph": round(res["graph"], 3),
                     "us_per_layer_direct_launch": round(res["direct"], 3),
                     "us_per_launch_hip_graph": round(res["graph"] / per_layer, 3)})
    return {"metric": "launch floor: dependent chain of near-empty kernels", "unit": "us/layer", "layers": L,
            "kernel": "merge_lse_kernel (1 head, 64 threads)", "rows": rows}


def _ctx_name(T):
    return "%dk" % (T // 1024) if T % 1024 == 0 else str(T)


def cpu_baseline(args, wl, inp, semvec, lengths, qsets, budget):
    """The CPU oracle, as it stands, on the same inputs: whole decode steps (all layers) until ~10 s."""
    import oracle
    orc = oracle.get("f32")
    L, H = wl.n_layers, wl.n_kv_heads
    off = gen.offsets_of(lengths)
    n_layers = min(L, args.cpu_layers)
    Kh = [gen.to_numpy(inp.K[l]) for l in range(n_layers)]
    Vh = [gen.to_numpy(inp.V[l]) for l in range(n_layers)]
    svh = [gen.to_numpy(semvec[l]) for l in range(n_layers)]
    qh = [gen.to_numpy(qsets[0, l]) for l in range(n_layers)]
    done, t_total, n_tok_sum = 0, 0.0, 0
    t_end = time.perf_counter() + args.cpu_seconds
    while True:
        for l in range(n_layers):
            t0 = time.perf_counter()
            r = orc.decode_step(qh[l], qh[l], Kh[l], Vh[l], svh[l], off, lengths, budget)
            t_total += time.perf_counter() - t0
            n_tok_sum += int(r["n_tok"].sum())
            done += 1
        if time.perf_counter() > t_end:
            break
    us_layer = t_total / done * 1e6
    b = decode_bytes(wl, len(lengths), n_tok_sum / done, n_tok_sum / done / float(lengths.mean()), fused=True)
    res = {"value": round(b["total"] / (us_layer * 1e-6) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
           "us_per_layer": round(us_layer, 1),
           "sample": "%d layer-steps of the same workload (layers 0..%d, query set 0), score+select+gather+attend, "
                     "single thread, fp32" % (done, n_layers - 1)}
    # The same oracle calls on all host cores of the box's share: independent layers side by side, one call per thread
    # (the C library runs outside the interpreter lock).  Nothing in the oracle is tuned for this.
    from concurrent.futures import ThreadPoolExecutor
    threads = max(1, min(16, os.cpu_count() or 1, n_layers))
    budget_s = max(2.0, args.cpu_seconds / 2)

    def one(l):
        orc.decode_step(qh[l], qh[l], Kh[l], Vh[l], svh[l], off, lengths, budget)

    done_p, t0 = 0, time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as pool:
        while True:
            list(pool.map(one, range(n_layers)))
            done_p += n_layers
            if time.perf_counter() - t0 > budget_s:
                break
    us_layer_p = (time.perf_counter() - t0) / done_p * 1e6
    res["all_cores"] = {"value": round(b["total"] / (us_layer_p * 1e-6) / 1e9, 4), "unit": "GB/s", "cores": threads,
                        "us_per_layer": round(us_layer_p, 1),
                        "sample": "%d layer-steps, %d threads each running whole layers of the same workload" % (done_p, threads)}
    return res


def measured_copy_peak(dev="cuda:0", mib=1024, reps=5):
    """Device-to-device copy rate of this GPU (a library copy kernel on 1 GiB: bytes read + bytes written per second),
    the achievable yardstick beside the datasheet figure."""
    src = torch.empty(mib << 20, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    with Timer() as t:
        for _ in range(reps):
            dst.copy_(src)
    return 2.0 * reps * (mib << 20) / (t.ms * 1e-3) / 1e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg1", choices=["cfg0", "cfg1", "cfg2", "cfg3", "cfg3-retain", "cfg4", "floor"])
    ap.add_argument("--window", type=int, default=32, help="cfg3-retain: observation-window tokens")
    ap.add_argument("--keep", type=int, default=4096, help="cfg3-retain: tokens retained per layer (floor(r tau))")
    ap.add_argument("--resident-layers", type=int, default=4, help="cfg4: layers of the pool kept in HBM")
    ap.add_argument("--batch", type=int, default=0, help="cfg4: number of sequences (default 16); cfg1, cfg2: that many sequences of the workload's context in one batch")
    ap.add_argument("--batched-sequences", default="16,64",
                    help="cfg1 without --batch: also time the step for these many sequences in one batch (comma-separated) "
                         "and report them under \"batched\" (0: skip)")
    ap.add_argument("--budget", type=int, default=0, help="token budget (default: the workload's largest)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--semvec-dtype", default="f32", choices=["f32", "bf16", "fp8"],
                    help="storage of the mean key vectors (decode workloads); bf16 = the fp32 mean rounded once")
    ap.add_argument("--launch", default="graph", choices=["graph", "direct"],
                    help="graph: the step's launches replayed as one HIP graph; direct: one host call per layer")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--cpu-layers", type=int, default=32)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="cfg1: skip the cfg2 (128K) and cfg4 (ragged batch) measurements reported under \"extras\"")
    ap.add_argument("--phase-stamps", action="store_true",
                    help="decode workloads: load the profiling build (python -m paper_2504_00970_amd._build --stamps) and "
                         "print where the blocks of the step's last kernel spend their time instead of the benchmark line")
    ap.add_argument("--host-pool-layers", type=int, default=-1,
                    help="layers of the K/V pool also kept in pinned host memory for the host-pool gather measurement "
                         "(default: 2 for cfg2, 0 otherwise)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no multi-GPU form in this build (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    if args.phase_stamps:
        from paper_2504_00970_amd import _build
        if _build.stale(_build.LIB_STAMPS):
            print("no profiling build of the current sources: run `python -m paper_2504_00970_amd._build --stamps` first",
                  file=sys.stderr)
            sys.exit(2)
        _build.LIB = _build.LIB_STAMPS
    if args.workload == "floor":
        print(json.dumps(run_launch_floor(args)), flush=True)
        return
    retain = args.workload == "cfg3-retain"
    wl = gen.CONFIGS["cfg3" if retain else args.workload]
    if args.batch > 0 and args.workload == "cfg4":
        wl = wl.scaled(batch=args.batch)
    elif args.batch > 1 and args.workload in ("cfg1", "cfg2"):
        # The same decode step for `batch` sequences of the workload's context, each with its own sentence structure.
        wl = wl.scaled(name="%s_x%d" % (wl.name, args.batch), batch=args.batch, t_range=(wl.n_tokens, wl.n_tokens),
                       budgets=(args.budget or max(wl.budgets),))
    if args.host_pool_layers < 0:
        args.host_pool_layers = 2 if args.workload == "cfg2" else 0
    if args.phase_stamps and not retain and args.workload != "cfg3":
        res = run_phase_stamps(args, wl, args.budget or max(wl.budgets))
        print(json.dumps(res), flush=True)
        return
    if retain:
        res = run_retention(args, wl)
    elif args.workload == "cfg3":
        res = run_prefill(args, wl)
    elif wl.batch > 1:
        res = run_ragged(args, wl)
    else:
        res = run_single_sequence(args, wl, args.budget or max(wl.budgets))
        import copy
        sizes = [int(x) for x in args.batched_sequences.split(",") if x.strip()] if args.workload == "cfg1" else []
        for Bs in [b for b in sizes if b > 1]:
            # the same step for a batch of sequences of the same context, each with its own buckets: what the kernels reach
            # once a launch has enough work (reported extras, never `value`)
            a2 = copy.copy(args)
            a2.steps, a2.warmup, a2.no_cpu_baseline = min(args.steps, 10), min(args.warmup, 2), True
            wb = wl.scaled(name="%s_x%d" % (wl.name, Bs), batch=Bs, t_range=(wl.n_tokens, wl.n_tokens),
                           budgets=(args.budget or max(wl.budgets),))
            rb = run_ragged(a2, wb)
            res.setdefault("batched", []).append(
                {"workload": wb.name, "sequences": Bs, "us_per_layer": rb["us_per_layer"], "value": rb["value"],
                 "unit": rb["unit"], "hbm_frac": rb["hbm_frac"], "bytes_per_layer": rb["bytes_per_layer"],
                 "resident_layers": args.resident_layers, "steps": a2.steps})
            torch.cuda.empty_cache()
        if args.workload == "cfg1" and not args.no_extras:
            # The other configurations the target names, each measured like the headline (never `value`): the 128K
            # context (pool in HBM; the gather from a pinned host pool separately) and the ragged 70B-shaped batch.
            res["extras"] = []
            a2 = copy.copy(args)
            a2.steps, a2.warmup, a2.no_cpu_baseline, a2.host_pool_layers = min(args.steps, 10), min(args.warmup, 2), True, 2
            torch.cuda.empty_cache()
            r2 = run_single_sequence(a2, gen.CONFIGS["cfg2"], max(gen.CONFIGS["cfg2"].budgets))
            res["extras"].append({"workload": r2["config"]["workload"], "context": r2["config"]["context"],
                                  "sentences": r2["config"]["sentences"], "budget": r2["config"]["budget"], "kv_pool": "hbm",
                                  "us_per_layer": r2["us_per_layer"], "value": r2["value"], "unit": r2["unit"],
                                  "hbm_frac": r2["hbm_frac"], "bytes_per_layer": r2["bytes_per_layer"], "steps": a2.steps,
                                  "frac_of_measured_copy_peak": r2["roofline"]["frac_of_measured_copy_peak"],
                                  "host_pool_gather": r2["host_pool_gather"]})
            del r2
            torch.cuda.empty_cache()
            a4 = copy.copy(a2)
            a4.steps = min(args.steps, 5)
            r4 = run_ragged(a4, gen.CONFIGS["cfg4"])
            res["extras"].append({"workload": r4["config"]["workload"], "sequences": r4["config"]["batch"],
                                  "tokens_total": r4["config"]["tokens_total"], "budget": r4["config"]["budget"],
                                  "resident_layers": r4["config"]["resident_layers"], "us_per_layer": r4["us_per_layer"],
                                  "value": r4["value"], "unit": r4["unit"], "hbm_frac": r4["hbm_frac"],
                                  "bytes_per_layer": r4["bytes_per_layer"], "steps": a4.steps,
                                  "launches_per_layer": 2})
            torch.cuda.empty_cache()
    res["host"] = {"nproc": os.cpu_count()}
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
