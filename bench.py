#!/usr/bin/env python3
"""Benchmark of the SLA chunked forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

A step is one pass of the whole hot path (one ``sla_forward`` call: head softmax, decay products,
intra-block scores and outputs, state read-out, gated epilogue, state update, final state) over one
batch of seeded synthetic input that is already resident in HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "tokens/sec SLA-GLA chunked fwd (B=8,T=2048,H=16,d=128 bf16); % MFMA peak"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


def rel_err(x, ref) -> float:
    """max|x - ref| / max|ref| (the parity gate's error measure)."""
    import numpy as np

    denom = float(np.max(np.abs(ref)))
    if denom == 0.0:
        return float(np.max(np.abs(x)))
    return float(np.max(np.abs(x - ref))) / denom


def source_digest() -> str:
    """sha256 over the kernel sources (csrc/*, include/sla.h), in name order: what a profile summary was taken from."""
    import hashlib

    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2602_01744_amd", "csrc")
    files = sorted(os.path.join(csrc, f) for f in os.listdir(csrc) if f.endswith((".hip", ".h")))
    for f in files + [os.path.join(ROOT, "include", "sla.h")]:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(key: str):
    """HBM bytes per call measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and calibrated against a plain copy
    of known size, as recorded in the summaries under profiles/ (a line `traffic-json: {...}` per summary; commands
    and raw counters are in the same file).  Returns {"bytes", "profile", "commit", "stale"} or None.  stale = the
    kernel sources have changed since the summary was taken."""
    pdir = os.path.join(ROOT, "profiles")
    best = None
    for name in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not name.endswith(".md"):
            continue
        for line in open(os.path.join(pdir, name), encoding="utf-8"):
            if line.startswith("traffic-json:"):
                try:
                    rec = json.loads(line[len("traffic-json:"):])
                except ValueError:
                    continue
                if key in rec.get("bytes", {}):
                    best = {"bytes": rec["bytes"][key], "profile": "profiles/" + name, "commit": rec.get("commit"),
                            "stale": rec.get("sources") != source_digest()}
    return best


def traffic_fields(key: str) -> dict:
    t = measured_traffic(key)
    if t is None:
        return {"traffic": None}
    out = {"traffic": t["bytes"], "traffic_source": t["profile"], "traffic_commit": t["commit"]}
    if t["stale"]:
        out["traffic_warning"] = "kernel sources changed since this profile summary was taken"
    return out


MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
BLOCK = 16                      # tokens per state step in the kernels (for the causal flop count)


def algorithmic_bytes(w) -> int:
    """One read of every input and one write of every output (the per-token figure of the design notes
    times the tokens of the workload, plus the final state)."""
    es = 2 if w.dtype == "bf16" else 4
    per_token_head = (2 * w.dk + 2 * w.dv) * es + 8  # q, k, v, out + two fp32 gate logits
    if w.variant == 1:
        per_token_head += w.dk * es  # per-dimension log-decay
    elif w.variant == 2:
        per_token_head += 8  # scalar log-decay and beta
    return w.B * w.T * w.H * per_token_head + w.B * w.H * w.dk * w.dv * 4


def algorithmic_flops(w) -> int:
    """Multiply-adds the method needs, counted as 2 flops, with only the causal half of the score tiles:
    read-out and state update 4*dk*dv per token-head, scores and their product with V (C+1)(dk+dv) for
    a chunk of C = 64 (the staging size); the delta rule adds its own products."""
    C = 64
    per = 4 * w.dk * w.dv + (C + 1) * (w.dk + w.dv)
    if w.variant == 2:
        per += 2 * w.dk * w.dv + (C + 1) * (w.dk + w.dv) + (C * C) // 3
    return w.B * w.T * w.H * per


def decode_bytes(w) -> int:
    """One decode step: the fp32 state is read and rewritten; q, k, v, out, decay, logits once."""
    es = 2 if w.dtype == "bf16" else 4
    per_head = 2 * w.dk * w.dv * 4 + (2 * w.dk + 2 * w.dv) * es + 8
    if w.variant == 1:
        per_head += w.dk * es
    elif w.variant == 2:
        per_head += 8
    return w.B * w.H * per_head


def backward_bytes(w) -> int:
    """One read of every input of sla_backward (q, k, v, d_out, logits, GLA decay) and one write of every
    gradient (dq, dk, dv, logit gradients, GLA decay gradient)."""
    es = 2
    per = (2 * w.dk + 2 * w.dv) * es + 8 + (2 * w.dk + w.dv) * es + 8
    if w.variant == 1:
        per += 2 * w.dk * es
    if w.variant == 2:  # scalar decay and beta read, their gradients written (fp32)
        per += 16
    return w.B * w.T * w.H * per


def bench_backward(args, w, sla, si, torch, np) -> int:
    """--backward: a step is one sla_backward call (gate evaluation, the dq / dv / dk sweeps, softmax backward)
    over the workload's batch, inputs and cotangents resident in HBM."""
    to_device = si.to_device

    if w.dtype != "bf16" or (w.variant == 2 and args.head_major):
        print("bench.py: --backward covers the bf16 workloads ([B,T,H,d] layout only for the delta rule)",
              file=sys.stderr)
        return 2
    d = si.generate(w)
    cot = si.cotangents(w.B, w.T, w.H, w.dk, w.dv, seed=w.seed + 50)
    g, tdt = to_device(d, w.dtype, w.variant)
    dev = torch.device("cuda:0")
    dout = torch.from_numpy(cot["d_out"]).to(torch.bfloat16).to(dev)
    hm = args.head_major
    if hm:  # the same values, q / k / v / d_out / decay (and the gradients) laid out [B,H,T,d]
        for n in ("q", "k", "v") + (("log_decay",) if w.variant == 1 else ()):
            g[n] = g[n].permute(0, 2, 1, 3).contiguous()
        dout = dout.permute(0, 2, 1, 3).contiguous()
    gdn = w.variant == 2
    params = sla.SlaParams(w.variant, 1, w.B, w.T, w.H, w.dk, w.dv, 0, sla.FLAG_HEAD_MAJOR if hm else 0, 1)
    # the backward cuts rows into segments only when told to; --segments 0 (the default) takes the library's advice
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    nseg = 1 if (gdn or hm) else (args.segments if args.segments > 0 else max(sla.sla_backward_segments(params, cus), 1))
    params.segments = nseg
    need = sla.sla_backward_gdn_workspace_bytes(params) if gdn else sla.sla_backward_workspace_bytes(params)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    gr = {
        "dq": torch.empty_like(g["q"]), "dk": torch.empty_like(g["k"]), "dv": torch.empty_like(g["v"]),
        "dq_logits": torch.empty_like(g["q_logits"]), "dk_logits": torch.empty_like(g["k_logits"]),
        "dlog_decay": torch.empty_like(g["log_decay"]) if w.variant != 0 else None,
        "dbeta": torch.empty_like(g["beta"]) if gdn else None,
    }
    ptr = lambda t: None if t is None else t.data_ptr()
    raw_gdn = (ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(g["q_logits"]), ptr(g["k_logits"]), ptr(g["log_decay"]),
               ptr(g["beta"]), None, ptr(dout), None, ptr(gr["dq"]), ptr(gr["dk"]), ptr(gr["dv"]), ptr(gr["dq_logits"]),
               ptr(gr["dk_logits"]), ptr(gr["dlog_decay"]), ptr(gr["dbeta"]), None, ptr(ws), need,
               torch.cuda.current_stream(dev).cuda_stream)
    raw = (ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(g["q_logits"]), ptr(g["k_logits"]), ptr(g["log_decay"]), None,
           ptr(dout), None, ptr(gr["dq"]), ptr(gr["dk"]), ptr(gr["dv"]), ptr(gr["dq_logits"]), ptr(gr["dk_logits"]),
           ptr(gr["dlog_decay"]), None, ptr(ws), need, torch.cuda.current_stream(dev).cuda_stream)

    def step():
        rc = sla.sla_backward_gdn(params, *raw_gdn) if gdn else sla.sla_backward(params, *raw)
        if rc != 0:
            raise sla.SlaError(rc, sla.sla_status_string(rc))

    for _ in range(args.settle + args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(args.steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_call_ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps)]
    call_ms = float(np.mean(per_call_ms))
    ms_per_step = wall * 1e3 / args.steps
    abytes = backward_bytes(w)
    achieved = abytes / (call_ms * 1e-3) / 1e9
    result = {
        "metric": f"tokens/sec SLA-{si.VARIANT_NAMES[w.variant].upper()} chunked bwd",
        "value": w.tokens() / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_launches": args.settle,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: backward of SLA-{si.VARIANT_NAMES[w.variant].upper()} B={w.B} T={w.T} H={w.H} "
                        f"dk={w.dk} dv={w.dv} bf16 in/out, dual head-softmax gates, no state cotangents"
                        + (", wide tensors laid out [B,H,T,d]" if hm else "")
                        + (f", {nseg} segments per batch row" if nseg > 1 else ""),
            "kernel": ("sla_backward_gdn (block form): sla_bwd_gates_kernel, gdn_blk_pre_kernel, gdn_blk_state_kernel, "
                       "gdn_blk_cotangent_kernel, gdn_blk_key_kernel, gdn_blk_query_kernel, "
                       "gdn_bwd_finish_kernel, gdn_bwd_decay_scan_kernel") if gdn else
                      "sla_backward: sla_bwd_gates_kernel, sla_bwd_dq_kernel, sla_bwd_dv_kernel, sla_bwd_dk_kernel, "
                      "sla_bwd_logits_kernel x2"
                      + (" after the segment pre-passes (sla_fwd_kernel state-only, sla_segment_combine_kernel, "
                         "sla_bwd_dv_kernel state-only, sla_bwd_segment_combine_kernel)" if nseg > 1 else ""),
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            **({"traffic": None} if hm else traffic_fields(w.name + ":backward")),
            "kernel_us": call_ms * 1e3,
            "kernel_us_min": float(np.min(per_call_ms)) * 1e3,
            "algorithmic_bytes": abytes,
            "note": "whole call (%s launches); achieved = algorithmic bytes / call time"
                    % ("nine" if gdn else "six" if nseg == 1 else "thirteen")
                    + ("; the sweeps pass res, w, the 32 x 32 block matrices and part of dk through the workspace, "
                       "about five times the algorithmic bytes, and run at the memory system's speed on those" if gdn else ""),
        },
    }
    if not args.no_cpu_baseline or not args.no_parity:
        import oracle

        bt = d["beta"] if gdn else None
        t0 = time.perf_counter()  # the C gradient oracle on the whole workload, all host threads
        ref = oracle.backward(w.variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"],
                              cot["d_out"], beta=bt)
        cpu_s = time.perf_counter() - t0
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = {
                "value": w.tokens() / cpu_s,
                "unit": "tokens/s",
                "cores": oracle.threads(0),
                "kind": "oracle",
                "sample": f"C gradient oracle (fp64) on the full workload, {w.tokens()} tokens x {w.H} heads, {cpu_s:.2f} s wall",
            }
        if not args.no_parity:
            step()
            torch.cuda.synchronize()
            def f64(t):
                if hm and t.dim() == 4:
                    t = t.permute(0, 2, 1, 3)
                return t.to(torch.float32).cpu().numpy().astype(np.float64)
            names = {"dq": "dq", "dk": "dk", "dv": "dv", "dq_logits": "dq_logits", "dk_logits": "dk_logits"}
            if w.variant != 0:
                names["dlog_decay"] = "dlog_decay"
            if gdn:
                names["dbeta"] = "dbeta"
            result["parity"] = {n + "_rel_err": rel_err(f64(gr[n]), ref[rn]) for n, rn in names.items()}
            result["parity"]["definition"] = "max|x - oracle| / max|oracle| per gradient tensor, every batch row"
    print(json.dumps(result), flush=True)
    return 0


def bench_train_step(args, w, sla, si, torch, np) -> int:
    """--train-step: a step is everything the mixer's hot path does in one training iteration: the gate logits
    (sla_gate_logits), the forward (sla_forward) and the backward (sla_backward / sla_backward_gdn), launched back to
    back on one stream with all buffers allocated up front."""
    to_device = si.to_device

    if w.dtype != "bf16":
        print("bench.py: --train-step covers the bf16 workloads", file=sys.stderr)
        return 2
    d = si.generate(w)
    g, tdt = to_device(d, w.dtype, w.variant)
    dev = torch.device("cuda:0")
    gw = si.gate_weights(w.H, w.dk, seed=w.seed + 60)
    wq, wk = torch.from_numpy(gw["w_gq"]).to(dev), torch.from_numpy(gw["w_gk"]).to(dev)
    dout = torch.from_numpy(si.cotangents(w.B, w.T, w.H, w.dk, w.dv, seed=w.seed + 50)["d_out"]).to(torch.bfloat16).to(dev)
    gdn = w.variant == 2
    pf = sla.SlaParams(w.variant, 1, w.B, w.T, w.H, w.dk, w.dv, 0, 0, 1)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    nseg = 1 if gdn else (args.segments if args.segments > 0 else max(sla.sla_backward_segments(pf, cus), 1))
    pb = sla.SlaParams(w.variant, 1, w.B, w.T, w.H, w.dk, w.dv, 0, 0, nseg)
    ql = torch.empty((w.B, w.T, w.H), dtype=torch.float32, device=dev)
    kl = torch.empty_like(ql)
    out = torch.empty_like(g["v"])
    fin = torch.empty((w.B, w.H, w.dk, w.dv), dtype=torch.float32, device=dev)
    grads = [torch.empty_like(g["q"]), torch.empty_like(g["k"]), torch.empty_like(g["v"]), torch.empty_like(ql),
             torch.empty_like(kl)]
    dld = torch.empty_like(g["log_decay"]) if w.variant != 0 else None
    dbeta = torch.empty_like(g["beta"]) if gdn else None
    need = sla.sla_backward_gdn_workspace_bytes(pb) if gdn else sla.sla_backward_workspace_bytes(pb)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    dwq, dwk = torch.empty_like(wq), torch.empty_like(wk)
    gneed = sla.sla_gate_logits_backward_workspace_bytes(pf)
    gws = torch.empty(max(gneed, 16), dtype=torch.uint8, device=dev)
    ptr = lambda t: None if t is None else t.data_ptr()
    st = torch.cuda.current_stream(dev).cuda_stream

    def step():
        rc = sla.sla_gate_logits(pf, ptr(g["q"]), ptr(g["k"]), ptr(wq), ptr(wk), ptr(ql), ptr(kl), st)
        rc = rc or sla.sla_forward(pf, ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(ql), ptr(kl), ptr(g["log_decay"]),
                                   ptr(g["beta"]), None, ptr(out), ptr(fin), st)
        if gdn:
            rc = rc or sla.sla_backward_gdn(pb, ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(ql), ptr(kl),
                                            ptr(g["log_decay"]), ptr(g["beta"]), None, ptr(dout), None,
                                            *(ptr(t) for t in grads), ptr(dld), ptr(dbeta), None, ptr(ws), need, st)
        else:
            rc = rc or sla.sla_backward(pb, ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(ql), ptr(kl), ptr(g["log_decay"]),
                                        None, ptr(dout), None, *(ptr(t) for t in grads), ptr(dld), None, ptr(ws), need, st)
        # the projections' share of dq, dk (added in place) and the gate matrices' gradients
        rc = rc or sla.sla_gate_logits_backward(pf, ptr(g["q"]), ptr(wq), ptr(grads[3]), ptr(grads[0]), ptr(dwq),
                                                ptr(gws), gneed, st)
        rc = rc or sla.sla_gate_logits_backward(pf, ptr(g["k"]), ptr(wk), ptr(grads[4]), ptr(grads[1]), ptr(dwk),
                                                ptr(gws), gneed, st)
        if rc != 0:
            raise sla.SlaError(rc, sla.sla_status_string(rc))

    settle = min(args.settle, 50) if gdn else args.settle
    for _ in range(settle + args.warmup):
        step()
    torch.cuda.synchronize()
    steps = min(args.steps, 50) if gdn else args.steps
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]
    call_ms = float(np.mean(per_ms))
    ms_per_step = wall * 1e3 / steps
    es = 2
    # gate logits: q, k read, two logit tensors written; their backward: q, k, dq, dk, the logit cotangents read,
    # dq, dk written, the gate matrices' gradients written
    abytes = ((2 * w.B * w.T * w.H * (w.dk * es + 4) + 2 * w.H * w.dk * 4) + algorithmic_bytes(w) + backward_bytes(w)
              + 2 * w.B * w.T * w.H * (3 * w.dk * es + 4) + 2 * w.H * w.dk * 4)
    achieved = abytes / (call_ms * 1e-3) / 1e9
    result = {
        "metric": f"tokens/sec SLA-{si.VARIANT_NAMES[w.variant].upper()} mixer training step (gate logits + fwd + bwd + gate projections' bwd)",
        "value": w.tokens() / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "settle_launches": settle,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: gate logits, forward and backward of SLA-{si.VARIANT_NAMES[w.variant].upper()} "
                        f"B={w.B} T={w.T} H={w.H} dk={w.dk} dv={w.dv} bf16"
                        + (f", backward in {nseg} segments per batch row" if nseg > 1 else ""),
            "kernel": "sla_gate_logits + sla_forward + " + ("sla_backward_gdn" if gdn else "sla_backward")
                      + " + 2 x sla_gate_logits_backward",
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": None,
            "kernel_us": call_ms * 1e3,
            "kernel_us_min": float(np.min(per_ms)) * 1e3,
            "algorithmic_bytes": abytes,
            "note": "three entry points back to back; achieved = the sum of their algorithmic bytes / step time",
        },
    }
    print(json.dumps(result), flush=True)
    return 0


def bench_prologue(args, w, sla, si, torch, np) -> int:
    """--prologue: a step is one sla_gate_logits call (both gates) over the workload's q and k."""
    to_device = si.to_device

    d = si.generate(w)
    gw = si.gate_weights(w.H, w.dk, seed=w.seed + 60)
    g, tdt = to_device(d, w.dtype, w.variant)
    dev = torch.device("cuda:0")
    wq, wk = torch.from_numpy(gw["w_gq"]).to(dev), torch.from_numpy(gw["w_gk"]).to(dev)
    ql = torch.empty((w.B, w.T, w.H), dtype=torch.float32, device=dev)
    kl = torch.empty_like(ql)
    params = sla.SlaParams(w.variant, 1 if w.dtype == "bf16" else 0, w.B, w.T, w.H, w.dk, w.dv, 0, 0, 1)
    raw = (g["q"].data_ptr(), g["k"].data_ptr(), wq.data_ptr(), wk.data_ptr(), ql.data_ptr(), kl.data_ptr(),
           torch.cuda.current_stream(dev).cuda_stream)

    def step():
        rc = sla.sla_gate_logits(params, *raw)
        if rc != 0:
            raise sla.SlaError(rc, sla.sla_status_string(rc))

    for _ in range(args.settle + args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(args.steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps)]
    kernel_ms = float(np.mean(per_ms))
    ms_per_step = wall * 1e3 / args.steps
    es = 2 if w.dtype == "bf16" else 4
    abytes = 2 * w.B * w.T * w.H * (w.dk * es + 4) + 2 * w.H * w.dk * 4
    achieved = abytes / (kernel_ms * 1e-3) / 1e9
    result = {
        "metric": "tokens/sec SLA gate logits (q W_GQ, k W_GK)",
        "value": w.tokens() / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_launches": args.settle,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: gate logits of both gates, B={w.B} T={w.T} H={w.H} dk={w.dk} {w.dtype} q and k, "
                        f"fp32 weights [H,dk] and logits",
            "kernel": f"sla_gate_logits_kernel<{'true' if w.dtype == 'bf16' else 'false'}, {w.dk}>",
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            **traffic_fields(w.name + ":prologue"),
            "kernel_us": kernel_ms * 1e3,
            "kernel_us_min": float(np.min(per_ms)) * 1e3,
            "algorithmic_bytes": abytes,
        },
    }
    if not args.no_cpu_baseline or not args.no_parity:
        from oracle import sla_numpy

        passes, cpu_s = 0, 0.0
        while True:
            t0 = time.perf_counter()
            rq = sla_numpy.gate_logits(d["q"], gw["w_gq"])
            rk = sla_numpy.gate_logits(d["k"], gw["w_gk"])
            cpu_s += time.perf_counter() - t0
            passes += 1
            if args.no_cpu_baseline or cpu_s >= 10.0 or passes >= 50:
                break
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = {
                "value": w.tokens() * passes / cpu_s,
                "unit": "tokens/s",
                "cores": 1,
                "kind": "oracle",
                "sample": f"the full workload, {passes} pass(es) of the numpy fp64 statement, {cpu_s:.2f} s wall",
            }
        if not args.no_parity:
            step()
            torch.cuda.synchronize()
            result["parity"] = {
                "q_logits_rel_err": rel_err(ql.cpu().numpy().astype(np.float64), rq),
                "k_logits_rel_err": rel_err(kl.cpu().numpy().astype(np.float64), rk),
                "definition": "max|x - oracle| / max|oracle| per tensor",
            }
    print(json.dumps(result), flush=True)
    return 0


def bench_short_conv(args, w, sla, si, torch, np) -> int:
    """--short-conv: a step is one sla_short_conv_silu call (4 taps) over a [B, T, H*dk] tensor of the workload's
    dtype, the shape of the query projection in front of the mixer."""
    dev = torch.device("cuda:0")
    C, taps = w.H * w.dk, 4
    r = np.random.default_rng(w.seed + 80)
    x = r.standard_normal(size=(w.B, w.T, C), dtype=np.float32)
    if w.dtype == "bf16":
        x = si.round_to_bf16(x)
    wt = (r.standard_normal(size=(C, taps), dtype=np.float32) / 2).astype(np.float32)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    xt, wtt = torch.from_numpy(x).to(tdt).to(dev), torch.from_numpy(wt).to(dev)
    y = torch.empty_like(xt)
    raw = (1 if w.dtype == "bf16" else 0, w.B, w.T, C, taps, xt.data_ptr(), wtt.data_ptr(), y.data_ptr(),
           torch.cuda.current_stream(dev).cuda_stream)

    def step():
        rc = sla.sla_short_conv_silu(*raw)
        if rc != 0:
            raise sla.SlaError(rc, sla.sla_status_string(rc))

    for _ in range(args.settle + args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(args.steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps)]
    kernel_ms = float(np.mean(per_ms))
    ms_per_step = wall * 1e3 / args.steps
    es = 2 if w.dtype == "bf16" else 4
    abytes = 2 * w.B * w.T * C * es + C * taps * 4
    achieved = abytes / (kernel_ms * 1e-3) / 1e9
    result = {
        "metric": "tokens/sec short causal convolution + SiLU (4 taps)",
        "value": w.tokens() / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_launches": args.settle,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: short convolution + SiLU over [B={w.B}, T={w.T}, C={C}] {w.dtype}, {taps} taps, fp32 weights",
            "kernel": f"sla_short_conv_silu_kernel<{'true' if w.dtype == 'bf16' else 'false'}, {taps}>",
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": None,
            "kernel_us": kernel_ms * 1e3,
            "kernel_us_min": float(np.min(per_ms)) * 1e3,
            "algorithmic_bytes": abytes,
        },
    }
    if not args.no_cpu_baseline or not args.no_parity:
        from oracle import sla_numpy

        rows = min(w.B, 2)
        t0 = time.perf_counter()
        want = sla_numpy.short_conv_silu(x[:rows], wt)
        cpu_s = time.perf_counter() - t0
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = {
                "value": rows * w.T / cpu_s,
                "unit": "tokens/s",
                "cores": 1,
                "kind": "oracle",
                "sample": f"numpy fp64 statement on {rows} batch row(s), {cpu_s:.2f} s wall",
            }
        if not args.no_parity:
            step()
            torch.cuda.synchronize()
            result["parity"] = {
                "rel_err": rel_err(y[:rows].to(torch.float32).cpu().numpy().astype(np.float64), want),
                "definition": "max|x - oracle| / max|oracle|",
            }
    print(json.dumps(result), flush=True)
    return 0


def bench_decode(args, w, sla, si, torch, np) -> int:
    """--workload decode_*: a step is one recurrent decode step (sla_decode_step) over the batch; the state
    stays resident and is updated in place, as in serving."""
    to_device = si.to_device

    d = si.generate(w)
    s0 = si.initial_state(w.B, w.H, w.dk, w.dv, seed=w.seed)
    g, tdt = to_device(d, w.dtype, w.variant)
    dev = torch.device("cuda:0")
    sq = lambda t: None if t is None else (t if t.dim() == 1 else t[:, 0].contiguous())
    q, k, v, ql, kl, beta = (sq(g[n]) for n in ("q", "k", "v", "q_logits", "k_logits", "beta"))
    ld = sq(g["log_decay"])
    state = torch.from_numpy(s0).to(dev)
    out = torch.empty((w.B, w.H, w.dv), dtype=tdt, device=dev)
    params = sla.SlaParams(w.variant, 1 if w.dtype == "bf16" else 0, w.B, 1, w.H, w.dk, w.dv, 0, 0, 1)
    ptr = lambda t: None if t is None else t.data_ptr()
    raw = (ptr(q), ptr(k), ptr(v), ptr(ql), ptr(kl), ptr(ld), ptr(beta), ptr(state), ptr(out),
           torch.cuda.current_stream(dev).cuda_stream)

    def step():
        rc = sla.sla_decode_step(params, *raw)
        if rc != 0:
            raise sla.SlaError(rc, sla.sla_status_string(rc))

    chain_us, raw_f = None, None
    if args.fused_gates:
        # The logits come from q, k and seeded gate matrices: either by sla_gate_logits in front of the step (two
        # launches) or inside sla_decode_step_fused (one).  Both are timed; the fused one is the reported step.
        from oracle import sla_numpy

        wts = si.gate_weights(w.H, w.dk, seed=w.seed + 77)
        wq, wk = torch.from_numpy(wts["w_gq"]).to(dev), torch.from_numpy(wts["w_gk"]).to(dev)
        d["q_logits"] = sla_numpy.gate_logits(d["q"], wts["w_gq"])
        d["k_logits"] = sla_numpy.gate_logits(d["k"], wts["w_gk"])
        raw_f = (ptr(q), ptr(k), ptr(v), ptr(wq), ptr(wk), ptr(ld), ptr(beta), ptr(state), ptr(out), raw[-1])
        gl = (ptr(q), ptr(k), ptr(wq), ptr(wk), ptr(ql), ptr(kl), raw[-1])

        def chain():
            rc = sla.sla_gate_logits(params, *gl) or sla.sla_decode_step(params, *raw)
            if rc != 0:
                raise sla.SlaError(rc, sla.sla_status_string(rc))

        def step():  # noqa: F811
            rc = sla.sla_decode_step_fused(params, *raw_f)
            if rc != 0:
                raise sla.SlaError(rc, sla.sla_status_string(rc))

        keep = state.clone()
        for _ in range(args.settle + args.warmup):
            chain()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            chain()
        e1.record()
        torch.cuda.synchronize()
        chain_us = e0.elapsed_time(e1) * 1e3 / args.steps
        state.copy_(keep)

    result_parity = None
    if not args.no_parity or not args.no_cpu_baseline:
        import oracle

        nthreads = oracle.threads(0)
        passes, cpu_s = 0, 0.0
        while True:
            t0 = time.perf_counter()
            ro, rf = oracle.forward(w.variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"],
                                    d["beta"], s0)
            cpu_s += time.perf_counter() - t0
            passes += 1
            if args.no_cpu_baseline or cpu_s * nthreads >= 15.0 or passes >= 200:
                break
        step()  # the first step from the seeded state is the one compared
        torch.cuda.synchronize()
        result_parity = {
            "out_rel_err": rel_err(out.to(torch.float32).cpu().numpy().astype(np.float64), ro[:, 0]),
            "state_rel_err": rel_err(state.cpu().numpy().astype(np.float64), rf),
            "definition": "max|x - oracle| / max|oracle| per tensor, first step from the seeded state",
        }
    per = args.graph if args.graph > 0 else 1  # steps per timed launch
    if args.steps % per:
        print(f"bench.py: --steps must be a multiple of --graph ({per})", file=sys.stderr)
        return 2
    launch = step
    if args.graph > 0:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        raw = raw[:-1] + (side.cuda_stream,)  # the captured calls go to the capture stream
        if args.fused_gates:
            raw_f = raw_f[:-1] + (side.cuda_stream,)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(per):
                step()
        launch = graph.replay
    for _ in range((args.settle + args.warmup + per - 1) // per):
        launch()
    torch.cuda.synchronize()
    nl = args.steps // per
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(nl + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(nl):
        launch()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_launch_ms = [evs[i].elapsed_time(evs[i + 1]) / per for i in range(nl)]
    kernel_ms = float(np.mean(per_launch_ms))
    ms_per_step = wall * 1e3 / args.steps
    abytes = decode_bytes(w)
    achieved = abytes / (kernel_ms * 1e-3) / 1e9
    result = {
        "metric": "tokens/sec SLA decode step (one token per sequence)",
        "value": w.B / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_launches": args.settle,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: SLA-{si.VARIANT_NAMES[w.variant].upper()} decode step B={w.B} H={w.H} dk={w.dk} "
                        f"dv={w.dv} {w.dtype} in/out, fp32 state updated in place, dual head-softmax gates",
            "kernel": "sla_decode_kernel" + (" with the gate projection fused (sla_decode_step_fused)" if args.fused_gates else ""),
            "launch": f"HIP graph of {per} steps per replay" if args.graph > 0 else "one launch per step",
            **({"unfused_chain_us": chain_us,
                "unfused_chain": "sla_gate_logits + sla_decode_step, back to back, same inputs"} if chain_us else {}),
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            **traffic_fields(w.name),
            "kernel_us": kernel_ms * 1e3,
            "kernel_us_min": float(np.min(per_launch_ms)) * 1e3,
            "algorithmic_bytes": abytes,
        },
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = {
            "value": w.B * passes / cpu_s,
            "unit": "tokens/s",
            "cores": nthreads,
            "kind": "oracle",
            "sample": f"the full decode batch, {passes} pass(es) ({w.B} tokens x {w.H} heads each, {cpu_s:.2f} s wall)",
        }
    if result_parity is not None and not args.no_parity:
        result["parity"] = result_parity
    print(json.dumps(result), flush=True)
    return 0


def measure_config(name, sla, si, torch, np, steps, warmup, settle):
    """One of the benchmark definition's other configurations, timed like the headline (raw C-ABI call, HIP events
    on the launch stream, the library's own schedule) and checked against the oracle on the full workload."""
    import oracle

    w = si.workload(name)
    d = si.generate(w)
    g, tdt = si.to_device(d, w.dtype, w.variant)
    dev = torch.device("cuda:0")
    out = torch.empty((w.B, w.T, w.H, w.dv), dtype=tdt, device=dev)
    fin = torch.empty((w.B, w.H, w.dk, w.dv), dtype=torch.float32, device=dev)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    params = sla.SlaParams(w.variant, 1 if w.dtype == "bf16" else 0, w.B, w.T, w.H, w.dk, w.dv, 0, 0, 0)
    nseg = sla.sla_segments(params, cus)
    ws_bytes = sla.sla_workspace_bytes(params, cus)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
    params.segments = nseg
    ptr = lambda t: None if t is None else t.data_ptr()
    raw = (ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(g["q_logits"]), ptr(g["k_logits"]), ptr(g["log_decay"]),
           ptr(g["beta"]), None, ptr(out), ptr(fin), ptr(ws), ws_bytes, torch.cuda.current_stream(dev).cuda_stream)

    def step():
        rc = sla.sla_forward_ws(params, *raw)
        if rc != 0:
            raise sla.SlaError(rc, sla.sla_status_string(rc))

    for _ in range(settle + warmup):
        step()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]
    call_ms = float(np.mean(per_ms))
    abytes = algorithmic_bytes(w)
    ro, rf = oracle.forward(w.variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"], d["beta"], None)
    return {
        "workload": f"{w.name}: SLA-{si.VARIANT_NAMES[w.variant].upper()} B={w.B} T={w.T} H={w.H} dk={w.dk} dv={w.dv} {w.dtype}",
        "segments": nseg,
        "launches_per_call": 1 if nseg == 1 else 3,
        "steps": steps,
        "ms_per_step": wall * 1e3 / steps,
        "call_us": call_ms * 1e3,
        "tokens_per_s": w.tokens() / (wall / steps),
        "algorithmic_bytes": abytes,
        "frac": abytes / (call_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        **traffic_fields(w.name),
        "out_rel_err": rel_err(out.to(torch.float32).cpu().numpy().astype(np.float64), ro),
        "state_rel_err": rel_err(fin.cpu().numpy().astype(np.float64), rf),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--settle", type=int, default=300,
                    help="untimed launches before the warm-up steps: the device's clocks dip for the first ~100 "
                         "launches of a burst and then recover; timing starts from the settled state")
    ap.add_argument("--workload", default="gla_train")
    ap.add_argument("--dv-split", type=int, default=0)
    ap.add_argument("--segments", type=int, default=0,
                    help="segment-parallel schedule: 0 = the library chooses (one pass when the batch fills the "
                         "device, as for the headline workload), 1 = one fused pass, n = n segments")
    ap.add_argument("--copy-bytes", type=int, default=0,
                    help="also run one plain device-to-device copy of this many bytes before the timed region "
                         "(a known-size kernel to calibrate the profiler's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--graph", type=int, default=50,
                    help="decode workloads only: steps per captured HIP graph (0 = plain launches).  A decode step "
                         "is shorter than the gap between two launches from Python; a serving loop replays a graph")
    ap.add_argument("--train-step", action="store_true",
                    help="time gate logits + forward + backward of the workload, back to back")
    ap.add_argument("--fused-gates", action="store_true",
                    help="decode workloads only: time sla_decode_step_fused (gate logits formed in the kernel) and, "
                         "beside it, the two-launch chain sla_gate_logits + sla_decode_step")
    ap.add_argument("--backward", action="store_true",
                    help="time sla_backward (RetNet / GLA) or sla_backward_gdn (--workload gdn) instead of the forward")
    ap.add_argument("--flush-mb", type=int, default=0,
                    help="forward only: overwrite a scratch buffer of this many MB between the timed launches, so that "
                         "no input is left in the 256 MB memory-side cache from the previous launch; each launch is "
                         "then timed by its own pair of events and `value` is computed from that time")
    ap.add_argument("--flush-kind", choices=("read", "write"), default="read",
                    help="how --flush-mb displaces the cache: by reading the scratch buffer (lines left clean) or by "
                         "rewriting it (lines left dirty: their write-back then overlaps the timed launch)")
    ap.add_argument("--head-major", action="store_true",
                    help="forward only: q, k, v, out (and the GLA decay) in the [B,H,T,d] layout (SLA_FLAG_HEAD_MAJOR) "
                         "instead of the benchmark definition's [B,T,H,d]; a secondary figure, not the headline")
    ap.add_argument("--varlen", action="store_true",
                    help="forward only: the workload's B*T tokens as one packed batch of mixed-length sequences "
                         "(sla_forward_varlen; lengths from sla_inputs.packed_lengths)")
    ap.add_argument("--short-conv", action="store_true",
                    help="time sla_short_conv_silu (the delta-rule blocks' feature map) on a [B,T,H*dk] tensor")
    ap.add_argument("--prologue", action="store_true",
                    help="time sla_gate_logits (the projections in front of the head softmax) on the workload's q, k")
    ap.add_argument("--no-configs", action="store_true",
                    help="headline run only: do not also time the benchmark definition's other four configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no collectives or sharding are built)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2602_01744_amd as sla
    import sla_inputs as si

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    sla.load_library()  # fails loudly if the HIP library is not built
    w = si.workload(args.workload)
    if w.name in si.DECODE_WORKLOAD_NAMES:
        return bench_decode(args, w, sla, si, torch, np)
    if args.backward:
        return bench_backward(args, w, sla, si, torch, np)
    if args.train_step:
        return bench_train_step(args, w, sla, si, torch, np)
    if args.prologue:
        return bench_prologue(args, w, sla, si, torch, np)
    if args.short_conv:
        return bench_short_conv(args, w, sla, si, torch, np)
    d = si.generate(w)

    to_device = si.to_device

    g, tdt = to_device(d, w.dtype, w.variant)
    dev = torch.device("cuda:0")
    out = torch.empty((w.B, w.T, w.H, w.dv), dtype=tdt, device=dev)
    if args.head_major:
        if args.varlen:
            print("bench.py: --head-major and --varlen do not combine", file=sys.stderr)
            return 2
        for n in ("q", "k", "v") + (("log_decay",) if w.variant == 1 else ()):
            g[n] = g[n].permute(0, 2, 1, 3).contiguous()
        out = torch.empty((w.B, w.H, w.T, w.dv), dtype=tdt, device=dev)
    lengths = si.packed_lengths(w.B * w.T, seed=w.seed + 70) if args.varlen else None
    nstates = len(lengths) if args.varlen else w.B
    fin = torch.empty((nstates, w.H, w.dk, w.dv), dtype=torch.float32, device=dev)

    cus = torch.cuda.get_device_properties(0).multi_processor_count
    params = sla.SlaParams(w.variant, 1 if w.dtype == "bf16" else 0, w.B, w.T, w.H, w.dk, w.dv, args.dv_split,
                           sla.FLAG_HEAD_MAJOR if args.head_major else 0, args.segments)
    nseg = sla.sla_segments(params, cus)
    if nseg < 1:
        print(f"bench.py: {sla.sla_status_string(nseg)}", file=sys.stderr)
        return 2
    ws_bytes = sla.sla_workspace_bytes(params, cus)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None

    # The timed call is the raw C-ABI entry point with addresses taken once: the Python wrapper's argument
    # checks would otherwise take about as long as the kernel and leave the GPU waiting for the host.
    params.segments = nseg
    stream = torch.cuda.current_stream(dev).cuda_stream
    ptr = lambda t: None if t is None else t.data_ptr()
    raw = (ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(g["q_logits"]), ptr(g["k_logits"]), ptr(g["log_decay"]),
           ptr(g["beta"]), None, ptr(out), ptr(fin), ptr(ws), ws_bytes, stream)

    def step():
        rc = sla.sla_forward_ws(params, *raw)
        if rc != 0:
            raise sla.SlaError(rc, sla.sla_status_string(rc))

    if args.varlen:
        # the same tensors read as one row of B*T tokens (the generator's batch rows laid end to end)
        cu_host = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
        cu = torch.from_numpy(cu_host).to(dev)
        vparams = sla.SlaParams(w.variant, 1 if w.dtype == "bf16" else 0, len(lengths), w.B * w.T, w.H, w.dk, w.dv, 0, 0, 1)
        vraw = raw[:7] + (cu.data_ptr(), None, ptr(out), ptr(fin), stream)

        def step():  # noqa: F811
            rc = sla.sla_forward_varlen(vparams, *vraw)
            if rc != 0:
                raise sla.SlaError(rc, sla.sla_status_string(rc))

    if args.copy_bytes > 0:
        src = torch.empty(args.copy_bytes, dtype=torch.uint8, device=dev).fill_(3)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # The settle phase is timed too, so that what it hides is on record: the mean of the burst's first launches
    # (after one untimed call, which loads the kernel's code object).
    step()
    torch.cuda.synchronize()
    nfirst = min(100, args.settle + args.warmup)
    f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    f0.record()
    for i in range(args.settle + args.warmup):
        step()
        if i + 1 == nfirst:
            f1.record()
    torch.cuda.synchronize()
    first_burst_us = f0.elapsed_time(f1) * 1e3 / nfirst if nfirst > 0 else None
    # per-launch kernel time: HIP events on the stream the kernel is enqueued on (torch's current stream)
    if args.flush_mb > 0:
        scratch = torch.zeros(args.flush_mb * (1 << 20) // 4, dtype=torch.float32, device=dev)
        flush_sink = torch.zeros((), dtype=torch.float32, device=dev)
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for e0, e1 in pairs:
            if args.flush_kind == "write":
                scratch.add_(1.0)  # reads and rewrites the buffer: the cache holds (dirty) scratch, not inputs
            else:
                flush_sink.copy_(scratch.max())  # reads the buffer: the cache holds clean scratch lines
            e0.record()
            step()
            e1.record()
        torch.cuda.synchronize()
        per_launch_ms = [e0.elapsed_time(e1) for e0, e1 in pairs]
        kernel_ms = float(np.mean(per_launch_ms))
        ms_per_step = kernel_ms
    else:
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        t0 = time.perf_counter()
        evs[0].record()
        for i in range(args.steps):
            step()
            evs[i + 1].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        per_launch_ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps)]
        kernel_ms = float(np.mean(per_launch_ms))
        ms_per_step = wall * 1e3 / args.steps
    tokens = w.tokens()
    value = tokens / (ms_per_step * 1e-3)

    abytes = algorithmic_bytes(w)
    aflops = algorithmic_flops(w)
    achieved_gbs = abytes / (kernel_ms * 1e-3) / 1e9
    dvw = args.dv_split or sla.sla_default_dv_split(params, cus)

    result = {
        "metric": METRIC,
        "value": value,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_launches": args.settle,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: SLA-{si.VARIANT_NAMES[w.variant].upper()} B={w.B} T={w.T} H={w.H} dk={w.dk} dv={w.dv} "
                        f"{w.dtype} in/out, fp32 state, dual head-softmax gates"
                        + (", q/k/v/out/decay laid out [B,H,T,d]" if args.head_major else ""),
            "kernel": sla.sla_kernel_name(params),
            "dv_split": dvw,
            "segments": nseg,
            "compute_units": cus,
            **({"cache_flush_mb_between_launches": args.flush_mb, "cache_flush_kind": args.flush_kind}
               if args.flush_mb > 0 else {}),
            **({"packed_lengths": [int(x) for x in lengths], "entry_point": "sla_forward_varlen"} if args.varlen else {}),
        },
        "roofline": {
            "bound": "hbm",
            "achieved": achieved_gbs,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved_gbs / HBM_PEAK_GBS,
            **({"traffic": None} if (args.varlen or args.head_major) else traffic_fields(w.name)),
            "kernel_us": kernel_ms * 1e3,
            "kernel_us_min": float(np.min(per_launch_ms)) * 1e3,
            "unsettled_first_launches_us": first_burst_us,
            "unsettled_first_launches": nfirst,
            "algorithmic_bytes": abytes,
            "mfma_tflops_causal": aflops / (kernel_ms * 1e-3) / 1e12,
            "mfma_frac_of_bf16_peak": aflops / (kernel_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        },
    }

    ro = None
    if not args.no_cpu_baseline or not args.no_parity:
        import oracle

        nthreads = oracle.threads(0)
        passes, cpu_s = 0, 0.0
        while True:  # whole passes over the workload until about 15 core-seconds have been spent (at most 8 passes)
            t0 = time.perf_counter()
            ro, rf = oracle.forward(w.variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"],
                                    d["beta"], None)
            cpu_s += time.perf_counter() - t0
            passes += 1
            if args.no_cpu_baseline or cpu_s * nthreads >= 15.0 or passes >= 8:
                break
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = {
                "value": tokens * passes / cpu_s,
                "unit": "tokens/s",
                "cores": nthreads,
                "kind": "oracle",
                "sample": f"the full workload, {passes} pass(es) ({tokens} tokens x {w.H} heads each, {cpu_s:.2f} s wall)",
            }
        if not args.no_parity and not args.varlen:
            step()
            torch.cuda.synchronize()
            og = out.permute(0, 2, 1, 3) if args.head_major else out
            result["parity"] = {
                "out_rel_err": rel_err(og.to(torch.float32).cpu().numpy().astype(np.float64), ro),
                "state_rel_err": rel_err(fin.cpu().numpy().astype(np.float64), rf),
                "definition": "max|x - oracle| / max|oracle| per tensor",
            }
        if not args.no_parity and args.varlen:
            step()
            torch.cuda.synchronize()
            flat = lambda a: None if a is None else (a if a.ndim == 1 else a.reshape((1, w.B * w.T) + a.shape[2:]))
            og = out.to(torch.float32).cpu().numpy().astype(np.float64).reshape((w.B * w.T, w.H, w.dv))
            fg = fin.cpu().numpy().astype(np.float64)
            eo = ef = 0.0
            for i in (0, len(lengths) // 2, len(lengths) - 1):  # the longest, a middle and the shortest sequence
                a0, a1 = int(cu_host[i]), int(cu_host[i + 1])
                cut = lambda x: None if x is None else (x if x.ndim == 1 else flat(x)[:, a0:a1])
                so, sf = oracle.forward(w.variant, cut(d["q"]), cut(d["k"]), cut(d["v"]), cut(d["q_logits"]),
                                        cut(d["k_logits"]), cut(d["log_decay"]), cut(d["beta"]), None)
                eo, ef = max(eo, rel_err(og[a0:a1], so[0])), max(ef, rel_err(fg[i], sf[0]))
            result["parity"] = {"out_rel_err": eo, "state_rel_err": ef,
                                "definition": "max|x - oracle| / max|oracle| over three sequences of the pack, each "
                                              "against the oracle run on that sequence alone"}
    plain = not (args.varlen or args.head_major or args.flush_mb or args.dv_split or args.segments)
    if w.name == "gla_train" and plain and not args.no_configs:
        # The other configurations of the benchmark definition (the headline is the third), each a few hundred
        # launches: the tiny fp32 correctness shape, the two few-sequence shapes (segment schedule), the delta rule.
        result["configs"] = {
            n: measure_config(n, sla, si, torch, np, steps=(50 if n == "gla_long" else 200), warmup=args.warmup,
                              settle=(50 if n == "gla_long" else 200))
            for n in ("gla_tiny", "retnet", "gdn", "gla_long")
        }
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
