#!/usr/bin/env python3
"""Benchmark of the Ouroboros verification step on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input:
ouro_verify_attn -> ouro_lmhead_argmax -> ouro_accept, enqueued back to back on one
stream with inputs resident in HBM.  The default workload is the Llama-2-7B-shaped
config (batch 1, 32 heads x 128, KV length 2048, draft block 64, vocabulary 32000).

Prints ONE JSON line: whole-job throughput in draft tokens verified per second, the
roofline of the dominant kernel (measured with HIP events on the launch stream inside
the timed region), and the CPU oracle timed on the host as a reported baseline.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="workload id 1..5 (default 2: Llama-2-7B-shaped layer)")
    ap.add_argument("--rotate", type=int, default=0, help="copies of KV cache and LM-head weight cycled through "
                    "(0: enough copies to exceed 1 GB, so that the 256 MB last-level cache cannot hold them)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="budget of the CPU-oracle baseline leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--branch", default="uniform", choices=["uniform", "last"])
    ap.add_argument("--event-every", type=int, default=8,
                    help="record the per-call and per-kernel HIP events on every Nth timed step (each record is a "
                         "packet on the stream and costs launch time; 1: every step)")
    ap.add_argument("--with-layer", action="store_true",
                    help="also time the rest of one verifying layer around the attention (RMSNorm, fused QKV projection, "
                         "rotary embedding at the draft positions, attention, output projection, RMSNorm, SwiGLU MLP) and "
                         "report it as an extra 'layer' object; the headline value is unchanged")
    ap.add_argument("--lm-rows", default="", help="comma-separated row counts (e.g. 1024,2048,4096): also time the LM "
                    "head alone at these R on the workload's vocabulary x hidden (MFMA-bound regime); adds lmhead_large_R")
    ap.add_argument("--kv-layout", default="head", choices=["head", "row"],
                    help="KV-cache layout: [Hkv, rows, D] (every (sequence, KV head) stream contiguous; default) or "
                         "[rows, Hkv, D]")
    ap.add_argument("--w-layout", default="tiled", choices=["tiled", "row"],
                    help="LM-head weight layout: re-blocked once at set-up into contiguous 128x64 tiles "
                         "(ouro_lmhead_pack_w; default) or the row-major [V, hidden] matrix as is")
    return ap.parse_args()


def attn_algorithmic_bytes(cfg, total_cache_rows):
    e = 2 if cfg.dtype == "bf16" else 4
    kv = 2 * (total_cache_rows + cfg.B * cfg.T) * cfg.Hkv * cfg.D * e
    qo = 2 * cfg.B * cfg.T * cfg.Hq * cfg.D * e
    return kv + qo + 4 * cfg.B * cfg.T


def attn_flops(cfg, seqlens):
    return sum(4 * cfg.T * cfg.Hq * (int(L) + cfg.T) * cfg.D for L in seqlens)


def lmhead_algorithmic_bytes(cfg):
    e = 2 if cfg.dtype == "bf16" else 4
    return cfg.V * cfg.hidden * e + cfg.R * cfg.hidden * e + 4 * cfg.R


def lmhead_flops(cfg):
    return 2 * cfg.R * cfg.hidden * cfg.V


def cpu_baseline(cfg, inp, w, draws, budget_s):
    """Time the oracle (as it stands) on the host on a bounded sample and scale to one full step."""
    import numpy as np
    from oracle import verify_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    # attention: sample (sequence, head) pairs until a third of the budget is spent
    pairs = [(b, h) for b in range(cfg.B) for h in range(cfg.Hq)]
    rng = np.random.default_rng(0)
    rng.shuffle(pairs)
    seqlens = np.diff(inp["cu_seqlens"])
    t0 = time.perf_counter()
    done, work_done = 0, 0.0
    for (b, h) in pairs:
        O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"], inp["k_blk"], inp["v_blk"],
                           inp["pid"], inp["boff"], heads=[(b, h)])
        done += 1
        work_done += float(seqlens[b] + cfg.T)
        if time.perf_counter() - t0 > budget_s / 3:
            break
    t_att_sample = time.perf_counter() - t0
    work_all = float(sum((seqlens[b] + cfg.T) for b in range(cfg.B)) * cfg.Hq)
    t_att = t_att_sample * work_all / work_done
    # LM head: sample rows (cost is linear in rows)
    rows = min(cfg.R, 64)
    hid = inp["q"].reshape(cfg.R, cfg.hidden)[:rows]          # any [rows, hidden] values: timing only
    t0 = time.perf_counter()
    lm = O.lmhead_argmax(hid, w)
    t_lm_sample = time.perf_counter() - t0
    t_lm = t_lm_sample * cfg.R / rows
    # acceptance: full
    amax = np.resize(lm["argmax"], (cfg.B, cfg.T))
    t0 = time.perf_counter()
    O.accept(draws["tok"], amax, inp["pid"], inp["boff"], draws["root_pred"], cfg.gamma, cfg.K, cfg.beta_p)
    t_acc = time.perf_counter() - t0
    t_step = t_att + t_lm + t_acc
    return {
        "value": cfg.R / t_step, "unit": "draft tokens verified/s", "cores": int(cores), "kind": "oracle",
        "sample": "attention on %d of %d (sequence, head) pairs, LM head on %d of %d rows, acceptance in full; "
                  "scaled linearly to one step" % (done, len(pairs), rows, cfg.R),
        "step_seconds_scaled": t_step,
        "stage_seconds_scaled": {"attention": t_att, "lmhead_argmax": t_lm, "accept": t_acc},
    }


def time_lmhead_rows(cfg, ob, torch, ws, rows_list, iters=60, warm=60):
    """ouro_lmhead_argmax alone at large row counts R (hidden ~ N(0,1)), the weight copies cycled through as in the
    step.  Returns one record per R: microseconds per call (whole call, both kernels) and the bf16 MFMA fraction."""
    import ctypes as C
    dev = torch.device("cuda:0")
    out = []
    stream = torch.cuda.current_stream()
    hs = stream.cuda_stream or None
    gen = torch.Generator().manual_seed(20240213)
    for R in rows_list:
        h = torch.randn(R, cfg.hidden, generator=gen).to(torch.bfloat16).to(dev)
        arg = torch.empty(R, dtype=torch.int32, device=dev)
        wsp = ob.alloc_workspace(ob.ouro_lmhead_argmax_workspace(h, ws[0]), dev)
        descs = [ob.make_lmhead_desc(h, w, arg, None, wsp) for w in ws]
        for i in range(warm):
            ob.lib.ouro_lmhead_argmax(C.byref(descs[i % len(descs)]), hs)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(iters):
            if ob.lib.ouro_lmhead_argmax(C.byref(descs[i % len(descs)]), hs) != 0:
                raise RuntimeError("ouro_lmhead_argmax failed")
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / iters
        tflops = 2.0 * R * cfg.hidden * cfg.V / us / 1e6
        out.append({"R": R, "us_per_call": us, "TFLOP/s": tflops, "frac_of_mfma_peak": tflops / MFMA_BF16_PEAK_TFLOPS})
    return out


def time_layer(cfg, ob, torch, q, k_blk, v_blk, kcs, vcs, cu, meta, max_seqlen, head_major, steps):
    """One Llama-shaped verifying layer (synthetic weights ~ N(0, 1/fan_in)) replayed from a HIP graph; the weights are
    cycled through copies like W.  Returns microseconds per layer and the bytes of weights + KV it must stream."""
    dev, dt = q.device, q.dtype
    Hd, D = cfg.hidden, cfg.D
    F = {4096: 11008, 5120: 13824, 8192: 28672}.get(Hd, (8 * Hd // 3 + 255) // 256 * 256)
    R = cfg.R
    nqkv = (cfg.Hq + 2 * cfg.Hkv) * D
    shapes = {"qkv": (nqkv, Hd), "o": (Hd, Hd), "gu": (2 * F, Hd), "down": (Hd, F)}
    wbytes = sum(n * k * 2 for n, k in shapes.values())
    ncopy = max(1, min(4, int(1.0e9 // wbytes) + 1))
    gen = torch.Generator(device=dev).manual_seed(1234)
    ws = [{name: ob.ouro_lmhead_pack_w((torch.randn(n, k, generator=gen, device=dev) * k ** -0.5).to(dt))
           for name, (n, k) in shapes.items()} for _ in range(ncopy)]
    x = torch.randn(R, Hd, generator=gen, device=dev).to(dt)
    qkv = torch.empty(R, nqkv, device=dev, dtype=dt)
    qb, kb, vb = torch.empty_like(q), torch.empty_like(k_blk), torch.empty_like(v_blk)
    att = torch.empty_like(q)
    x1, out = torch.empty_like(x), torch.empty_like(x)
    act = torch.empty(R, F, device=dev, dtype=dt)
    lin_ws = ob.alloc_workspace(64 << 20, dev)
    att_ws = ob.alloc_workspace(ob.ouro_verify_attn_workspace(q, k_blk, max_seqlen), dev)

    def layer(r, stream):
        w = ws[r % ncopy]
        ob.ouro_linear(x, w["qkv"], out=qkv, workspace=lin_ws, stream=stream, rms_eps=1e-5)      # RMSNorm folded in
        ob.ouro_rope_block(qb, kb, meta, cu, stream=stream, qkv=qkv, v_blk=vb)    # rotary + split of the fused output
        ob.ouro_verify_attn(qb, kcs[r % len(kcs)], vcs[r % len(vcs)], cu, kb, vb, meta, max_seqlen, out=att,
                            workspace=att_ws, stream=stream, head_major=head_major)
        ob.ouro_linear(att.view(R, Hd), w["o"], residual=x, out=x1, workspace=lin_ws, stream=stream)
        ob.ouro_linear(x1, w["gu"], out=act, workspace=lin_ws, stream=stream, swiglu=True, rms_eps=1e-5)   # norm + gate
        ob.ouro_linear(act, w["down"], residual=x1, out=out, workspace=lin_ws, stream=stream)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for r in range(2):
            layer(r, side)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for r in range(ncopy):
                layer(r, side)
        graph.replay()
        torch.cuda.synchronize()
        reps = max(1, steps // ncopy)
        g0, g1e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record(side)
        for _ in range(reps):
            graph.replay()
        g1e.record(side)
        torch.cuda.synchronize()
    us = g0.elapsed_time(g1e) * 1e3 / (reps * ncopy)
    return us, wbytes, F


def load_traffic(workload_key):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, each scaled by the plain-copy calibration) of the
    main kernels, from the committed rocprofv3 --pmc summary for this workload, if present."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        with open(path) as f:
            return json.load(f).get(workload_key)
    except Exception:
        return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (use --gpus 1)." % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2402_13720_amd import binding as ob, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    cfg = W.CONFIGS[args.config]
    seed = W.seed_for(args.config)
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32

    inp = W.make_attention_inputs(cfg, seed, branch=args.branch)
    w = W.make_lmhead_weight(cfg, seed)
    draws = W.make_token_draws(cfg, seed)
    seqlens = np.diff(inp["cu_seqlens"])
    total_rows = int(inp["cu_seqlens"][-1])
    max_seqlen = int(seqlens.max())

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, inp, w, draws, args.cpu_seconds)

    # ---- device-resident inputs; KV cache and W in several copies that the steps cycle through ----
    e = 2 if cfg.dtype == "bf16" else 4
    rot_bytes = 2 * total_rows * cfg.Hkv * cfg.D * e + cfg.V * cfg.hidden * e
    nrot = args.rotate if args.rotate > 0 else max(1, min(8, int(np.ceil(1.0e9 / rot_bytes))))
    up = lambda x: torch.from_numpy(x).to(dev).to(dt).contiguous()
    q, k_blk, v_blk = up(inp["q"]), up(inp["k_blk"]), up(inp["v_blk"])
    kc0, vc0, w0 = up(inp["k_cache"]), up(inp["v_cache"]), up(w)
    head_major = args.kv_layout == "head"
    if head_major:                                        # a re-layout of the same values, done once at set-up
        kc0, vc0 = kc0.permute(1, 0, 2).contiguous(), vc0.permute(1, 0, 2).contiguous()
    kcs = [kc0] + [kc0.clone() for _ in range(nrot - 1)]
    vcs = [vc0] + [vc0.clone() for _ in range(nrot - 1)]
    ws = [w0] + [w0.clone() for _ in range(nrot - 1)]
    if args.w_layout == "tiled" and cfg.dtype == "bf16":
        ws = [ob.ouro_lmhead_pack_w(x) for x in ws]       # load-time step, outside the timed region
        torch.cuda.synchronize()
        del w0
    cu = torch.from_numpy(inp["cu_seqlens"]).to(dev)
    meta = ob.pack_meta(inp["pid"], inp["boff"]).to(dev)
    root = torch.from_numpy(draws["root_pred"]).to(dev)

    out = torch.empty_like(q)
    hidden = out.view(cfg.R, cfg.hidden)
    arg = torch.empty(cfg.R, dtype=torch.int32, device=dev)
    ws_attn = ob.alloc_workspace(ob.ouro_verify_attn_workspace(q, k_blk, max_seqlen), dev)
    ws_lm = ob.alloc_workspace(ob.ouro_lmhead_argmax_workspace(hidden, ws[0]), dev)
    acc_out = ob.alloc_accept_outputs(cfg.B, cfg.gamma, cfg.K, cfg.beta_p, dev)

    # draft ids: half of the block positions carry the token they will be compared with (the greedy
    # token of their parent row); the other half are uniform.  Values do not affect timing.
    ob.ouro_verify_attn(q, kcs[0], vcs[0], cu, k_blk, v_blk, meta, max_seqlen, out=out, workspace=ws_attn,
                        head_major=head_major)
    ob.ouro_lmhead_argmax(hidden, ws[0], argmax_out=arg, workspace=ws_lm)
    torch.cuda.synchronize()
    amax = arg.cpu().numpy().reshape(cfg.B, cfg.T)
    exp = np.empty_like(amax)
    for b in range(cfg.B):
        for t in range(cfg.T):
            if inp["pid"][b, t] == 0:
                p = t - 1
            elif t > 0 and inp["pid"][b, t - 1] == inp["pid"][b, t]:
                p = t - 1
            else:
                p = int(inp["boff"][b, t])
            exp[b, t] = draws["root_pred"][b] if p < 0 else amax[b, p]
    tok = torch.from_numpy(W.plant_tokens(draws["tok"], draws["chosen"], exp)).to(dev)

    stream = torch.cuda.current_stream()
    hs = stream.cuda_stream or None
    import ctypes as C
    # descriptors are built once per rotated copy; a step is then three C-ABI calls
    d_attn = [ob.make_attn_desc(q, kcs[r], vcs[r], cu, k_blk, v_blk, meta, out, max_seqlen, None, ws_attn,
                                head_major=head_major)
              for r in range(nrot)]
    d_lm = [ob.make_lmhead_desc(hidden, ws[r], arg, None, ws_lm) for r in range(nrot)]
    d_acc = ob.make_accept_desc(tok, arg.view(cfg.B, cfg.T), meta, root, cfg.gamma, cfg.K, cfg.beta_p, acc_out)
    f_attn, f_lm, f_acc = ob.lib.ouro_verify_attn, ob.lib.ouro_lmhead_argmax, ob.lib.ouro_accept

    # raw HIP events handed to the library: it records them right around the main kernel of a call,
    # on the launch stream, so that kernel's duration is measured inside the timed region
    hip = C.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]

    def new_event():
        e = C.c_void_p()
        if hip.hipEventCreate(C.byref(e)) != 0:
            raise RuntimeError("hipEventCreate failed")
        return e

    def elapsed_us(e0, e1):
        ms = C.c_float()
        if hip.hipEventElapsedTime(C.byref(ms), e0, e1) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return ms.value * 1e3

    every = max(1, args.event_every)
    sampled = [i for i in range(args.steps) if i % every == 0]
    kev = {i: [new_event() for _ in range(4)] for i in sampled}

    def step(i, ev=None, kv=None):
        r = i % nrot
        d_attn[r].ev_start, d_attn[r].ev_stop = (kv[0], kv[1]) if kv else (None, None)
        d_lm[r].ev_start, d_lm[r].ev_stop = (kv[2], kv[3]) if kv else (None, None)
        if ev is not None:
            ev[0].record(stream)
        st = f_attn(C.byref(d_attn[r]), hs)
        if ev is not None:
            ev[1].record(stream)
        st |= f_lm(C.byref(d_lm[r]), hs)
        if ev is not None:
            ev[2].record(stream)
        st |= f_acc(C.byref(d_acc), hs)
        if ev is not None:
            ev[3].record(stream)
        if st != 0:
            raise RuntimeError("a verification-step call failed (status bits %d)" % st)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    events = {i: [torch.cuda.Event(enable_timing=True) for _ in range(4)] for i in sampled}
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, events.get(i), kev.get(i))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # ---- extra: the same steps replayed from a HIP graph (launch gaps removed); not the headline value ----
    graph_us = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            hs_side = side.cuda_stream

            def gstep(r):
                d_attn[r].ev_start = d_attn[r].ev_stop = d_lm[r].ev_start = d_lm[r].ev_stop = None
                return (f_attn(C.byref(d_attn[r]), hs_side) | f_lm(C.byref(d_lm[r]), hs_side)
                        | f_acc(C.byref(d_acc), hs_side))

            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                st = 0
                for r in range(nrot):
                    st |= gstep(r)
            if st == 0:
                reps = max(1, args.steps // nrot)
                graph.replay()
                torch.cuda.synchronize()
                g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                g0.record(side)
                for _ in range(reps):
                    graph.replay()
                g1.record(side)
                torch.cuda.synchronize()
                graph_us = g0.elapsed_time(g1) * 1e3 / (reps * nrot)
    except Exception as exc:      # graph capture is optional; report why it was skipped
        graph_us = "unavailable: %s" % type(exc).__name__

    layer = None
    if args.with_layer and cfg.dtype == "bf16":
        us, wbytes, F = time_layer(cfg, ob, torch, q, k_blk, v_blk, kcs, vcs, cu, meta, max_seqlen, head_major,
                                   args.steps)
        lbytes = wbytes + attn_algorithmic_bytes(cfg, total_rows)
        layer = {"us_per_layer": us, "mlp_width": F, "weight_bytes": wbytes, "algorithmic_bytes": lbytes,
                 "achieved_GBs": lbytes / us / 1e3, "frac_of_hbm_peak": lbytes / us / 1e3 / HBM_PEAK_GBS,
                 "how": "7 library calls (QKV with RMSNorm folded in, rotary + split, attention, o + residual, gate/up with RMSNorm folded in and the SwiGLU gate in its epilogue, down + residual), replayed from a HIP graph"}

    large_r = None
    if args.lm_rows and cfg.dtype == "bf16":
        large_r = time_lmhead_rows(cfg, ob, torch, ws, [int(x) for x in args.lm_rows.split(",") if x])

    ms_step = elapsed * 1e3 / args.steps
    seg = np.array([[ev[j].elapsed_time(ev[j + 1]) for j in range(3)] for ev in events.values()])   # ms
    t_attn, t_lm, t_acc = (float(x) for x in seg.mean(axis=0))
    tokens = cfg.R
    # main-kernel durations (ms): attention split-KV kernel, LM-head weight-streaming kernel
    k_attn = float(np.mean([elapsed_us(k[0], k[1]) for k in kev.values()])) * 1e-3
    k_lm = float(np.mean([elapsed_us(k[2], k[3]) for k in kev.values()])) * 1e-3

    lm_bytes = lmhead_algorithmic_bytes(cfg)
    at_bytes = attn_algorithmic_bytes(cfg, total_rows)
    lm_gbs = lm_bytes / (k_lm * 1e-3) / 1e9
    at_gbs = at_bytes / (k_attn * 1e-3) / 1e9
    lm_tflops = lmhead_flops(cfg) / (k_lm * 1e-3) / 1e12
    at_tflops = attn_flops(cfg, seqlens) / (k_attn * 1e-3) / 1e12
    workload = "cfg%d:%s" % (cfg.cfg_id, cfg.name)
    lm_mfma_bound = cfg.R >= 312          # arithmetic intensity ~R flop/B against a machine balance of ~312
    traffic = load_traffic(workload) or {}
    if lm_mfma_bound:
        roofline = {"kernel": "lmhead_bf16_tile_kernel (main kernel of ouro_lmhead_argmax)", "bound": "mfma",
                    "achieved": lm_tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": lm_tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic.get("lmhead_bytes"),
                    "kernel_us": k_lm * 1e3, "algorithmic_bytes": lm_bytes}
    else:
        roofline = {"kernel": "lmhead_bf16_kernel (main kernel of ouro_lmhead_argmax)", "bound": "hbm",
                    "achieved": lm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": lm_gbs / HBM_PEAK_GBS,
                    "traffic": traffic.get("lmhead_bytes"), "kernel_us": k_lm * 1e3, "algorithmic_bytes": lm_bytes}
    result = {
        "metric": "draft tokens verified per second (one verification step: attention + LM head/argmax + accept)",
        "value": tokens / (ms_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "verify_step_latency_us": ms_step * 1e3,
        "graph_replay_step_latency_us": graph_us,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": workload, "B": cfg.B, "T": cfg.T, "gamma": cfg.gamma, "K": cfg.K, "beta": cfg.beta_p,
                   "Hq": cfg.Hq, "Hkv": cfg.Hkv, "D": cfg.D, "cache_rows": total_rows, "V": cfg.V,
                   "branch": args.branch, "rotated_copies": nrot, "events_on_every_nth_step": every,
                   "w_layout": args.w_layout if cfg.dtype == "bf16" else "row", "kv_layout": args.kv_layout},
        "call_us": {"ouro_verify_attn": t_attn * 1e3, "ouro_lmhead_argmax": t_lm * 1e3, "ouro_accept": t_acc * 1e3},
        "roofline": roofline,
        "roofline_attn": {"kernel": "%s (main kernel of ouro_verify_attn)"
                                    % ("attn_bf16_kernel" if cfg.T * (cfg.Hq // cfg.Hkv) <= 64 else "attn_bf16_rows_kernel"),
                          "bound": "hbm",
                          "achieved": at_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": at_gbs / HBM_PEAK_GBS,
                          "traffic": traffic.get("attn_bytes"), "kernel_us": k_attn * 1e3,
                          "algorithmic_bytes": at_bytes, "mfma_tflops": at_tflops},
        "lmhead_mfma_frac": lm_tflops / MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else None,
        "layer": layer,
        "lmhead_large_R": large_r,
        "cpu_baseline": cpu,
        "accepted_per_sequence": acc_out["n_accept"].cpu().tolist()[:16],
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
