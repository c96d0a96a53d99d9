#!/usr/bin/env python3
"""Benchmark of the Ouroboros verification step on one MI355X.

A step = one pass of the whole hot path over one batch of synthetic input:
ouro_verify_attn -> ouro_lmhead_argmax -> ouro_accept, enqueued back to back on one
stream with inputs resident in HBM.  The headline workload is the largest single-GPU one,
the batched Llama-2-7B-shaped verification (16 sequences with cached lengths in [512, 8192],
draft blocks of 32 tokens, vocabulary 32000: 512 rows, 1.15 GB of K/V per step).

Prints ONE JSON line: whole-job throughput in draft tokens verified per second, the
roofline of the kernel that takes the largest share of the step (measured with HIP events
on the launch stream), the other main kernel beside it, one record per workload
(``per_config``), and the CPU oracle timed on the host as a reported baseline.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
FP32_VALU_PEAK_TFLOPS = 157.3    # MI355X fp32 vector
MACHINE_BALANCE = MFMA_BF16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)   # flop per byte above which bf16 work is MFMA-bound


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=5,
                    help="headline workload id 1..5 (default 5: batched Llama-2-7B-shaped verification, the largest)")
    ap.add_argument("--rotate", type=int, default=0, help="copies of KV cache and LM-head weight cycled through "
                    "(0: enough copies to exceed 1 GB, so that the 256 MB last-level cache cannot hold them)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0, help="budget of the CPU-oracle baseline leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="skip the records of the other workloads")
    ap.add_argument("--branch", default="uniform", choices=["uniform", "last"])
    ap.add_argument("--event-every", type=int, default=8,
                    help="inside the timed region, record the per-call and per-kernel HIP events on every Nth step only "
                         "(each record is a packet on the stream and costs launch time); the kernel durations quoted "
                         "come from a separate block of instrumented steps after it")
    ap.add_argument("--settle-steps", type=int, default=64,
                    help="untimed steps of the workload run as the last part of the set-up, before the W warm-up steps: "
                         "after the host-side set-up the chip needs some tens of milliseconds of load to reach the "
                         "clocks it then sustains (measured: 20 timed steps behind 5 warm-up steps read 4-5 %% slower "
                         "than behind 60)")
    ap.add_argument("--instrumented-steps", type=int, default=64,
                    help="untimed steps after the timed region with events around every call and main kernel (>= 50)")
    ap.add_argument("--with-layer", action="store_true",
                    help="also time the rest of one verifying layer around the attention (RMSNorm, fused QKV projection, "
                         "rotary embedding at the draft positions, attention, output projection, RMSNorm, SwiGLU MLP) and "
                         "report it as an extra 'layer' object; the headline value is unchanged")
    ap.add_argument("--lm-rows", default="", help="comma-separated row counts (e.g. 1024,2048,4096): also time the LM "
                    "head alone at these R on the workload's vocabulary x hidden (MFMA-bound regime); adds lmhead_large_R")
    ap.add_argument("--attn-plan", default="", help="tuning: force the attention launch shape of the --config workload, "
                    "as ROWBLOCKS,KEYS (row blocks per workgroup 1/2/4, 132 = 4 with the four-wave kernel; keys per "
                    "workgroup, multiple of 128; 0 = the library's choice)")
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


class Hip:
    """Raw HIP events: the library records them right around the main kernel of a call, on the launch stream."""

    def __init__(self):
        self.lib = C.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.lib.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.lib.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.lib.hipEventDestroy.argtypes = [C.c_void_p]

    def event(self):
        e = C.c_void_p()
        if self.lib.hipEventCreate(C.byref(e)) != 0:
            raise RuntimeError("hipEventCreate failed")
        return e

    def record(self, e, stream):
        if self.lib.hipEventRecord(e, stream) != 0:
            raise RuntimeError("hipEventRecord failed")

    def elapsed_us(self, e0, e1):
        ms = C.c_float()
        if self.lib.hipEventElapsedTime(C.byref(ms), e0, e1) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return ms.value * 1e3

    def destroy(self, events):
        for e in events:
            self.lib.hipEventDestroy(e)


def measured_peaks(ob, torch, hip):
    """What a plain streaming read of 2 GiB and a bare bf16 matrix-core loop reach on this GPU (the library's probes)."""
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    hs = stream.cuda_stream or None
    nbytes = 2 << 30
    buf = torch.ones(nbytes // 4, dtype=torch.int32, device=dev)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    e0, e1 = hip.event(), hip.event()
    out = {}

    def timed(call, iters, warm):
        for _ in range(warm):
            call()
        hip.record(e0, hs)
        for _ in range(iters):
            if call() != 0:
                raise RuntimeError("probe failed")
        hip.record(e1, hs)
        torch.cuda.synchronize()
        return hip.elapsed_us(e0, e1) / iters

    us = timed(lambda: ob.lib.ouro_probe_stream_read(buf.data_ptr(), nbytes, sink.data_ptr(), hs), 20, 5)
    out["hbm_stream_read_GBs"] = nbytes / us / 1e3
    out["hbm_stream_read"] = "2 GiB, 16-byte non-temporal loads, 16 KB per wave in flight, 2048 workgroups; %.1f us" % us
    wgs, rounds = 1024, 2048
    us = timed(lambda: ob.lib.ouro_probe_mfma_bf16(wgs, rounds, sink.data_ptr(), hs), 10, 3)
    out["mfma_bf16_loop_TFLOPs"] = wgs * 4 * rounds * 16 * 32768.0 / us / 1e6
    out["mfma_bf16_loop"] = "%d workgroups x 4 waves x %d x 16 v_mfma_f32_32x32x16_bf16 on register operands; %.1f us" % (wgs, rounds, us)
    hip.destroy([e0, e1])
    del buf
    return out


def time_lmhead_rows(cfg, ob, torch, ws, rows_list, iters=60, warm=60):
    """ouro_lmhead_argmax alone at large row counts R (hidden ~ N(0,1)), the weight copies cycled through as in the
    step.  Returns one record per R: microseconds per call (whole call, both kernels) and the bf16 MFMA fraction."""
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


def attn_kernel_name(cfg, plan=None):
    if cfg.dtype != "bf16":
        return "attn_f32_kernel"
    if plan is not None:
        if plan["row_blocks_per_workgroup"] == 1:
            return "attn_bf16_kernel"
        return "attn_bf16_rows8_kernel" if plan["waves_per_workgroup"] == 8 else "attn_bf16_rows_kernel"
    return "attn_bf16_kernel" if cfg.T * (cfg.Hq // cfg.Hkv) <= 64 else "attn_bf16_rows8_kernel"


def lmhead_kernel_name(cfg):
    if cfg.dtype != "bf16":
        return "lmhead_f32_kernel"
    return "lmhead_bf16_kernel" if cfg.R <= 128 else "lmhead_bf16_tile_kernel"


def kernel_roofline(kind, cfg, kernel_us, call_us, bytes_, flops, traffic, peaks, extra=None):
    """Roofline object of one main kernel.  The bound is the one its arithmetic intensity puts it under: HBM below the
    machine balance (~312 flop/byte for bf16), the matrix cores above it (the fp32 workload: the vector ALU)."""
    gbs = bytes_ / kernel_us / 1e3
    tfl = flops / kernel_us / 1e6
    intensity = flops / bytes_
    if cfg.dtype == "bf16" and intensity >= MACHINE_BALANCE:
        bound, achieved, peak, unit = "mfma", tfl, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
        measured = peaks.get("mfma_bf16_loop_TFLOPs") if peaks else None
    else:
        bound, achieved, peak, unit = "hbm", gbs, HBM_PEAK_GBS, "GB/s"
        measured = peaks.get("hbm_stream_read_GBs") if peaks else None
    r = {"kernel": "%s (main kernel of %s)" % (attn_kernel_name(cfg, (extra or {}).get("launch")) if kind == "attn" else lmhead_kernel_name(cfg),
                                               "ouro_verify_attn" if kind == "attn" else "ouro_lmhead_argmax"),
         "bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
         "traffic": traffic, "kernel_us": kernel_us, "whole_call_us": call_us,
         "frac_whole_call": achieved / peak * kernel_us / call_us,
         "frac_of_measured_peak": (achieved / measured) if measured else None,
         "algorithmic_bytes": bytes_, "flops": flops, "flop_per_byte": intensity,
         "hbm_GBs": gbs, "hbm_frac": gbs / HBM_PEAK_GBS,
         "mfma_TFLOPs": tfl if cfg.dtype == "bf16" else None,
         "mfma_frac": tfl / MFMA_BF16_PEAK_TFLOPS if cfg.dtype == "bf16" else None}
    if extra:
        r.update(extra)
    return r


def run_config(cfg_id, args, ob, W, torch, hip, peaks, headline):
    """Set one workload up on the device, run W warm-up + K timed steps (value), then the instrumented block (kernel and
    call durations).  Returns the record of the workload; the headline also gets the graph replay and the options."""
    import numpy as np
    dev = torch.device("cuda:0")
    cfg = W.CONFIGS[cfg_id]
    seed = W.seed_for(cfg_id)
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    attn_plan = 0
    if headline and args.attn_plan:
        rb, keys = (int(x) for x in args.attn_plan.split(","))
        attn_plan = ob.plan_override(rb & 0x7f, keys, bool(rb & 0x80))

    inp = W.make_attention_inputs(cfg, seed, branch=args.branch)
    w = W.make_lmhead_weight(cfg, seed)
    draws = W.make_token_draws(cfg, seed)
    seqlens = np.diff(inp["cu_seqlens"])
    total_rows = int(inp["cu_seqlens"][-1])
    max_seqlen = int(seqlens.max())

    cpu = None
    if headline and not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, inp, w, draws, args.cpu_seconds)

    # ---- device-resident inputs; KV cache and W in several copies that the steps cycle through ----
    e = 2 if cfg.dtype == "bf16" else 4
    rot_bytes = 2 * total_rows * cfg.Hkv * cfg.D * e + cfg.V * cfg.hidden * e
    nrot = args.rotate if args.rotate > 0 else max(2, min(8, int(np.ceil(1.0e9 / rot_bytes))))   # never the same copy twice in a row
    up = lambda x: torch.from_numpy(x).to(dev).to(dt).contiguous()
    q, k_blk, v_blk = up(inp["q"]), up(inp["k_blk"]), up(inp["v_blk"])
    kc0, vc0, w0 = up(inp["k_cache"]), up(inp["v_cache"]), up(w)
    head_major = args.kv_layout == "head"
    if head_major:                                        # a re-layout of the same values, done once at set-up
        kc0, vc0 = kc0.permute(1, 0, 2).contiguous(), vc0.permute(1, 0, 2).contiguous()
    kcs = [kc0] + [kc0.clone() for _ in range(nrot - 1)]
    vcs = [vc0] + [vc0.clone() for _ in range(nrot - 1)]
    ws = [w0] + [w0.clone() for _ in range(nrot - 1)]
    tiled = args.w_layout == "tiled" and cfg.dtype == "bf16"
    if tiled:
        ws = [ob.ouro_lmhead_pack_w(x) for x in ws]       # load-time step, outside the timed region
        torch.cuda.synchronize()
        del w0
    cu = torch.from_numpy(inp["cu_seqlens"]).to(dev)
    meta = ob.pack_meta(inp["pid"], inp["boff"]).to(dev)
    root = torch.from_numpy(draws["root_pred"]).to(dev)

    out = torch.empty_like(q)
    hidden = out.view(cfg.R, cfg.hidden)
    arg = torch.empty(cfg.R, dtype=torch.int32, device=dev)
    ws_attn = ob.alloc_workspace(max(ob.ouro_verify_attn_workspace(q, k_blk, max_seqlen, plan=attn_plan),
                                     ob.ouro_verify_attn_workspace(q, k_blk, max_seqlen)), dev)
    ws_lm = ob.alloc_workspace(ob.ouro_lmhead_argmax_workspace(hidden, ws[0]), dev)
    acc_out = ob.alloc_accept_outputs(cfg.B, cfg.gamma, cfg.K, cfg.beta_p, dev)

    # Draft ids: half of the block positions carry the token they will be compared with, the other half are uniform
    # (values do not affect timing).  The token a position is compared with is taken from the library itself: a first
    # acceptance call on the uniform draft returns, per phrase, the target's greedy token at each of its positions
    # (the `repaired` by-product); the main draft is a plain sequence, position i follows position i-1.
    ob.ouro_verify_attn(q, kcs[0], vcs[0], cu, k_blk, v_blk, meta, max_seqlen, out=out, workspace=ws_attn,
                        head_major=head_major)
    ob.ouro_lmhead_argmax(hidden, ws[0], argmax_out=arg, workspace=ws_lm)
    tok0 = torch.from_numpy(draws["tok"]).to(dev)
    probe_out = dict(acc_out)
    probe_out.update(ob.alloc_pool_outputs(cfg.B, cfg.gamma, cfg.K, cfg.beta_p, dev))
    ob.ouro_accept(tok0, arg.view(cfg.B, cfg.T), meta, root, cfg.gamma, cfg.K, cfg.beta_p, outs=probe_out)
    torch.cuda.synchronize()
    amax = arg.view(cfg.B, cfg.T)
    expected = torch.empty_like(amax)
    expected[:, 0] = root
    expected[:, 1:cfg.gamma] = amax[:, :cfg.gamma - 1]
    if cfg.K:
        expected[:, cfg.gamma:] = probe_out["repaired"][:, :, 1:].reshape(cfg.B, cfg.K * cfg.beta_p)
    tok = torch.from_numpy(W.plant_tokens(draws["tok"], draws["chosen"], expected.cpu().numpy())).to(dev)

    stream = torch.cuda.current_stream()
    hs = stream.cuda_stream or None
    # descriptors are built once per rotated copy; a step is then three C-ABI calls
    d_attn = [ob.make_attn_desc(q, kcs[r], vcs[r], cu, k_blk, v_blk, meta, out, max_seqlen, None, ws_attn,
                                head_major=head_major, plan=attn_plan)
              for r in range(nrot)]
    d_lm = [ob.make_lmhead_desc(hidden, ws[r], arg, None, ws_lm) for r in range(nrot)]
    d_acc = ob.make_accept_desc(tok, arg.view(cfg.B, cfg.T), meta, root, cfg.gamma, cfg.K, cfg.beta_p, acc_out)
    f_attn, f_lm, f_acc = ob.lib.ouro_verify_attn, ob.lib.ouro_lmhead_argmax, ob.lib.ouro_accept

    def step(i, ev=None, kv=None):
        r = i % nrot
        d_attn[r].ev_start, d_attn[r].ev_stop = (kv[0], kv[1]) if kv else (None, None)
        d_lm[r].ev_start, d_lm[r].ev_stop = (kv[2], kv[3]) if kv else (None, None)
        if ev is not None:
            hip.record(ev[0], hs)
        st = f_attn(C.byref(d_attn[r]), hs)
        if ev is not None:
            hip.record(ev[1], hs)
        st |= f_lm(C.byref(d_lm[r]), hs)
        if ev is not None:
            hip.record(ev[2], hs)
        st |= f_acc(C.byref(d_acc), hs)
        if ev is not None:
            hip.record(ev[3], hs)
        if st != 0:
            raise RuntimeError("a verification-step call failed (status bits %d)" % st)

    steps, warmup = args.steps, args.warmup
    every = max(1, args.event_every)
    sampled = [i for i in range(steps) if i % every == 0]
    ev_timed = {i: ([hip.event() for _ in range(4)], [hip.event() for _ in range(4)]) for i in sampled}
    n_inst = max(50, args.instrumented_steps)
    ev_inst = [([hip.event() for _ in range(4)], [hip.event() for _ in range(4)]) for _ in range(n_inst)]

    # ---- end of the set-up: bring the chip to its sustained clocks; then W warm-up steps, then exactly K timed steps ----
    for i in range(max(0, args.settle_steps)):
        step(i)
    torch.cuda.synchronize()
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        pair = ev_timed.get(i)
        step(warmup + i, pair[0] if pair else None, pair[1] if pair else None)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # ---- untimed: a block of instrumented steps (events around every call and around both main kernels) ----
    for i in range(n_inst):
        step(warmup + steps + i, ev_inst[i][0], ev_inst[i][1])
    torch.cuda.synchronize()

    # ---- untimed: the same K steps on one and the same copy of the cache and the weight (what the last-level cache adds
    # when a caller's data happens to fit it; the rotated figure above is the one that is quoted) ----
    unrot_us = None
    if nrot > 1:
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(steps):
            step(0)
        torch.cuda.synchronize()
        unrot_us = (time.perf_counter() - t1) / steps * 1e6

    def durations(pairs):
        calls = np.array([[hip.elapsed_us(c[j], c[j + 1]) for j in range(3)] for c, _ in pairs])
        kern = np.array([[hip.elapsed_us(k[0], k[1]), hip.elapsed_us(k[2], k[3])] for _, k in pairs])
        return calls, kern

    calls_i, kern_i = durations(ev_inst)
    calls_t, kern_t = durations(list(ev_timed.values()))
    t_attn, t_lm, t_acc = (float(x) for x in calls_i.mean(axis=0))
    k_attn, k_lm = (float(x) for x in kern_i.mean(axis=0))
    for c, k in list(ev_timed.values()) + ev_inst:
        hip.destroy(c + k)

    # ---- extra (headline): the same steps replayed from a HIP graph (launch gaps removed); not the headline value ----
    graph_us = None
    if headline:
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
                    reps = max(1, steps // nrot)
                    for _ in range(1 + max(0, args.settle_steps) // nrot):      # warm-up replays (clocks, as above)
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
    if headline and args.with_layer and cfg.dtype == "bf16":
        us, wbytes, F = time_layer(cfg, ob, torch, q, k_blk, v_blk, kcs, vcs, cu, meta, max_seqlen, head_major, steps)
        lbytes = wbytes + attn_algorithmic_bytes(cfg, total_rows)
        layer = {"us_per_layer": us, "mlp_width": F, "weight_bytes": wbytes, "algorithmic_bytes": lbytes,
                 "achieved_GBs": lbytes / us / 1e3, "frac_of_hbm_peak": lbytes / us / 1e3 / HBM_PEAK_GBS,
                 "how": "7 library calls (QKV with RMSNorm folded in, rotary + split, attention, o + residual, gate/up with RMSNorm folded in and the SwiGLU gate in its epilogue, down + residual), replayed from a HIP graph"}
    large_r = None
    if headline and args.lm_rows and cfg.dtype == "bf16":
        large_r = time_lmhead_rows(cfg, ob, torch, ws, [int(x) for x in args.lm_rows.split(",") if x])

    ms_step = elapsed * 1e3 / steps
    workload = "cfg%d:%s" % (cfg.cfg_id, cfg.name)
    traffic = load_traffic(workload) or {}
    samples = {"kernel_us_from": "%d instrumented steps after the timed region (events around every call and main kernel)" % n_inst,
               "kernel_us_std": None, "kernel_us_in_timed_region": None}
    r_attn = kernel_roofline("attn", cfg, k_attn, t_attn, attn_algorithmic_bytes(cfg, total_rows), attn_flops(cfg, seqlens),
                             traffic.get("attn_bytes"), peaks,
                             {**samples, "kernel_us_std": float(kern_i[:, 0].std()),
                              "kernel_us_in_timed_region": {"mean": float(kern_t[:, 0].mean()), "n": int(len(kern_t))},
                              "combine_and_gaps_us": t_attn - k_attn,
                              "launch": ob.ouro_verify_attn_plan(q, k_blk, max_seqlen, plan=attn_plan),
                              "whole_call_is": "main kernel + the launch that merges the chunk partials (when a sequence spans several chunks)"})
    r_lm = kernel_roofline("lmhead", cfg, k_lm, t_lm, lmhead_algorithmic_bytes(cfg), lmhead_flops(cfg),
                           traffic.get("lmhead_bytes"), peaks,
                           {**samples, "kernel_us_std": float(kern_i[:, 1].std()),
                            "kernel_us_in_timed_region": {"mean": float(kern_t[:, 1].mean()), "n": int(len(kern_t))},
                            "whole_call_is": "main kernel + the cross-slab arg-max launch"})
    rec = {
        "workload": workload, "dtype": cfg.dtype, "rows": cfg.R, "step_us": ms_step * 1e3,
        "tokens_per_s": cfg.R / (ms_step * 1e-3), "steps": steps, "warmup": warmup,
        "step_us_same_copy_every_step": unrot_us,
        "call_us": {"ouro_verify_attn": t_attn, "ouro_lmhead_argmax": t_lm, "ouro_accept": t_acc},
        "attn": r_attn, "lmhead": r_lm,
        "accepted_per_sequence": acc_out["n_accept"].cpu().tolist()[:16],
    }
    extras = {"cfg": cfg, "ms_step": ms_step, "graph_us": graph_us, "layer": layer, "large_r": large_r, "cpu": cpu,
              "total_rows": total_rows, "nrot": nrot, "every": every}
    del kcs, vcs, ws, d_attn, d_lm
    torch.cuda.empty_cache()
    return rec, extras


def brief(rec):
    """The per_config form of a workload record: step time and both main kernels' fractions."""
    def k(r):
        return {"kernel": r["kernel"].split(" ")[0], "bound": r["bound"], "kernel_us": r["kernel_us"],
                "whole_call_us": r["whole_call_us"], "frac": r["frac"], "frac_whole_call": r["frac_whole_call"],
                "frac_of_measured_peak": r["frac_of_measured_peak"], "hbm_frac": r["hbm_frac"], "mfma_frac": r["mfma_frac"]}
    return {"workload": rec["workload"], "dtype": rec["dtype"], "rows": rec["rows"], "step_us": rec["step_us"],
            "tokens_per_s": rec["tokens_per_s"], "step_us_same_copy_every_step": rec["step_us_same_copy_every_step"],
            "attn": k(rec["attn"]), "lmhead": k(rec["lmhead"]),
            "accept_call_us": rec["call_us"]["ouro_accept"]}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (use --gpus 1)." % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2402_13720_amd import binding as ob, workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    hip = Hip()
    peaks = measured_peaks(ob, torch, hip)

    # the other workloads first (their launches also bring the clocks up), the headline workload last
    per_config = {}
    if not args.no_per_config:
        for cid in sorted(W.CONFIGS):
            if cid != args.config:
                rec, _ = run_config(cid, args, ob, W, torch, hip, peaks, headline=False)
                per_config[cid] = brief(rec)
    rec, x = run_config(args.config, args, ob, W, torch, hip, peaks, headline=True)
    per_config[args.config] = brief(rec)
    cfg = x["cfg"]

    # the roofline object names the kernel that takes the largest share of the step; the other one sits beside it
    dom, other = ("attn", "lmhead") if rec["attn"]["kernel_us"] >= rec["lmhead"]["kernel_us"] else ("lmhead", "attn")
    result = {
        "metric": "draft tokens verified per second (one verification step: attention + LM head/argmax + accept)",
        "value": rec["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": x["ms_step"],
        "verify_step_latency_us": x["ms_step"] * 1e3,
        "graph_replay_step_latency_us": x["graph_us"],
        "step_latency_us_same_copy_every_step": rec["step_us_same_copy_every_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": rec["workload"], "B": cfg.B, "T": cfg.T, "gamma": cfg.gamma, "K": cfg.K, "beta": cfg.beta_p,
                   "Hq": cfg.Hq, "Hkv": cfg.Hkv, "D": cfg.D, "cache_rows": x["total_rows"], "V": cfg.V,
                   "branch": args.branch, "rotated_copies": x["nrot"], "events_on_every_nth_timed_step": x["every"],
                   "settle_steps_before_warmup": max(0, args.settle_steps),
                   "w_layout": args.w_layout if cfg.dtype == "bf16" else "row", "kv_layout": args.kv_layout},
        "call_us": rec["call_us"],
        "roofline": rec[dom],
        "roofline_other_kernel": rec[other],
        "measured_peaks": peaks,
        "per_config": [per_config[c] for c in sorted(per_config)],
        "layer": x["layer"],
        "lmhead_large_R": x["large_r"],
        "cpu_baseline": x["cpu"],
        "accepted_per_sequence": rec["accepted_per_sequence"],
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
