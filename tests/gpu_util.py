"""Helpers shared by the GPU parity tests: upload seeded host inputs, call the C ABI through the binding."""
import functools

import numpy as np
import torch

from paper_2402_13720_amd import workloads as W

DEV = "cuda:0"


def torch_dtype(cfg):
    return torch.bfloat16 if cfg.dtype == "bf16" else torch.float32


def upload_attention(cfg, inp, head_major=False):
    """head_major: the caches go up as [Hkv, rows, D] (a pure re-layout of the same values)."""
    from paper_2402_13720_amd import binding as ob
    dt = torch_dtype(cfg)
    t = {}
    for k in ("q", "k_cache", "v_cache", "k_blk", "v_blk"):
        t[k] = torch.from_numpy(inp[k]).to(DEV).to(dt).contiguous()
    if head_major:
        for k in ("k_cache", "v_cache"):
            t[k] = t[k].permute(1, 0, 2).contiguous()
    t["cu_seqlens"] = torch.from_numpy(inp["cu_seqlens"]).to(DEV)
    t["meta"] = ob.pack_meta(inp["pid"], inp["boff"]).to(DEV)
    t["max_seqlen"] = int(np.diff(inp["cu_seqlens"]).max()) if cfg.B else 0
    return t


def run_attention(cfg, inp, want_lse=True, max_seqlen=None, head_major=False, rw=0, chunk=0):
    """rw, chunk: force the bf16 kernel variant (row blocks per workgroup; 4 + 0x80: 4 row blocks with the four-wave
    kernel) and the keys per workgroup (0: heuristic)."""
    from paper_2402_13720_amd import binding as ob
    t = upload_attention(cfg, inp, head_major)
    lse = torch.full((cfg.B, cfg.Hq, cfg.T), float("nan"), dtype=torch.float32, device=DEV) if want_lse else None
    out = ob.ouro_verify_attn(t["q"], t["k_cache"], t["v_cache"], t["cu_seqlens"], t["k_blk"], t["v_blk"], t["meta"],
                              max_seqlen=t["max_seqlen"] if max_seqlen is None else max_seqlen, lse=lse,
                              head_major=head_major, plan=ob.plan_override(rw & 0x7f, chunk, bool(rw & 0x80)))
    torch.cuda.synchronize()
    return out, lse, t


@functools.lru_cache(maxsize=2)
def full_size_attention_case(cfg_id):
    """(inputs, oracle result on every head) of a workload at full size; kept so that tests of the same workload in
    several layouts pay for the inputs and the oracle once."""
    from oracle import verify_oracle as O
    cfg = W.CONFIGS[cfg_id]
    inp = W.make_attention_inputs(cfg, W.seed_for(cfg_id))
    ref = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"], inp["k_blk"], inp["v_blk"],
                             inp["pid"], inp["boff"])
    return inp, ref


def to_np64(x):
    return x.detach().float().cpu().numpy().astype(np.float64)


def attn_tol(cfg):
    # spec tolerances: max-abs 2e-2 for bf16 outputs, 1e-5 for fp32
    return 2e-2 if cfg.dtype == "bf16" else 1e-5
