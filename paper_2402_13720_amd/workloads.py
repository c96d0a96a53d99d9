"""Seeded synthetic inputs for the Ouroboros verification step.

This module holds shapes and random-number recipes only: it draws tensors,
block layouts and token ids, and contains none of the method's arithmetic
(no visibility rule, no attention, no argmax, no acceptance).  Both the CPU
oracle's tests and the HIP path's tests/bench draw their inputs from here.

Block layout (Sec. 3.2, Eq. (7)): a verify block of T tokens is the main draft
of ``gamma`` tokens followed by K candidate phrases of ``beta_p`` tokens each
(``beta_p`` is the paper's beta-1: the phrase's first token equals the draft
token it hangs off and is not repeated), so T = gamma + K*beta_p.  Every block
token carries ``(phrase_id, branch_off)``: main token i has (0, i); a token of
phrase j (1-based) has (j, b_j) where b_j is the 0-based main-draft index the
phrase hangs off (the paper's own case is b_j = gamma-1 for every j).

All floating-point tensors are returned as float32 numpy arrays.  For the bf16
workloads every value is already rounded to the nearest bf16 (ties to even), so
a later cast to bf16 on the device is exact and the oracle sees the very same
numbers the kernels see.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple, Union

import numpy as np

BASE_SEED = 20240213


@dataclass(frozen=True)
class VerifyConfig:
    """One synthetic verify-step workload (shapes only)."""
    cfg_id: int
    name: str
    dtype: str                      # "f32" or "bf16"
    B: int                          # sequences
    Hq: int                         # query heads
    Hkv: int                        # key/value heads
    D: int                          # head dim
    L: Union[int, Tuple[int, int]]  # cache length, or inclusive (lo, hi) range drawn per sequence
    gamma: int                      # main draft length
    K: int                          # number of candidate phrases
    beta_p: int                     # tokens per phrase inside the block (paper's beta - 1)
    V: int                          # vocabulary

    @property
    def T(self) -> int:
        return self.gamma + self.K * self.beta_p

    @property
    def hidden(self) -> int:
        return self.Hq * self.D

    @property
    def R(self) -> int:
        return self.B * self.T


CONFIGS: Dict[int, VerifyConfig] = {
    1: VerifyConfig(1, "tiny-fp32", "f32", 1, 4, 4, 64, 128, 8, 2, 4, 1000),
    2: VerifyConfig(2, "llama2-7b-layer", "bf16", 1, 32, 32, 128, 2048, 16, 8, 6, 32000),
    3: VerifyConfig(3, "llama2-13b-layer", "bf16", 1, 40, 40, 128, 4096, 32, 16, 6, 32000),
    4: VerifyConfig(4, "llama2-70b-layer-gqa", "bf16", 1, 64, 8, 128, 4096, 16, 8, 6, 32000),
    5: VerifyConfig(5, "llama2-7b-batched-varlen", "bf16", 16, 32, 32, 128, (512, 8192), 8, 4, 6, 32000),
}


def seed_for(cfg_id: int, trial: int = 0) -> int:
    return BASE_SEED + 1000 * cfg_id + trial


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even), keep float32 storage."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _normal(rng: np.random.Generator, shape, std: float, bf16: bool) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return round_to_bf16(x) if bf16 else x


def draw_seqlens(cfg: VerifyConfig, rng: np.random.Generator) -> np.ndarray:
    if isinstance(cfg.L, tuple):
        lo, hi = cfg.L
        return rng.integers(lo, hi + 1, size=cfg.B).astype(np.int64)
    return np.full(cfg.B, int(cfg.L), dtype=np.int64)


def make_block_meta(cfg: VerifyConfig, rng: np.random.Generator,
                    branch: str = "uniform") -> Tuple[np.ndarray, np.ndarray]:
    """Per-token (phrase_id, branch_off), each int16 [B, T].

    branch = "uniform": b_j drawn uniformly from {0..gamma-1} per phrase;
    branch = "last":    b_j = gamma-1 for every phrase (the paper's own layout);
    branch = "any":     b_j drawn uniformly from {-1, 0..gamma-1}: -1 is a phrase that hangs off the last
                        cached token and sees no main token (parity sweeps only).
    """
    B, T, g, K, bp = cfg.B, cfg.T, cfg.gamma, cfg.K, cfg.beta_p
    pid = np.zeros((B, T), dtype=np.int16)
    boff = np.zeros((B, T), dtype=np.int16)
    for b in range(B):
        boff[b, :g] = np.arange(g, dtype=np.int16)
        for j in range(1, K + 1):
            lo = g + (j - 1) * bp
            if branch == "uniform":
                bj = int(rng.integers(0, g))
            elif branch == "last":
                bj = g - 1
            elif branch == "any":
                bj = int(rng.integers(-1, g))
            else:
                raise ValueError(branch)
            pid[b, lo:lo + bp] = j
            boff[b, lo:lo + bp] = bj
    return pid, boff


def make_attention_inputs(cfg: VerifyConfig, seed: int, branch: str = "uniform",
                          seqlens: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Q, cache K/V (packed per sequence), block K/V, metadata for one verify step.

    Layouts: q [B,T,Hq,D]; k_cache, v_cache [sum L_b, Hkv, D]; cu_seqlens [B+1]
    int64; k_blk, v_blk [B,T,Hkv,D]; pid, boff [B,T] int16.
    """
    ss = np.random.SeedSequence(seed)
    r_len, r_meta, r_q, r_kc, r_vc, r_kb, r_vb = (np.random.default_rng(s) for s in ss.spawn(7))
    bf16 = cfg.dtype == "bf16"
    if seqlens is None:
        seqlens = draw_seqlens(cfg, r_len)
    seqlens = np.asarray(seqlens, dtype=np.int64)
    assert seqlens.shape == (cfg.B,)
    cu = np.zeros(cfg.B + 1, dtype=np.int64)
    cu[1:] = np.cumsum(seqlens)
    total = int(cu[-1])
    pid, boff = make_block_meta(cfg, r_meta, branch)
    B, T, Hq, Hkv, D = cfg.B, cfg.T, cfg.Hq, cfg.Hkv, cfg.D
    return {
        "q": _normal(r_q, (B, T, Hq, D), 1.0, bf16),
        "k_cache": _normal(r_kc, (total, Hkv, D), 1.0, bf16),
        "v_cache": _normal(r_vc, (total, Hkv, D), 1.0, bf16),
        "cu_seqlens": cu,
        "k_blk": _normal(r_kb, (B, T, Hkv, D), 1.0, bf16),
        "v_blk": _normal(r_vb, (B, T, Hkv, D), 1.0, bf16),
        "pid": pid,
        "boff": boff,
    }


def make_lmhead_weight(cfg: VerifyConfig, seed: int) -> np.ndarray:
    """LM-head weight, physical layout [V, hidden] (row v = output embedding of token v), N(0, 0.02^2)."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x1A]))
    return _normal(rng, (cfg.V, cfg.hidden), 0.02, cfg.dtype == "bf16")


def make_hidden(cfg: VerifyConfig, seed: int, rows: Optional[int] = None) -> np.ndarray:
    """Stand-alone LM-head input [R, hidden] ~ N(0,1) (used when the LM head is exercised without attention)."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x2B]))
    return _normal(rng, (cfg.R if rows is None else rows, cfg.hidden), 1.0, cfg.dtype == "bf16")


def make_token_draws(cfg: VerifyConfig, seed: int) -> Dict[str, np.ndarray]:
    """Uniform draft ids [B,T], uniform root_pred [B], and the per-sequence choice of
    exactly floor(T/2) block positions whose id is to be overwritten by the caller with
    the value that position will be compared against (``plant_tokens``)."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 0x3C]))
    tok = rng.integers(0, cfg.V, size=(cfg.B, cfg.T)).astype(np.int32)
    root = rng.integers(0, cfg.V, size=cfg.B).astype(np.int32)
    chosen = np.zeros((cfg.B, cfg.T), dtype=bool)
    for b in range(cfg.B):
        chosen[b, rng.permutation(cfg.T)[: cfg.T // 2]] = True
    return {"tok": tok, "root_pred": root, "chosen": chosen}


def plant_tokens(tok: np.ndarray, chosen: np.ndarray, expected: np.ndarray) -> np.ndarray:
    """Copy ``expected`` (supplied by the caller) into the chosen positions of ``tok``."""
    out = tok.copy()
    out[chosen] = expected[chosen]
    return out.astype(np.int32)


def scaled(cfg: VerifyConfig, **kw) -> VerifyConfig:
    """A variant of a config with some fields replaced (for reduced-size parity cases)."""
    return replace(cfg, **kw)
