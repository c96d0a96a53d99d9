"""CPU oracle for the rest of the verifying layer around the draft-block attention.  TEST INFRASTRUCTURE ONLY.

The paper verifies a draft block with ONE forward pass of the target model (Sec. 3.2); it is silent on the layer
itself, which is the target model's (Llama-2 in Sec. 4).  What the paper does fix is the position every block token
must be given: each lengthened draft of Eq. (7) is an ordinary linear sequence, so a token's position is the
number of tokens before it in ITS OWN draft -- the cached prefix plus its ancestors in the block -- not its index
in the block.  The other operations are the published Llama-2 formulation (RMSNorm, rotary embedding in the
rotate-half form, SwiGLU MLP), written out plainly in fp64.

Shares no code with the HIP library; only tests may import it.  Pins: tests/test_oracle_layer.py (positions
against the linearised drafts and the visibility row sums; rotary embedding against complex multiplication, norm
preservation and the relative-position property; RMSNorm and SiLU against closed forms; the projections against a
library matmul).  No function here is "parity unpinned".
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from oracle import verify_oracle as V


def block_depth(pid: np.ndarray, boff: np.ndarray) -> np.ndarray:
    """depth[t] = number of block tokens that precede t in its own lengthened draft (its ancestors)."""
    par = V.parents(pid, boff)
    T = par.shape[0]
    depth = np.zeros(T, dtype=np.int64)
    for t in range(T):
        n, u = 0, par[t]
        while u != V.ROOT:
            n += 1
            u = par[u]
        depth[t] = n
    return depth


def block_positions(pid: np.ndarray, boff: np.ndarray, seq_len: np.ndarray) -> np.ndarray:
    """pos[b, t] = seq_len[b] + depth of token t: its index in the linear sequence [prefix, ancestors, t]."""
    B = pid.shape[0]
    return np.stack([int(seq_len[b]) + block_depth(pid[b], boff[b]) for b in range(B)])


def rope(x: np.ndarray, pos: np.ndarray, base: float = 10000.0) -> np.ndarray:
    """Rotary position embedding, rotate-half form: x [B,T,H,D], pos [B,T].  Pair (x[i], x[i+D/2]) is rotated by
    the angle pos * base^(-2i/D)."""
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[-1]
    half = D // 2
    inv = base ** (-2.0 * np.arange(half) / D)
    ang = np.asarray(pos, dtype=np.float64)[:, :, None, None] * inv            # [B,T,1,half]
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * g over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=np.float64)


def linear(x: np.ndarray, w: np.ndarray, residual: Optional[np.ndarray] = None) -> np.ndarray:
    """out[r, n] = sum_k x[r, k] * w[n, k] (+ residual[r, n]); w is [out features, in features]."""
    out = np.zeros((x.shape[0], w.shape[0]), dtype=np.float64)
    xs, ws = np.asarray(x, dtype=np.float64), np.asarray(w, dtype=np.float64)
    for r in range(xs.shape[0]):
        out[r] = (ws * xs[r][None, :]).sum(axis=1)
    if residual is not None:
        out = out + np.asarray(residual, dtype=np.float64)
    return out


def silu_mul(gate_up: np.ndarray) -> np.ndarray:
    """[R, 2F] -> [R, F]: silu(gate) * up with gate = first F columns, up = last F; silu(z) = z / (1 + exp(-z))."""
    gu = np.asarray(gate_up, dtype=np.float64)
    F = gu.shape[1] // 2
    g, u = gu[:, :F], gu[:, F:]
    return g / (1.0 + np.exp(-g)) * u
