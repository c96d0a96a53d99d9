"""Pins for the oracle's softmax attention arithmetic (no GPU)."""
import math

import numpy as np
import torch

from oracle import verify_oracle as O
from paper_2402_13720_amd import workloads as W


def _brute(q, k, v, mask, scale):
    """Pure-Python definition, one scalar at a time."""
    T, D = q.shape
    N = k.shape[0]
    out = np.zeros((T, D))
    lse = np.zeros(T)
    for i in range(T):
        s = [sum(float(q[i, d]) * float(k[j, d]) for d in range(D)) * scale if mask[i, j] else None
             for j in range(N)]
        mx = max(x for x in s if x is not None)
        e = [math.exp(x - mx) if x is not None else 0.0 for x in s]
        den = sum(e)
        for d in range(D):
            out[i, d] = sum(e[j] * float(v[j, d]) for j in range(N)) / den
        lse[i] = mx + math.log(den)
    return out, lse


def test_masked_softmax_matches_scalar_brute_force():
    rng = np.random.default_rng(0)
    q, k, v = rng.standard_normal((5, 7)), rng.standard_normal((11, 7)), rng.standard_normal((11, 3 + 4))
    mask = rng.random((5, 11)) < 0.6
    mask[:, 0] = True
    o, l = O.masked_softmax_attention(q, k, v, mask, 0.37)
    bo, bl = _brute(q, k, v, mask, 0.37)
    np.testing.assert_allclose(o, bo, atol=1e-13)
    np.testing.assert_allclose(l, bl, atol=1e-13)


def test_full_path_matches_brute_force_on_config1_shape():
    cfg = W.scaled(W.CONFIGS[1], L=20, D=8)
    inp = W.make_attention_inputs(cfg, W.seed_for(1))
    res = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"],
                             inp["k_blk"], inp["v_blk"], inp["pid"], inp["boff"])
    mask = O.dense_mask(inp["pid"][0], inp["boff"][0], 20)
    for h in range(cfg.Hq):
        k = np.concatenate([inp["k_cache"][:, h], inp["k_blk"][0, :, h]])
        v = np.concatenate([inp["v_cache"][:, h], inp["v_blk"][0, :, h]])
        bo, bl = _brute(inp["q"][0, :, h], k, v, mask, 1.0 / math.sqrt(8))
        np.testing.assert_allclose(res["out"][0, :, h], bo, atol=1e-12)
        np.testing.assert_allclose(res["lse"][0, h], bl, atol=1e-12)


def test_default_scale_is_inverse_sqrt_head_dim_and_gqa_groups_consecutive_heads():
    """Library SDPA (default scale 1/sqrt(D)) with KV heads repeated explicitly per group."""
    cfg = W.scaled(W.CONFIGS[1], Hq=6, Hkv=2, D=16, L=13, gamma=4, K=0, beta_p=0)
    inp = W.make_attention_inputs(cfg, 21)
    res = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"],
                             inp["k_blk"], inp["v_blk"], inp["pid"], inp["boff"])["out"]
    k = np.concatenate([inp["k_cache"], inp["k_blk"][0]])          # [N, Hkv, D]
    v = np.concatenate([inp["v_cache"], inp["v_blk"][0]])
    k = np.repeat(k, 3, axis=1)                                     # head h <- kv head h // 3
    v = np.repeat(v, 3, axis=1)
    N, Tq = k.shape[0], 4
    mask = torch.ones(Tq, N, dtype=torch.bool).tril(diagonal=N - Tq)
    o = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(inp["q"][0]).double().permute(1, 0, 2)[None],
        torch.from_numpy(k).double().permute(1, 0, 2)[None],
        torch.from_numpy(v).double().permute(1, 0, 2)[None], attn_mask=mask)
    np.testing.assert_allclose(res[0], o[0].permute(1, 0, 2).numpy(), atol=1e-12)


def test_split_cache_merged_by_logsumexp_equals_unsplit():
    """Attention over two halves of the keys, merged with weights exp(lse_i - lse), equals the whole."""
    rng = np.random.default_rng(4)
    q, k, v = rng.standard_normal((6, 8)), rng.standard_normal((30, 8)), rng.standard_normal((30, 8))
    mask = np.ones((6, 30), bool)
    o, l = O.masked_softmax_attention(q, k, v, mask, 0.3)
    o1, l1 = O.masked_softmax_attention(q, k[:13], v[:13], mask[:, :13], 0.3)
    o2, l2 = O.masked_softmax_attention(q, k[13:], v[13:], mask[:, 13:], 0.3)
    lm = np.logaddexp(l1, l2)
    merged = o1 * np.exp(l1 - lm)[:, None] + o2 * np.exp(l2 - lm)[:, None]
    np.testing.assert_allclose(merged, o, atol=1e-13)
    np.testing.assert_allclose(lm, l, atol=1e-13)


def test_single_visible_key_returns_its_value_and_score_as_lse():
    q = np.array([[1.0, 2.0]])
    k = np.array([[3.0, -1.0], [100.0, 100.0]])
    v = np.array([[7.0, 8.0], [1e9, 1e9]])
    o, l = O.masked_softmax_attention(q, k, v, np.array([[True, False]]), 0.5)
    np.testing.assert_allclose(o, [[7.0, 8.0]])
    np.testing.assert_allclose(l, [0.5 * (3.0 - 2.0)])


def test_two_keys_closed_form():
    """softmax over two scores a, b is the logistic function of their difference."""
    q = np.array([[2.0]])
    k = np.array([[1.0], [-0.5]])
    v = np.array([[1.0], [0.0]])
    o, _ = O.masked_softmax_attention(q, k, v, np.ones((1, 2), bool), 1.0)
    np.testing.assert_allclose(o[0, 0], 1.0 / (1.0 + math.exp(-(2.0 - (-1.0)))), atol=1e-15)
