"""Pins for the oracle's chained verification step (no GPU): the wiring between its stages."""
import numpy as np
import torch

from oracle import verify_oracle as O
from paper_2402_13720_amd import workloads as W
from golden_io import meta_from_layout


def _inputs(cfg, seed, branch):
    inp = W.make_attention_inputs(cfg, seed, branch=branch)
    return inp, int(inp["cu_seqlens"][1])


def test_planted_greedy_tokens_through_a_library_attention():
    """K = 0 is plain speculative decoding: the block is causal after the prefix, so a library SDPA with an explicit
    mask gives every row's hidden state.  Planting w[v_r] = hidden_r / |hidden_r| makes v_r the greedy token of row r
    (Cauchy-Schwarz: no other unit vector scores higher), so the chain's arg-max must return the planted ids: this
    fails if the heads are laid side by side in the wrong order, if rows and sequences are swapped, or if the LM head
    is fed anything but the attention output."""
    cfg = W.scaled(W.CONFIGS[1], B=3, Hq=4, Hkv=2, D=16, L=(5, 9), gamma=6, K=0, beta_p=0, V=40)
    inp = W.make_attention_inputs(cfg, 11)
    B, T, Hq, D, G = cfg.B, cfg.T, cfg.Hq, cfg.D, cfg.Hq // cfg.Hkv
    hidden = np.zeros((B * T, Hq * D))
    for b in range(B):
        lo, hi = int(inp["cu_seqlens"][b]), int(inp["cu_seqlens"][b + 1])
        L = hi - lo
        mask = torch.ones(T, L + T, dtype=torch.bool)
        mask[:, L:] = torch.tril(torch.ones(T, T, dtype=torch.bool))
        for h in range(Hq):
            k = torch.from_numpy(np.concatenate([inp["k_cache"][lo:hi, h // G], inp["k_blk"][b, :, h // G]])).double()
            v = torch.from_numpy(np.concatenate([inp["v_cache"][lo:hi, h // G], inp["v_blk"][b, :, h // G]])).double()
            q = torch.from_numpy(inp["q"][b, :, h]).double()
            o = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], attn_mask=mask[None])[0]
            hidden[b * T:(b + 1) * T, h * D:(h + 1) * D] = o.numpy()
    rng = np.random.default_rng(3)
    plant = rng.permutation(cfg.V)[:B * T]
    w = rng.standard_normal((cfg.V, Hq * D)) * 1e-3
    w[plant] = hidden / np.linalg.norm(hidden, axis=1, keepdims=True)
    root = np.array([7, 8, 9])
    seen = {}

    def draft(amax):
        seen["amax"] = amax.copy()
        return np.stack([O.expected_tokens(amax[b], inp["pid"][b], inp["boff"][b], int(root[b])) for b in range(B)])

    r = O.verify_step(inp, w, draft, root, cfg.gamma, 0, 0)
    assert np.array_equal(r["lm"]["argmax"], plant)
    assert np.array_equal(seen["amax"], plant.reshape(B, T))
    assert np.allclose(r["hidden"], hidden, atol=1e-12)
    # the draft built from the chain's own greedy tokens is all-correct: fully accepted, bonus = the last row's token
    assert r["accept"]["n_accept"].tolist() == [cfg.gamma] * B
    assert r["accept"]["bonus"].tolist() == plant.reshape(B, T)[:, -1].tolist()


def test_all_correct_draft_is_fully_accepted_through_the_whole_chain():
    """The invariant the method rests on (Eq. (4)): a draft that agrees with the target everywhere is accepted to the end
    of the longest lengthened draft, gamma + beta' tokens with a phrase hanging off the last main token."""
    cfg = W.scaled(W.CONFIGS[1], B=2, L=(3, 40), V=200)
    inp = W.make_attention_inputs(cfg, 5, branch="last")
    w = W.make_lmhead_weight(cfg, 5)
    root = np.array([4, 150])
    r = O.verify_step(inp, w, lambda amax: np.stack(
        [O.expected_tokens(amax[b], inp["pid"][b], inp["boff"][b], int(root[b])) for b in range(cfg.B)]),
        root, cfg.gamma, cfg.K, cfg.beta_p)
    assert r["accept"]["n_accept"].tolist() == [cfg.gamma + cfg.beta_p] * cfg.B
    assert r["accept"]["path"].tolist() == [1, 1]
    # an array draft is taken as it is, and a hidden_round hook is applied before the LM head
    tok = np.full((cfg.B, cfg.T), -5)
    r2 = O.verify_step(inp, w, tok, root, cfg.gamma, cfg.K, cfg.beta_p, hidden_round=lambda h: np.zeros_like(h))
    assert r2["accept"]["n_accept"].tolist() == [0, 0] and (r2["lm"]["argmax"] == 0).all()     # all logits tie at 0
