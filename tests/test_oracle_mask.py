"""Pins for the oracle's block visibility and masked attention (no GPU).

The masked single pass must reproduce verifying the K lengthened drafts one by one
(Sec. 3.2): each pin below is independent of the oracle's own ancestor walk.
"""
import numpy as np
import pytest
import torch

from oracle import verify_oracle as O
from paper_2402_13720_amd import workloads as W
from golden_io import load_mask, meta_from_layout


@pytest.mark.parametrize("name", ["mask_paper_layout_g3_K2_b2.txt",
                                  "mask_branch_offsets_g4_K2_b2.txt",
                                  "mask_root_branch_g2_K1_b3.txt"])
def test_visibility_matches_handwritten_mask(name):
    gamma, K, bp, branch, want = load_mask(name)
    pid, boff = meta_from_layout(gamma, K, bp, branch)
    got = O.block_visibility(pid, boff)
    assert got.shape == want.shape
    assert np.array_equal(got, want)
    full = O.dense_mask(pid, boff, 5)
    assert full[:, :5].all() and np.array_equal(full[:, 5:], want)


def _sdpa_causal_with_prefix(q, k, v):
    """Library routine: causal attention of the last len(q) positions of a linear sequence of len(k)."""
    Tq, N = q.shape[0], k.shape[0]
    mask = torch.ones(Tq, N, dtype=torch.bool).tril(diagonal=N - Tq)
    o = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None].double(), torch.from_numpy(k)[None, None].double(),
        torch.from_numpy(v)[None, None].double(), attn_mask=mask[None, None])
    return o[0, 0].numpy()


@pytest.mark.parametrize("branch_mode", ["uniform", "last"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_masked_pass_equals_one_by_one_causal_verification(branch_mode, seed):
    """Enumeration pin: linearise each lengthened draft [cache, main 0..b_j, phrase j] and run
    ordinary causal attention on it; every block row of the masked pass must equal its row there."""
    cfg = W.scaled(W.CONFIGS[1], B=2, Hq=4, Hkv=2, D=16, L=(3, 40), gamma=5, K=3, beta_p=4)
    inp = W.make_attention_inputs(cfg, 100 + seed, branch=branch_mode)
    res = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"],
                             inp["k_blk"], inp["v_blk"], inp["pid"], inp["boff"])
    G = cfg.Hq // cfg.Hkv
    for b in range(cfg.B):
        lo, hi = inp["cu_seqlens"][b], inp["cu_seqlens"][b + 1]
        for h in range(cfg.Hq):
            g = h // G
            kc, vc = inp["k_cache"][lo:hi, g], inp["v_cache"][lo:hi, g]
            kb, vb, qb = inp["k_blk"][b, :, g], inp["v_blk"][b, :, g], inp["q"][b, :, h]
            # the main draft alone
            rows = list(range(cfg.gamma))
            want = _sdpa_causal_with_prefix(qb[rows], np.concatenate([kc, kb[rows]]),
                                            np.concatenate([vc, vb[rows]]))
            np.testing.assert_allclose(res["out"][b, rows, h], want, rtol=0, atol=1e-12)
            for j in range(1, cfg.K + 1):
                p0 = cfg.gamma + (j - 1) * cfg.beta_p
                bj = int(inp["boff"][b, p0])
                rows = list(range(bj + 1)) + list(range(p0, p0 + cfg.beta_p))
                want = _sdpa_causal_with_prefix(qb[rows], np.concatenate([kc, kb[rows]]),
                                                np.concatenate([vc, vb[rows]]))
                np.testing.assert_allclose(res["out"][b, rows, h], want, rtol=0, atol=1e-12)


def test_probe_zero_queries_onehot_values_recover_the_mask():
    """Q = 0 gives a uniform softmax over the visible keys; with V = one-hot(key index) the
    output times the number of visible keys is the mask row itself (closed form)."""
    gamma, K, bp, branch, want = load_mask("mask_branch_offsets_g4_K2_b2.txt")
    pid, boff = meta_from_layout(gamma, K, bp, branch)
    T, L = gamma + K * bp, 6
    N = L + T
    q = np.zeros((1, T, 1, N), np.float32)
    rng = np.random.default_rng(3)
    kc = rng.standard_normal((L, 1, N)).astype(np.float32)
    kb = rng.standard_normal((1, T, 1, N)).astype(np.float32)
    eye = np.eye(N, dtype=np.float32)
    res = O.verify_attention(q, kc, eye[:L, None, :], np.array([0, L]), kb, eye[None, L:, None, :],
                             pid[None], boff[None])
    out = res["out"][0, :, 0, :]
    nvis = L + want.sum(axis=1)
    rec = out * nvis[:, None]
    np.testing.assert_allclose(rec[:, :L], 1.0, atol=1e-12)
    np.testing.assert_allclose(rec[:, L:], want.astype(float), atol=1e-12)
    np.testing.assert_allclose(res["lse"][0, 0], np.log(nvis), atol=1e-12)


def test_rows_sum_to_one_and_phrases_are_independent():
    cfg = W.scaled(W.CONFIGS[1], B=1, Hq=2, Hkv=2, D=8, L=9, gamma=4, K=3, beta_p=3)
    inp = W.make_attention_inputs(cfg, 7)
    ones_c, ones_b = np.ones_like(inp["v_cache"]), np.ones_like(inp["v_blk"])
    r = O.verify_attention(inp["q"], inp["k_cache"], ones_c, inp["cu_seqlens"], inp["k_blk"], ones_b,
                           inp["pid"], inp["boff"])
    np.testing.assert_allclose(r["out"], 1.0, atol=1e-13)
    base = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"],
                              inp["k_blk"], inp["v_blk"], inp["pid"], inp["boff"])["out"]
    # perturb everything belonging to phrase 2: no row outside phrase 2 may change
    sel = inp["pid"][0] == 2
    p = {k: v.copy() for k, v in inp.items()}
    for key in ("q", "k_blk", "v_blk"):
        p[key][0, sel] += 3.0
    pert = O.verify_attention(p["q"], p["k_cache"], p["v_cache"], p["cu_seqlens"], p["k_blk"], p["v_blk"],
                              p["pid"], p["boff"])["out"]
    assert np.array_equal(pert[0, ~sel], base[0, ~sel])
    assert not np.allclose(pert[0, sel], base[0, sel])


def test_cache_permutation_invariance():
    cfg = W.scaled(W.CONFIGS[1], B=1, Hq=2, Hkv=1, D=8, L=17, gamma=3, K=2, beta_p=2)
    inp = W.make_attention_inputs(cfg, 11)
    base = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"],
                              inp["k_blk"], inp["v_blk"], inp["pid"], inp["boff"])["out"]
    perm = np.random.default_rng(0).permutation(17)
    out = O.verify_attention(inp["q"], inp["k_cache"][perm], inp["v_cache"][perm], inp["cu_seqlens"],
                             inp["k_blk"], inp["v_blk"], inp["pid"], inp["boff"])["out"]
    np.testing.assert_allclose(out, base, atol=1e-13)


def test_single_phrase_off_single_main_token_is_plain_causal():
    """gamma = 1, K = 1, branch 0: the whole block is one linear sequence (spec invariant)."""
    cfg = W.scaled(W.CONFIGS[1], B=1, Hq=1, Hkv=1, D=8, L=5, gamma=1, K=1, beta_p=6)
    inp = W.make_attention_inputs(cfg, 5)
    assert inp["boff"][0, 1] == 0
    assert np.array_equal(O.block_visibility(inp["pid"][0], inp["boff"][0]), np.tril(np.ones((7, 7), bool)))
    out = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"],
                             inp["k_blk"], inp["v_blk"], inp["pid"], inp["boff"])["out"]
    want = _sdpa_causal_with_prefix(inp["q"][0, :, 0], np.concatenate([inp["k_cache"][:, 0], inp["k_blk"][0, :, 0]]),
                                    np.concatenate([inp["v_cache"][:, 0], inp["v_blk"][0, :, 0]]))
    np.testing.assert_allclose(out[0, :, 0], want, atol=1e-12)


def test_no_phrases_is_speculative_decoding_causal_mask():
    cfg = W.scaled(W.CONFIGS[1], gamma=6, K=0, beta_p=0)
    pid, boff = W.make_block_meta(cfg, np.random.default_rng(0))
    assert np.array_equal(O.block_visibility(pid[0], boff[0]), np.tril(np.ones((6, 6), bool)))


def test_empty_cache_rows_still_see_themselves():
    cfg = W.scaled(W.CONFIGS[1], B=2, L=(0, 0), gamma=2, K=1, beta_p=2, Hq=1, Hkv=1, D=4)
    inp = W.make_attention_inputs(cfg, 9)
    r = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"],
                           inp["k_blk"], inp["v_blk"], inp["pid"], inp["boff"])
    assert np.isfinite(r["out"]).all()
    np.testing.assert_allclose(r["out"][:, 0, 0], inp["v_blk"][:, 0, 0].astype(np.float64), atol=1e-13)
