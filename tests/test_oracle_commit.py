"""Pins of the oracle's commit of accepted tokens and of its cache-with-room attention option."""
import numpy as np
import pytest

from golden_io import load_commit_examples
from oracle import verify_oracle as O
from paper_2402_13720_amd import workloads as W


def _roomy(cfg, inp, room, rng):
    """Re-lay a packed cache into regions with `room` spare rows per sequence (spare rows hold noise)."""
    lens = np.diff(inp["cu_seqlens"]).astype(np.int64)
    cu = np.concatenate([[0], np.cumsum(lens + room)]).astype(np.int64)
    shape = (int(cu[-1]),) + inp["k_cache"].shape[1:]
    k = rng.standard_normal(shape).astype(np.float32)
    v = rng.standard_normal(shape).astype(np.float32)
    for b in range(cfg.B):
        lo = int(inp["cu_seqlens"][b])
        k[cu[b]:cu[b] + lens[b]] = inp["k_cache"][lo:lo + lens[b]]
        v[cu[b]:cu[b] + lens[b]] = inp["v_cache"][lo:lo + lens[b]]
    return k, v, cu, lens


def test_commit_matches_the_hand_worked_example():
    for ex in load_commit_examples("kv_commit_example.txt"):
        B = len(ex["seq_len"])
        kc = ex["k_cache"].astype(np.float64).reshape(-1, 1, 1)
        k_blk = np.stack([ex["k_blk%d" % b] for b in range(B)]).astype(np.float64)[:, :, None, None]
        idx = np.stack([ex["idx%d" % b] for b in range(B)])
        r = O.kv_commit(kc, -kc, ex["cu"], ex["seq_len"], k_blk, -k_blk, idx, ex["n_accept"])
        assert np.array_equal(r["k_cache"].ravel(), ex["want_k"])
        assert np.array_equal(r["v_cache"].ravel(), -ex["want_k"])
        assert np.array_equal(r["seq_len"], ex["want_len"])
        assert np.array_equal(r["overflow"], ex["want_overflow"])


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_commit_equals_concatenation_with_library_routines(seed):
    """Per sequence the new cached tokens are concatenate(old tokens, block rows taken at the accepted indices)."""
    rng = np.random.default_rng(seed)
    cfg = W.scaled(W.CONFIGS[1], B=3, L=(0, 40))
    inp = W.make_attention_inputs(cfg, 50 + seed)
    k, v, cu, lens = _roomy(cfg, inp, room=cfg.gamma + cfg.beta_p, rng=rng)
    n_acc = rng.integers(0, cfg.gamma + cfg.beta_p + 1, size=cfg.B)
    idx = np.full((cfg.B, cfg.gamma + cfg.beta_p), -1, dtype=np.int32)
    for b in range(cfg.B):
        idx[b, :n_acc[b]] = rng.choice(cfg.T, size=n_acc[b], replace=False)
    r = O.kv_commit(k, v, cu, lens, inp["k_blk"], inp["v_blk"], idx, n_acc)
    assert not r["overflow"].any()
    for b in range(cfg.B):
        want_k = np.concatenate([k[cu[b]:cu[b] + lens[b]], np.take(inp["k_blk"][b], idx[b, :n_acc[b]], axis=0)])
        want_v = np.concatenate([v[cu[b]:cu[b] + lens[b]], np.take(inp["v_blk"][b], idx[b, :n_acc[b]], axis=0)])
        got = slice(int(cu[b]), int(cu[b] + r["seq_len"][b]))
        assert r["seq_len"][b] == lens[b] + n_acc[b]
        assert np.array_equal(r["k_cache"][got], want_k) and np.array_equal(r["v_cache"][got], want_v)
        spare = slice(int(cu[b] + r["seq_len"][b]), int(cu[b + 1]))
        assert np.array_equal(r["k_cache"][spare], k[spare]) and np.array_equal(r["v_cache"][spare], v[spare])
    assert r["k_cache"] is not k and r["v_cache"] is not v          # the inputs are not modified in place


def test_attention_ignores_the_unused_room_of_a_region():
    """seq_len option: attention over regions with spare rows equals attention over the packed cache."""
    rng = np.random.default_rng(3)
    cfg = W.scaled(W.CONFIGS[1], B=3, L=(0, 40))
    inp = W.make_attention_inputs(cfg, 60)
    k, v, cu, lens = _roomy(cfg, inp, room=5, rng=rng)
    a = O.verify_attention(inp["q"], inp["k_cache"], inp["v_cache"], inp["cu_seqlens"], inp["k_blk"], inp["v_blk"],
                           inp["pid"], inp["boff"])
    b = O.verify_attention(inp["q"], k, v, cu, inp["k_blk"], inp["v_blk"], inp["pid"], inp["boff"], seq_len=lens)
    assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["lse"], b["lse"])


def test_committed_cache_gives_the_next_step_the_accepted_context():
    """After the accepted path of one step is committed, a one-token block of the next step must attend to the
    old cache followed by the accepted tokens in accepted order (Eq. (2): v_i is conditioned on x and the accepted
    v_1..i-1).  The expected value is a textbook softmax over that concatenation."""
    rng = np.random.default_rng(4)
    cfg = W.scaled(W.CONFIGS[1], B=2, L=(5, 30))
    inp = W.make_attention_inputs(cfg, 70)
    k, v, cu, lens = _roomy(cfg, inp, room=cfg.gamma + cfg.beta_p + 1, rng=rng)
    idx = np.full((cfg.B, cfg.gamma + cfg.beta_p), -1, dtype=np.int32)
    # sequence 0: whole main draft then phrase 1 (its block indices follow the main draft); sequence 1: main 0, 1
    idx[0, :cfg.gamma + cfg.beta_p] = np.arange(cfg.gamma + cfg.beta_p)
    idx[1, :2] = [0, 1]
    n_acc = np.array([cfg.gamma + cfg.beta_p, 2])
    r = O.kv_commit(k, v, cu, lens, inp["k_blk"], inp["v_blk"], idx, n_acc)
    # step 2: one new token per sequence (gamma = 1, no phrases)
    q2 = rng.standard_normal((cfg.B, 1, cfg.Hq, cfg.D))
    k2 = rng.standard_normal((cfg.B, 1, cfg.Hkv, cfg.D))
    v2 = rng.standard_normal((cfg.B, 1, cfg.Hkv, cfg.D))
    pid2 = np.zeros((cfg.B, 1), dtype=np.int16)
    boff2 = np.zeros((cfg.B, 1), dtype=np.int16)
    got = O.verify_attention(q2, r["k_cache"], r["v_cache"], cu, k2, v2, pid2, boff2, seq_len=r["seq_len"])["out"]
    G = cfg.Hq // cfg.Hkv
    for b in range(cfg.B):
        for h in range(cfg.Hq):
            g = h // G
            keys = np.concatenate([k[cu[b]:cu[b] + lens[b], g], inp["k_blk"][b, idx[b, :n_acc[b]], g], k2[b, :, g]])
            vals = np.concatenate([v[cu[b]:cu[b] + lens[b], g], inp["v_blk"][b, idx[b, :n_acc[b]], g], v2[b, :, g]])
            s = keys.astype(np.float64) @ q2[b, 0, h] / np.sqrt(cfg.D)
            p = np.exp(s - s.max())
            want = (p / p.sum()) @ vals.astype(np.float64)
            assert np.allclose(got[b, 0, h], want, rtol=1e-12, atol=1e-12)
