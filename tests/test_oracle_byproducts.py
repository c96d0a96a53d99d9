"""Pins of the oracle's phrase-pool by-products (Sec. 3.3)."""
import re

import numpy as np
import pytest

from golden_io import meta_from_layout
from oracle import verify_oracle as O
from paper_2402_13720_amd import workloads as W


def _examples():
    import os
    from golden_io import GOLDEN, _clean
    out, cur = [], {}
    with open(os.path.join(GOLDEN, "pool_byproducts_example.txt")) as f:
        for ln in list(_clean(f)) + [""]:
            if not ln.strip():
                if cur:
                    out.append(cur)
                    cur = {}
                continue
            k, v = ln.split(":", 1)
            cur[k.strip()] = v.split()
    return out


def test_hand_worked_examples():
    for ex in _examples():
        gamma, K, bp = int(ex["gamma"][0]), int(ex["K"][0]), int(ex["beta_p"][0])
        pid, boff = meta_from_layout(gamma, K, bp, [int(x) for x in ex["branch"]])
        root = None if ex["root"][0] == "none" else int(ex["root"][0])
        ints = lambda k: np.array([int(x) for x in ex[k]])
        r = O.pool_byproducts_one(ints("tok"), ints("argmax"), pid, boff, root, gamma, K, bp)
        assert np.array_equal(r["match"], ints("match"))
        assert r["n_seg"] == int(ex["n_seg"][0])
        assert np.array_equal(r["seg_start"], ints("seg_start")) and np.array_equal(r["seg_len"], ints("seg_len"))
        assert np.array_equal(r["repaired"].ravel(), ints("repaired"))


@pytest.mark.parametrize("cfg_id", [1, 2, 5])
@pytest.mark.parametrize("with_root", [True, False])
def test_against_independent_restatements(cfg_id, with_root):
    """#Match is the sum of Eq. (10); segments are the '1+' runs of the match string after the first mismatch
    (regular-expression scan); repaired phrases restate expected_tokens, which has its own pins; the accepted
    length of the main draft is the position of the first 0."""
    cfg = W.scaled(W.CONFIGS[cfg_id], B=min(W.CONFIGS[cfg_id].B, 4))
    for trial in range(3):
        rng = np.random.default_rng(cfg_id * 100 + trial)
        pid, boff = W.make_block_meta(cfg, rng)
        argmax = rng.integers(0, 6, size=(cfg.B, cfg.T))           # few distinct ids: many chance matches
        tok = rng.integers(0, 6, size=(cfg.B, cfg.T))
        root = rng.integers(0, 6, size=cfg.B) if with_root else None
        got = O.pool_byproducts(tok, argmax, pid, boff, root, cfg.gamma, cfg.K, cfg.beta_p)
        acc = O.accept(tok, argmax, pid, boff, root, cfg.gamma, cfg.K, cfg.beta_p)
        for b in range(cfg.B):
            v = O.expected_tokens(argmax[b], pid[b], boff[b], None if root is None else int(root[b]))
            sm = "".join("1" if (v[i] == tok[b, i] or (i == 0 and root is None)) else "0" for i in range(cfg.gamma))
            assert got["match"][b, :cfg.gamma].sum() == sm.count("1") == acc["n_match"][b]
            A = len(sm) if "0" not in sm else sm.index("0")
            assert A == acc["main_A"][b]
            runs = [(A + m.start(), m.end() - m.start()) for m in re.finditer("1+", sm[A:])]
            assert got["n_seg"][b] == len(runs)
            assert [(int(s), int(l)) for s, l in zip(got["seg_start"][b], got["seg_len"][b]) if l > 0] == runs
            for o in range(cfg.K):
                lo = cfg.gamma + o * cfg.beta_p
                bo = int(boff[b, lo])
                assert got["repaired"][b, o, 0] == (tok[b, bo] if bo >= 0 else -1)
                assert np.array_equal(got["repaired"][b, o, 1:], v[lo:lo + cfg.beta_p])


def test_all_correct_and_all_wrong_drafts():
    cfg = W.CONFIGS[1]
    rng = np.random.default_rng(5)
    pid, boff = W.make_block_meta(cfg, rng)
    argmax = rng.integers(0, cfg.V, size=(1, cfg.T))
    v = O.expected_tokens(argmax[0], pid[0], boff[0], 7)
    r = O.pool_byproducts(v[None, :], argmax, pid, boff, np.array([7]), cfg.gamma, cfg.K, cfg.beta_p)
    assert r["match"].all() and r["n_seg"][0] == 0                     # nothing is discarded
    for o in range(cfg.K):                                             # a correct phrase is its own repair
        lo = cfg.gamma + o * cfg.beta_p
        assert np.array_equal(r["repaired"][0, o, 1:], v[lo:lo + cfg.beta_p])
    r = O.pool_byproducts(v[None, :] + 1, argmax, pid, boff, np.array([7]), cfg.gamma, cfg.K, cfg.beta_p)
    assert not r["match"].any() and r["n_seg"][0] == 0
